"""GPU parity of the share calls when the weight-side operands F and B_i are passed as digit
planes (``comet_open_weight_planes`` + ``COMET_WEIGHT_PLANES``): every output element against the
oracle's Eq. 1 on the same words, for both kinds of product, full-size and compact triple shares,
every tile shape of the matrix-core kernel, ragged sizes and spare block capacity; plus the plane
bytes themselves against the format the header documents."""
import sys

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

import oracle as co                                   # noqa: E402
from workloads import rng                             # noqa: E402


def say(msg):
    print("[gpu-planes] " + msg, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def ctx():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2505_07239_amd as comet
    c = comet.Context(0)
    yield c
    c.close()


def up(a):
    return torch.from_numpy(np.ascontiguousarray(a).view(np.int64)).cuda()


def down(t):
    return t.cpu().numpy().view(np.uint64)


def u64(seed, stream, *shape):
    return rng.uniform_u64(seed, stream, int(np.prod(shape))).reshape(shape)


def planes_by_definition(w):
    """The documented format, written out on the host: signed base-256 digits d_t of every word
    (x = sum d_t 2^(8t) mod 2^64, d_t in [-128, 127]); unit (s, t, g, c) = digit t of rows
    32 s + 16 g + 0..15 of column c, units ordered (s, c / 64, t, g, c % 64); rows beyond k are
    zero.  Returns the bytes and a mask of the bytes that belong to real columns (the padding of
    the last chunk is never written)."""
    k, n = w.shape
    ks, nch = (k + 31) // 32, (n + 63) // 64
    pad = np.zeros((ks * 32, nch * 64), np.uint64)
    pad[:k, :n] = w
    out = np.zeros((ks, nch, 8, 2, 64, 16), np.int8)
    rest = pad.copy()
    for t in range(8):
        d = (rest & np.uint64(0xFF)).astype(np.uint8).view(np.int8)          # signed residue mod 256
        rest = (rest - d.astype(np.int64).view(np.uint64)) >> np.uint64(8)   # exact: removes the digit, carries
        # d[32 s + 16 g + i, 64 ch + c] -> out[s, ch, t, g, c, i]
        out[:, :, t] = d.reshape(ks, 2, 16, nch, 64).transpose(0, 3, 1, 4, 2)
    real = np.zeros((ks, nch, 8, 2, 64, 16), bool)
    real.reshape(ks, nch, 8, 2, 64 * 16)[...] = (np.arange(nch * 64).reshape(nch, 1, 1, 64) < n).repeat(16, axis=-1)
    return out.reshape(-1).view(np.uint8), real.reshape(-1)


def test_plane_bytes_follow_the_documented_format(ctx):
    import paper_2505_07239_amd as comet
    for seed, (k, n) in enumerate([(64, 40), (33, 7), (130, 300), (16, 64), (1, 1)]):
        g0, g1 = u64(70 + seed, 1, k, n), u64(70 + seed, 2, k, n)
        g0[0, 0] = np.uint64(0x8080808080808080)                  # all digits -128 after the carries
        g1[0, 0] = 0
        say("plane bytes k=%d n=%d" % (k, n))
        both = ctx.open_weight_planes(up(g0), up(g1))
        single = ctx.open_weight_planes(up(g0))
        torch.cuda.synchronize()
        need = comet.binding.load_library().comet_weight_planes_bytes(k, n)
        assert need == (k + 31) // 32 * 32 * ((n + 63) // 64 * 64) * 8
        for got, words in ((both, co.open_(g0, g1)), (single, g0)):
            want, real = planes_by_definition(words)
            assert len(want) == need
            assert np.array_equal(got.buf.cpu().numpy()[:need][real], want[real])


@pytest.mark.parametrize("k,n", [(64, 64), (33, 7), (130, 300), (16, 65), (1, 1), (257, 129), (4096, 96), (31, 200)])
def test_plane_bytes_from_neuron_major_operands(ctx, k, n):
    """Operands stored one row per column of the matrix give the planes of the row-major call on
    their transposes, byte for byte (both shares, one share; odd k takes the word-by-word loads)."""
    import paper_2505_07239_amd as comet
    g0, g1 = u64(75, k + n, k, n), u64(76, k + n, k, n)
    t0, t1 = up(np.ascontiguousarray(g0.T)), up(np.ascontiguousarray(g1.T))
    say("plane bytes from neuron-major operands k=%d n=%d" % (k, n))
    need = comet.binding.load_library().comet_weight_planes_bytes(k, n)
    for pair in ((0, 1), (0,)):
        want = ctx.open_weight_planes(up(g0), up(g1) if len(pair) == 2 else None)
        fill = torch.full((max(need, 16),), 0x5A, dtype=torch.uint8, device="cuda")
        got = ctx.open_weight_planes(t0, t1 if len(pair) == 2 else None, out=fill, neuron_major=True)
        torch.cuda.synchronize()
        assert got.shape == (k, n)
        _, real = planes_by_definition(co.open_(g0, g1) if len(pair) == 2 else g0)
        assert np.array_equal(got.buf.cpu().numpy()[:need][real], want.buf.cpu().numpy()[:need][real])
        # the padding of the last chunk is never written
        assert np.all(got.buf.cpu().numpy()[:need][~real] == 0x5A)


def _case(seed, kind, m, k, n, bs, kept, cap_extra=0):
    """Random words for one share call.  SOMM: n = number of neurons (columns of B_i), SIMM: k =
    number of neurons (rows of B_i).  Returns host arrays, index list and the oracle result."""
    idx = np.array(sorted(kept), dtype=np.int32)
    t = len(idx)
    cap = t + cap_extra
    kc = t * bs
    if kind == "somm":
        e, a = u64(seed, 1, m, k), [u64(seed, 2 + i, m, k) for i in (0, 1)]
        f, b = u64(seed, 4, k, kc), [u64(seed, 5 + i, k, n) for i in (0, 1)]
        c = [u64(seed, 7 + i, m, kc) for i in (0, 1)]
        a_sel = a
        b_sel = [co.index_cols(v, idx, bs) for v in b]
    else:
        e, a = u64(seed, 1, m, kc), [u64(seed, 2 + i, m, k) for i in (0, 1)]
        f, b = u64(seed, 4, kc, n), [u64(seed, 5 + i, k, n) for i in (0, 1)]
        c = [u64(seed, 7 + i, m, n) for i in (0, 1)]
        a_sel = [co.index_cols(v, idx, bs) for v in a]
        b_sel = [co.index_rows(v, idx, bs) for v in b]
    want = [co.beaver_share(i, e, f, a_sel[i], b_sel[i], c[i]) for i in (0, 1)]
    return dict(kind=kind, m=m, k=k, n=n, bs=bs, idx=idx, t=t, cap=cap, e=e, f=f, a=a, b=b, c=c,
                a_sel=a_sel, b_sel=b_sel, want=want)


def _pad(arr, shape, seed):
    out = u64(seed, 99, *shape)                     # junk where nothing may be read
    out[:arr.shape[0], :arr.shape[1]] = arr
    return out


SENTINEL = np.uint64(0x0123456789ABCDEF)


def _run(ctx, cs, party, b_full):
    kind, m, bs, t, cap = cs["kind"], cs["m"], cs["bs"], cs["t"], cs["cap"]
    ld, kc = cap * bs, t * bs
    gi = torch.zeros(max(cap, 1), dtype=torch.int32, device="cuda")
    gi[:t] = torch.from_numpy(cs["idx"]).cuda()
    n_dev = torch.tensor([t], dtype=torch.int32, device="cuda")
    seed = 500 + m
    if kind == "somm":
        f_words = _pad(cs["f"], (cs["k"], ld), seed)
        b_words = cs["b"][party] if b_full else _pad(cs["b_sel"][party], (cs["k"], ld), seed + 1)
        c_words = _pad(cs["c"][party], (m, ld), seed + 2)
        f_pl, b_pl = ctx.open_weight_planes(up(f_words)), ctx.open_weight_planes(up(b_words))
        out = torch.full((m, ld), int(SENTINEL.view(np.int64)), dtype=torch.int64, device="cuda")
        z = ctx.somm_share(party, bs, gi, n_dev, cap, up(cs["e"]), f_pl, up(cs["a"][party]), b_pl, up(c_words),
                           b_full=b_full, out=out)
        torch.cuda.synchronize()
        got = down(z)
        assert np.array_equal(got[:, :kc], cs["want"][party])
        assert np.all(got[:, kc:] == SENTINEL)
    else:
        e_words = _pad(cs["e"], (m, ld), seed)
        f_words = _pad(cs["f"], (ld, cs["n"]), seed + 1)
        b_words = cs["b"][party] if b_full else _pad(cs["b_sel"][party], (ld, cs["n"]), seed + 2)
        a_words = cs["a"][party] if b_full else _pad(cs["a_sel"][party], (m, ld), seed + 3)
        f_pl, b_pl = ctx.open_weight_planes(up(f_words)), ctx.open_weight_planes(up(b_words))
        z = ctx.simm_share(party, bs, gi, n_dev, cap, up(e_words), f_pl, up(a_words), b_pl, up(cs["c"][party]),
                           a_full=b_full, b_full=b_full)
        torch.cuda.synchronize()
        assert np.array_equal(down(z), cs["want"][party])


# (m, contraction / neurons, other dimension, bs, kept blocks, spare capacity): every tile shape
# (m <= 32: 32 x 128, m <= 64: 64 x 64, else 128 x 64 or 64 x 64), ragged tails, one and several
# blocks per contraction step
SHAPES = [
    (5, 96, 8, (0, 3, 4, 9), 0), (20, 130, 16, (1, 2, 6), 1), (32, 64, 32, (0, 2), 0),
    (50, 200, 16, (0, 5, 6, 7, 11), 2), (64, 96, 48, (1, 3), 0),
    (100, 70, 64, (0, 2, 3), 0), (129, 256, 32, (1, 2, 3, 8, 9, 15), 1), (300, 512, 32, tuple(range(0, 30, 2)), 0),
    (260, 33, 16, (0, 1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 11, 12, 13, 14, 15, 16, 17, 18, 19, 20), 0),
]


@pytest.mark.parametrize("m,other,bs,kept,spare", SHAPES)
@pytest.mark.parametrize("b_full", [True, False])
def test_somm_share_with_weight_planes(ctx, m, other, bs, kept, spare, b_full):
    nb = max(kept) + 2
    cs = _case(700 + m, "somm", m, other, nb * bs, bs, kept, spare)
    for party in (0, 1):
        say("somm planes m=%d k=%d bs=%d blocks=%d b_full=%s party %d" % (m, other, bs, len(kept), b_full, party))
        _run(ctx, cs, party, b_full)


@pytest.mark.parametrize("m,other,bs,kept,spare", SHAPES)
@pytest.mark.parametrize("b_full", [True, False])
def test_simm_share_with_weight_planes(ctx, m, other, bs, kept, spare, b_full):
    if b_full and bs % 16:
        pytest.skip("planes of a full-size B_i are gathered in units of sixteen rows")
    nb = max(kept) + 2
    cs = _case(800 + m, "simm", m, nb * bs, other, bs, kept, spare)
    for party in (0, 1):
        say("simm planes m=%d n=%d bs=%d blocks=%d b_full=%s party %d" % (m, other, bs, len(kept), b_full, party))
        _run(ctx, cs, party, b_full)


# A decoding batch (m <= 32) on weight planes takes the kernel in which every wavefront streams
# its own fragments: several column groups of 128 with a ragged last one, contraction lengths that
# are no multiple of 32, blocks of 16 / 48 / 64, every row count that matters for the 32-row
# matrix-instruction tile; grids of 1, 3 and 7 workgroups make the runs of steps cross from one
# column group into the next.
FEW_SHAPES = [
    (1, 96, 16, (0, 3, 4, 9, 10, 11, 12, 20, 21), 0), (8, 130, 64, (1, 2, 6), 1), (9, 70, 48, (0, 2, 3, 5), 0),
    (17, 200, 32, tuple(range(0, 22, 2)), 2), (31, 33, 16, tuple(range(19)), 0), (32, 515, 64, (0, 1, 4, 5, 6), 0),
]


@pytest.mark.parametrize("grid", [0, 1, 3, 7])
@pytest.mark.parametrize("m,other,bs,kept,spare", FEW_SHAPES)
@pytest.mark.parametrize("kind", ["somm", "simm"])
def test_few_rows_on_weight_planes(ctx, kind, m, other, bs, kept, spare, grid):
    import paper_2505_07239_amd as comet
    nb = max(kept) + 2
    cs = _case(900 + m, kind, m, other if kind == "somm" else nb * bs, nb * bs if kind == "somm" else other,
               bs, kept, spare)
    ctx.set_tuning(comet.TUNE_GEMM_GRID, grid)
    try:
        for b_full in (True, False):
            if kind == "simm" and b_full and bs % 16:
                continue
            for party in (0, 1):
                say("few rows planes %s m=%d other=%d bs=%d blocks=%d grid=%d b_full=%s party %d"
                    % (kind, m, other, bs, len(kept), grid, b_full, party))
                _run(ctx, cs, party, b_full)
    finally:
        ctx.set_tuning(comet.TUNE_GEMM_GRID, 0)


@pytest.mark.parametrize("m", [3, 32])
def test_few_rows_long_contraction_worst_case_digits(ctx, m):
    """All digits -128 over runs of steps longer than one accumulation segment (one workgroup
    takes all 2 x 257 steps of a column group)."""
    import paper_2505_07239_amd as comet
    k, n, bs = 8224, 160, 32
    worst = np.uint64(0x8080808080808080)
    e, a = np.full((m, k), worst), np.full((m, k), worst)
    f, b = np.full((k, n), worst), np.full((k, n), worst)
    e[::3, ::5] = u64(55, 2, m, k)[::3, ::5]
    f[::7, ::2] = u64(55, 3, k, n)[::7, ::2]
    c = u64(55, 1, m, n)
    idx = torch.arange(n // bs, dtype=torch.int32, device="cuda")
    want = [co.beaver_share(party, e, f, a, b, c) for party in (0, 1)]
    for grid in (0, 1, 2):
        ctx.set_tuning(comet.TUNE_GEMM_GRID, grid)
        try:
            for party in (0, 1):
                say("few rows worst-case digits m=%d grid=%d party %d" % (m, grid, party))
                z = ctx.somm_share(party, bs, idx, None, n // bs, up(e), ctx.open_weight_planes(up(f)), up(a),
                                   ctx.open_weight_planes(up(b)), up(c))
                torch.cuda.synchronize()
                assert np.array_equal(down(z), want[party])
        finally:
            ctx.set_tuning(comet.TUNE_GEMM_GRID, 0)


def test_planes_long_contraction_worst_case_digits(ctx):
    """All digits -128 over a contraction longer than one accumulation segment."""
    m, k, n, bs = 33, 8224, 32, 32
    worst = np.uint64(0x8080808080808080)
    e, a = np.full((m, k), worst), np.full((m, k), worst)
    f, b = np.full((k, n), worst), np.full((k, n), worst)
    e[::3, ::5] = u64(54, 2, m, k)[::3, ::5]
    f[::7, ::2] = u64(54, 3, k, n)[::7, ::2]
    c = u64(54, 1, m, n)
    idx = torch.zeros(1, dtype=torch.int32, device="cuda")
    import paper_2505_07239_amd as comet
    for grid in (0, 1, 8):
        ctx.set_tuning(comet.TUNE_GEMM_GRID, grid)
        try:
            for party in (0, 1):
                say("planes worst-case digits grid=%d party %d" % (grid, party))
                z = ctx.somm_share(party, bs, idx, None, 1, up(e), ctx.open_weight_planes(up(f)), up(a),
                                   ctx.open_weight_planes(up(b)), up(c))
                torch.cuda.synchronize()
                assert np.array_equal(down(z), co.beaver_share(party, e, f, a, b, c))
        finally:
            ctx.set_tuning(comet.TUNE_GEMM_GRID, 0)


def test_planes_flag_combinations_are_checked(ctx):
    import paper_2505_07239_amd as comet
    m, k, bs, t = 40, 64, 8, 2
    idx = torch.arange(t, dtype=torch.int32, device="cuda")
    e, a, c = up(u64(1, 1, m, k)), up(u64(1, 2, m, k)), up(u64(1, 3, m, t * bs))
    f = ctx.open_weight_planes(up(u64(1, 4, k, t * bs)))
    b_words = up(u64(1, 5, k, 4 * bs))
    with pytest.raises(TypeError):
        ctx.somm_share(0, bs, idx, None, t, e, f, a, b_words, c)             # planes and words mixed
    # planes have a layout of their own: not together with neuron-major weights (raw C-ABI call)
    import ctypes
    ptr = lambda x: ctypes.c_void_p(x.data_ptr())
    b_pl = ctx.open_weight_planes(b_words)
    z = torch.empty((m, t * bs), dtype=torch.int64, device="cuda")
    need = comet.workspace_bytes(comet.OP_SOMM, m, k, t * bs, bs)
    ws = ctx.workspace(need)
    flags = comet.FULL_B | comet.WEIGHT_PLANES
    args = lambda fl: (ctx.h, 0, m, k, 4 * bs, bs, ptr(idx), None, t, fl, ptr(e), ptr(f), ptr(a), ptr(b_pl), ptr(c),
                       ptr(z), ptr(ws), need)
    assert ctx.lib.comet_somm_share(*args(flags | comet.WEIGHTS_NEURON_MAJOR)) == -1
    assert ctx.lib.comet_somm_share(*args(flags)) == 0
    torch.cuda.synchronize()
    # SIMM with a full-size B_i in planes: bs must be a multiple of 16
    e2, a2, c2 = up(u64(2, 1, m, t * bs)), up(u64(2, 2, m, 4 * bs)), up(u64(2, 3, m, k))
    f2 = ctx.open_weight_planes(up(u64(2, 4, t * bs, k)))
    b2 = ctx.open_weight_planes(up(u64(2, 5, 4 * bs, k)))
    with pytest.raises(comet.CometError) as ei:
        ctx.simm_share(0, bs, idx, None, t, e2, f2, a2, b2, c2)
    assert ei.value.code == -1
