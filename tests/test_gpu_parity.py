"""GPU parity: every HIP entry point against the CPU oracle, bit for bit.

All calls go through the C ABI (ctypes binding).  Inputs are the seeded
synthetic workloads; expected values come from ``oracle/`` only.
"""
import os
import sys

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

import oracle as co                                   # noqa: E402
from oracle import cases, protocols                   # noqa: E402
from workloads import configs, masks, rng             # noqa: E402


def say(msg):
    print("[gpu-parity] " + msg, flush=True)
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


# ---------------------------------------------------------------------------
# (1) mask / open
# ---------------------------------------------------------------------------

@pytest.mark.parametrize("n", [0, 1, 2, 3, 1023, 2048, (1 << 20) + 3, 5_000_001])
def test_mask_share_and_open(ctx, n):
    say("mask_share/open n=%d" % n)
    x, a = u64(31, 1, n), u64(31, 2, n)
    gx, ga = up(x), up(a)
    d = ctx.mask_share(gx, ga)
    e = ctx.open(gx, ga)
    torch.cuda.synchronize()
    assert np.array_equal(down(d), co.mask_share(x, a))
    assert np.array_equal(down(e), co.open_(x, a))


def test_mask_share_rejects_bad_arguments(ctx):
    import paper_2505_07239_amd as comet
    x = up(u64(32, 1, 16))
    with pytest.raises(comet.CometError) as ei:
        ctx.mask_share(x[1:9], x[1:9])          # 8-byte aligned only
    assert ei.value.code == -2


@pytest.mark.parametrize("rows,cols,bs,nb_keep,axis", [
    (5, 48, 4, 3, 0), (7, 33, 3, 4, 0), (48, 10, 4, 5, 1), (33, 7, 3, 2, 1),
    (128, 3072, 32, 10, 0), (3072, 768, 32, 10, 1)])
def test_mask_share_gather(ctx, rows, cols, bs, nb_keep, axis):
    import paper_2505_07239_amd as comet
    say("mask_share_gather %dx%d bs=%d axis=%d" % (rows, cols, bs, axis))
    extent = cols if axis == comet.AXIS_COLS else rows
    nb = extent // bs
    mask = masks.uniform_block_mask(33, rows + cols, nb, nb_keep / nb)
    idx = co.compact_mask(mask)
    w, b = u64(33, 1, rows, cols), u64(33, 2, rows, cols)
    cap = len(idx) + 2 if len(idx) + 2 <= nb else len(idx)
    gi = torch.zeros(nb, dtype=torch.int32, device="cuda")
    gi[:len(idx)] = torch.from_numpy(idx).cuda()
    n_dev = torch.tensor([len(idx)], dtype=torch.int32, device="cuda")
    shape = (rows, cap * bs) if axis == comet.AXIS_COLS else (cap * bs, cols)
    out = torch.full(shape, -1, dtype=torch.int64, device="cuda")
    ctx.mask_share_gather(up(w), up(b), axis, bs, gi, n_dev, cap, out=out)
    torch.cuda.synchronize()
    got = down(out)
    if axis == comet.AXIS_COLS:
        want = co.mask_share(co.index_cols(w, idx, bs), co.index_cols(b, idx, bs))
        assert np.array_equal(got[:, :len(idx) * bs], want)
        assert np.all(got[:, len(idx) * bs:] == np.uint64(2 ** 64 - 1))     # beyond n_blk: untouched
    else:
        want = co.mask_share(co.index_rows(w, idx, bs), co.index_rows(b, idx, bs))
        assert np.array_equal(got[:len(idx) * bs], want)
        assert np.all(got[len(idx) * bs:] == np.uint64(2 ** 64 - 1))


# ---------------------------------------------------------------------------
# (2) compaction
# ---------------------------------------------------------------------------

def _check_compact(ctx, mask_np):
    m = torch.from_numpy(mask_np).cuda()
    idx, n_dev = ctx.compact_mask(m)
    torch.cuda.synchronize()
    want = co.compact_mask(mask_np)
    t = int(n_dev.item())
    assert t == len(want)
    assert np.array_equal(idx[:t].cpu().numpy(), want)


@pytest.mark.parametrize("cid", [1, 2, 3, 4, 5])
def test_compact_mask_configs(ctx, cid):
    cfg = configs.config(cid, 0.25 if cid == 5 else None)
    say("compact config %d" % cid)
    _check_compact(ctx, configs.token_masks(cfg))


@pytest.mark.parametrize("n_tok,nb", [(1, 1), (1, 15), (1, 16), (1, 17), (3, 100), (8, 216), (5, 4096),
                                      (1, 4097), (1, 16384), (1, 16385), (3, 50_000), (4, 65536),
                                      (1, 1_000_003), (2, 3_000_000),
                                      # several super-chunks of the pipelined form, one token and two
                                      (1, 20_000_003), (2, 34_000_000)])
def test_compact_mask_shapes(ctx, n_tok, nb):
    say("compact n_tok=%d nb=%d" % (n_tok, nb))
    m = np.stack([masks.stress_mask(34, 10 * t + nb % 7, nb, 0.15) for t in range(n_tok)])
    # any non-zero byte is an active flag
    m = (m * (1 + (rng.uniform_u64(34, 99, n_tok * nb) % np.uint64(255)).astype(np.uint8).reshape(n_tok, nb)))
    _check_compact(ctx, np.ascontiguousarray(m.astype(np.uint8)))


def _token_masks(seed, n_tok, nb, density=0.3, shared=0.4):
    """[n_tok, nb] flags: clustered draws per position, restricted to a shared set of columns
    (tokens of a batch agree on most of their active neurons), any non-zero byte active."""
    flat = masks.stress_mask(seed, 1, n_tok * nb, density).reshape(n_tok, nb)
    common = masks.stress_mask(seed, 3, nb, shared)
    vals = 1 + (rng.uniform_u64(seed, 5, n_tok * nb) % np.uint64(255)).astype(np.uint8).reshape(n_tok, nb)
    return np.ascontiguousarray((flat & common[None, :]) * vals).astype(np.uint8)


@pytest.mark.parametrize("n_tok,nb", [
    (2, 1), (2, 3), (7, 5), (33, 15), (16, 16), (9, 17), (64, 344), (512, 344), (513, 343), (380, 345),
    (31, 4095), (32, 4096), (4096, 344), (1000, 1001), (300, 4096), (129, 4097), (40, 13824), (333, 11008),
    (17, 65535), (9, 65536), (700, 65536), (5, 65537), (3, 200_003), (300, 70_001), (2100, 16400),
    # column periods of exactly one trip of the narrow and of the wide workgroup, and in between
    (40, 16384), (20, 32768), (50, 2049), (66, 8190), (2, 65536), (8200, 344)])
def test_compact_mask_many_tokens(ctx, n_tok, nb):
    """Several token rows: one workgroup over the flat mask, the flat pass with merged bitmaps,
    and (beyond 65536 columns) the token split per column chunk; row lengths of every
    alignment."""
    say("compact many tokens n_tok=%d nb=%d" % (n_tok, nb))
    _check_compact(ctx, _token_masks(41, n_tok, nb))


@pytest.mark.parametrize("lead", [1, 4, 15])
@pytest.mark.parametrize("n_tok,nb", [(50, 344), (700, 344), (90, 4096), (600, 13824), (11, 65537)])
def test_compact_mask_many_tokens_unaligned_pointer(ctx, n_tok, nb, lead):
    say("compact many tokens n_tok=%d nb=%d lead=%d" % (n_tok, nb, lead))
    m = _token_masks(42 + lead, n_tok, nb)
    # surrounded by set flags that are not part of the mask
    backing = torch.full((lead + n_tok * nb + 64,), 1, dtype=torch.uint8, device="cuda")
    backing[lead:lead + n_tok * nb] = torch.from_numpy(m.reshape(-1)).cuda()
    view = backing[lead:lead + n_tok * nb].view(n_tok, nb)
    idx, n_dev = ctx.compact_mask(view)
    torch.cuda.synchronize()
    want = co.compact_mask(m)
    assert int(n_dev.item()) == len(want) and np.array_equal(idx[:len(want)].cpu().numpy(), want)


def test_compact_mask_many_tokens_corners(ctx):
    say("compact many tokens corners")
    for n_tok, nb in ((2, 16), (100, 344), (2000, 344), (50, 5000), (40, 70_000)):
        _check_compact(ctx, np.zeros((n_tok, nb), np.uint8))
        _check_compact(ctx, np.full((n_tok, nb), 255, np.uint8))
        for r, c in ((0, 0), (n_tok - 1, nb - 1), (n_tok - 1, 0), (0, nb - 1), (n_tok // 2, nb // 2)):
            m = np.zeros((n_tok, nb), np.uint8)
            m[r, c] = 128
            _check_compact(ctx, m)


def test_compact_mask_degenerate(ctx):
    say("compact degenerate")
    for nb in (7, 5000, 70_000):
        _check_compact(ctx, np.zeros((2, nb), np.uint8))
        _check_compact(ctx, np.ones((1, nb), np.uint8))
    # unaligned mask pointer
    base = torch.from_numpy(masks.stress_mask(35, 1, 20_001, 0.3)).cuda()
    idx, n_dev = ctx.compact_mask(base[1:])
    torch.cuda.synchronize()
    want = co.compact_mask(base[1:].cpu().numpy())
    assert int(n_dev.item()) == len(want) and np.array_equal(idx[:len(want)].cpu().numpy(), want)


@pytest.mark.parametrize("shift", [0, 1, 2, 3])
@pytest.mark.parametrize("density", [0.001, 0.15, 0.9])
def test_compact_mask_output_alignment(ctx, shift, density):
    """The index list may start at any 4-byte boundary; the large path writes whole 16-byte
    quads in the middle of each workgroup's run and single words at its ragged ends.  Dense
    masks overflow the LDS stage and take the direct path."""
    nb = 200_003
    say("compact output shift %d density %.3f" % (shift, density))
    m = masks.stress_mask(36, 3 + shift, nb, density)[None, :]
    backing = torch.full((nb + 8,), -7, dtype=torch.int32, device="cuda")
    n_dev = torch.zeros(1, dtype=torch.int32, device="cuda")
    ctx.compact_mask(torch.from_numpy(m).cuda(), backing[shift:shift + nb], n_dev)
    torch.cuda.synchronize()
    want = co.compact_mask(m)
    got = backing.cpu().numpy()
    assert int(n_dev.item()) == len(want)
    assert np.array_equal(got[shift:shift + len(want)], want)
    # nothing outside the list is touched
    assert np.all(got[:shift] == -7) and np.all(got[shift + len(want):] == -7)


# ---------------------------------------------------------------------------
# (3) output shares
# ---------------------------------------------------------------------------

SENTINEL = np.uint64(0x5EA15EA15EA15EA1)


def _run_share(ctx, kind, party, bs, idx_np, cap, e, f, a_i, b_i, c_i, a_full=True, b_full=True,
               n_blk_on_device=True):
    """The output buffer starts out full of a sentinel, so that a caller can see what was written."""
    gi = torch.zeros(max(cap, 1), dtype=torch.int32, device="cuda")
    gi[:len(idx_np)] = torch.from_numpy(idx_np).cuda()
    n_dev = torch.tensor([len(idx_np)], dtype=torch.int32, device="cuda") if n_blk_on_device else None
    zshape = (e.shape[0], cap * bs) if kind == "somm" else (e.shape[0], f.shape[1])
    out = torch.full(zshape, int(SENTINEL.view(np.int64)), dtype=torch.int64, device="cuda")
    if kind == "somm":
        return ctx.somm_share(party, bs, gi, n_dev, cap, up(e), up(f), up(a_i), up(b_i), up(c_i),
                              b_full=b_full, out=out)
    return ctx.simm_share(party, bs, gi, n_dev, cap, up(e), up(f), up(a_i), up(b_i), up(c_i),
                          a_full=a_full, b_full=b_full, out=out)


def _pad_cols(a, ld):
    """Spare columns hold junk: nothing at or beyond n_blk * bs may be read."""
    out = u64(4242, a.shape[0] + 7 * ld, a.shape[0], ld)
    out[:, :a.shape[1]] = a
    return out


def _pad_rows(a, ld):
    out = u64(4243, a.shape[1] + 7 * ld, ld, a.shape[1])
    out[:a.shape[0]] = a
    return out


def _random_case(kind, m, k, n, bs, keep, seed):
    """Uniformly random ring elements everywhere (shares are uniform anyway)."""
    nb = (n if kind == "somm" else k) // bs
    mask = masks.uniform_block_mask(seed, 7, nb, keep / nb)[None, :]
    nk = int(mask.sum()) * bs
    shape_c = (m, nk) if kind == "somm" else (m, n)
    x_sh = (u64(seed, 1, m, k), u64(seed, 2, m, k))
    y_sh = (u64(seed, 3, k, n), u64(seed, 4, k, n))
    return protocols.block_case(kind, x_sh, y_sh, mask, bs, u64(seed, 5, m, k), u64(seed, 6, k, n),
                                u64(seed, 8, m, k), u64(seed, 9, k, n), u64(seed, 10, *shape_c))


@pytest.mark.parametrize("cid", [1, 2])
def test_share_configs_full(ctx, cid):
    cfg = configs.config(cid)
    for mm in cfg.matmuls:
        case, _ = cases.build(cfg, mm)
        for party in (0, 1):
            say("config %d %s party %d" % (cid, mm.name, party))
            z = _run_share(ctx, mm.kind, party, cfg.bs, case.idx, len(case.idx), case.e, case.f,
                           case.a[party], case.b[party], case.c[party])
            torch.cuda.synchronize()
            assert np.array_equal(down(z), case.z[party])


@pytest.mark.parametrize("kind,m,k,n,bs,keep", [
    ("somm", 1, 1, 4, 4, 1), ("somm", 37, 70, 96, 3, 5), ("somm", 130, 45, 200, 8, 9),
    ("somm", 65, 33, 64, 32, 1), ("somm", 200, 300, 512, 16, 20), ("somm", 9, 520, 600, 20, 17),
    ("simm", 1, 4, 1, 4, 1), ("simm", 37, 96, 70, 3, 5), ("simm", 130, 200, 45, 8, 9),
    ("simm", 65, 64, 33, 32, 1), ("simm", 200, 512, 300, 16, 20), ("simm", 9, 600, 520, 20, 17)])
def test_share_ragged_shapes(ctx, kind, m, k, n, bs, keep):
    case = _random_case(kind, m, k, n, bs, keep, 40 + m)
    t = len(case.idx)
    for party in (0, 1):
        say("ragged %s m=%d k=%d n=%d bs=%d party %d" % (kind, m, k, n, bs, party))
        z = _run_share(ctx, kind, party, bs, case.idx, t, case.e, case.f, case.a[party],
                       case.b[party], case.c[party])
        torch.cuda.synchronize()
        assert np.array_equal(down(z), case.z[party])


@pytest.mark.parametrize("kind,m,k,n,bs,keep", [
    ("somm", 1, 70, 96, 3, 5), ("somm", 2, 300, 512, 16, 20), ("somm", 5, 45, 200, 8, 9),
    ("somm", 8, 1100, 640, 64, 7), ("somm", 9, 520, 600, 20, 17), ("somm", 13, 33, 63, 7, 4),
    ("somm", 16, 777, 384, 32, 5),
    ("simm", 1, 96, 70, 3, 5), ("simm", 2, 512, 300, 16, 20), ("simm", 5, 200, 45, 8, 9),
    ("simm", 8, 640, 1100, 64, 7), ("simm", 9, 600, 520, 20, 17), ("simm", 13, 63, 33, 7, 4),
    ("simm", 16, 384, 777, 32, 5)])
@pytest.mark.parametrize("path", ["vector", "matrix"])
def test_share_few_rows(ctx, kind, m, k, n, bs, keep, path):
    """m <= 8 takes the vector-ALU kernel by default; the matrix-core kernel must give the
    same bits for the same call (odd widths and odd bs reach the one-column-per-lane variant)."""
    import paper_2505_07239_amd as comet
    case = _random_case(kind, m, k, n, bs, keep, 140 + m)
    t = len(case.idx)
    ctx.set_tuning(comet.TUNE_SKINNY, 1 if path == "matrix" else 0)
    try:
        for party in (0, 1):
            say("few rows (%s) %s m=%d k=%d n=%d bs=%d party %d" % (path, kind, m, k, n, bs, party))
            z = _run_share(ctx, kind, party, bs, case.idx, t, case.e, case.f, case.a[party],
                           case.b[party], case.c[party])
            torch.cuda.synchronize()
            assert np.array_equal(down(z), case.z[party])
    finally:
        ctx.set_tuning(comet.TUNE_SKINNY, 0)


@pytest.mark.parametrize("kind,m,k,n,bs,keep", [
    ("somm", 1, 70, 96, 3, 5), ("somm", 2, 300, 512, 16, 20), ("somm", 4, 45, 200, 8, 9), ("somm", 5, 130, 77, 7, 6),
    ("somm", 8, 1100, 640, 64, 7),
    ("simm", 1, 96, 70, 3, 5), ("simm", 2, 512, 300, 16, 20), ("simm", 3, 200, 45, 8, 9), ("simm", 7, 77, 131, 7, 6),
    ("simm", 8, 640, 1100, 64, 7)])
@pytest.mark.parametrize("b_full", [True, False])
def test_share_few_rows_unopened(ctx, kind, m, k, n, bs, keep, b_full):
    """The few-row share with the opening folded in: handed the two masked shares of the indexed
    weights (F = G_0 + G_1, Sec. 2.1) it must give the bits of Eq. 1 on the opened F.  The split of
    F into shares is random, so a dropped or doubled share cannot cancel."""
    case = _random_case(kind, m, k, n, bs, keep, 180 + m)
    t = len(case.idx)
    g_1 = u64(181, m + 3, *case.f.shape)
    g_0 = case.f - g_1                                      # mod 2^64
    assert np.array_equal(co.open_(g_0, g_1), case.f)
    gi = torch.from_numpy(case.idx).cuda() if t else torch.zeros(1, dtype=torch.int32, device="cuda")
    n_dev = torch.tensor([t], dtype=torch.int32, device="cuda")
    for party in (0, 1):
        say("few rows unopened %s m=%d k=%d n=%d bs=%d b_full=%s party %d" % (kind, m, k, n, bs, b_full, party))
        if kind == "somm":
            b_i = case.b[party] if b_full else co.index_cols(case.b[party], case.idx, bs)
            z = ctx.somm_share_unopened(party, bs, gi, n_dev, t, up(case.e), up(g_0), up(g_1), up(case.a[party]),
                                        up(b_i), up(case.c[party]), b_full=b_full)
        else:
            a_i = case.a[party] if b_full else co.index_cols(case.a[party], case.idx, bs)
            b_i = case.b[party] if b_full else co.index_rows(case.b[party], case.idx, bs)
            z = ctx.simm_share_unopened(party, bs, gi, n_dev, t, up(case.e), up(g_0), up(g_1), up(a_i), up(b_i),
                                        up(case.c[party]), a_full=b_full, b_full=b_full)
        torch.cuda.synchronize()
        assert np.array_equal(down(z), case.z[party])


def test_share_unopened_limits(ctx):
    """Beyond eight rows, or when the few-row kernel is switched off, the unopened form is refused
    with a clear error (and nothing is launched)."""
    import paper_2505_07239_amd as comet
    case = _random_case("somm", 9, 64, 96, 8, 4, 190)
    t = len(case.idx)
    gi, n_dev = torch.from_numpy(case.idx).cuda(), torch.tensor([t], dtype=torch.int32, device="cuda")
    args = (1, 8, gi, n_dev, t, up(case.e), up(case.f), up(case.f), up(case.a[1]), up(case.b[1]), up(case.c[1]))
    with pytest.raises(comet.CometError) as ei:
        ctx.somm_share_unopened(*args)
    assert ei.value.code == -1 and "few-row" in str(ei.value)
    case = _random_case("somm", 4, 64, 96, 8, 4, 191)
    args = (1, 8, gi, n_dev, t, up(case.e), up(case.f), up(case.f), up(case.a[1]), up(case.b[1]), up(case.c[1]))
    ctx.set_tuning(comet.TUNE_SKINNY, 1)
    try:
        with pytest.raises(comet.CometError):
            ctx.somm_share_unopened(*args)
    finally:
        ctx.set_tuning(comet.TUNE_SKINNY, 0)


@pytest.mark.parametrize("m,k,n,bs,keep", [
    (1, 2, 4, 4, 1), (37, 70, 96, 3, 5), (130, 46, 200, 8, 9), (65, 34, 64, 32, 1),
    (200, 300, 512, 16, 20), (9, 520, 600, 20, 17), (16, 778, 384, 32, 5), (256, 768, 3072, 32, 10)])
@pytest.mark.parametrize("b_full", [True, False])
def test_somm_neuron_major_weights(ctx, m, k, n, bs, keep, b_full):
    """B_i and F stored one row per neuron (the transposes of the row-major operands) give
    the same share, with B_i at full size (kept rows indexed in the kernel) or compact."""
    case = _random_case("somm", m, k, n, bs, keep, 240 + m)
    t = len(case.idx)
    gi = torch.zeros(max(t, 1), dtype=torch.int32, device="cuda")
    gi[:t] = torch.from_numpy(case.idx).cuda()
    n_dev = torch.tensor([t], dtype=torch.int32, device="cuda")
    f_t = np.ascontiguousarray(case.f.T)
    for party in (0, 1):
        say("neuron-major somm m=%d k=%d n=%d bs=%d b_full=%s party %d" % (m, k, n, bs, b_full, party))
        b_i = case.b[party] if b_full else co.index_cols(case.b[party], case.idx, bs)
        z = ctx.somm_share(party, bs, gi, n_dev, t, up(case.e), up(f_t), up(case.a[party]),
                           up(np.ascontiguousarray(b_i.T)), up(case.c[party]), b_full=b_full,
                           neuron_major=True)
        torch.cuda.synchronize()
        assert np.array_equal(down(z), case.z[party])


def test_somm_neuron_major_rejects_odd_k_and_simm(ctx):
    import paper_2505_07239_amd as comet
    case = _random_case("somm", 4, 7, 16, 4, 2, 260)
    t = len(case.idx)
    gi = torch.from_numpy(case.idx).cuda()
    n_dev = torch.tensor([t], dtype=torch.int32, device="cuda")
    with pytest.raises(comet.CometError) as ei:
        ctx.somm_share(0, 4, gi, n_dev, t, up(case.e), up(np.ascontiguousarray(case.f.T)),
                       up(case.a[0]), up(np.ascontiguousarray(case.b[0].T)), up(case.c[0]),
                       neuron_major=True)
    assert ei.value.code == -1


@pytest.mark.parametrize("slices", [1, 3, 64, 5000])
@pytest.mark.parametrize("kind", ["somm", "simm"])
def test_share_few_rows_any_split(ctx, kind, slices):
    """The split of the stacked contraction over workgroups never changes the result, also when
    most wavefronts get an empty run (more slices than contraction rows)."""
    import paper_2505_07239_amd as comet
    m, k, n, bs, keep = 7, 130, 192, 16, 6
    if kind == "simm":
        k, n = n, k
    case = _random_case(kind, m, k, n, bs, keep, 160)
    ctx.set_tuning(comet.TUNE_SKINNY_SLICES, slices)
    try:
        for party in (0, 1):
            say("few rows split %s slices=%d party %d" % (kind, slices, party))
            z = _run_share(ctx, kind, party, bs, case.idx, len(case.idx), case.e, case.f,
                           case.a[party], case.b[party], case.c[party])
            torch.cuda.synchronize()
            assert np.array_equal(down(z), case.z[party])
    finally:
        ctx.set_tuning(comet.TUNE_SKINNY_SLICES, 0)


@pytest.mark.parametrize("kind", ["somm", "simm"])
def test_share_few_rows_compact_triples(ctx, kind):
    """Vector-ALU kernel with already indexed triple shares and spare block capacity."""
    m, k, n, bs, keep = 6, 96, 128, 8, 5
    case = _random_case(kind, m, k, n, bs, keep, 161)
    t, cap = len(case.idx), len(case.idx) + 2
    ld = cap * bs
    for party in (0, 1):
        say("few rows compact triples %s party %d" % (kind, party))
        if kind == "somm":
            b_sel = co.index_cols(case.b[party], case.idx, bs)
            args = (case.e, _pad_cols(case.f, ld), case.a[party], _pad_cols(b_sel, ld),
                    _pad_cols(case.c[party], ld))
            z = _run_share(ctx, kind, party, bs, case.idx, cap, *args, b_full=False)
            torch.cuda.synchronize()
            assert np.array_equal(down(z)[:, :t * bs], case.z[party])
            assert np.all(down(z)[:, t * bs:] == SENTINEL)      # spare columns are never written
        else:
            a_sel = co.index_cols(case.a[party], case.idx, bs)
            b_sel = co.index_rows(case.b[party], case.idx, bs)
            args = (_pad_cols(case.e, ld), _pad_rows(case.f, ld), _pad_cols(a_sel, ld),
                    _pad_rows(b_sel, ld), case.c[party])
            z = _run_share(ctx, kind, party, bs, case.idx, cap, *args, a_full=False, b_full=False)
            torch.cuda.synchronize()
            assert np.array_equal(down(z), case.z[party])


@pytest.mark.parametrize("kind", ["somm", "simm"])
def test_share_compact_triples_and_spare_capacity(ctx, kind):
    """Triple shares passed already indexed; n_blk on the device below n_blk_cap."""
    m, k, n, bs, keep = 70, 96, 128, 8, 5
    case = _random_case(kind, m, k, n, bs, keep, 51)
    t, cap = len(case.idx), len(case.idx) + 3
    ld = cap * bs
    for party in (0, 1):
        say("compact triples %s party %d" % (kind, party))
        if kind == "somm":
            b_sel = co.index_cols(case.b[party], case.idx, bs)
            args = (case.e, _pad_cols(case.f, ld), case.a[party], _pad_cols(b_sel, ld),
                    _pad_cols(case.c[party], ld))
            z = _run_share(ctx, kind, party, bs, case.idx, cap, *args, b_full=False)
            torch.cuda.synchronize()
            got = down(z)
            assert np.array_equal(got[:, :t * bs], case.z[party])
            assert np.all(got[:, t * bs:] == SENTINEL)          # spare columns are never written
        else:
            a_sel = co.index_cols(case.a[party], case.idx, bs)
            b_sel = co.index_rows(case.b[party], case.idx, bs)
            args = (_pad_cols(case.e, ld), _pad_rows(case.f, ld), _pad_cols(a_sel, ld),
                    _pad_rows(b_sel, ld), case.c[party])
            z = _run_share(ctx, kind, party, bs, case.idx, cap, *args, a_full=False, b_full=False)
            torch.cuda.synchronize()
            assert np.array_equal(down(z), case.z[party])


def test_share_without_device_count(ctx):
    case = _random_case("somm", 40, 64, 96, 8, 4, 52)
    z = _run_share(ctx, "somm", 1, 8, case.idx, len(case.idx), case.e, case.f, case.a[1], case.b[1],
                   case.c[1], n_blk_on_device=False)
    torch.cuda.synchronize()
    assert np.array_equal(down(z), case.z[1])


def test_share_empty_mask(ctx):
    """No active block: SOMM has nothing to write, SIMM returns C_i."""
    m, k, n, bs = 16, 32, 24, 8
    e, a, c = u64(53, 1, m, bs), u64(53, 2, m, k), u64(53, 3, m, n)
    f, b = u64(53, 4, bs, n), u64(53, 5, k, n)
    gi = torch.zeros(1, dtype=torch.int32, device="cuda")
    n_dev = torch.zeros(1, dtype=torch.int32, device="cuda")
    z = ctx.simm_share(1, bs, gi, n_dev, 1, up(e), up(f), up(a), up(b), up(c))
    torch.cuda.synchronize()
    assert np.array_equal(down(z), c)


@pytest.mark.parametrize("m", [4, 16, 40])
def test_share_empty_mask_every_path(ctx, m):
    """No active block (count on the device is zero, capacity is not): SIMM returns C_i and SOMM
    writes nothing, on weight words, on weight planes (the few-row and the tile kernels) and with
    the opening folded in."""
    k, n, bs, cap = 64, 48, 16, 2
    gi = torch.zeros(cap, dtype=torch.int32, device="cuda")
    n_dev = torch.zeros(1, dtype=torch.int32, device="cuda")
    sent = int(SENTINEL.view(np.int64))
    # SIMM: E m x ld, F ld x n, A m x k, B k x n
    e, a, c = u64(57, 1, m, cap * bs), u64(57, 2, m, k), u64(57, 3, m, n)
    f, b = u64(57, 4, cap * bs, n), u64(57, 5, k, n)
    forms = [("words", up(f), up(b))]
    forms.append(("planes", ctx.open_weight_planes(up(f)), ctx.open_weight_planes(up(b))))
    for name, fw, bw in forms:
        say("empty mask simm %s m=%d" % (name, m))
        z = ctx.simm_share(1, bs, gi, n_dev, cap, up(e), fw, up(a), bw, up(c))
        torch.cuda.synchronize()
        assert np.array_equal(down(z), c)
    if m <= 8:
        z = ctx.simm_share_unopened(1, bs, gi, n_dev, cap, up(e), up(f), up(f), up(a), up(b), up(c))
        torch.cuda.synchronize()
        assert np.array_equal(down(z), c)
    # SOMM: E, A m x k, F k x ld, B k x n_full, C m x ld
    e, a, c = u64(58, 1, m, k), u64(58, 2, m, k), u64(58, 3, m, cap * bs)
    f, b = u64(58, 4, k, cap * bs), u64(58, 5, k, 6 * bs)
    forms = [("words", up(f), up(b)), ("planes", ctx.open_weight_planes(up(f)), ctx.open_weight_planes(up(b)))]
    for name, fw, bw in forms:
        say("empty mask somm %s m=%d" % (name, m))
        out = torch.full((m, cap * bs), sent, dtype=torch.int64, device="cuda")
        ctx.somm_share(0, bs, gi, n_dev, cap, up(e), fw, up(a), bw, up(c), out=out)
        torch.cuda.synchronize()
        assert np.all(down(out) == SENTINEL)
    if m <= 8:
        out = torch.full((m, cap * bs), sent, dtype=torch.int64, device="cuda")
        ctx.somm_share_unopened(0, bs, gi, n_dev, cap, up(e), up(f), up(f), up(a), up(b), up(c), out=out)
        torch.cuda.synchronize()
        assert np.all(down(out) == SENTINEL)


@pytest.mark.parametrize("grid", [0, 1, 8])
def test_share_extreme_digits_long_contraction(ctx, grid):
    """All-0x80 bytes make every signed digit -128, the worst case for the
    int32 digit-product planes; a contraction of 2 x 8224 words forces more
    than one accumulation segment when few workgroups share it."""
    import paper_2505_07239_amd as comet
    m, k, n, bs = 33, 8224, 32, 32
    worst = np.uint64(0x8080808080808080)
    e, a = np.full((m, k), worst), np.full((m, k), worst)
    f, b = np.full((k, n), worst), np.full((k, n), worst)
    c = u64(54, 1, m, n)
    e[::3, ::5] = u64(54, 2, m, k)[::3, ::5]
    f[::7, ::2] = u64(54, 3, k, n)[::7, ::2]
    idx = np.array([0], dtype=np.int32)
    ctx.set_tuning(comet.TUNE_GEMM_GRID, grid)
    try:
        for party in (0, 1):
            say("extreme digits grid=%d party %d" % (grid, party))
            z = _run_share(ctx, "somm", party, bs, idx, 1, e, f, a, b, c)
            torch.cuda.synchronize()
            assert np.array_equal(down(z), co.beaver_share(party, e, f, a, b, c))
    finally:
        ctx.set_tuning(comet.TUNE_GEMM_GRID, 0)


def test_share_is_deterministic(ctx):
    """Integer ring: two runs must agree bit for bit (any difference is a race)."""
    case = _random_case("simm", 150, 256, 200, 16, 9, 55)
    runs = []
    for _ in range(2):
        z = _run_share(ctx, "simm", 1, 16, case.idx, len(case.idx), case.e, case.f, case.a[1],
                       case.b[1], case.c[1])
        torch.cuda.synchronize()
        runs.append(down(z).copy())
    assert np.array_equal(runs[0], runs[1]) and np.array_equal(runs[0], case.z[1])


def test_share_kernel_timing_counts_and_leaves_results_alone(ctx):
    """Timed launches (event pairs attached to the kernel's dispatch), every launch and every
    third one: the launch counts, positive kernel times, and the same output as untimed calls."""
    import paper_2505_07239_amd as comet
    case = _random_case("somm", 96, 160, 256, 16, 7, 56)
    for m in (96, 5):                                  # the matrix-core kernel and the few-row kernel
        e, a, c = case.e[:m], case.a[0][:m], case.c[0][:m]
        want = case.z[0][:m]                            # output rows are independent of each other
        for stride, calls, timed in ((0, 4, 4), (3, 7, 3), (1, 2, 2)):
            say("timing m=%d stride=%d" % (m, stride))
            ctx.set_tuning(comet.TUNE_TIMING_STRIDE, stride)
            ctx.timing_begin(calls)
            try:
                for _ in range(calls):
                    z = _run_share(ctx, "somm", 0, 16, case.idx, len(case.idx), e, case.f, a, case.b[0], c)
            finally:
                ms, n = ctx.timing_end()
                ctx.set_tuning(comet.TUNE_TIMING_STRIDE, 0)
            torch.cuda.synchronize()
            assert n == timed and 0.0 < ms < 1000.0
            assert np.array_equal(down(z), want)


def test_end_to_end_pipeline_config2(ctx):
    """compact -> mask (indexed) -> open -> share, chained on the device with
    n_blk never leaving it; then reconstruction against the plaintext product."""
    import paper_2505_07239_amd as comet
    cfg = configs.config(2)
    for mm in cfg.matmuls:
        say("pipeline config 2 %s" % mm.name)
        case, plain = cases.build(cfg, mm)
        idx, n_dev = ctx.compact_mask(torch.from_numpy(plain["mask"]).cuda())
        cap = configs.masks.kept_blocks(cfg.density, cfg.nb)
        d, g = [], []
        for i in (0, 1):
            if mm.kind == "somm":
                d.append(ctx.mask_share(up(case.x[i]), up(case.a[i])))
                g.append(ctx.mask_share_gather(up(case.y[i]), up(case.b[i]), comet.AXIS_COLS, cfg.bs,
                                               idx, n_dev, cap))
            else:
                d.append(ctx.mask_share_gather(up(case.x[i]), up(case.a[i]), comet.AXIS_COLS, cfg.bs,
                                               idx, n_dev, cap))
                g.append(ctx.mask_share_gather(up(case.y[i]), up(case.b[i]), comet.AXIS_ROWS, cfg.bs,
                                               idx, n_dev, cap))
        e, f = ctx.open(d[0], d[1]), ctx.open(g[0], g[1])
        z = []
        for i in (0, 1):
            fn = ctx.somm_share if mm.kind == "somm" else ctx.simm_share
            z.append(fn(i, cfg.bs, idx, n_dev, cap, e, f, up(case.a[i]), up(case.b[i]), up(case.c[i])))
        torch.cuda.synchronize()
        assert np.array_equal(down(e), case.e) and np.array_equal(down(f), case.f)
        for i in (0, 1):
            assert np.array_equal(down(z[i]), case.z[i])
        cols = (case.idx.astype(np.int64)[:, None] * cfg.bs + np.arange(cfg.bs)[None, :]).ravel()
        rec = down(z[0]) + down(z[1])
        want = plain["xq"] @ plain["yq"][:, cols] if mm.kind == "somm" else \
            plain["xq"][:, cols] @ plain["yq"][cols, :]
        assert np.array_equal(rec, want)
