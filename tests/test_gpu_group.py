"""GPU parity of ``comet_share_group``: several share products of one shape in one call, every
output element of every member against the oracle's Eq. 1 on that member's own operands.

The grouped matrix-core launch is forced (``COMET_TUNE_GROUP`` = 1) on shapes the oracle finishes
quickly; the cases cover a workgroup range that runs across members, whole owned tiles (the grid
divides the tile count) and shared ones, contractions longer than one accumulation segment, a
device-side block count below the capacity, the most members a group takes, and the fallbacks
(word operands, few rows, grouping switched off), which must give the same result."""
import ctypes
import sys

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

import oracle as co                                   # noqa: E402
from workloads import rng                             # noqa: E402

SENTINEL = np.uint64(0x0123456789ABCDEF)


def say(msg):
    print("[gpu-group] " + msg, flush=True)
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


def _member(seed, kind, party, m, k, n, bs, idx, cap):
    """One member: its own random operands (full-size triple shares, compact opened operands with
    junk in the spare capacity) and the oracle's output share."""
    t, ld = len(idx), cap * bs
    kc = t * bs
    junk = lambda stream, *shape: u64(seed, 90 + stream, *shape)
    if kind == "somm":
        e, a, b = u64(seed, 1, m, k), u64(seed, 2, m, k), u64(seed, 3, k, n)
        f, c = junk(1, k, ld), junk(2, m, ld)
        want = (co.beaver_share(party, e, f[:, :kc], a, co.index_cols(b, idx, bs), c[:, :kc]) if t
                else np.zeros((m, 0), np.uint64))
    else:
        e, a, b = junk(3, m, ld), u64(seed, 2, m, k), u64(seed, 3, k, n)
        f, c = junk(4, ld, n), u64(seed, 5, m, n)
        want = co.beaver_share(party, e[:, :kc], f[:kc], co.index_cols(a, idx, bs), co.index_rows(b, idx, bs), c)
    return dict(party=party, e=e, f=f, a=a, b=b, c=c, want=want)


def _run_group(ctx, kind, m, k, n, bs, kept, spare, parties, planes=True, seed=0, single=False):
    """``single``: the members through one ``somm_share`` / ``simm_share`` call each instead."""
    idx = np.array(sorted(kept), dtype=np.int32)
    t, cap = len(idx), len(idx) + spare
    kc = t * bs
    gi = torch.zeros(max(cap, 1), dtype=torch.int32, device="cuda")
    gi[:t] = torch.from_numpy(idx).cuda()
    n_dev = torch.tensor([t], dtype=torch.int32, device="cuda")
    members, outs, wants = [], [], []
    for j, party in enumerate(parties):
        mb = _member(seed + 10 * j, kind, party, m, k, n, bs, idx, cap)
        wf = (lambda w: ctx.open_weight_planes(up(w))) if planes else up
        members.append((party, up(mb["e"]), wf(mb["f"]), up(mb["a"]), wf(mb["b"]), up(mb["c"])))
        zshape = (m, cap * bs) if kind == "somm" else (m, n)
        outs.append(torch.full(zshape, int(SENTINEL.view(np.int64)), dtype=torch.int64, device="cuda"))
        wants.append(mb["want"])
    if single:
        call = ctx.somm_share if kind == "somm" else ctx.simm_share
        got = [call(mb[0], bs, gi, n_dev, cap, *mb[1:], out=o) for mb, o in zip(members, outs)]
    else:
        got = ctx.share_group(kind, bs, gi, n_dev, cap, members, out=outs)
    torch.cuda.synchronize()
    for j, (z, want) in enumerate(zip(got, wants)):
        z = down(z)
        if kind == "somm":
            assert np.array_equal(z[:, :kc], want), "member %d" % j
            assert np.all(z[:, kc:] == SENTINEL), "member %d wrote beyond the kept columns" % j
        else:
            assert np.array_equal(z, want), "member %d" % j


# (kind, m, k, n, bs, kept blocks, spare capacity, parties of the members, forced grid)
# SOMM: n neurons = columns of B_i, output m x kept; SIMM: k neurons, output m x n.
CASES = [
    # 2 x 2 tiles per member, 4 members, 3 workgroups: ranges run across members and tiles
    ("somm", 200, 96, 16 * 32, 32, (0, 2, 3, 9), 1, (0, 1, 0, 1), 3),
    # the default grid (far more workgroups than tiles: many slices per tile, atomic adds)
    ("somm", 130, 200, 12 * 16, 16, (1, 2, 5, 6, 7, 10), 0, (1, 0), 0),
    # grid divides the tile count: 2 members x 4 tiles over 4 and over 8 workgroups, owned tiles
    ("somm", 256, 64, 8 * 32, 32, (0, 1, 4, 5), 0, (0, 1), 4),
    ("somm", 256, 64, 8 * 32, 32, (0, 1, 4, 5), 2, (0, 1), 8),
    # owned tiles with a contraction longer than one segment (2 * 4128 / 32 = 258 steps)
    ("somm", 128, 4128, 4 * 32, 32, (1, 2), 0, (1, 0), 2),
    # the same product on three workgroups: tiles cut into parts (some longer than one
    # accumulation segment), contraction steps taken in the rotated order
    ("somm", 128, 4128, 4 * 32, 32, (1, 2), 0, (1, 0), 3),
    ("somm", 256, 4128, 6 * 32, 32, (1, 2, 4), 1, (1, 0, 0), 5),
    # shared tiles, long contraction, one workgroup does everything
    ("somm", 70, 4128, 2 * 32, 32, (1,), 0, (0, 1, 1), 1),
    # eight members
    ("somm", 100, 40, 6 * 16, 16, (0, 3, 5), 0, (0, 1, 0, 1, 1, 0, 1, 0), 0),
    ("simm", 200, 16 * 32, 96, 32, (0, 2, 3, 9), 1, (0, 1, 0, 1), 3),
    ("simm", 130, 12 * 16, 200, 16, (1, 2, 5, 6, 7, 10), 0, (1, 0), 0),
    ("simm", 256, 8 * 32, 128, 32, (0, 1, 4, 5), 0, (0, 1), 4),
    ("simm", 256, 8 * 32, 128, 32, (0, 1, 4, 5), 2, (0, 1), 8),
    ("simm", 128, 140 * 32, 64, 32, tuple(range(0, 140, 1))[:130], 0, (1, 0), 2),
    ("simm", 128, 140 * 32, 64, 32, tuple(range(0, 140, 1))[:130], 0, (1, 0), 3),
    ("simm", 256, 140 * 32, 128, 32, tuple(range(3, 140, 1))[:131], 2, (0, 1, 1), 5),
    ("simm", 100, 6 * 16, 40, 16, (0, 3, 5), 0, (0, 1, 0, 1, 1, 0, 1, 0), 0),
]


@pytest.mark.parametrize("kind,m,k,n,bs,kept,spare,parties,grid", CASES)
def test_share_group_one_launch(ctx, kind, m, k, n, bs, kept, spare, parties, grid):
    import paper_2505_07239_amd as comet
    say("%s m=%d k=%d n=%d bs=%d kept=%d members=%d grid=%d" % (kind, m, k, n, bs, len(kept), len(parties), grid))
    ctx.set_tuning(comet.TUNE_GROUP, 1)
    ctx.set_tuning(comet.TUNE_GEMM_GRID, grid)
    try:
        _run_group(ctx, kind, m, k, n, bs, kept, spare, parties, seed=900)
    finally:
        ctx.set_tuning(comet.TUNE_GROUP, 0)
        ctx.set_tuning(comet.TUNE_GEMM_GRID, 0)


@pytest.mark.parametrize("single", [False, True])
@pytest.mark.parametrize("kept,spare", [((0, 1, 4, 5), 0), ((0, 4, 5), 1), ((1, 5), 2), ((3,), 3), ((), 4)])
def test_owned_tiles_follow_the_device_side_block_count(ctx, kept, spare, single):
    """A launch planned for owned tiles (capacity of four blocks: 2 x 2 tiles per product on a grid
    that divides their number) with fewer blocks on the device: a ragged last tile still owned,
    a tile count the grid no longer divides (shared tiles after all, and the packing kernel has to
    initialise Z after all), and no block at all.  Weight planes (single and grouped calls)."""
    import paper_2505_07239_amd as comet
    say("owned tiles, kept=%s capacity=%d single=%s" % (kept, len(kept) + spare, single))
    ctx.set_tuning(comet.TUNE_GROUP, 1)
    ctx.set_tuning(comet.TUNE_GEMM_GRID, 4)
    try:
        _run_group(ctx, "somm", 256, 64, 8 * 32, 32, kept, spare, (0, 1), seed=980, single=single)
    finally:
        ctx.set_tuning(comet.TUNE_GROUP, 0)
        ctx.set_tuning(comet.TUNE_GEMM_GRID, 0)


@pytest.mark.parametrize("kind", ["somm", "simm"])
@pytest.mark.parametrize("mode", [0, 2])
def test_share_group_automatic_and_switched_off(ctx, kind, mode):
    """Mode 0 decides by the size of a member (this one is far too small for a joint launch),
    mode 2 never groups: both run the members one after the other."""
    import paper_2505_07239_amd as comet
    ctx.set_tuning(comet.TUNE_GROUP, mode)
    try:
        dims = (200, 96, 16 * 32) if kind == "somm" else (200, 16 * 32, 96)
        _run_group(ctx, kind, *dims, 32, (0, 2, 3, 9), 1, (0, 1, 1), seed=950)
    finally:
        ctx.set_tuning(comet.TUNE_GROUP, 0)


@pytest.mark.parametrize("kind", ["somm", "simm"])
def test_share_group_fallbacks(ctx, kind):
    """Word operands and activations of at most 64 rows are not grouped even when asked to."""
    import paper_2505_07239_amd as comet
    ctx.set_tuning(comet.TUNE_GROUP, 1)
    try:
        dims = (150, 64, 8 * 16) if kind == "somm" else (150, 8 * 16, 64)
        say("%s group of word operands" % kind)
        _run_group(ctx, kind, *dims, 16, (1, 2, 6), 0, (0, 1), planes=False, seed=960)
        for m in (5, 64):
            say("%s group with m=%d" % (kind, m))
            _run_group(ctx, kind, m, *dims[1:], 16, (1, 2, 6), 0, (1, 0, 1), seed=970 + m)
    finally:
        ctx.set_tuning(comet.TUNE_GROUP, 0)


def test_share_group_at_bench_size_matches_single_calls(ctx):
    """The shape the automatic rule groups (LLaMA-7B gate projection, 256 tokens, 52 of 344 blocks):
    four members in one launch, bit for bit the result of the four single calls."""
    m, k, nb, bs, t = 256, 4096, 344, 32, 52
    idx = torch.arange(0, 2 * t, 2, dtype=torch.int32, device="cuda")
    n_dev = torch.tensor([t], dtype=torch.int32, device="cuda")
    words = lambda st, *shape: rng.uniform_u64_torch(77, st, int(np.prod(shape)), "cuda").view(*shape)
    members, single = [], []
    for j in range(4):
        e, a, c = words(10 * j + 1, m, k), words(10 * j + 2, m, k), words(10 * j + 3, m, t * bs)
        f = ctx.open_weight_planes(words(10 * j + 4, k, t * bs))
        b = ctx.open_weight_planes(words(10 * j + 5, k, nb * bs))
        members.append((j & 1, e, f, a, b, c))
        single.append(ctx.somm_share(j & 1, bs, idx, n_dev, t, e, f, a, b, c).clone())
    say("group of four at 256 x 4096 x 1664")
    outs = ctx.share_group("somm", bs, idx, n_dev, t, members)
    torch.cuda.synchronize()
    for z, want in zip(outs, single):
        assert torch.equal(z, want)
    # the oracle on a block of rows of the last member
    _, e, f, a, b, c = members[-1]
    rows = slice(100, 140)
    host = lambda x: x.cpu().numpy().view(np.uint64)
    f_w, b_w = host(words(34, k, t * bs)), host(words(35, k, nb * bs))
    want = co.beaver_share(1, host(e)[rows], f_w, host(a)[rows], co.index_cols(b_w, idx.cpu().numpy(), bs),
                           host(c)[rows])
    assert np.array_equal(host(outs[-1])[rows], want)


def test_share_group_argument_checks(ctx):
    import paper_2505_07239_amd as comet
    m, k, bs, t = 80, 64, 8, 2
    idx = torch.arange(t, dtype=torch.int32, device="cuda")
    mk = lambda s: (0, up(u64(s, 1, m, k)), ctx.open_weight_planes(up(u64(s, 4, k, t * bs))), up(u64(s, 2, m, k)),
                    ctx.open_weight_planes(up(u64(s, 5, k, 4 * bs))), up(u64(s, 3, m, t * bs)))
    with pytest.raises(ValueError):
        ctx.share_group("somm", bs, idx, None, t, [])
    with pytest.raises(ValueError):
        ctx.share_group("somm", bs, idx, None, t, [mk(1)] * 9)
    # raw C ABI: member count, operation code, null operand, party, workspace size
    from paper_2505_07239_amd.binding import ShareOperands
    one = mk(2)
    z = torch.empty((m, t * bs), dtype=torch.int64, device="cuda")
    arr = (ShareOperands * 2)()
    for j in range(2):
        arr[j] = ShareOperands(j, 0, *[x.data_ptr() for x in one[1:]], z.data_ptr())
    each = comet.workspace_bytes(comet.OP_SOMM, m, k, t * bs, bs)
    ws = ctx.workspace(2 * each)
    ptr = lambda x: ctypes.c_void_p(x.data_ptr())
    call = lambda op, n, members, wbytes: ctx.lib.comet_share_group(
        ctx.h, op, n, members, m, k, 4 * bs, bs, ptr(idx), None, t, comet.FULL_B | comet.WEIGHT_PLANES, ptr(ws), wbytes)
    assert call(comet.OP_SOMM, 0, arr, 2 * each) == -1
    assert call(comet.OP_SOMM, 9, arr, 2 * each) == -1
    assert call(comet.OP_COMPACT, 2, arr, 2 * each) == -1
    assert call(comet.OP_SOMM, 2, None, 2 * each) == -1
    assert call(comet.OP_SOMM, 2, arr, 2 * each - 1) != 0           # workspace too small
    bad = (ShareOperands * 2)()
    bad[0], bad[1] = arr[0], arr[1]
    bad[1].party = 2
    assert call(comet.OP_SOMM, 2, bad, 2 * each) == -1
    bad[1].party = 1
    bad[1].C_i = None
    assert call(comet.OP_SOMM, 2, bad, 2 * each) == -1
    assert call(comet.OP_SOMM, 1, arr, 2 * each) == 0               # a group of one is a single call
    torch.cuda.synchronize()


def _draw(case):
    r = rng.uniform_u64(4343, case, 12)
    pick = lambda i, lo, hi: lo + int(r[i] % np.uint64(hi - lo + 1))
    kind = "somm" if r[0] & np.uint64(1) else "simm"
    m = [65, 100, 128, 129, 200, 256, 300, 385][pick(1, 0, 7)]
    bs = [16, 32, 48, 64][pick(2, 0, 3)]
    nb = pick(3, 2, max(2, 640 // bs))
    keep = pick(4, 1, nb)
    other = pick(5, 1, 300)                       # the axis that is not indexed
    members = pick(6, 1, 5)
    grid = [0, 1, 2, 3, 4, 6, 8, 16][pick(7, 0, 7)]
    spare = pick(8, 0, 2)
    mode = 1 if r[9] & np.uint64(1) else 3        # with and without teams over the row tiles
    return kind, m, bs, nb, keep, other, members, grid, spare, mode


@pytest.mark.parametrize("case", range(40))
def test_share_group_sweep(ctx, case):
    """Seeded sweep of grouped launches over shapes, block sizes, member counts, grids and both
    ways of sharing out the row tiles, each member compared element by element with the oracle."""
    import paper_2505_07239_amd as comet
    from workloads import masks
    kind, m, bs, nb, keep, other, members, grid, spare, mode = _draw(case)
    mk = masks.uniform_block_mask(6000 + case, 1, nb, keep / nb)
    kept = tuple(int(v) for v in co.compact_mask(mk[None, :]))
    spare = min(spare, nb - len(kept))
    say("sweep %d: %s m=%d bs=%d nb=%d kept=%d other=%d members=%d grid=%d spare=%d mode=%d"
        % (case, kind, m, bs, nb, len(kept), other, members, grid, spare, mode))
    dims = (m, other, nb * bs) if kind == "somm" else (m, nb * bs, other)
    parties = tuple((case + j) & 1 for j in range(members))
    ctx.set_tuning(comet.TUNE_GROUP, mode)
    ctx.set_tuning(comet.TUNE_GEMM_GRID, grid)
    try:
        _run_group(ctx, kind, *dims, bs, kept, spare, parties, seed=7000 + 20 * case)
    finally:
        ctx.set_tuning(comet.TUNE_GROUP, 0)
        ctx.set_tuning(comet.TUNE_GEMM_GRID, 0)
