"""Error behaviour of the share calls through the binding (argument checks happen on the host, before
any launch) and the documented handling of block ids that do not fit the indexed axis."""
import ctypes
import sys

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

import oracle as co                                   # noqa: E402
from workloads import rng                             # noqa: E402


def say(msg):
    print("[gpu-errors] " + msg, flush=True)
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


def _raw_somm(ctx, party, m, k, n_full, bs, idx, cap, flags, e, f, a, b, c, z, ws, ws_bytes):
    p = lambda t: None if t is None else ctypes.c_void_p(t.data_ptr())
    return ctx.lib.comet_somm_share(ctx.h, party, m, k, n_full, bs, p(idx), None, cap, flags, p(e), p(f),
                                    p(a), p(b), p(c), p(z), p(ws), ws_bytes)


def test_share_argument_checks(ctx):
    import paper_2505_07239_amd as comet
    m, k, nb, bs, cap = 40, 64, 6, 8, 3
    n_full, ld = nb * bs, cap * bs
    e, a = up(u64(700, 1, m, k)), up(u64(700, 2, m, k))
    f, b = up(u64(700, 3, k, ld)), up(u64(700, 4, k, n_full))
    c, z = up(u64(700, 5, m, ld)), torch.empty((m, ld), dtype=torch.int64, device="cuda")
    idx = torch.tensor([0, 2, 5], dtype=torch.int32, device="cuda")
    need = comet.workspace_bytes(comet.OP_SOMM, m, k, ld, bs)
    ws = ctx.workspace(need)
    args = (m, k, n_full, bs, idx, cap, comet.FULL_B, e, f, a, b, c, z)
    say("argument checks")
    assert _raw_somm(ctx, 1, *args, ws, need) == 0
    assert _raw_somm(ctx, 2, *args, ws, need) == -1                       # party
    assert _raw_somm(ctx, 1, *args, ws, need - 1) == -5                   # workspace too small
    assert b"workspace" in ctx.lib.comet_last_error(ctx.h)
    assert _raw_somm(ctx, 1, *args, None, need) == -5
    assert _raw_somm(ctx, 1, m, k, n_full, bs, None, cap, comet.FULL_B, e, f, a, b, c, z, ws, need) == -1
    assert _raw_somm(ctx, 1, m, k, 2 * bs, bs, idx, cap, comet.FULL_B, e, f, a, b, c, z, ws, need) == -1
    assert _raw_somm(ctx, 1, m, k, n_full, bs, idx, cap, comet.FULL_A, e, f, a, b, c, z, ws, need) == -1
    assert _raw_somm(ctx, 1, m, k, n_full, bs, idx, cap, comet.FULL_B, e, f, a, b, None, z, ws, need) == -1
    mis = torch.empty(m * ld + 1, dtype=torch.int64, device="cuda")[1:].view(m, ld)
    assert _raw_somm(ctx, 1, m, k, n_full, bs, idx, cap, comet.FULL_B, e, f, a, b, c, mis, ws, need) == -2
    assert _raw_somm(ctx, 1, 1 << 23, k, n_full, bs, idx, cap, comet.FULL_B, e, f, a, b, c, z, ws, need) == -3
    torch.cuda.synchronize()


@pytest.mark.parametrize("m", [8, 70])
def test_block_ids_outside_the_axis_read_block_zero(ctx, m):
    """Documented behaviour: an id that does not fit the indexed axis is read as block 0; the call
    completes normally whatever the list holds (here: for both the few-row and the matrix kernel)."""
    k, nb, bs = 48, 6, 8
    n_full = nb * bs
    bad = np.array([1, 1 << 20, -7, 4], dtype=np.int32)
    as_read = np.array([1, 0, 0, 4], dtype=np.int32)
    t = len(bad)
    e, a = u64(710 + m, 1, m, k), u64(710 + m, 2, m, k)
    f, b = u64(710 + m, 3, k, t * bs), u64(710 + m, 4, k, n_full)
    c = u64(710 + m, 5, m, t * bs)
    say("bad block ids m=%d" % m)
    idx = torch.from_numpy(bad).cuda()
    z = ctx.somm_share(1, bs, idx, None, t, up(e), up(f), up(a), up(b), up(c))
    torch.cuda.synchronize()
    want = co.beaver_share(1, e, f, a, co.index_cols(b, as_read, bs), c)
    assert np.array_equal(down(z), want)


@pytest.mark.parametrize("m,bs", [(8, 8), (70, 8), (70, 6), (40, 16)])
@pytest.mark.parametrize("full", [True, False])
def test_simm_block_ids_outside_the_axis_read_block_zero(ctx, m, bs, full):
    """Same rule on the contraction axis: the rows of B_i and the columns of A_i of a block whose id
    does not fit are those of block 0 (few-row kernel, power-of-two and general block sizes)."""
    nb, n = 7, 40
    k_full = nb * bs
    bad = np.array([2, -1, 1 << 18, 5], dtype=np.int32)
    as_read = np.array([2, 0, 0, 5], dtype=np.int32)
    t = len(bad)
    seed = 730 + m + bs
    e, a = u64(seed, 1, m, t * bs), u64(seed, 2, m, k_full)
    f, b = u64(seed, 3, t * bs, n), u64(seed, 4, k_full, n)
    c = u64(seed, 5, m, n)
    say("bad block ids (simm) m=%d bs=%d full=%s" % (m, bs, full))
    idx = torch.from_numpy(bad).cuda()
    a_sel, b_sel = co.index_cols(a, as_read, bs), co.index_rows(b, as_read, bs)
    if full:
        z = ctx.simm_share(1, bs, idx, None, t, up(e), up(f), up(a), up(b), up(c))
    else:                                     # already indexed operands: the list is not consulted
        z = ctx.simm_share(1, bs, idx, None, t, up(e), up(f), up(a_sel), up(b_sel), up(c),
                           a_full=False, b_full=False)
    torch.cuda.synchronize()
    assert np.array_equal(down(z), co.beaver_share(1, e, f, a_sel, b_sel, c))


@pytest.mark.parametrize("axis", [0, 1])
def test_indexed_masking_skips_blocks_that_do_not_fit(ctx, axis):
    """comet_mask_share_gather leaves the outputs of a block whose id does not fit untouched."""
    import paper_2505_07239_amd as comet
    rows, cols, bs = (9, 48, 8) if axis == 0 else (48, 9, 8)
    bad = np.array([1, 999, -3, 4], dtype=np.int32)
    t = len(bad)
    w, b = u64(750 + axis, 1, rows, cols), u64(750 + axis, 2, rows, cols)
    shape = (rows, t * bs) if axis == 0 else (t * bs, cols)
    out = torch.full(shape, -5, dtype=torch.int64, device="cuda")
    say("indexed masking with ids that do not fit, axis %d" % axis)
    ctx.mask_share_gather(up(w), up(b), axis, bs, torch.from_numpy(bad).cuda(), None, t, out=out)
    torch.cuda.synchronize()
    got = down(out)
    d = w - b
    for pos, blk in enumerate(bad):
        sl = slice(pos * bs, (pos + 1) * bs)
        piece = got[:, sl] if axis == 0 else got[sl, :]
        if 0 <= blk and (blk + 1) * bs <= (cols if axis == 0 else rows):
            want = d[:, blk * bs:(blk + 1) * bs] if axis == 0 else d[blk * bs:(blk + 1) * bs, :]
            assert np.array_equal(piece, want)
        else:
            assert np.all(piece.view(np.int64) == -5)
