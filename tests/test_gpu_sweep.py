"""Seeded sweep of share calls over shapes, block sizes, densities and operand forms inside the
documented limits, each compared element by element with the oracle.  The shapes are drawn from
the counter-based generator, so the sweep is the same on every run."""
import sys

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

import oracle as co                                   # noqa: E402
from workloads import masks, rng                      # noqa: E402


def say(msg):
    print("[gpu-sweep] " + msg, flush=True)
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


def draw(case):
    r = rng.uniform_u64(4242, case, 12)
    pick = lambda i, lo, hi: lo + int(r[i] % np.uint64(hi - lo + 1))
    kind = "somm" if r[0] & np.uint64(1) else "simm"
    m = [1, 7, 16, 17, 33, 64, 65, 129, 200, 257][pick(1, 0, 9)]
    bs = [1, 2, 3, 8, 16, 20, 32, 64][pick(2, 0, 7)]
    nb = pick(3, 2, max(2, min(40, 640 // bs)))
    keep = pick(4, 1, nb)
    other = pick(5, 1, 300)                       # the axis that is not indexed
    party = pick(6, 0, 1)
    compact = bool(r[7] & np.uint64(1))            # triple shares passed already indexed
    spare = pick(8, 0, 2)                          # capacity beyond the kept blocks
    on_device = bool(r[9] & np.uint64(1))          # block count on the device or from the capacity
    return kind, m, bs, nb, keep, other, party, compact, spare, on_device


@pytest.mark.parametrize("fmt", ["words", "planes"])
@pytest.mark.parametrize("case", range(48))
def test_share_sweep(ctx, case, fmt):
    """``fmt``: the weight-side operands F and B_i as words or as digit planes."""
    kind, m, bs, nb, keep, other, party, compact, spare, on_device = draw(case)
    if fmt == "planes" and kind == "simm" and bs % 16:
        compact = True        # planes of a full-size B_i are gathered in units of sixteen rows
    wt = (lambda a: ctx.open_weight_planes(up(a))) if fmt == "planes" else up
    if not on_device:
        spare = 0                                  # without a device count the capacity is the count
    full = nb * bs
    say("case %d (%s): %s m=%d bs=%d nb=%d keep=%d other=%d party=%d compact=%s spare=%d device_count=%s"
        % (case, fmt, kind, m, bs, nb, keep, other, party, compact, spare, on_device))
    seed = 5000 + case
    mk = masks.uniform_block_mask(seed, 1, nb, keep / nb)
    idx_np = co.compact_mask(mk[None, :])
    t = len(idx_np)
    if not compact:
        spare = min(spare, nb - t)                 # a full-size operand bounds the capacity
    cap = t + spare
    ld = cap * bs
    gi = torch.zeros(max(cap, 1), dtype=torch.int32, device="cuda")
    gi[:t] = torch.from_numpy(idx_np).cuda()
    n_dev = torch.tensor([t], dtype=torch.int32, device="cuda") if on_device else None

    def pad_cols(a):
        out = u64(seed, 90, a.shape[0], ld)
        out[:, :a.shape[1]] = a
        return out

    def pad_rows(a):
        out = u64(seed, 91, ld, a.shape[1])
        out[:a.shape[0]] = a
        return out

    if kind == "somm":
        k, n_act = other, t * bs
        e, a = u64(seed, 2, m, k), u64(seed, 3, m, k)
        f, b = u64(seed, 4, k, n_act), u64(seed, 5, k, full)
        c = u64(seed, 6, m, n_act)
        b_sel = co.index_cols(b, idx_np, bs)
        want = co.beaver_share(party, e, f, a, b_sel, c)
        z = ctx.somm_share(party, bs, gi, n_dev, cap, up(e), wt(pad_cols(f)), up(a),
                           wt(pad_cols(b_sel)) if compact else wt(b), up(pad_cols(c)), b_full=not compact)
        torch.cuda.synchronize()
        assert np.array_equal(down(z)[:, :n_act], want)
    else:
        n, k_act = other, t * bs
        e, a = u64(seed, 2, m, k_act), u64(seed, 3, m, full)
        f, b = u64(seed, 4, k_act, n), u64(seed, 5, full, n)
        c = u64(seed, 6, m, n)
        a_sel, b_sel = co.index_cols(a, idx_np, bs), co.index_rows(b, idx_np, bs)
        want = co.beaver_share(party, e, f, a_sel, b_sel, c)
        z = ctx.simm_share(party, bs, gi, n_dev, cap, up(pad_cols(e)), wt(pad_rows(f)),
                           up(pad_cols(a_sel)) if compact else up(a),
                           wt(pad_rows(b_sel)) if compact else wt(b), up(c),
                           a_full=not compact, b_full=not compact)
        torch.cuda.synchronize()
        assert np.array_equal(down(z), want)
