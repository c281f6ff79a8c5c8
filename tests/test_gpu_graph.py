"""The whole chain (compact -> indexed masking -> open -> both parties' shares) captured in a HIP
graph and replayed: every call enqueues kernels only (no allocation, no memset, no host sync), so a
caller may capture it.  Each replay runs on new inputs written in place between replays, with eager
work and synchronisations in between, and is compared with the oracle."""
import sys

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

import oracle as co                                   # noqa: E402
from workloads import masks, rng                      # noqa: E402


def say(msg):
    print("[gpu-graph] " + msg, flush=True)
    sys.stdout.flush()


def up(a):
    return torch.from_numpy(np.ascontiguousarray(a).view(np.int64)).cuda()


def down(t):
    return t.cpu().numpy().view(np.uint64)


def u64(seed, stream, *shape):
    return rng.uniform_u64(seed, stream, int(np.prod(shape))).reshape(shape)


@pytest.mark.parametrize("m,grouped", [(8, False), (96, False), (96, True)])
def test_chain_replays_from_a_graph(m, grouped):
    """``grouped``: F is opened straight into digit planes and both parties' shares come out of one
    ``comet_share_group`` call (one packing launch, one matrix-core launch)."""
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2505_07239_amd as comet
    ctx = comet.Context(0)
    k, nb, bs, cap = 64, 24, 8, 9
    n_full, ld = nb * bs, cap * bs
    dev = torch.device("cuda:0")
    # static buffers the graph reads and writes
    mask = torch.zeros((1, nb), dtype=torch.uint8, device=dev)
    x = [torch.zeros((m, k), dtype=torch.int64, device=dev) for _ in (0, 1)]
    y = [up(u64(800, 3 + i, k, n_full)) for i in (0, 1)]
    a = [up(u64(800, 5 + i, m, k)) for i in (0, 1)]
    b = [up(u64(800, 7 + i, k, n_full)) for i in (0, 1)]
    c = [up(u64(800, 9 + i, m, ld)) for i in (0, 1)]
    idx = torch.zeros(nb, dtype=torch.int32, device=dev)
    n_dev = torch.zeros(1, dtype=torch.int32, device=dev)
    d = [torch.empty((m, k), dtype=torch.int64, device=dev) for _ in (0, 1)]
    g = [torch.empty((k, ld), dtype=torch.int64, device=dev) for _ in (0, 1)]
    e, f = torch.empty((m, k), dtype=torch.int64, device=dev), torch.empty((k, ld), dtype=torch.int64, device=dev)
    z = [torch.zeros((m, ld), dtype=torch.int64, device=dev) for _ in (0, 1)]
    if grouped:
        ctx.set_tuning(comet.TUNE_GROUP, 1)
        b_planes = [ctx.open_weight_planes(b[i]) for i in (0, 1)]      # offline, outside the graph
        f_planes = ctx.open_weight_planes(g[0], g[1])                   # buffer of the right size

    def chain():
        if grouped:
            ctx.compact_mask(mask, idx, n_dev)
            for i in (0, 1):
                ctx.mask_share(x[i], a[i], out=d[i])
                ctx.mask_share_gather(y[i], b[i], comet.AXIS_COLS, bs, idx, n_dev, cap, out=g[i])
            ctx.open(d[0], d[1], out=e)
            ctx.open_weight_planes(g[0], g[1], out=f_planes.buf)
            ctx.share_group("somm", bs, idx, n_dev, cap,
                            [(i, e, f_planes, a[i], b_planes[i], c[i]) for i in (0, 1)], out=z)
            return
        ctx.compact_mask(mask, idx, n_dev)
        for i in (0, 1):
            ctx.mask_share(x[i], a[i], out=d[i])
            ctx.mask_share_gather(y[i], b[i], comet.AXIS_COLS, bs, idx, n_dev, cap, out=g[i])
        ctx.open(d[0], d[1], out=e)
        ctx.open(g[0], g[1], out=f)
        for i in (0, 1):
            ctx.somm_share(i, bs, idx, n_dev, cap, e, f, a[i], b[i], c[i], out=z[i])

    def set_inputs(rep):
        mk = masks.uniform_block_mask(810 + rep, 1, nb, (3 + 2 * rep) / nb)[None, :]
        mask.copy_(torch.from_numpy(mk).to(dev))
        xs = [u64(820 + rep, i, m, k) for i in (0, 1)]
        for i in (0, 1):
            x[i].copy_(up(xs[i]))
        return mk, xs

    def expected(mk, xs):
        idx_np = co.compact_mask(mk)
        t = len(idx_np)
        yn, an, bn, cn = ([down(v) for v in q] for q in (y, a, b, c))
        e_ref = co.open_(co.mask_share(xs[0], an[0]), co.mask_share(xs[1], an[1]))
        f_ref = co.open_(co.mask_share(co.index_cols(yn[0], idx_np, bs), co.index_cols(bn[0], idx_np, bs)),
                         co.mask_share(co.index_cols(yn[1], idx_np, bs), co.index_cols(bn[1], idx_np, bs)))
        return t, [co.beaver_share(i, e_ref, f_ref, an[i], co.index_cols(bn[i], idx_np, bs),
                                   cn[i][:, :t * bs]) for i in (0, 1)]

    # warm up eagerly on a side stream (workspace allocation happens here, outside the capture)
    mk, xs = set_inputs(0)
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        chain()
    torch.cuda.current_stream().wait_stream(s)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        chain()
    for rep in range(1, 4):
        mk, xs = set_inputs(rep)
        for zz in z:
            zz.zero_()
        torch.cuda.synchronize()
        say("m=%d replay %d" % (m, rep))
        graph.replay()
        torch.cuda.synchronize()
        t, want = expected(mk, xs)
        assert int(n_dev.item()) == t
        for i in (0, 1):
            assert np.array_equal(down(z[i])[:, :t * bs], want[i]), "replay %d party %d" % (rep, i)
        # eager call on the same inputs gives the same bits
        chain()
        torch.cuda.synchronize()
        for i in (0, 1):
            assert np.array_equal(down(z[i])[:, :t * bs], want[i])
    ctx.close()
