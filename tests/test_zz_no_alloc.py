"""The entry point that allocates nothing (``comet_somm_share_static``): same result as
``comet_somm_share`` and as the oracle, on two calls in a row that share the library's static
scratch array, the second one smaller than the first.  Calls go through the C ABI with raw
pointers; every buffer, the output included, is allocated before the calls."""
import ctypes
import sys

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

import oracle as co                                   # noqa: E402
from workloads import rng                             # noqa: E402

STATIC_SCRATCH_BYTES = 32 * 1024 * 1024


def say(msg):
    print("[gpu-no-alloc] " + msg, flush=True)
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


def u64(stream, *shape):
    return rng.uniform_u64(rng.BASE_SEED, 88000 + stream, int(np.prod(shape))).reshape(shape)


def _case(tag, m, k, nb, bs, kept):
    """Operands of one SOMM share on the device plus the oracle's result for both parties."""
    idx_np = np.array(sorted(kept), dtype=np.int32)
    t = len(idx_np)
    e, f = u64(tag + 1, m, k), u64(tag + 2, k, t * bs)
    a = [u64(tag + 3 + i, m, k) for i in (0, 1)]
    b = [u64(tag + 5 + i, k, nb * bs) for i in (0, 1)]
    c = [u64(tag + 7 + i, m, t * bs) for i in (0, 1)]
    want = [co.beaver_share(i, e, f, a[i], co.index_cols(b[i], idx_np, bs), c[i]) for i in (0, 1)]
    dev = dict(idx=torch.from_numpy(idx_np).cuda(), n=torch.tensor([t], dtype=torch.int32, device="cuda"),
               e=up(e), f=up(f), a=[up(v) for v in a], b=[up(v) for v in b], c=[up(v) for v in c])
    return dict(m=m, k=k, nb=nb, bs=bs, t=t, dev=dev, want=want)


def _raw_static(ctx, party, cs, out):
    """comet_somm_share_static through the C ABI, raw pointers only."""
    import paper_2505_07239_amd as comet
    d = cs["dev"]
    p = lambda t: ctypes.c_void_p(t.data_ptr())
    ctx._sync_stream()
    return ctx.lib.comet_somm_share_static(ctx.h, party, cs["m"], cs["k"], cs["nb"] * cs["bs"], cs["bs"],
                                           p(d["idx"]), p(d["n"]), cs["t"], comet.FULL_B, p(d["e"]),
                                           p(d["f"]), p(d["a"][party]), p(d["b"][party]), p(d["c"][party]),
                                           p(out))


def test_static_scratch_matches_workspace_call_twice_in_a_row(ctx):
    big = _case(0, 300, 512, 40, 32, range(3, 31, 2))          # 14 blocks: 300 x 1024 x 448, three row tiles
    small = _case(20, 70, 96, 12, 8, (1, 4, 5, 9))             # a smaller call on the same scratch
    few = _case(40, 5, 130, 12, 16, (0, 7, 11))                # the few-row kernel keeps its copy there too
    for name, cs in (("big", big), ("small", small), ("few rows", few), ("big again", big)):
        for party in (0, 1):
            say("%s party %d" % (name, party))
            d = cs["dev"]
            ref = ctx.somm_share(party, cs["bs"], d["idx"], d["n"], cs["t"], d["e"], d["f"], d["a"][party],
                                 d["b"][party], d["c"][party])
            out = torch.full_like(ref, 0x5A5A5A5A5A5A5A5A)
            torch.cuda.synchronize()
            before = torch.cuda.memory_allocated()
            rc = _raw_static(ctx, party, cs, out)
            assert rc == 0, ctx.lib.comet_last_error(ctx.h)
            torch.cuda.synchronize()
            assert torch.cuda.memory_allocated() == before          # torch's allocator was not touched
            assert np.array_equal(down(out), down(ref))
            assert np.array_equal(down(out), cs["want"][party])


def test_static_scratch_rejects_what_does_not_fit(ctx):
    import paper_2505_07239_amd as comet
    m, k, bs, t = 1024, 4096, 32, 4
    assert comet.workspace_bytes(comet.OP_SOMM, m, k, t * bs, bs) > STATIC_SCRATCH_BYTES
    z = torch.zeros((m, t * bs), dtype=torch.int64, device="cuda")
    e = torch.zeros((m, k), dtype=torch.int64, device="cuda")
    f = torch.zeros((k, t * bs), dtype=torch.int64, device="cuda")
    idx = torch.arange(t, dtype=torch.int32, device="cuda")
    with pytest.raises(comet.CometError) as ei:
        ctx.somm_share_static(0, bs, idx, None, t, e, f, e, f, z, b_full=False, out=z.clone())
    assert ei.value.code == -3 and "static" in str(ei.value)
    # the largest headline shape that fits: config 3's gate projection (256 x 4096, 52 blocks of 32)
    assert comet.workspace_bytes(comet.OP_SOMM, 256, 4096, 52 * 32, 32) <= STATIC_SCRATCH_BYTES
