"""GPU parity of the local steps around the products: oblivious shuffle steps, merge back to the
full width, share-local rescaling -- element by element against the oracle."""
import sys

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

import oracle as co                                   # noqa: E402
from oracle import protocols                          # noqa: E402
from workloads import rng                             # noqa: E402


def say(msg):
    print("[gpu-glue] " + msg, flush=True)
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


def perm(seed, stream, n):
    return np.argsort(rng.uniform_u64(seed, stream, n), kind="stable").astype(np.int32)


@pytest.mark.parametrize("rows,cols,axis", [(1, 7, 0), (5, 9, 0), (64, 11008, 0), (3, 20000, 0), (2, 16384, 0),
                                            (300, 1000, 0), (33, 17, 1), (200, 4096, 1), (7, 1025, 1),
                                            (1, 1, 0), (1, 1, 1)])
@pytest.mark.parametrize("sign", [1, -1])
def test_permute_mask(ctx, rows, cols, axis, sign):
    say("permute rows=%d cols=%d axis=%d sign=%d" % (rows, cols, axis, sign))
    seed = 500 + rows + cols
    src, mask = u64(seed, 1, rows, cols), u64(seed, 2, rows, cols)
    p = perm(seed, 3, cols if axis == 0 else rows)
    got = ctx.permute_mask(up(src), torch.from_numpy(p).cuda(), up(mask), axis, sign)
    torch.cuda.synchronize()
    assert np.array_equal(down(got), co.permute_mask(src, p, mask, axis, sign))


@pytest.mark.parametrize("rows,cols,axis", [(16, 3072, 0), (344, 64, 1)])
def test_oblivious_shuffle_both_parties(ctx, rows, cols, axis):
    """Protocol 1 end to end with the GPU doing every local step of both parties."""
    say("shuffle rows=%d cols=%d axis=%d" % (rows, cols, axis))
    n = cols if axis == 0 else rows
    seed = 520 + axis
    pi, t1, t2 = perm(seed, 1, n), perm(seed, 2, n), perm(seed, 3, n)
    mat = protocols.shuffle_offline(pi, t1, t2, u64(seed, 4, rows, cols), u64(seed, 5, rows, cols),
                                    u64(seed, 6, rows, cols), axis)
    x = u64(seed, 7, rows, cols)
    x_sh = co.share(x, u64(seed, 8, rows, cols))
    z_ref, y_ref = protocols.shuffle_online(x_sh, mat, axis)
    dev = lambda p: torch.from_numpy(p).cuda()
    y = [ctx.permute_mask(up(x_sh[i]), dev(mat.tau[i]), up(mat.a[i]), axis, +1) for i in (0, 1)]
    z = [ctx.permute_mask(y[1 - i], dev(mat.rho[i]), up(mat.b[i]), axis, -1) for i in (0, 1)]
    torch.cuda.synchronize()
    for i in (0, 1):
        assert np.array_equal(down(y[i]), y_ref[i]) and np.array_equal(down(z[i]), z_ref[i])
    want = x[:, pi] if axis == 0 else x[pi, :]
    assert np.array_equal(down(z[0]) + down(z[1]), want)


@pytest.mark.parametrize("m,nb,bs,keep,spare", [(5, 9, 4, 3, 0), (16, 344, 32, 52, 0), (7, 11, 3, 4, 2),
                                                (33, 20, 5, 20, 0), (4, 6, 8, 0, 1)])
def test_scatter_cols(ctx, m, nb, bs, keep, spare):
    say("scatter m=%d nb=%d bs=%d keep=%d" % (m, nb, bs, keep))
    seed = 540 + m
    idx = np.sort(perm(seed, 1, nb)[:keep]).astype(np.int32)
    cap = keep + spare
    c = u64(seed, 2, m, cap * bs)
    gi = torch.zeros(max(cap, 1), dtype=torch.int32, device="cuda")
    gi[:keep] = torch.from_numpy(idx).cuda()
    n_dev = torch.tensor([keep], dtype=torch.int32, device="cuda")
    out = torch.full((m, nb * bs), -1, dtype=torch.int64, device="cuda")
    ctx.scatter_cols(up(c), bs, gi, n_dev, cap, nb * bs, out=out)
    torch.cuda.synchronize()
    assert np.array_equal(down(out), co.scatter_cols(c[:, :keep * bs], idx, bs, nb * bs))


@pytest.mark.parametrize("n", [1, 2, 1001, 1 << 20])
@pytest.mark.parametrize("party", [0, 1])
def test_truncate_share(ctx, n, party):
    say("truncate n=%d party %d" % (n, party))
    z = u64(560, party, n)
    z[:4] = np.array([0, 1, 2 ** 64 - 1, 1 << 63], dtype=np.uint64)[:min(4, n)]
    for f in (16, 1, 0):
        got = ctx.truncate_share(party, up(z), f)
        torch.cuda.synchronize()
        assert np.array_equal(down(got), co.truncate_share(party, z, f))
