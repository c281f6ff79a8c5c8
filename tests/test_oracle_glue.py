"""Pins of the oracle's glue steps around the hot path: oblivious shuffle (Protocol 1),
merge back to the full width, share-local rescaling."""
import os

import numpy as np
import pytest

import oracle as co
from oracle import protocols
from workloads import rng

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def u64(seed, stream, *shape):
    return rng.uniform_u64(seed, stream, int(np.prod(shape))).reshape(shape)


def perm(seed, stream, n):
    return np.argsort(rng.uniform_u64(seed, stream, n), kind="stable").astype(np.int32)


def test_permutation_convention_matches_the_papers_example():
    rows = {}
    for line in open(os.path.join(GOLDEN, "shuffle_example.txt")):
        if line.startswith("#") or not line.strip():
            continue
        key, *vals = line.split()
        rows[key] = [int(v) for v in vals]
    pi = np.array(rows["pi"], dtype=np.int32) - 1
    x = np.array([rows["x"]], dtype=np.uint64)
    out = co.permute_mask(x, pi, np.zeros_like(x), 0, +1)
    assert out[0].tolist() == rows["out"]


@pytest.mark.parametrize("rows,cols,axis", [(1, 7, 0), (5, 9, 0), (6, 4, 1), (33, 17, 1), (17, 33, 0)])
def test_shuffle_reconstructs_to_the_permuted_secret(rows, cols, axis):
    n = cols if axis == 0 else rows
    seed = 50 + rows
    pi, t1, t2 = perm(seed, 1, n), perm(seed, 2, n), perm(seed, 3, n)
    mat = protocols.shuffle_offline(pi, t1, t2, u64(seed, 4, rows, cols), u64(seed, 5, rows, cols),
                                    u64(seed, 6, rows, cols), axis)
    # the two decompositions of pi: rho_i o tau_other = pi
    for i in (0, 1):
        assert np.array_equal(protocols.compose(mat.rho[i], mat.tau[1 - i]), pi)
    x = u64(seed, 7, rows, cols)
    x_sh = co.share(x, u64(seed, 8, rows, cols))
    z, y = protocols.shuffle_online(x_sh, mat, axis)
    want = x[:, pi] if axis == 0 else x[pi, :]
    assert np.array_equal(co.reconstruct(*z), want)
    # neither output share alone is the permuted input share
    assert not np.array_equal(z[0], x_sh[0][:, pi] if axis == 0 else x_sh[0][pi, :])
    # what is exchanged is masked: y_i - a_i is tau_i(x_i), y_i itself is not
    tx = x_sh[0][:, mat.tau[0]] if axis == 0 else x_sh[0][mat.tau[0], :]
    assert np.array_equal(y[0] - mat.a[0], tx) and not np.array_equal(y[0], tx)


def test_same_sub_permutations_align_two_tensors_and_unshuffle_restores():
    rows, cols, axis, seed = 4, 12, 0, 61
    pi, t1, t2 = perm(seed, 1, cols), perm(seed, 2, cols), perm(seed, 3, cols)
    x, s = u64(seed, 7, rows, cols), u64(seed, 9, rows, cols)
    outs = []
    for k, v in enumerate((x, s)):          # same (rho, tau), fresh masks each time
        mat = protocols.shuffle_offline(pi, t1, t2, u64(seed, 20 + k, rows, cols),
                                        u64(seed, 30 + k, rows, cols), u64(seed, 40 + k, rows, cols), axis)
        z, _ = protocols.shuffle_online(co.share(v, u64(seed, 50 + k, rows, cols)), mat, axis)
        outs.append(z)
        assert np.array_equal(co.reconstruct(*z), v[:, pi])
    back = protocols.unshuffle_material(mat, u64(seed, 60, rows, cols), u64(seed, 61, rows, cols),
                                        u64(seed, 62, rows, cols), axis)
    for i in (0, 1):
        assert np.array_equal(protocols.compose(back.rho[i], back.tau[1 - i]), protocols.inverse(pi))
    z, _ = protocols.shuffle_online(outs[0], back, axis)
    assert np.array_equal(co.reconstruct(*z), x)


def test_scatter_is_the_inverse_of_indexing_and_zero_elsewhere():
    m, nb, bs = 5, 9, 4
    idx = np.array([1, 4, 7], dtype=np.int32)
    c = u64(70, 1, m, len(idx) * bs)
    full = co.scatter_cols(c, idx, bs, nb * bs)
    assert np.array_equal(co.index_cols(full, idx, bs), c)
    rest = np.setdiff1d(np.arange(nb), idx).astype(np.int32)
    assert not co.index_cols(full, rest, bs).any()
    # shares scattered separately reconstruct to the scattered secret
    sh = co.share(c, u64(70, 2, *c.shape))
    assert np.array_equal(co.reconstruct(co.scatter_cols(sh[0], idx, bs, nb * bs),
                                         co.scatter_cols(sh[1], idx, bs, nb * bs)), full)


def test_share_local_rescaling_is_within_one_unit():
    """Products of two Q16 values carry 32 fractional bits; each party shifts its own share."""
    n, f = 20000, 16
    a = (rng.gaussian_f64(80, 1, n) * 3.0)
    b = (rng.gaussian_f64(80, 2, n) * 3.0)
    prod = co.encode(a) * co.encode(b)                        # scale 2^32, exact in the ring
    sh = co.share(prod, u64(80, 3, n))
    t = [co.truncate_share(i, sh[i], f) for i in (0, 1)]
    got = co.reconstruct(*t).view(np.int64)
    exact = prod.view(np.int64) >> f                          # floor of the true quotient
    assert np.all(np.abs(got - exact) <= 1)
    # decoded, the result is the product to within fixed-point resolution
    assert np.max(np.abs(co.decode(co.reconstruct(*t)) - a * b)) < 2 ** -12
    # with a zero share for party 1 the rule is exactly the floor
    z = prod
    assert np.array_equal(co.truncate_share(0, z, f).view(np.int64), exact)
    assert not co.truncate_share(1, np.zeros(4, np.uint64), f).any()
    # party 1 rounds towards +inf: -floor(-v / 2^f) = ceil(v / 2^f)
    v = np.array([5 << 16, (5 << 16) + 1, np.uint64(2 ** 64 - 3)], dtype=np.uint64)
    want = np.array([5, 6, 0], dtype=np.int64)                # ceil(-3 / 65536) = 0
    assert np.array_equal(co.truncate_share(1, v, f).view(np.int64), want)


def test_share_local_rescaling_wraps_when_the_shares_straddle_the_ring():
    """The known failure mode: a small secret whose shares wrap around 2^64 comes out wrong by
    2^(64-f); it happens with probability about |z| / 2^63 over the sharing randomness."""
    f = 16
    z = np.array([1 << 20], dtype=np.uint64)
    z0 = np.array([(1 << 63) + 5], dtype=np.uint64)           # negative as a signed word
    z1 = z - z0                                               # also negative as a signed word
    t = [co.truncate_share(i, s, f) for i, s in enumerate((z0, z1))]
    got = int(co.reconstruct(*t).view(np.int64)[0])
    assert abs(got - (1 << 4)) > 1 and abs((got - (1 << 4)) % (1 << 48)) <= 1


def test_mha_masks_shape_and_structure():
    from workloads import configs
    cfg = configs.mha_config()
    qkv, out = configs.mha_head_masks(cfg)
    h = cfg.n_heads
    assert qkv.shape == (cfg.rows, 3 * h) and out.shape == (cfg.tokens, h)
    assert np.all(out.sum(axis=1) == round(cfg.head_density * h))
    # current tokens keep Q, K and V of their heads; refill rows ask for K and V only
    assert np.array_equal(qkv[:cfg.tokens, :h], out) and np.array_equal(qkv[:cfg.tokens, h:2 * h], out)
    assert not qkv[cfg.tokens:, :h].any()
    assert np.array_equal(qkv[cfg.tokens:, h:2 * h], qkv[cfg.tokens:, 2 * h:])
    assert np.all(qkv[cfg.tokens:].sum(axis=1) >= 2)
