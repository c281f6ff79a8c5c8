"""Pins for the oracle's primitives: ring product, fixed point, sharing, Eq. 1.

Each check compares the C oracle with something that is not the oracle:
Python big integers reduced mod 2^64, numpy's integer matmul, hand-worked
numbers (tests/golden/eq1_scalar.txt), or float64 arithmetic.
"""
import os

import numpy as np
import pytest

import oracle as co
from workloads import rng

M64 = (1 << 64) - 1


def big(a):
    """numpy uint64 array -> nested lists of Python ints."""
    return [[int(v) for v in row] for row in np.asarray(a)]


def big_matmul(x, y):
    x, y = big(x), big(y)
    m, k, n = len(x), len(y), len(y[0])
    return np.array([[sum(x[i][l] * y[l][j] for l in range(k)) & M64 for j in range(n)]
                     for i in range(m)], dtype=np.uint64)


def u64(seed, stream, *shape):
    return rng.uniform_u64(seed, stream, int(np.prod(shape))).reshape(shape)


@pytest.mark.parametrize("m,k,n", [(1, 1, 1), (2, 3, 4), (4, 2, 3), (3, 5, 2), (7, 4, 1)])
def test_ring_matmul_brute_force_bigint(m, k, n):
    # full-range operands: every product overflows 64 bits, so the wrap is exercised;
    # non-square shapes catch transposed operands and swapped strides
    x, y = u64(11, 1, m, k), u64(11, 2, k, n)
    assert np.array_equal(co.ring_matmul(x, y), big_matmul(x, y))


def test_ring_matmul_known_values():
    x = np.array([[1, 2], [3, 4]], dtype=np.uint64)
    y = np.array([[5, 6, 7], [8, 9, 10]], dtype=np.uint64)
    assert co.ring_matmul(x, y).tolist() == [[21, 24, 27], [47, 54, 61]]
    # (2^64 - 1)^2 = 1 mod 2^64;  2^63 * 2 = 0 mod 2^64
    top = np.array([[M64]], dtype=np.uint64)
    assert co.ring_matmul(top, top).tolist() == [[1]]
    assert co.ring_matmul(np.array([[1 << 63]], dtype=np.uint64),
                          np.array([[2]], dtype=np.uint64)).tolist() == [[0]]


def test_ring_matmul_vs_numpy_integer_matmul():
    x, y = u64(12, 1, 37, 129), u64(12, 2, 129, 53)
    assert np.array_equal(co.ring_matmul(x, y), x @ y)


def test_ring_matmul_is_not_commutative_guard():
    # a transposed-operand bug would pass on symmetric inputs; make sure ours are not
    x, y = u64(13, 1, 3, 3), u64(13, 2, 3, 3)
    assert not np.array_equal(co.ring_matmul(x, y), co.ring_matmul(y, x))
    assert np.array_equal(co.ring_matmul(x, y), big_matmul(x, y))


def test_encode_decode_fixed_point():
    x = np.array([0.0, 1.0, -1.0, 0.5, -0.5, 1.5 / 65536, -1.5 / 65536, 2.5 / 65536, 1e-9, 3.25])
    q = co.encode(x, 16)
    expect = [0, 65536, (1 << 64) - 65536, 32768, (1 << 64) - 32768, 2, (1 << 64) - 2, 3, 0, 212992]
    assert [int(v) for v in q] == expect          # ties round away from zero
    back = co.decode(q, 16)
    assert back[:5].tolist() == [0.0, 1.0, -1.0, 0.5, -0.5]
    assert np.max(np.abs(back - x)) <= 0.5 / 65536
    # decode at 32 fractional bits (the scale of a product of two Q16 values)
    assert co.decode(np.array([1 << 32, M64], dtype=np.uint64), 32).tolist() == [1.0, -(2.0 ** -32)]


def test_encode_error_bound_random():
    x = rng.gaussian_f64(5, 1, 10000)
    back = co.decode(co.encode(x, 16), 16)
    assert np.max(np.abs(back - x)) <= 2.0 ** -17


def test_share_reconstruct_bigint():
    v, r = u64(14, 1, 5, 7), u64(14, 2, 5, 7)
    v0, v1 = co.share(v, r)
    assert np.array_equal(v0, r)
    for a, b, c in zip(v0.ravel(), v1.ravel(), v.ravel()):
        assert (int(a) + int(b)) & M64 == int(c)
    assert np.array_equal(co.reconstruct(v0, v1), v)
    # reconstruction is a sum, not a difference
    assert co.reconstruct(np.array([3], dtype=np.uint64), np.array([M64], dtype=np.uint64)).tolist() == [2]


def test_mask_share_and_open_bigint():
    x, a = u64(15, 1, 9), u64(15, 2, 9)
    d = co.mask_share(x, a)
    assert [int(v) for v in d] == [(int(p) - int(q)) & M64 for p, q in zip(x, a)]
    e = co.open_(x, a)
    assert [int(v) for v in e] == [(int(p) + int(q)) & M64 for p, q in zip(x, a)]


def _golden(path):
    vals = {}
    with open(path) as fh:
        for line in fh:
            if line.startswith("#") or not line.strip():
                continue
            k, v = line.split()
            vals[k] = int(v) & M64
    return vals


def test_eq1_hand_worked_scalar(golden_dir):
    g = _golden(os.path.join(golden_dir, "eq1_scalar.txt"))
    arr = lambda key: np.array([[g[key]]], dtype=np.uint64)
    d = [co.mask_share(arr("x_%d" % i), arr("a_%d" % i)) for i in (1, 2)]
    f = [co.mask_share(arr("y_%d" % i), arr("b_%d" % i)) for i in (1, 2)]
    dd, ee = co.open_(d[0], d[1]), co.open_(f[0], f[1])
    assert int(dd[0, 0]) == g["d"] and int(ee[0, 0]) == g["e"]
    # the paper's P_1 is party 0 here, P_2 is party 1 (the one that adds d*e)
    z1 = co.beaver_share(0, dd, ee, arr("a_1"), arr("b_1"), arr("c_1"))
    z2 = co.beaver_share(1, dd, ee, arr("a_2"), arr("b_2"), arr("c_2"))
    assert int(z1[0, 0]) == g["z_1"]
    assert int(z2[0, 0]) == g["z_2"]
    assert int(co.beaver_share_at(1, dd, ee, arr("a_2"), arr("b_2"), arr("c_2"), 0, 0)) == g["z_2"]


@pytest.mark.parametrize("party", [0, 1])
@pytest.mark.parametrize("m,k,n", [(2, 3, 4), (4, 3, 2), (1, 5, 3)])
def test_beaver_share_formula_bigint(party, m, k, n):
    e, a = u64(16, 1, m, k), u64(16, 2, m, k)
    f, b = u64(16, 3, k, n), u64(16, 4, k, n)
    c = u64(16, 5, m, n)
    eb, af, ef = big_matmul(e, b), big_matmul(a, f), big_matmul(e, f)
    want = [[(int(c[i, j]) + int(eb[i, j]) + int(af[i, j]) + party * int(ef[i, j])) & M64
             for j in range(n)] for i in range(m)]
    got = co.beaver_share(party, e, f, a, b, c)
    assert big(got) == want
    rows = co.beaver_share_rows(party, e, f, a, b, c, m - 1, m)
    assert big(rows) == want[m - 1:]
    assert co.beaver_share_at(party, e, f, a, b, c, m - 1, n - 1) == want[m - 1][n - 1]


def test_beaver_degenerate_triples():
    m, k, n = 3, 4, 5
    x, w = u64(17, 1, m, k), u64(17, 2, k, n)
    zero_mk, zero_kn = np.zeros((m, k), np.uint64), np.zeros((k, n), np.uint64)
    c0, c1 = u64(17, 3, m, n), u64(17, 4, m, n)
    # A = B = 0: E = X, F = W; party 0 keeps C_0, party 1 gets C_1 + X W
    assert np.array_equal(co.beaver_share(0, x, w, zero_mk, zero_kn, c0), c0)
    assert np.array_equal(co.beaver_share(1, x, w, zero_mk, zero_kn, c1), c1 + big_matmul(x, w))
    # X = A: E = 0, so Z_i = C_i + A_i F for both parties
    a_i, b_i = u64(17, 5, m, k), u64(17, 6, k, n)
    for party in (0, 1):
        got = co.beaver_share(party, zero_mk, w, a_i, b_i, c0)
        assert np.array_equal(got, c0 + big_matmul(a_i, w))


def test_index_cols_rows_vs_numpy():
    mat = u64(18, 1, 6, 12)
    idx = np.array([0, 2], dtype=np.int32)
    assert np.array_equal(co.index_cols(mat, idx, 4), mat[:, [0, 1, 2, 3, 8, 9, 10, 11]])
    assert np.array_equal(co.index_rows(mat, idx, 2), mat[[0, 1, 4, 5], :])
    assert co.index_cols(mat, np.array([], dtype=np.int32), 4).shape == (6, 0)


def test_compact_mask_brute_force():
    for seed in range(20):
        nb, n_tok = 1 + seed * 7, 1 + seed % 4
        m = (rng.uniform_u64(seed, 3, nb * n_tok) % np.uint64(4) == 0).astype(np.uint8).reshape(n_tok, nb)
        idx = co.compact_mask(m)
        want = [b for b in range(nb) if any(m[t, b] for t in range(n_tok))]
        assert idx.tolist() == want
        assert all(idx[i] < idx[i + 1] for i in range(len(idx) - 1))
    assert co.compact_mask(np.zeros((2, 9), np.uint8)).tolist() == []
    assert co.compact_mask(np.ones((1, 5), np.uint8)).tolist() == [0, 1, 2, 3, 4]
    # any non-zero byte counts as active
    assert co.compact_mask(np.array([[0, 7, 0, 255]], np.uint8)).tolist() == [1, 3]
