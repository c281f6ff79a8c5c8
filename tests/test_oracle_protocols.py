"""Pins for the oracle's protocol layer (Pi_MatMul, Protocols 2 and 3).

What fixes the expected values here is the mathematics of the paper, never the
oracle itself: the reconstruction identity of Eq. 1 against a plaintext ring
product formed from the *unshared* secrets, the all-ones mask collapsing to a
dense product, the step-by-step protocols agreeing with the single indexed
Pi_MatMul, the cost model of the optimality appendix, the float64 product of
the dequantised secrets, and a communication figure printed in the paper.
"""
import os

import numpy as np
import pytest

import oracle as co
from oracle import cases, protocols
from workloads import configs, rng

M64 = (1 << 64) - 1


def u64(seed, stream, *shape):
    return rng.uniform_u64(seed, stream, int(np.prod(shape))).reshape(shape)


def small_q(seed, stream, *shape):
    """Signed fixed-point-like secrets of about 20 bits, as two's complement."""
    return co.encode(rng.gaussian_f64(seed, stream, int(np.prod(shape))).reshape(shape), 16)


def plain_product(kind, xq, yq, idx, bs):
    """Plaintext ring product on the kept positions, from the unshared secrets,
    with numpy's integer matmul (wraps mod 2^64) and numpy fancy indexing."""
    cols = (np.asarray(idx, dtype=np.int64)[:, None] * bs + np.arange(bs)[None, :]).ravel()
    if kind == "somm":
        return xq @ yq[:, cols]
    return xq[:, cols] @ yq[cols, :]


@pytest.mark.parametrize("cid", [1, 2])
def test_reconstruction_identity_on_configs(cid):
    cfg = configs.config(cid)
    for mm in cfg.matmuls:
        case, plain = cases.build(cfg, mm)
        z = co.reconstruct(*case.z)
        assert np.array_equal(z, plain_product(mm.kind, plain["xq"], plain["yq"], case.idx, cfg.bs))
        # the opened values are what Eq. 1 says they are: E = X - A on the indexed operands
        if mm.kind == "somm":
            assert np.array_equal(case.e, case.x[0] + case.x[1] - case.a[0] - case.a[1])
        # shares really are shares: neither equals the result on its own
        assert not np.array_equal(case.z[0], z) and not np.array_equal(case.z[1], z)


def test_reconstruction_tiny_bigint():
    # bs = 1, tiny shapes, Python integers
    m, k, n = 3, 4, 5
    xq, yq = small_q(21, 1, m, k), small_q(21, 2, k, n)
    mask = np.array([[1, 0, 1, 1, 0]], dtype=np.uint8)
    case = protocols.block_case("somm", co.share(xq, u64(21, 3, m, k)), co.share(yq, u64(21, 4, k, n)),
                                mask, 1, u64(21, 5, m, k), u64(21, 6, k, n), u64(21, 7, m, k),
                                u64(21, 8, k, n), u64(21, 9, m, 3))
    kept = [0, 2, 3]
    for i in range(m):
        for c, j in enumerate(kept):
            want = sum(int(xq[i, l]) * int(yq[l, j]) for l in range(k)) & M64
            assert (int(case.z[0][i, c]) + int(case.z[1][i, c])) & M64 == want
    # SIMM: contraction over kept neurons only
    mask = np.array([[0, 1, 1, 0]], dtype=np.uint8)
    case = protocols.block_case("simm", co.share(xq, u64(21, 3, m, k)), co.share(yq, u64(21, 4, k, n)),
                                mask, 1, u64(21, 5, m, k), u64(21, 6, k, n), u64(21, 7, m, k),
                                u64(21, 8, k, n), u64(21, 9, m, n))
    for i in range(m):
        for j in range(n):
            want = sum(int(xq[i, l]) * int(yq[l, j]) for l in (1, 2)) & M64
            assert (int(case.z[0][i, j]) + int(case.z[1][i, j])) & M64 == want


@pytest.mark.parametrize("kind", ["somm", "simm"])
def test_all_ones_mask_is_dense_product(kind):
    m, k, n, bs = 5, 8, 12, 4
    xq, yq = small_q(22, 1, m, k), small_q(22, 2, k, n)
    nb = (n if kind == "somm" else k) // bs
    mask = np.ones((1, nb), dtype=np.uint8)
    case = protocols.block_case(kind, co.share(xq, u64(22, 3, m, k)), co.share(yq, u64(22, 4, k, n)),
                                mask, bs, u64(22, 5, m, k), u64(22, 6, k, n), u64(22, 7, m, k),
                                u64(22, 8, k, n), u64(22, 9, m, n))
    assert np.array_equal(co.reconstruct(*case.z), xq @ yq)
    # and the triple is the dense one: C_0 + C_1 = A B
    assert np.array_equal(co.reconstruct(*case.c),
                          co.reconstruct(*case.a) @ co.reconstruct(*case.b))


def test_components_against_union_find():
    for seed in range(12):
        m, n = 2 + seed % 5, 3 + seed % 7
        s = (u64(seed, 30, m, n) % np.uint64(4) == 0).astype(np.uint8)
        comps = protocols.components(s)
        parent = list(range(m + n))

        def find(v):
            while parent[v] != v:
                parent[v] = parent[parent[v]]
                v = parent[v]
            return v
        for i in range(m):
            for j in range(n):
                if s[i, j]:
                    parent[find(i)] = find(m + j)
        groups = {}
        for i in range(m):
            if s[i].any():
                groups.setdefault(find(i), (set(), set()))[0].add(i)
        for j in range(n):
            if s[:, j].any():
                groups.setdefault(find(m + j), (set(), set()))[1].add(j)
        want = sorted((sorted(r), sorted(c)) for r, c in groups.values())
        got = sorted((r.tolist(), c.tolist()) for r, c in comps)
        assert got == want
    # the figure's situation: two rows sharing a column form one component
    s = np.array([[1, 0, 0], [1, 0, 0], [0, 0, 1]], dtype=np.uint8)
    got = [(r.tolist(), c.tolist()) for r, c in protocols.components(s)]
    assert got == [([0, 1], [0]), ([2], [2])]


def test_somm_literal_general_mask():
    m, k, n = 4, 3, 6
    xq, yq = small_q(23, 1, m, k), small_q(23, 2, k, n)
    s = np.array([[1, 1, 0, 0, 0, 0],
                  [0, 1, 0, 0, 0, 0],
                  [0, 0, 0, 1, 0, 1],
                  [0, 0, 0, 0, 0, 0]], dtype=np.uint8)
    cost = protocols.Cost()
    z = protocols.somm_literal(co.share(xq, u64(23, 3, m, k)), co.share(yq, u64(23, 4, k, n)), s,
                               u64(23, 5, m, k), u64(23, 6, k, n), u64(23, 7, m, k),
                               u64(23, 8, k, n), u64(23, 9, m, n), cost)
    full = xq @ yq
    rec = co.reconstruct(*z)
    assert np.array_equal(rec[s != 0], full[s != 0])          # every wanted output is right
    # blocks: rows {0,1} x cols {0,1}, rows {2} x cols {3,5}; nothing else is computed
    block = np.zeros_like(s)
    block[np.ix_([0, 1], [0, 1])] = 1
    block[np.ix_([2], [3, 5])] = 1
    assert np.array_equal(rec[block == 0], np.zeros(int((block == 0).sum()), np.uint64))
    assert np.array_equal(rec[block != 0], full[block != 0])
    # cost model: C1 = 2(|X|+|Y|) and C2 = 3|X||Y| summed over the two components
    assert cost.calls == 2
    assert cost.vectors == 2 * (2 + 2) + 2 * (1 + 2)
    assert cost.dot_products == 3 * 2 * 2 + 3 * 1 * 2


def test_somm_literal_equals_block_form_on_column_masks():
    m, k, n, bs = 6, 5, 12, 2
    xq, yq = small_q(24, 1, m, k), small_q(24, 2, k, n)
    mask = np.array([[1, 0, 0, 1, 1, 0]], dtype=np.uint8)
    args = (u64(24, 5, m, k), u64(24, 6, k, n), u64(24, 7, m, k), u64(24, 8, k, n))
    x_sh, y_sh = co.share(xq, u64(24, 3, m, k)), co.share(yq, u64(24, 4, k, n))
    c_split_full = u64(24, 9, m, n)
    s = np.repeat(np.repeat(mask, bs, axis=1), m, axis=0)
    comps = protocols.components(s)
    assert len(comps) == 1 and comps[0][0].tolist() == list(range(m))     # a single component
    lit = protocols.somm_literal(x_sh, y_sh, s, *args, c_split_full)
    idx = co.compact_mask(mask)
    case = protocols.block_case("somm", x_sh, y_sh, mask, bs, *args,
                                co.index_cols(c_split_full, idx, bs))
    for i in (0, 1):
        assert np.array_equal(co.index_cols(lit[i], idx, bs), case.z[i])   # share by share


def test_simm_literal_equals_block_form_on_column_masks():
    m, k, p, bs = 4, 8, 5, 2
    xq, yq = small_q(25, 1, m, k), small_q(25, 2, k, p)
    mask = np.array([[0, 1, 1, 0]], dtype=np.uint8)
    args = (u64(25, 5, m, k), u64(25, 6, k, p), u64(25, 7, m, k), u64(25, 8, k, p))
    x_sh, y_sh = co.share(xq, u64(25, 3, m, k)), co.share(yq, u64(25, 4, k, p))
    s = np.repeat(np.repeat(mask, bs, axis=1), m, axis=0)
    c_cols = [u64(25, 100 + j, m, p) for j in range(k)]
    cost = protocols.Cost()
    lit = protocols.simm_literal(x_sh, y_sh, s, *args, c_cols, cost)
    kept = [2, 3, 4, 5]
    c0 = np.zeros((m, p), np.uint64)
    for j in kept:
        c0 = c0 + c_cols[j]                      # Merge&Sum of the per-column triples' shares
    case = protocols.block_case("simm", x_sh, y_sh, mask, bs, *args, c0)
    for i in (0, 1):
        assert np.array_equal(lit[i], case.z[i])
    assert np.array_equal(co.reconstruct(*lit), xq[:, kept] @ yq[kept, :])
    # N p scalar multiplications per local product (N = non-zeros of X), three products
    assert cost.scalar_mults == 3 * (m * len(kept)) * p


def test_simm_literal_ragged_row_sets():
    m, k, p = 4, 3, 2
    xq, yq = small_q(26, 1, m, k), small_q(26, 2, k, p)
    s = np.array([[1, 0, 0], [0, 0, 1], [1, 0, 1], [0, 0, 0]], dtype=np.uint8)
    lit = protocols.simm_literal(co.share(xq, u64(26, 3, m, k)), co.share(yq, u64(26, 4, k, p)), s,
                                 u64(26, 5, m, k), u64(26, 6, k, p), u64(26, 7, m, k),
                                 u64(26, 8, k, p), [u64(26, 100 + j, m, p) for j in range(k)])
    xs = np.where(s != 0, xq, np.uint64(0))
    assert np.array_equal(co.reconstruct(*lit), xs @ yq)


def test_cost_counters_on_config():
    cfg = configs.config(1)
    for mm in cfg.matmuls:
        case, _ = cases.build(cfg, mm)
        n_act = len(case.idx) * cfg.bs
        if mm.kind == "somm":
            assert case.cost.opened_elems == mm.m * mm.k + mm.k * n_act
            assert case.cost.dot_products == 3 * mm.m * n_act
            assert case.cost.scalar_mults == 3 * mm.m * mm.k * n_act
        else:
            assert case.cost.opened_elems == mm.m * n_act + n_act * mm.n
            assert case.cost.scalar_mults == 3 * mm.m * n_act * mm.n


def test_paper_communication_reduction(golden_dir):
    vals = {}
    with open(os.path.join(golden_dir, "comm_reduction.txt")) as fh:
        for line in fh:
            if not line.startswith("#") and line.strip():
                k, v = line.split()
                vals[k] = float(v)
    m, k, n = int(vals["m"]), int(vals["k"]), int(vals["n"])
    dense, sparse = protocols.Cost(), protocols.Cost()
    dense.add(m, k, n)
    sparse.add(m, k, int(round(vals["density"] * n)))
    ratio = dense.opened_elems / sparse.opened_elems
    assert abs(ratio / ((m * k + k * n) / (m * k + k * vals["density"] * n)) - 1.0) < 1e-3
    assert abs(ratio - vals["paper_reduction_at_90pct"]) / vals["paper_reduction_at_90pct"] < 0.05


@pytest.mark.parametrize("cid", [1, 2])
def test_fixed_point_decode_vs_float64(cid):
    cfg = configs.config(cid)
    for mm in cfg.matmuls:
        case, plain = cases.build(cfg, mm)
        got = co.decode(co.reconstruct(*case.z), 32)
        cols = (case.idx.astype(np.int64)[:, None] * cfg.bs + np.arange(cfg.bs)[None, :]).ravel()
        xd, yd = co.decode(plain["xq"], 16), co.decode(plain["yq"], 16)
        if mm.kind == "somm":
            deq, raw = xd @ yd[:, cols], plain["x"] @ plain["y"][:, cols]
        else:
            deq, raw = xd[:, cols] @ yd[cols, :], plain["x"][:, cols] @ plain["y"][cols, :]
        assert np.max(np.abs(got - deq)) < 1e-9           # exact up to float64 summation error
        if cid == 1:
            assert np.max(np.abs(got - raw)) < 2.0 ** -10  # quantisation error at K = 64


def test_shares_look_uniform():
    cfg = configs.config(2)
    case, _ = cases.build(cfg, cfg.matmuls[0])
    for arr in (case.d[0], case.e, case.f, case.z[0], case.z[1]):
        top = (arr.ravel() >> np.uint64(56)).astype(np.int64)
        counts = np.bincount(top, minlength=256)
        expect = top.size / 256.0
        chi2 = float(((counts - expect) ** 2 / expect).sum())
        assert chi2 < 400.0        # 255 dof: mean 255, sd 22.6


# ---------------------------------------------------------------------------
# one-pass general forms (what the GPU path is compared with) against the
# literal protocols
# ---------------------------------------------------------------------------

def _random_s(seed, m, n, one_in):
    return (u64(seed, 40, m, n) % np.uint64(one_in) == 0).astype(np.uint8)


@pytest.mark.parametrize("seed,m,k,n,one_in", [(31, 5, 4, 7, 4), (32, 9, 6, 11, 6), (33, 6, 3, 6, 2),
                                               (34, 12, 5, 16, 9), (35, 3, 2, 4, 1)])
def test_somm_one_pass_equals_literal_per_party(seed, m, k, n, one_in):
    """Protocol 2 evaluated in one pass over all components gives each party the very share
    the component-by-component protocol gives it (same triples, same splits)."""
    s = _random_s(seed, m, n, one_in)
    x_sh, y_sh = (u64(seed, 1, m, k), u64(seed, 2, m, k)), (u64(seed, 3, k, n), u64(seed, 4, k, n))
    args = (u64(seed, 5, m, k), u64(seed, 6, k, n), u64(seed, 7, m, k), u64(seed, 8, k, n), u64(seed, 9, m, n))
    lit = protocols.somm_literal(x_sh, y_sh, s, *args)
    gen = protocols.somm_general(x_sh, y_sh, s, *args)
    for i in (0, 1):
        assert np.array_equal(gen.z[i], lit[i])
    # the merged result holds X Y on the result blocks and nothing elsewhere
    xy = co.ring_matmul(co.reconstruct(*x_sh), co.reconstruct(*y_sh))
    on_blocks = (gen.row_comp[:, None] >= 0) & (gen.row_comp[:, None] == gen.col_comp[None, :])
    assert np.array_equal(co.reconstruct(*gen.z), np.where(on_blocks, xy, np.uint64(0)))
    # every requested output lies on a block
    assert np.all(on_blocks[s != 0])


def test_somm_one_pass_all_ones_is_the_dense_share():
    m, k, n = 4, 5, 6
    s = np.ones((m, n), np.uint8)
    x_sh, y_sh = (u64(36, 1, m, k), u64(36, 2, m, k)), (u64(36, 3, k, n), u64(36, 4, k, n))
    gen = protocols.somm_general(x_sh, y_sh, s, u64(36, 5, m, k), u64(36, 6, k, n), u64(36, 7, m, k),
                                 u64(36, 8, k, n), u64(36, 9, m, n))
    assert len(gen.comps) == 1
    for i in (0, 1):
        assert np.array_equal(gen.z[i], co.beaver_share(i, gen.e, gen.f, gen.a[i], gen.b[i], gen.c[i]))


@pytest.mark.parametrize("seed,m,k,p,one_in", [(41, 5, 7, 4, 3), (42, 9, 11, 6, 5), (43, 4, 6, 3, 1),
                                               (44, 8, 16, 5, 8)])
def test_simm_one_pass_equals_literal_per_party(seed, m, k, p, one_in):
    """Protocol 3 summed over its columns in one pass gives each party the share the
    column-by-column protocol gives it."""
    s = _random_s(seed, m, k, one_in)
    x_sh, y_sh = (u64(seed, 1, m, k), u64(seed, 2, m, k)), (u64(seed, 3, k, p), u64(seed, 4, k, p))
    args = (u64(seed, 5, m, k), u64(seed, 6, k, p), u64(seed, 7, m, k), u64(seed, 8, k, p),
            [u64(seed, 100 + j, m, p) for j in range(k)])
    lit = protocols.simm_literal(x_sh, y_sh, s, *args)
    gen = protocols.simm_general(x_sh, y_sh, s, *args)
    for i in (0, 1):
        assert np.array_equal(gen.z[i], lit[i])
    xs = np.where(s != 0, co.reconstruct(*x_sh), np.uint64(0))
    assert np.array_equal(co.reconstruct(*gen.z), co.ring_matmul(xs, co.reconstruct(*y_sh)))


def test_simm_one_pass_ignores_entries_outside_s():
    """Entries of the opened X side outside the sparsity distribution are never sent; whatever
    stands there must not influence the share."""
    m, k, p = 6, 9, 4
    s = _random_s(45, m, k, 3)
    x_sh, y_sh = (u64(45, 1, m, k), u64(45, 2, m, k)), (u64(45, 3, k, p), u64(45, 4, k, p))
    gen = protocols.simm_general(x_sh, y_sh, s, u64(45, 5, m, k), u64(45, 6, k, p), u64(45, 7, m, k),
                                 u64(45, 8, k, p), [u64(45, 100 + j, m, p) for j in range(k)])
    junk_e = np.where(s != 0, gen.e, u64(45, 50, m, k))
    junk_a = np.where(s != 0, gen.a[1], u64(45, 51, m, k))
    assert np.array_equal(co.beaver_share_sparse_input(1, junk_e, gen.f, junk_a, gen.b[1], gen.c[1], s),
                          gen.z[1])


# ---------------------------------------------------------------------------
# Optimality appendix: the grouping Protocol 2 uses, and the work of Protocol 3
# ---------------------------------------------------------------------------

def _set_partitions(items):
    """Every partition of a list into non-empty groups."""
    if not items:
        yield []
        return
    head, rest = items[0], items[1:]
    for part in _set_partitions(rest):
        for i in range(len(part)):
            yield part[:i] + [[head] + part[i]] + part[i + 1:]
        yield [[head]] + part


def test_components_are_the_optimal_grouping_by_brute_force():
    """Theorem 1: over every way of splitting the requested outputs (edges)
    into disjoint result blocks, the split into connected components has the
    smallest total node count S1 and, among the splits that reach it, the
    smallest total of |X_i| |Y_i|.  Checked by listing all partitions of the
    edge set of tiny graphs (at most 7 edges, 877 partitions)."""
    checked = 0
    for seed in range(40):
        m, n = 2 + seed % 3, 2 + seed % 4
        s = (u64(seed, 31, m, n) % np.uint64(3) == 0).astype(np.uint8)
        edges = [(i, j) for i in range(m) for j in range(n) if s[i, j]]
        if not 2 <= len(edges) <= 7:
            continue
        comps = protocols.components(s)
        s1_comp = sum(len(r) + len(c) for r, c in comps)
        s2_comp = sum(len(r) * len(c) for r, c in comps)
        best_s1, best_s2 = None, None
        for part in _set_partitions(edges):
            s1 = sum(len({i for i, _ in g}) + len({j for _, j in g}) for g in part)
            s2 = sum(len({i for i, _ in g}) * len({j for _, j in g}) for g in part)
            if best_s1 is None or s1 < best_s1:
                best_s1, best_s2 = s1, s2
            elif s1 == best_s1 and s2 < best_s2:
                best_s2 = s2
        assert (s1_comp, s2_comp) == (best_s1, best_s2), (seed, s.tolist())
        # the minimum of S1 is the number of nodes that take part at all
        assert s1_comp == int(s.any(axis=1).sum() + s.any(axis=0).sum())
        checked += 1
    assert checked >= 15


def test_somm_literal_counts_the_cost_of_its_components():
    """The counters of Protocol 2 on a general mask are the appendix's sums
    over the components: C1 = 2 sum(|X_i| + |Y_i|), C2 = 3 sum |X_i| |Y_i|."""
    m, k, n = 6, 5, 9
    s = (u64(27, 1, m, n) % np.uint64(4) == 0).astype(np.uint8)
    xq, yq = small_q(27, 2, m, k), small_q(27, 3, k, n)
    cost = protocols.Cost()
    protocols.somm_literal(co.share(xq, u64(27, 4, m, k)), co.share(yq, u64(27, 5, k, n)), s,
                           u64(27, 6, m, k), u64(27, 7, k, n), u64(27, 8, m, k), u64(27, 9, k, n),
                           u64(27, 10, m, n), cost)
    comps = protocols.components(s)
    assert cost.calls == len(comps)
    assert cost.vectors == 2 * sum(len(r) + len(c) for r, c in comps)
    assert cost.dot_products == 3 * sum(len(r) * len(c) for r, c in comps)


def test_simm_literal_does_n_times_p_multiplications_per_product():
    """Theorem 2: the column-by-row form spends p scalar multiplications per
    non-zero of X, N p in all (times the three local products of Pi_MatMul),
    and opens each non-zero of X once plus each used row of Y once."""
    m, k, p = 5, 7, 4
    s = (u64(28, 1, m, k) % np.uint64(3) == 0).astype(np.uint8)
    s[:, 2] = 0                                      # a column nobody uses: its row of Y is never sent
    xq, yq = small_q(28, 2, m, k), small_q(28, 3, k, p)
    cost = protocols.Cost()
    protocols.simm_literal(co.share(xq, u64(28, 4, m, k)), co.share(yq, u64(28, 5, k, p)), s,
                           u64(28, 6, m, k), u64(28, 7, k, p), u64(28, 8, m, k), u64(28, 9, k, p),
                           [u64(28, 100 + j, m, p) for j in range(k)], cost)
    nnz = int(s.sum())
    used_cols = int(s.any(axis=0).sum())
    assert cost.scalar_mults == 3 * nnz * p
    assert cost.opened_elems == nnz + used_cols * p
    assert cost.calls == used_cols
