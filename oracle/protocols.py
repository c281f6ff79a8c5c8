"""Two-party simulation of the paper's protocols on top of the C oracle.

TEST INFRASTRUCTURE ONLY (see ``oracle/__init__.py``).

Both parties live in one process; "sending" a value is handing the array to
the other party's step.  Parties are 0-based here: party 1 is the paper's
P_2, the one whose share carries the extra ``E F`` term of Eq. 1.

Functions
---------
ttp_triple        trusted third party of Sec. 3.2: shares of (A, B, C = A B)
pi_matmul         Pi_MatMul of Sec. 2.1 / 5.1 on explicit shares
components        connected components of the bipartite graph of Sec. 5.1
somm_literal      Protocol 2, step by step, for an arbitrary 0/1 matrix S
simm_literal      Protocol 3, step by step, for an arbitrary 0/1 matrix S
block_case        Protocols 2 / 3 when S keeps the same neuron blocks for every row
Cost              counters of the cost model in the optimality appendix
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

import oracle as co


@dataclass
class Cost:
    """Cost model of the optimality appendix, accumulated over Pi_MatMul calls.

    ``vectors``: row vectors of X plus column vectors of Y that are masked and
    sent, counted for both directions: C1 = 2(|X| + |Y|).
    ``dot_products``: local dot products, C2 = 3 |X| |Y|.
    ``opened_elems``: ring elements each party sends (|X| k + k |Y|).
    ``scalar_mults``: scalar ring multiplications of the three local products.
    """
    vectors: int = 0
    dot_products: int = 0
    opened_elems: int = 0
    scalar_mults: int = 0
    calls: int = 0

    def add(self, m: int, k: int, n: int) -> None:
        self.vectors += 2 * (m + n)
        self.dot_products += 3 * m * n
        self.opened_elems += m * k + k * n
        self.scalar_mults += 3 * m * k * n
        self.calls += 1


@dataclass
class Triple:
    a: Tuple[np.ndarray, np.ndarray]
    b: Tuple[np.ndarray, np.ndarray]
    c: Tuple[np.ndarray, np.ndarray]


def ttp_triple(a: np.ndarray, b: np.ndarray, a_split: np.ndarray, b_split: np.ndarray,
               c_split: np.ndarray) -> Triple:
    """Beaver triple for one Pi_MatMul: C = A B (mod 2^64), all three shared."""
    c = co.ring_matmul(a, b)
    return Triple(co.share(a, a_split), co.share(b, b_split), co.share(c, c_split))


def pi_matmul(x: Sequence[np.ndarray], y: Sequence[np.ndarray], t: Triple,
              cost: Optional[Cost] = None, trace: Optional[Dict[str, np.ndarray]] = None):
    """Pi_MatMul.  ``x``, ``y``: the two parties' shares.  Returns ``(Z_0, Z_1)``.

    Each party masks its shares with its triple shares, the masked values are
    exchanged and summed (opened), then Eq. 1 is evaluated locally.
    """
    d = [co.mask_share(x[i], t.a[i]) for i in (0, 1)]      # [E]_i = [X]_i - [A]_i
    g = [co.mask_share(y[i], t.b[i]) for i in (0, 1)]      # [F]_i = [Y]_i - [B]_i
    e = co.open_(d[0], d[1])
    f = co.open_(g[0], g[1])
    z = tuple(co.beaver_share(i, e, f, t.a[i], t.b[i], t.c[i]) for i in (0, 1))
    if cost is not None:
        cost.add(x[0].shape[0], x[0].shape[1], y[0].shape[1])
    if trace is not None:
        trace.update(d0=d[0], d1=d[1], g0=g[0], g1=g[1], e=e, f=f)
    return z


# ---------------------------------------------------------------------------
# Protocol 2 (SOMM), general form
# ---------------------------------------------------------------------------

def components(s: np.ndarray) -> List[Tuple[np.ndarray, np.ndarray]]:
    """Connected components of the bipartite graph whose left nodes are the
    rows of X, right nodes the columns of Y and edges the ones of ``s``
    (``m x n``).  Isolated nodes are dropped.  Depth-first search with an
    explicit stack.  Each component is ``(sorted rows, sorted cols)``;
    components are ordered by their smallest row."""
    s = np.asarray(s) != 0
    m, n = s.shape
    seen_r = np.zeros(m, dtype=bool)
    seen_c = np.zeros(n, dtype=bool)
    out = []
    for r0 in range(m):
        if seen_r[r0] or not s[r0].any():
            continue
        rows, cols = [], []
        stack = [("r", r0)]
        seen_r[r0] = True
        while stack:
            side, v = stack.pop()
            if side == "r":
                rows.append(v)
                for c in np.nonzero(s[v])[0]:
                    if not seen_c[c]:
                        seen_c[c] = True
                        stack.append(("c", int(c)))
            else:
                cols.append(v)
                for r in np.nonzero(s[:, v])[0]:
                    if not seen_r[r]:
                        seen_r[r] = True
                        stack.append(("r", int(r)))
        out.append((np.array(sorted(rows), dtype=np.int32), np.array(sorted(cols), dtype=np.int32)))
    return out


def _rows(mat, idx):
    return co.index_rows(mat, np.ascontiguousarray(idx, dtype=np.int32), 1)


def _cols(mat, idx):
    return co.index_cols(mat, np.ascontiguousarray(idx, dtype=np.int32), 1)


def somm_literal(x, y, s, a, b, a_split, b_split, c_split, cost: Optional[Cost] = None):
    """Protocol 2 (Sec. 5.1).  ``x``, ``y``: share pairs (``m x k``, ``k x n``); ``s``: 0/1
    ``m x n``, the sparsity distribution of ``X Y``.

    The requested outputs are grouped by connected component of the bipartite graph of ``s``.
    For a component with rows ``I_x`` and columns ``I_y`` the result block is
    ``Z[I_x, I_y] = Pi_MatMul(X[I_x, :], Y[:, I_y])`` with a triple of its own; the output is zero
    everywhere else.  Triple material ``a`` (m x k), ``b`` (k x n) and the splitting randomness
    are given at full shape; a component's triple is their restriction to ``I_x`` / ``I_y`` with
    ``C = A[I_x, :] B[:, I_y]``.  Returns the two parties' full-size ``m x n`` shares."""
    m, n = np.asarray(s).shape
    z = [np.zeros((m, n), dtype=np.uint64) for _ in (0, 1)]
    for i_x, i_y in components(s):
        triple = ttp_triple(_rows(a, i_x), _cols(b, i_y), _rows(a_split, i_x), _cols(b_split, i_y),
                            _cols(_rows(c_split, i_x), i_y))
        block = pi_matmul([_rows(x[i], i_x) for i in (0, 1)], [_cols(y[i], i_y) for i in (0, 1)],
                          triple, cost)
        for i in (0, 1):
            z[i][np.ix_(i_x, i_y)] = block[i]
    return tuple(z)


# ---------------------------------------------------------------------------
# Protocol 3 (SIMM), general form
# ---------------------------------------------------------------------------

def simm_literal(x, y, s, a, b, a_split, b_split, c_split_cols, cost: Optional[Cost] = None):
    """Protocol 3 (Sec. 5.2).  ``x``: shares of the ``m x k`` sparse-input matrix, ``s``: its
    0/1 sparsity distribution, ``y``: shares of ``k x p``.

    Column by row: ``Z = sum_j X[:, j] Y[j, :]``, and column ``j`` of ``X`` is non-zero only on
    its row set ``R_j = {r : s[r, j] != 0}``.  So every column with a non-empty ``R_j`` adds the
    outer product ``Pi_MatMul(X[R_j, j], Y[j, :])`` (an ``|R_j| x 1`` by ``1 x p`` product with a
    triple of its own) onto rows ``R_j`` of the output; a row of ``Y`` is masked once.
    ``c_split_cols[j]`` is the ``m x p`` randomness that splits the triple of column ``j``
    (rows outside ``R_j`` unused).  Returns the two parties' ``m x p`` shares."""
    s = np.asarray(s) != 0
    m, k = s.shape
    p = y[0].shape[1]
    z = [np.zeros((m, p), dtype=np.uint64) for _ in (0, 1)]
    for j in range(k):
        r_j = np.nonzero(s[:, j])[0]
        if not len(r_j):
            continue
        col = lambda mat: _rows(_cols(mat, [j]), r_j)          # mat[R_j, j] as |R_j| x 1
        row = lambda mat: _rows(mat, [j])                      # mat[j, :]   as 1 x p
        triple = ttp_triple(col(a), row(b), col(a_split), row(b_split),
                            _rows(np.ascontiguousarray(c_split_cols[j]), r_j))
        outer = pi_matmul([col(x[i]) for i in (0, 1)], [row(y[i]) for i in (0, 1)], triple, cost)
        for i in (0, 1):
            z[i][r_j, :] += outer[i]
    return tuple(z)


# ---------------------------------------------------------------------------
# The hot path: whole column blocks kept for every row
# ---------------------------------------------------------------------------

@dataclass
class BlockCase:
    """Everything both parties hold for one block-sparse matmul, plus results."""
    kind: str
    m: int
    k: int
    n: int
    bs: int
    idx: np.ndarray
    x: Tuple[np.ndarray, np.ndarray]            # full-size shares
    y: Tuple[np.ndarray, np.ndarray]
    a: Tuple[np.ndarray, np.ndarray]            # full-size triple shares
    b: Tuple[np.ndarray, np.ndarray]
    c: Tuple[np.ndarray, np.ndarray]            # compact: C = A_sel B_sel
    d: Tuple[np.ndarray, np.ndarray] = None     # masked X-side shares (compact for simm)
    g: Tuple[np.ndarray, np.ndarray] = None     # masked Y-side shares (compact)
    e: np.ndarray = None
    f: np.ndarray = None
    z: Tuple[np.ndarray, np.ndarray] = None
    cost: Cost = field(default_factory=Cost)


def _sel(kind: str, x, y, idx, bs):
    """IndexCols / IndexRows of Protocols 2 and 3 for block-granular index sets."""
    if kind == "somm":
        return x, co.index_cols(y, idx, bs)
    return co.index_cols(x, idx, bs), co.index_rows(y, idx, bs)


def block_case(kind: str, x_sh, y_sh, mask: np.ndarray, bs: int, a: np.ndarray, b: np.ndarray,
               a_split: np.ndarray, b_split: np.ndarray, c_split: np.ndarray,
               with_result: bool = True) -> BlockCase:
    """Run SOMM (``kind="somm"``) or SIMM (``kind="simm"``) when the sparsity
    distribution keeps the same neuron blocks for every token: a single
    Pi_MatMul on the indexed sub-matrices.

    ``mask``: per-token block flags ``[n_tok, nb]``; the union over tokens is
    kept.  Triple parts ``a``, ``b`` are full-shape draws; the TTP forms the
    triple on their indexed restriction, ``C = A_sel B_sel``, split with
    ``c_split`` (already of the compact output shape)."""
    idx = co.compact_mask(mask)
    m, k = x_sh[0].shape
    n = y_sh[0].shape[1]
    a_sel, b_sel = _sel(kind, a, b, idx, bs)
    as_sel, bs_sel = _sel(kind, a_split, b_split, idx, bs)
    a_sh = co.share(a, a_split)
    b_sh = co.share(b, b_split)
    case = BlockCase(kind, m, k, n, bs, idx, tuple(x_sh), tuple(y_sh), a_sh, b_sh, None)
    c = co.ring_matmul(a_sel, b_sel)
    case.c = co.share(c, c_split)
    xs = [_sel(kind, x_sh[i], y_sh[i], idx, bs) for i in (0, 1)]
    t = Triple(co.share(a_sel, as_sel), co.share(b_sel, bs_sel), case.c)
    # the indexed restriction of a full-size share pair is the share pair of the restriction
    assert np.array_equal(t.a[1], _sel(kind, a_sh[1], b_sh[1], idx, bs)[0])
    if with_result:
        trace: Dict[str, np.ndarray] = {}
        case.z = pi_matmul([xs[0][0], xs[1][0]], [xs[0][1], xs[1][1]], t, case.cost, trace)
        case.d = (trace["d0"], trace["d1"])
        case.g = (trace["g0"], trace["g1"])
        case.e, case.f = trace["e"], trace["f"]
    return case


# ---------------------------------------------------------------------------
# Protocols 2 and 3 in one pass (what a party computes locally, all components
# / all columns at once), from the same material as the literal forms above
# ---------------------------------------------------------------------------

@dataclass
class GeneralCase:
    """Material of one general-form protocol run in the layout of the full matrices.

    ``a``, ``b``, ``c``: the two parties' triple shares (for SOMM ``c`` is
    defined on the result blocks and zero elsewhere; for SIMM it is the sum of
    the scattered column triples); ``e``, ``f``: opened masked operands;
    ``z``: the two parties' output shares by the one-pass formula.
    ``row_comp`` / ``col_comp`` (SOMM only): component number of every row of
    X / column of Y, -1 for the ones that take part in no dot product;
    ``comps``: the components as (rows, cols), ordered by smallest row."""
    kind: str
    s: np.ndarray
    a: Tuple[np.ndarray, np.ndarray]
    b: Tuple[np.ndarray, np.ndarray]
    c: Tuple[np.ndarray, np.ndarray]
    e: np.ndarray
    f: np.ndarray
    z: Tuple[np.ndarray, np.ndarray]
    row_comp: Optional[np.ndarray] = None
    col_comp: Optional[np.ndarray] = None
    comps: Optional[list] = None


def component_numbers(s: np.ndarray):
    """(components, row_comp, col_comp) of the bipartite graph of ``s``."""
    m, n = np.asarray(s).shape
    comps = components(s)
    row_comp = np.full(m, -1, dtype=np.int32)
    col_comp = np.full(n, -1, dtype=np.int32)
    for t, (i_x, i_y) in enumerate(comps):
        row_comp[i_x] = t
        col_comp[i_y] = t
    return comps, row_comp, col_comp


def somm_general(x, y, s, a, b, a_split, b_split, c_split) -> GeneralCase:
    """Protocol 2 with the per-component triples of :func:`somm_literal` laid out
    at their rows and columns, evaluated by ``oracle.beaver_share_blocks``."""
    comps, row_comp, col_comp = component_numbers(s)
    a_sh, b_sh = co.share(a, a_split), co.share(b, b_split)
    m, n = np.asarray(s).shape
    c_sh = [np.zeros((m, n), dtype=np.uint64) for _ in (0, 1)]
    for i_x, i_y in comps:                                # the TTP's C = A[I_x] B[:, I_y], shared
        ct = co.ring_matmul(co.index_rows(a, i_x, 1), co.index_cols(b, i_y, 1))
        c0 = co.index_cols(co.index_rows(c_split, i_x, 1), i_y, 1)
        c_sh[0][np.ix_(i_x, i_y)] = c0
        c_sh[1][np.ix_(i_x, i_y)] = ct - c0
    d = [co.mask_share(x[i], a_sh[i]) for i in (0, 1)]
    g = [co.mask_share(y[i], b_sh[i]) for i in (0, 1)]
    e, f = co.open_(d[0], d[1]), co.open_(g[0], g[1])
    z = tuple(co.beaver_share_blocks(i, e, f, a_sh[i], b_sh[i], c_sh[i], row_comp, col_comp)
              for i in (0, 1))
    return GeneralCase("somm", np.asarray(s), a_sh, b_sh, tuple(c_sh), e, f, z, row_comp, col_comp, comps)


def simm_general(x, y, s, a, b, a_split, b_split, c_split_cols) -> GeneralCase:
    """Protocol 3 with the column triples of :func:`simm_literal` laid out at their
    positions, evaluated by ``oracle.beaver_share_sparse_input``."""
    s = (np.asarray(s) != 0).astype(np.uint8)
    m, k = s.shape
    p = y[0].shape[1]
    a_sh, b_sh = co.share(a, a_split), co.share(b, b_split)
    c_sh = [np.zeros((m, p), dtype=np.uint64) for _ in (0, 1)]
    for j in range(k):
        r_j = np.nonzero(s[:, j])[0].astype(np.int32)
        if not len(r_j):
            continue
        jj = np.array([j], dtype=np.int32)
        cj = co.ring_matmul(co.index_rows(co.index_cols(a, jj, 1), r_j, 1), co.index_rows(b, jj, 1))
        c0 = co.index_rows(np.ascontiguousarray(c_split_cols[j]), r_j, 1)
        c_sh[0][r_j, :] += c0
        c_sh[1][r_j, :] += cj - c0
    d = [co.mask_share(x[i], a_sh[i]) for i in (0, 1)]
    g = [co.mask_share(y[i], b_sh[i]) for i in (0, 1)]
    e, f = co.open_(d[0], d[1]), co.open_(g[0], g[1])
    z = tuple(co.beaver_share_sparse_input(i, e, f, a_sh[i], b_sh[i], c_sh[i], s) for i in (0, 1))
    return GeneralCase("simm", s, a_sh, b_sh, tuple(c_sh), e, f, z)


# ---------------------------------------------------------------------------
# Protocol 1: oblivious shuffle
# ---------------------------------------------------------------------------

@dataclass
class ShuffleMaterial:
    """What the trusted third party hands out at the offline stage (0-based parties)."""
    pi: np.ndarray
    rho: Tuple[np.ndarray, np.ndarray]
    tau: Tuple[np.ndarray, np.ndarray]
    a: Tuple[np.ndarray, np.ndarray]
    b: Tuple[np.ndarray, np.ndarray]


def compose(f: np.ndarray, g: np.ndarray) -> np.ndarray:
    """Index array of f o g (apply g first): (f o g)(x)_j = g(x)[f[j]] = x[g[f[j]]]."""
    return np.asarray(g)[np.asarray(f)].astype(np.int32)


def inverse(p: np.ndarray) -> np.ndarray:
    inv = np.empty(len(p), dtype=np.int32)
    inv[np.asarray(p)] = np.arange(len(p), dtype=np.int32)
    return inv


def shuffle_offline(pi, tau1, tau2, a1, a2, c, axis: int) -> ShuffleMaterial:
    """Offline stage of Protocol 1 from given randomness: rho_1 = pi o tau_2^-1,
    rho_2 = pi o tau_1^-1, b_1 = rho_1(a_2) + c, b_2 = rho_2(a_1) - c."""
    pi, tau1, tau2 = (np.asarray(v, dtype=np.int32) for v in (pi, tau1, tau2))
    rho1, rho2 = compose(pi, inverse(tau2)), compose(pi, inverse(tau1))
    zero = np.zeros_like(a1)
    b1 = co.permute_mask(a2, rho1, zero, axis, +1) + c
    b2 = co.permute_mask(a1, rho2, zero, axis, +1) - c
    return ShuffleMaterial(pi, (rho1, rho2), (tau1, tau2), (a1, a2), (b1, b2))


def shuffle_online(x: Sequence[np.ndarray], mat: ShuffleMaterial, axis: int):
    """Online stage: y_i = tau_i(x_i) + a_i is sent to the other party, which computes
    z = rho(y) - b.  Returns (z_0, z_1) and the exchanged (y_0, y_1)."""
    y = [co.permute_mask(x[i], mat.tau[i], mat.a[i], axis, +1) for i in (0, 1)]
    z = tuple(co.permute_mask(y[1 - i], mat.rho[i], mat.b[i], axis, -1) for i in (0, 1))
    return z, tuple(y)


def unshuffle_material(mat: ShuffleMaterial, a1, a2, c, axis: int) -> ShuffleMaterial:
    """Material of the shuffle that restores the original order ("unshuffle"): every party
    inverts its own sub-permutations locally, tau_i' = rho_i^-1 and rho_i' = tau_i^-1, so that
    rho_i' o tau_other' = tau_i^-1 o rho_other^-1 = (rho_other o tau_i)^-1 = pi^-1; fresh masks."""
    tau = (inverse(mat.rho[0]), inverse(mat.rho[1]))
    rho = (inverse(mat.tau[0]), inverse(mat.tau[1]))
    zero = np.zeros_like(a1)
    b1 = co.permute_mask(a2, rho[0], zero, axis, +1) + c
    b2 = co.permute_mask(a1, rho[1], zero, axis, +1) - c
    return ShuffleMaterial(inverse(mat.pi), rho, tau, (a1, a2), (b1, b2))
