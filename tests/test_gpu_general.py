"""GPU parity of Protocols 2 and 3 in general form (per-token sparsity at block granularity):
the component search, the result-block share of Protocol 2 and the per-token row sets of
Protocol 3, element by element against the oracle's one-pass forms (which are pinned against
the literal protocols in the CPU suite)."""
import sys

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

import oracle as co                                   # noqa: E402
from oracle import protocols                          # noqa: E402
from workloads import configs, masks, rng             # noqa: E402


def say(msg):
    print("[gpu-general] " + msg, flush=True)
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


def grouped_mask(seed, n_tok, nb, groups, per_tok):
    """Tokens fall into ``groups`` clusters that draw their blocks from disjoint ranges (several
    components), plus a few tokens without any block."""
    r = rng.uniform_u64(seed, 60, n_tok * (per_tok + 1)).reshape(n_tok, per_tok + 1)
    m = np.zeros((n_tok, nb), np.uint8)
    span = nb // groups
    for t in range(n_tok):
        g = int(r[t, 0] % np.uint64(groups + 1))
        if g == groups:
            continue                              # this token predicts nothing
        for j in range(per_tok):
            m[t, g * span + int(r[t, 1 + j] % np.uint64(span))] = 1
    return m


def flat_components(mask_blk, comps=None):
    if comps is None:
        comps = protocols.components(mask_blk)
    row_idx = np.concatenate([r for r, _ in comps]) if comps else np.zeros(0, np.int32)
    blk_idx = np.concatenate([c for _, c in comps]) if comps else np.zeros(0, np.int32)
    row_comp = np.concatenate([np.full(len(r), t, np.int32) for t, (r, _) in enumerate(comps)]) \
        if comps else np.zeros(0, np.int32)
    blk_comp = np.concatenate([np.full(len(c), t, np.int32) for t, (_, c) in enumerate(comps)]) \
        if comps else np.zeros(0, np.int32)
    return comps, row_idx.astype(np.int32), row_comp, blk_idx.astype(np.int32), blk_comp


def fast_components(mask):
    """Connected components by union-find on the host (test-side, for masks too large for the
    oracle's depth-first search in pure Python); same listing convention as the oracle: ordered
    by smallest row, rows and columns ascending inside a component.  Checked against the oracle's
    search on small masks in test_fast_components_agree_with_the_oracle."""
    m, n = mask.shape
    parent = list(range(m + n))

    def find(v):
        while parent[v] != v:
            parent[v] = parent[parent[v]]
            v = parent[v]
        return v

    rs, cs = np.nonzero(mask)
    for r, c in zip(rs.tolist(), cs.tolist()):
        a, b = find(r), find(m + c)
        if a != b:
            parent[max(a, b)] = min(a, b)
    groups = {}
    for r in sorted(set(rs.tolist())):
        groups.setdefault(find(r), ([], []))[0].append(r)
    for c in sorted(set(cs.tolist())):
        groups[find(m + c)][1].append(c)
    return [(np.array(g[0], np.int32), np.array(g[1], np.int32)) for _, g in sorted(groups.items())]


def test_fast_components_agree_with_the_oracle():
    for seed, (m, nb, groups, per_tok) in enumerate([(8, 216, 3, 5), (40, 96, 4, 2), (200, 344, 6, 3)]):
        mk = grouped_mask(900 + seed, m, nb, groups, per_tok)
        a, b = fast_components(mk), protocols.components(mk)
        assert len(a) == len(b)
        for (r1, c1), (r2, c2) in zip(a, b):
            assert np.array_equal(r1, r2) and np.array_equal(c1, c2)


def check_components(ctx, mask_blk, comps=None):
    out = ctx.components(torch.from_numpy(mask_blk).cuda())
    torch.cuda.synchronize()
    comps, row_idx, row_comp, blk_idx, blk_comp = flat_components(mask_blk, comps)
    assert int(out["n_comp"].item()) == len(comps)
    assert int(out["n_row"].item()) == len(row_idx) and int(out["n_blk"].item()) == len(blk_idx)
    assert np.array_equal(out["row_idx"][:len(row_idx)].cpu().numpy(), row_idx)
    assert np.array_equal(out["row_comp"][:len(row_idx)].cpu().numpy(), row_comp)
    assert np.array_equal(out["blk_idx"][:len(blk_idx)].cpu().numpy(), blk_idx)
    assert np.array_equal(out["blk_comp"][:len(blk_idx)].cpu().numpy(), blk_comp)
    return out


@pytest.mark.parametrize("n_tok,nb,groups,per_tok", [(1, 1, 1, 1), (8, 216, 3, 5), (40, 96, 4, 2),
                                                     (200, 344, 6, 3), (512, 344, 1, 8), (1024, 500, 9, 2),
                                                     (33, 4096, 7, 4), (5, 37, 5, 1)])
def test_components_match_depth_first_search(ctx, n_tok, nb, groups, per_tok):
    say("components n_tok=%d nb=%d groups=%d" % (n_tok, nb, groups))
    check_components(ctx, grouped_mask(70 + n_tok, n_tok, nb, groups, per_tok))


def test_components_chain_needs_many_rounds(ctx):
    """A path token 0 - block 0 - token 1 - block 1 - ... is the slowest case for label
    propagation (one hop per round)."""
    n = 300
    m = np.zeros((n, n), np.uint8)
    for t in range(n):
        m[t, t] = 1
        if t + 1 < n:
            m[t + 1, t] = 1
    say("components chain of %d" % n)
    out = check_components(ctx, m[::-1].copy())      # reversed, so that labels travel the whole way
    assert int(out["n_comp"].item()) == 1


def test_components_degenerate_and_config_masks(ctx):
    say("components degenerate")
    check_components(ctx, np.zeros((7, 50), np.uint8))
    check_components(ctx, np.ones((9, 70), np.uint8))
    check_components(ctx, np.eye(64, dtype=np.uint8))
    for cid in (1, 2, 4):
        cfg = configs.config(cid)
        mk = configs.token_masks(cfg)
        if mk.shape[0] == 1:                          # one mask for the whole batch
            mk = np.repeat(mk, 4, axis=0)
        check_components(ctx, np.ascontiguousarray(mk))


def test_components_rejects_oversize(ctx):
    import paper_2505_07239_amd as comet
    for shape in ((4097, 8), (2, 16385)):
        with pytest.raises(comet.CometError) as ei:
            ctx.components(torch.zeros(shape, dtype=torch.uint8, device="cuda"))
        assert ei.value.code == -3      # COMET_ECAP


@pytest.fixture
def big_search(ctx):
    """Every comet_components call of the test takes the multi-workgroup search."""
    import paper_2505_07239_amd as comet
    ctx.set_tuning(comet.TUNE_COMPONENTS, 1)
    yield ctx
    ctx.set_tuning(comet.TUNE_COMPONENTS, 0)


@pytest.mark.parametrize("n_tok,nb,groups,per_tok", [(1, 1, 1, 1), (8, 216, 3, 5), (40, 96, 4, 2),
                                                     (200, 344, 6, 3), (512, 344, 1, 8), (1024, 500, 9, 2),
                                                     (33, 4096, 7, 4), (5, 37, 5, 1), (300, 1000, 300, 1)])
def test_components_multi_workgroup_search_on_small_graphs(big_search, n_tok, nb, groups, per_tok):
    say("components (multi-workgroup) n_tok=%d nb=%d groups=%d" % (n_tok, nb, groups))
    check_components(big_search, grouped_mask(70 + n_tok, n_tok, nb, groups, per_tok))


def test_components_multi_workgroup_search_degenerate(big_search):
    say("components (multi-workgroup) degenerate")
    check_components(big_search, np.zeros((7, 50), np.uint8))
    check_components(big_search, np.ones((9, 70), np.uint8))
    check_components(big_search, np.eye(64, dtype=np.uint8))
    n = 300                                       # a path: the deepest trees for the union-find
    m = np.zeros((n, n), np.uint8)
    for t in range(n):
        m[t, t] = 1
        if t + 1 < n:
            m[t + 1, t] = 1
    out = check_components(big_search, m[::-1].copy())
    assert int(out["n_comp"].item()) == 1


def element_mask(seed, n_tok, n_neurons, groups, density, mean_run=4.0):
    """Element-granular sparsity distribution (bs = 1) at FFN width: the tokens of ``groups``
    unrelated requests draw clustered neuron masks from disjoint ranges of the neurons."""
    return masks.grouped_token_masks(seed, 7000, n_tok, n_neurons, groups, density, mean_run)


@pytest.mark.parametrize("n_tok,n_neurons,groups,density", [(512, 13824, 6, 0.02), (256, 11008, 1, 0.15),
                                                            (2048, 4096, 16, 0.01), (4096, 16384, 40, 0.002),
                                                            (700, 16000, 9, 0.05)])
def test_components_element_granular_at_ffn_width(ctx, n_tok, n_neurons, groups, density):
    """Beyond the one-workgroup limits: hundreds of tokens by more than ten thousand neurons."""
    mk = element_mask(1234 + n_tok, n_tok, n_neurons, groups, density)
    say("components element-granular %d x %d, %d edges" % (n_tok, n_neurons, int(mk.sum())))
    out = check_components(ctx, mk, fast_components(mk))
    assert int(out["n_comp"].item()) >= 1


# ---------------------------------------------------------------------------
# Protocol 3 with per-token row sets
# ---------------------------------------------------------------------------

@pytest.mark.parametrize("m,nb,bs,n,groups,per_tok", [(3, 12, 8, 40, 2, 2), (8, 24, 16, 96, 3, 3),
                                                      # element-granular masks (bs = 1)
                                                      (6, 50, 1, 40, 2, 5), (45, 200, 1, 70, 4, 9),
                                                      (150, 333, 1, 64, 3, 20),
                                                      (13, 10, 3, 33, 2, 2), (40, 20, 32, 70, 4, 2),
                                                      (130, 16, 16, 200, 3, 4), (70, 9, 5, 64, 1, 3),
                                                      # several row tiles with different step lists
                                                      (300, 40, 32, 96, 5, 3), (200, 30, 64, 70, 4, 2),
                                                      # more listed steps than one accumulation segment holds
                                                      (100, 300, 32, 64, 1, 290)])
@pytest.mark.parametrize("compact_triples", [False, True])
def test_simm_per_token_row_sets(ctx, m, nb, bs, n, groups, per_tok, compact_triples):
    seed = 300 + m
    k = nb * bs
    mask_blk = grouped_mask(seed, m, nb, groups, per_tok)
    s = np.repeat(mask_blk, bs, axis=1)
    x_sh, y_sh = (u64(seed, 1, m, k), u64(seed, 2, m, k)), (u64(seed, 3, k, n), u64(seed, 4, k, n))
    gen = protocols.simm_general(x_sh, y_sh, s, u64(seed, 5, m, k), u64(seed, 6, k, n), u64(seed, 7, m, k),
                                 u64(seed, 8, k, n), [u64(seed, 100 + j, m, n) for j in range(k)])
    idx_np = co.compact_mask(mask_blk)
    t = len(idx_np)
    idx, n_dev = ctx.compact_mask(torch.from_numpy(mask_blk).cuda())
    # what is never exchanged may hold anything
    e_sent = np.where(s != 0, gen.e, u64(seed, 50, m, k))
    e_c, f_c = co.index_cols(e_sent, idx_np, bs), co.index_rows(gen.f, idx_np, bs)
    tm = torch.from_numpy(mask_blk).cuda()
    for party in (0, 1):
        say("simm row sets m=%d nb=%d bs=%d n=%d party %d compact=%s" % (m, nb, bs, n, party, compact_triples))
        if compact_triples:
            a_arg, b_arg = co.index_cols(gen.a[party], idx_np, bs), co.index_rows(gen.b[party], idx_np, bs)
        else:
            a_arg, b_arg = gen.a[party], gen.b[party]
        z = ctx.simm_share_masked(party, bs, idx, n_dev, t, tm, up(e_c), up(f_c), up(a_arg), up(b_arg),
                                  up(gen.c[party]), a_full=not compact_triples, b_full=not compact_triples)
        torch.cuda.synchronize()
        assert np.array_equal(down(z), gen.z[party])


# ---------------------------------------------------------------------------
# Protocol 2 with result blocks
# ---------------------------------------------------------------------------

def _somm_blocks_case(ctx, seed, m, k, nb, bs, groups, per_tok, spare_rows=0, spare_blocks=0, b_full=True,
                      neuron_major=False):
    n_full = nb * bs
    mask_blk = grouped_mask(seed, m, nb, groups, per_tok)
    s = np.repeat(mask_blk, bs, axis=1)
    x_sh, y_sh = (u64(seed, 1, m, k), u64(seed, 2, m, k)), (u64(seed, 3, k, n_full), u64(seed, 4, k, n_full))
    gen = protocols.somm_general(x_sh, y_sh, s, u64(seed, 5, m, k), u64(seed, 6, k, n_full),
                                 u64(seed, 7, m, k), u64(seed, 8, k, n_full), u64(seed, 9, m, n_full))
    comp = check_components(ctx, mask_blk)
    comps, row_idx, row_comp, blk_idx, blk_comp = flat_components(mask_blk)
    n_row, n_blk = len(row_idx), len(blk_idx)
    m_cap, cap = n_row + spare_rows, n_blk + spare_blocks
    ld = cap * bs
    cols = (blk_idx.astype(np.int64)[:, None] * bs + np.arange(bs)[None, :]).ravel()

    def rows_padded(a):                       # listed rows first, then spare rows of junk
        out = u64(seed, 77, m_cap, a.shape[1])
        out[:n_row] = a[row_idx]
        return out

    def cols_padded(a):
        out = u64(seed, 78, a.shape[0], ld)
        out[:, :n_blk * bs] = a[:, cols]
        return out

    e_p, f_c = rows_padded(gen.e), cols_padded(gen.f)
    got = []
    for party in (0, 1):
        a_p = rows_padded(gen.a[party])
        c_p = cols_padded(rows_padded(gen.c[party]))
        b_arg = gen.b[party] if b_full else cols_padded(gen.b[party])
        f_arg = f_c
        if neuron_major:                      # the same weights stored one row per neuron
            b_arg, f_arg = np.ascontiguousarray(b_arg.T), np.ascontiguousarray(f_c.T)
        z = ctx.somm_share_blocks(party, bs, comp["blk_idx"], comp["blk_comp"], comp["n_blk"], cap,
                                  comp["row_comp"], comp["n_row"], up(e_p), up(f_arg), up(a_p), up(b_arg),
                                  up(c_p), b_full=b_full, neuron_major=neuron_major)
        torch.cuda.synchronize()
        zz = down(z)
        want = gen.z[party][np.ix_(row_idx, cols)] if n_row and n_blk else np.zeros((n_row, n_blk * bs), np.uint64)
        assert np.array_equal(zz[:n_row, :n_blk * bs], want), "party %d" % party
        got.append(zz[:n_row, :n_blk * bs])
    if n_row and n_blk:
        # merged result: X Y on the result blocks, zero between them
        xy = co.ring_matmul(co.reconstruct(*x_sh), co.reconstruct(*y_sh))[np.ix_(row_idx, cols)]
        on = row_comp[:, None] == np.repeat(blk_comp, bs)[None, :]
        assert np.array_equal(got[0] + got[1], np.where(on, xy, np.uint64(0)))
    return len(comps)


@pytest.mark.parametrize("m,k,nb,bs,groups,per_tok", [(8, 64, 24, 16, 3, 3), (5, 40, 12, 8, 2, 2),
                                                      # element-granular masks (bs = 1)
                                                      (7, 40, 60, 1, 2, 6), (40, 64, 200, 1, 4, 9),
                                                      (130, 96, 300, 1, 3, 20), (300, 33, 500, 1, 5, 12),
                                                      (16, 96, 10, 3, 2, 2), (40, 70, 20, 32, 4, 2),
                                                      (200, 130, 16, 16, 3, 3), (300, 64, 40, 32, 5, 2),
                                                      (70, 33, 9, 5, 1, 3)])
def test_somm_result_blocks(ctx, m, k, nb, bs, groups, per_tok):
    say("somm blocks m=%d k=%d nb=%d bs=%d groups=%d" % (m, k, nb, bs, groups))
    n_comp = _somm_blocks_case(ctx, 400 + m, m, k, nb, bs, groups, per_tok)
    assert n_comp >= 1


@pytest.mark.parametrize("m,k,nb,bs,groups,per_tok,b_full", [(8, 64, 24, 16, 3, 3, True),
                                                             (40, 70, 20, 32, 4, 2, False),
                                                             (200, 130, 16, 16, 3, 3, True),
                                                             (300, 64, 40, 32, 5, 2, False)])
def test_somm_result_blocks_neuron_major_weights(ctx, m, k, nb, bs, groups, per_tok, b_full):
    say("somm blocks, neuron-major weights m=%d k=%d nb=%d bs=%d groups=%d" % (m, k, nb, bs, groups))
    n_comp = _somm_blocks_case(ctx, 430 + m, m, k, nb, bs, groups, per_tok, spare_rows=3,
                               spare_blocks=0 if b_full else 1, b_full=b_full, neuron_major=True)
    assert n_comp >= 1


@pytest.mark.parametrize("m", [6, 150])
def test_somm_result_blocks_spare_capacity_and_compact_triples(ctx, m):
    say("somm blocks spare capacity m=%d" % m)
    _somm_blocks_case(ctx, 450 + m, m, 48, 14, 16, 3, 2, spare_rows=5, spare_blocks=2, b_full=False)


def test_somm_result_blocks_matrix_path_for_few_rows(ctx):
    """m <= 8 with the vector-ALU path switched off: the matrix-core kernel's 32-row tile."""
    import paper_2505_07239_amd as comet
    ctx.set_tuning(comet.TUNE_SKINNY, 1)
    try:
        _somm_blocks_case(ctx, 470, 12, 64, 18, 16, 3, 2)
    finally:
        ctx.set_tuning(comet.TUNE_SKINNY, 0)


# ---------------------------------------------------------------------------
# MHA-shaped workload: head-granular sparsity (block = one attention head)
# ---------------------------------------------------------------------------

def test_mha_sparse_qkv_and_output_layers(ctx):
    """Sparse QKV layer with merged cache-refill rows (Protocol 2, result blocks) and sparse
    output layer (Protocol 3, per-token head sets) at the LLaMA-2-7B attention shape.  Operands are
    uniform random words (shares and opened values are uniform anyway; the C shares are not
    tied to A B, the per-party share is checked for exactly the C that is passed in).  Both layers
    are compared in full."""
    cfg = configs.mha_config()
    qkv_mask, out_mask = configs.mha_head_masks(cfg)
    d, h, bs = cfg.d_model, cfg.n_heads, cfg.head_dim
    seed = 600

    # --- sparse QKV: rows = current tokens + refill rows, 96 column blocks of 128 ---
    comp = check_components(ctx, qkv_mask)
    comps, row_idx, row_comp, blk_idx, blk_comp = flat_components(qkv_mask)
    n_row, n_blk = len(row_idx), len(blk_idx)
    n_act = n_blk * bs
    say("mha qkv: %d rows, %d of %d blocks, %d components" % (n_row, n_blk, 3 * h, len(comps)))
    e, a = u64(seed, 1, n_row, d), u64(seed, 2, n_row, d)
    f, b = u64(seed, 3, d, n_act), u64(seed, 4, d, 3 * h * bs)
    c = u64(seed, 5, n_row, n_act)
    z = ctx.somm_share_blocks(1, bs, comp["blk_idx"], comp["blk_comp"], comp["n_blk"], n_blk,
                              comp["row_comp"], comp["n_row"], up(e), up(f), up(a), up(b), up(c))
    torch.cuda.synchronize()
    got = down(z)
    cols = (blk_idx.astype(np.int64)[:, None] * bs + np.arange(bs)[None, :]).ravel()
    b_sel = np.ascontiguousarray(b[:, cols])
    col_comp = np.repeat(blk_comp, bs)
    want = co.beaver_share_blocks(1, e, f, a, b_sel, c, row_comp, col_comp)
    assert np.array_equal(got, want)
    on = row_comp[:, None] == col_comp[None, :]
    assert not got[~on].any()                    # zero between the result blocks

    # --- sparse output layer: contraction over the heads each token activated ---
    idx_np = co.compact_mask(out_mask)
    t = len(idx_np)
    idx, n_dev = ctx.compact_mask(torch.from_numpy(out_mask).cuda())
    m = cfg.tokens
    kc = t * bs
    say("mha output layer: %d tokens, %d of %d heads in the union" % (m, t, h))
    e2, a2 = u64(seed, 11, m, kc), u64(seed, 12, m, h * bs)
    f2, b2 = u64(seed, 13, kc, d), u64(seed, 14, h * bs, d)
    c2 = u64(seed, 15, m, d)
    tm = torch.from_numpy(out_mask).cuda()
    z2 = ctx.simm_share_masked(1, bs, idx, n_dev, t, tm, up(e2), up(f2), up(a2), up(b2), up(c2))
    torch.cuda.synchronize()
    s_el = np.repeat(out_mask[:, idx_np], bs, axis=1)
    want2 = co.beaver_share_sparse_input(1, e2, f2, co.index_cols(a2, idx_np, bs),
                                         co.index_rows(b2, idx_np, bs), c2, s_el)
    assert np.array_equal(down(z2), want2)


# ---------------------------------------------------------------------------
# element-granular sparsity distributions at FFN width (bs = 1)
# ---------------------------------------------------------------------------

def test_general_forms_element_granular_at_ffn_width(ctx):
    """512 tokens x 13824 neurons (the LLaMA-2-13B FFN width), every neuron its own block: the
    component search beyond the one-workgroup limits, Protocol 2 on the result blocks and
    Protocol 3 with per-token row sets, each compared in full with the oracle's one-pass form.
    The other dimension of each product is kept short so that the oracle stays in seconds."""
    m, neurons, k, n_out, groups = 512, 13824, 96, 64, 6
    mk = element_mask(4321, m, neurons, groups, 0.02)
    comps = fast_components(mk)
    comp = check_components(ctx, mk, comps)
    _, row_idx, row_comp, blk_idx, blk_comp = flat_components(mk, comps)
    n_row, n_blk = len(row_idx), len(blk_idx)
    say("element-granular FFN width: %d edges, %d components, %d rows, %d neurons" %
        (int(mk.sum()), len(comps), n_row, n_blk))
    seed = 4400
    # --- Protocol 2, result blocks, bs = 1 ---
    e, a = u64(seed, 1, n_row, k), u64(seed, 2, n_row, k)
    f, b = u64(seed, 3, k, n_blk), u64(seed, 4, k, neurons)
    c = u64(seed, 5, n_row, n_blk)
    z = ctx.somm_share_blocks(1, 1, comp["blk_idx"], comp["blk_comp"], comp["n_blk"], n_blk, comp["row_comp"],
                              comp["n_row"], up(e), up(f), up(a), up(b), up(c))
    torch.cuda.synchronize()
    want = co.beaver_share_blocks(1, e, f, a, np.ascontiguousarray(b[:, blk_idx]), c, row_comp, blk_comp)
    assert np.array_equal(down(z), want)
    # --- Protocol 3, per-token row sets, bs = 1 ---
    idx_np = co.compact_mask(mk)
    t = len(idx_np)
    idx, n_dev = ctx.compact_mask(torch.from_numpy(mk).cuda())
    e2, a2 = u64(seed, 11, m, t), u64(seed, 12, m, neurons)
    f2, b2 = u64(seed, 13, t, n_out), u64(seed, 14, neurons, n_out)
    c2 = u64(seed, 15, m, n_out)
    z2 = ctx.simm_share_masked(0, 1, idx, n_dev, t, torch.from_numpy(mk).cuda(), up(e2), up(f2), up(a2), up(b2),
                               up(c2))
    torch.cuda.synchronize()
    assert int(n_dev.item()) == t and np.array_equal(idx[:t].cpu().numpy(), idx_np)
    want2 = co.beaver_share_sparse_input(0, e2, f2, co.index_cols(a2, idx_np, 1), co.index_rows(b2, idx_np, 1), c2,
                                         np.ascontiguousarray(mk[:, idx_np]))
    assert np.array_equal(down(z2), want2)


# ---------------------------------------------------------------------------
# seeded sweep over both general forms
# ---------------------------------------------------------------------------

def _draw_general(case):
    r = rng.uniform_u64(4343, case, 10)
    pick = lambda i, lo, hi: lo + int(r[i] % np.uint64(hi - lo + 1))
    m = [2, 9, 16, 17, 40, 64, 100, 129, 260][pick(0, 0, 8)]
    bs = [1, 2, 3, 8, 16, 32, 64][pick(1, 0, 6)]
    nb = pick(2, 3, max(3, min(36 if bs > 1 else 300, 576 // bs)))
    groups = pick(3, 1, min(5, nb))
    per_tok = pick(4, 1, 4)
    other = pick(5, 8, 200)
    return m, bs, nb, groups, per_tok, other


@pytest.mark.parametrize("case", range(20))
def test_general_forms_sweep(ctx, case):
    m, bs, nb, groups, per_tok, other = _draw_general(case)
    say("sweep %d: m=%d bs=%d nb=%d groups=%d per_tok=%d other=%d" % (case, m, bs, nb, groups, per_tok, other))
    # Protocol 2 with result blocks (other = contraction length)
    _somm_blocks_case(ctx, 6000 + case, m, other, nb, bs, groups, per_tok, spare_rows=case % 3,
                      spare_blocks=0, b_full=bool(case & 1))
    # Protocol 3 with per-token row sets (other = output width)
    seed = 6500 + case
    k = nb * bs
    mask_blk = grouped_mask(seed, m, nb, groups, per_tok)
    if not mask_blk.any():
        return
    s = np.repeat(mask_blk, bs, axis=1)
    idx_np = co.compact_mask(mask_blk)
    t = len(idx_np)
    # the one-pass oracle on operands drawn directly (its agreement with the literal protocol is
    # pinned in the CPU suite); entries outside the sparsity distribution hold junk
    e, a = u64(seed, 1, m, t * bs), u64(seed, 2, m, k)
    f, b = u64(seed, 3, t * bs, other), u64(seed, 4, k, other)
    c = u64(seed, 5, m, other)
    idx, n_dev = ctx.compact_mask(torch.from_numpy(mask_blk).cuda())
    z = ctx.simm_share_masked(1, bs, idx, n_dev, t, torch.from_numpy(mask_blk).cuda(), up(e), up(f), up(a),
                              up(b), up(c))
    torch.cuda.synchronize()
    want = co.beaver_share_sparse_input(1, e, f, co.index_cols(a, idx_np, bs), co.index_rows(b, idx_np, bs), c,
                                        np.ascontiguousarray(s[:, np.repeat(idx_np, bs) * bs + np.tile(np.arange(bs), t)]))
    assert np.array_equal(down(z), want)
