"""GPU parity at the benchmark's full sizes (configs 3, 4 and 5), in the launch
configurations bench.py times: the whole pipeline (compact -> indexed masking ->
open -> both parties' shares) runs on the device with n_blk never leaving it,
once with word operands and one share call per product and party, and once as
bench.py's default step does it: F opened straight into digit planes, B_i packed
into planes beforehand, and the share products that are ready together in one
grouped call (gate and up of both parties; down of both parties).

Everything is compared element by element: compaction, masking, opening and
both parties' output shares on every row and column (the oracle needs a few
seconds per configuration on the host cores of the GPU machine).  One case per kind
of product also runs with spare block capacity (n_blk_cap above the number of
kept blocks, the count only on the device) and checks that nothing beyond
n_blk * bs is read or written.

Triples: the C shares here are uniform random words rather than shares of
A_sel B_sel.  The per-party share Z_i = C_i + ... is checked against the oracle
for exactly the C_i that is passed in, so the check is as strict as with a true
triple; the reconstruction identity itself is covered at the smaller sizes.
"""
import sys

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

import oracle as co                                   # noqa: E402
from workloads import configs, rng                    # noqa: E402


def say(msg):
    print("[gpu-fullsize] " + msg, flush=True)
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


_raw_cache = {}


def _raw(cfg, mm):
    """Uniform share / triple words of one projection (cached across the density sweep)."""
    key = (cfg.cid, mm.index)
    if key not in _raw_cache:
        _raw_cache.clear()
        sid = lambda role: configs.stream_id(cfg, mm.index, role)
        mk, kn = mm.m * mm.k, mm.k * mm.n
        u = lambda role, n, shape: rng.uniform_u64(rng.BASE_SEED, sid(role), n).reshape(shape)
        _raw_cache[key] = dict(
            x=[u(configs.R_XSPLIT, mk, (mm.m, mm.k)), u(configs.R_X, mk, (mm.m, mm.k))],
            y=[u(configs.R_YSPLIT, kn, (mm.k, mm.n)), u(configs.R_Y, kn, (mm.k, mm.n))],
            a=[u(configs.R_ASPLIT, mk, (mm.m, mm.k)), u(configs.R_A, mk, (mm.m, mm.k))],
            b=[u(configs.R_BSPLIT, kn, (mm.k, mm.n)), u(configs.R_B, kn, (mm.k, mm.n))])
    return _raw_cache[key]


SENTINEL = np.uint64(0xA5A5A5A5A5A5A5A5)


def _sentinel(*shape):
    return torch.full(shape, int(SENTINEL.view(np.int64)), dtype=torch.int64, device="cuda")


def _run_projection(ctx, cfg, mm, mask_np, spare=0):
    """Whole path of one projection on the device, every buffer against the oracle.  ``spare``
    extra blocks of capacity: compact operands get ``(t + spare) * bs`` columns / rows, the part
    beyond the kept blocks holds a sentinel that must survive (outputs) or must not matter
    (inputs)."""
    import paper_2505_07239_amd as comet
    raw = _raw(cfg, mm)
    bs = cfg.bs
    idx_np = co.compact_mask(mask_np)
    t = len(idx_np)
    cap = t + spare
    n_act, ld = t * bs, cap * bs
    idx, n_dev = ctx.compact_mask(torch.from_numpy(mask_np).cuda())
    gx = [up(v) for v in raw["x"]]
    gy = [up(v) for v in raw["y"]]
    ga = [up(v) for v in raw["a"]]
    gb = [up(v) for v in raw["b"]]
    zshape = (mm.m, n_act) if mm.kind == "somm" else (mm.m, mm.n)
    c = [rng.uniform_u64(rng.BASE_SEED, configs.stream_id(cfg, mm.index, configs.R_CSPLIT) + 50 * i,
                         zshape[0] * zshape[1]).reshape(zshape) for i in (0, 1)]
    d, g = [], []
    for i in (0, 1):
        if mm.kind == "somm":
            d.append(ctx.mask_share(gx[i], ga[i]))
            g.append(ctx.mask_share_gather(gy[i], gb[i], comet.AXIS_COLS, bs, idx, n_dev, cap,
                                           out=_sentinel(mm.k, ld)))
        else:
            d.append(ctx.mask_share_gather(gx[i], ga[i], comet.AXIS_COLS, bs, idx, n_dev, cap,
                                           out=_sentinel(mm.m, ld)))
            g.append(ctx.mask_share_gather(gy[i], gb[i], comet.AXIS_ROWS, bs, idx, n_dev, cap,
                                           out=_sentinel(ld, mm.n)))
    e, f = ctx.open(d[0], d[1]), ctx.open(g[0], g[1])
    z = []
    for i in (0, 1):
        if mm.kind == "somm":
            c_dev = _sentinel(mm.m, ld)
            c_dev[:, :n_act] = up(c[i])
            z.append(ctx.somm_share(i, bs, idx, n_dev, cap, e, f, ga[i], gb[i], c_dev,
                                    out=_sentinel(mm.m, ld)))
        else:
            z.append(ctx.simm_share(i, bs, idx, n_dev, cap, e, f, ga[i], gb[i], up(c[i])))
    torch.cuda.synchronize()
    assert int(n_dev.item()) == t and np.array_equal(idx[:t].cpu().numpy(), idx_np)

    # oracle side: indexing, masking, opening, Eq. 1, all in full
    if mm.kind == "somm":
        a_sel = raw["a"]
        b_sel = [co.index_cols(v, idx_np, bs) for v in raw["b"]]
        d_ref = [co.mask_share(raw["x"][i], raw["a"][i]) for i in (0, 1)]
        g_ref = [co.mask_share(co.index_cols(raw["y"][i], idx_np, bs), b_sel[i]) for i in (0, 1)]
        cut_d = lambda v: v
        cut_g = lambda v: v[:, :n_act]
        spare_g = lambda v: v[:, n_act:]
    else:
        a_sel = [co.index_cols(v, idx_np, bs) for v in raw["a"]]
        b_sel = [co.index_rows(v, idx_np, bs) for v in raw["b"]]
        d_ref = [co.mask_share(co.index_cols(raw["x"][i], idx_np, bs), a_sel[i]) for i in (0, 1)]
        g_ref = [co.mask_share(co.index_rows(raw["y"][i], idx_np, bs), b_sel[i]) for i in (0, 1)]
        cut_d = lambda v: v[:, :n_act]
        cut_g = lambda v: v[:n_act]
        spare_g = lambda v: v[n_act:]
    e_ref, f_ref = co.open_(d_ref[0], d_ref[1]), co.open_(g_ref[0], g_ref[1])
    for i in (0, 1):
        assert np.array_equal(cut_d(down(d[i])), d_ref[i]), "masked X-side share %d" % i
        assert np.array_equal(cut_g(down(g[i])), g_ref[i]), "masked W-side share %d" % i
        assert np.all(spare_g(down(g[i])) == SENTINEL), "W-side share %d written beyond the kept blocks" % i
        if mm.kind == "simm":
            assert np.all(down(d[i])[:, n_act:] == SENTINEL), "X-side share %d written beyond the kept blocks" % i
    assert np.array_equal(cut_d(down(e)), e_ref) and np.array_equal(cut_g(down(f)), f_ref)

    for i in (0, 1):
        got = down(z[i])
        want = co.beaver_share(i, e_ref, f_ref, a_sel[i], b_sel[i], c[i])
        if mm.kind == "somm":
            assert np.array_equal(got[:, :n_act], want), "share %d" % i
            assert np.all(got[:, n_act:] == SENTINEL), "share %d written beyond the kept blocks" % i
        else:
            assert np.array_equal(got, want), "share %d" % i


def test_config3_llama7b_ffn(ctx):
    cfg = configs.config(3)
    mask = configs.token_masks(cfg)
    for mm in cfg.matmuls:
        say("config 3 %s (%s) m=%d k=%d n=%d" % (mm.name, mm.kind, mm.m, mm.k, mm.n))
        _run_projection(ctx, cfg, mm, mask)


def test_config3_spare_block_capacity(ctx):
    """Gate (SOMM) and down (SIMM) projection of config 3 with five blocks of spare capacity."""
    cfg = configs.config(3)
    mask = configs.token_masks(cfg)
    for mm in (cfg.matmuls[0], cfg.matmuls[2]):
        say("config 3 %s (%s) with spare capacity" % (mm.name, mm.kind))
        _run_projection(ctx, cfg, mm, mask, spare=5)


def test_config4_llama13b_decode(ctx):
    cfg = configs.config(4)
    mask = configs.token_masks(cfg)
    for mm in cfg.matmuls:
        say("config 4 %s (%s) m=%d k=%d n=%d" % (mm.name, mm.kind, mm.m, mm.k, mm.n))
        _run_projection(ctx, cfg, mm, mask)


@pytest.mark.parametrize("density", configs.C5_DENSITIES)
def test_config5_density_sweep(ctx, density):
    cfg = configs.config(5, density)
    mask = configs.token_masks(cfg)
    mm = cfg.matmuls[0]
    say("config 5 density %.2f down-projection m=%d k=%d n=%d" % (density, mm.m, mm.k, mm.n))
    _run_projection(ctx, cfg, mm, mask)


def _run_grouped(ctx, cfg, mms, mask_np, neuron_major=False):
    """bench.py's default step for the projections ``mms`` (one kind, one shape): weight-side
    operands as digit planes, all products of both parties in one ``share_group`` call (the
    library decides whether that is one launch).  Every output element against the oracle.
    ``neuron_major`` (SOMM): the weights and their triple shares are stored one row per neuron,
    the kept neurons are gathered as rows and the planes are packed from that layout."""
    import paper_2505_07239_amd as comet
    bs, kind = cfg.bs, mms[0].kind
    idx_np = co.compact_mask(mask_np)
    t = len(idx_np)
    n_act = t * bs
    idx, n_dev = ctx.compact_mask(torch.from_numpy(mask_np).cuda())
    members, wants = [], []
    for mm in mms:
        sid = lambda role: configs.stream_id(cfg, mm.index, role)
        u = lambda role, *shape: rng.uniform_u64(rng.BASE_SEED, sid(role), int(np.prod(shape))).reshape(shape)
        x = [u(configs.R_XSPLIT, mm.m, mm.k), u(configs.R_X, mm.m, mm.k)]
        y = [u(configs.R_YSPLIT, mm.k, mm.n), u(configs.R_Y, mm.k, mm.n)]
        a = [u(configs.R_ASPLIT, mm.m, mm.k), u(configs.R_A, mm.m, mm.k)]
        b = [u(configs.R_BSPLIT, mm.k, mm.n), u(configs.R_B, mm.k, mm.n)]
        zshape = (mm.m, n_act) if kind == "somm" else (mm.m, mm.n)
        c = [rng.uniform_u64(rng.BASE_SEED, sid(configs.R_CSPLIT) + 50 * i, zshape[0] * zshape[1]).reshape(zshape)
             for i in (0, 1)]
        ga, gb = [up(v) for v in a], [up(v) for v in b]
        d, g = [], []
        for i in (0, 1):
            if kind == "somm" and neuron_major:
                d.append(ctx.mask_share(up(x[i]), ga[i]))
                g.append(ctx.mask_share_gather(up(np.ascontiguousarray(y[i].T)), up(np.ascontiguousarray(b[i].T)),
                                               comet.AXIS_ROWS, bs, idx, n_dev, t))
            elif kind == "somm":
                d.append(ctx.mask_share(up(x[i]), ga[i]))
                g.append(ctx.mask_share_gather(up(y[i]), gb[i], comet.AXIS_COLS, bs, idx, n_dev, t))
            else:
                d.append(ctx.mask_share_gather(up(x[i]), ga[i], comet.AXIS_COLS, bs, idx, n_dev, t))
                g.append(ctx.mask_share_gather(up(y[i]), gb[i], comet.AXIS_ROWS, bs, idx, n_dev, t))
        e = ctx.open(d[0], d[1])
        nm = neuron_major and kind == "somm"
        f = ctx.open_weight_planes(g[0], g[1], neuron_major=nm)
        for i in (0, 1):
            b_pl = ctx.open_weight_planes(up(np.ascontiguousarray(b[i].T)), neuron_major=True) if nm \
                else ctx.open_weight_planes(gb[i])
            members.append((i, e, f, ga[i], b_pl, up(c[i])))
        torch.cuda.synchronize()
        del gb, g, d
        # oracle side, in full
        if kind == "somm":
            a_sel, b_sel = a, [co.index_cols(v, idx_np, bs) for v in b]
            e_ref = co.open_(co.mask_share(x[0], a[0]), co.mask_share(x[1], a[1]))
            f_ref = co.open_(*[co.mask_share(co.index_cols(y[i], idx_np, bs), b_sel[i]) for i in (0, 1)])
        else:
            a_sel = [co.index_cols(v, idx_np, bs) for v in a]
            b_sel = [co.index_rows(v, idx_np, bs) for v in b]
            e_ref = co.open_(*[co.mask_share(co.index_cols(x[i], idx_np, bs), a_sel[i]) for i in (0, 1)])
            f_ref = co.open_(*[co.mask_share(co.index_rows(y[i], idx_np, bs), b_sel[i]) for i in (0, 1)])
        assert np.array_equal(down(e), e_ref)
        wants += [co.beaver_share(i, e_ref, f_ref, a_sel[i], b_sel[i], c[i]) for i in (0, 1)]
        del x, y, a, b, a_sel, b_sel
    outs = [_sentinel(*w.shape) for w in wants]
    ctx.share_group(kind, bs, idx, n_dev, t, members, out=outs)
    torch.cuda.synchronize()
    assert int(n_dev.item()) == t
    for j, (z, want) in enumerate(zip(outs, wants)):
        assert np.array_equal(down(z), want), "member %d (projection %s, party %d)" % (j, mms[j // 2].name, j % 2)


def test_config3_grouped_calls_on_weight_planes(ctx):
    """The step bench.py times by default: gate and up of both parties in one grouped call (four
    products, one launch), then down of both parties."""
    cfg = configs.config(3)
    mask = configs.token_masks(cfg)
    somm = [mm for mm in cfg.matmuls if mm.kind == "somm"]
    simm = [mm for mm in cfg.matmuls if mm.kind == "simm"]
    say("config 3 grouped: %s" % "+".join(mm.name for mm in somm))
    _run_grouped(ctx, cfg, somm, mask)
    say("config 3 grouped: %s" % "+".join(mm.name for mm in simm))
    _run_grouped(ctx, cfg, simm, mask)


def test_config3_gate_and_up_from_neuron_major_weights(ctx):
    """bench.py keeps the gate / up weights one row per neuron: row gather of the kept neurons,
    planes packed from that layout, the same grouped share call; every output element."""
    cfg = configs.config(3)
    mask = configs.token_masks(cfg)
    somm = [mm for mm in cfg.matmuls if mm.kind == "somm"]
    say("config 3 grouped, neuron-major weights: %s" % "+".join(mm.name for mm in somm))
    _run_grouped(ctx, cfg, somm, mask, neuron_major=True)


@pytest.mark.parametrize("density", configs.C5_DENSITIES)
def test_config5_density_sweep_grouped_calls_on_weight_planes(ctx, density):
    """Config 5 the way bench.py runs it: both parties' down-projection shares through one grouped
    call on weight planes (one launch at 10 % and 5 %, two launches with owned tiles above)."""
    cfg = configs.config(5, density)
    mask = configs.token_masks(cfg)
    say("config 5 density %.2f grouped call on weight planes" % density)
    _run_grouped(ctx, cfg, [cfg.matmuls[0]], mask)
