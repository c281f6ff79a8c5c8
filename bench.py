#!/usr/bin/env python3
"""Benchmark of the hot path on one MI355X.

One *step* is one pass of the whole local path of a sparse FFN layer over one
batch of synthetic input: compact the predicted block mask, then for every
projection of the layer (gate / up: SOMM, down: SIMM) mask both parties'
shares, open them, and compute both parties' output shares.  All inputs are
resident in HBM before the timed region starts.

Prints ONE JSON line.  ``value`` is ring-GEMM throughput: algorithmic ring
operations (1 multiply-accumulate mod 2^64 = 2 ops, two products per party per
projection -- the minimum for Eq. 1) of one step divided by the step time.
Both simulated parties run on the same GPU one after the other, so this is the
rate one party's GPU sustains.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c3]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

METRIC = "sparse secret-shared FFN ring-GEMM Gop/s (mod 2^64) per party; % of roofline"
PEAK_INT8_TOPS = 5000.0      # MI355X dense int8 MFMA, published
PEAK_HBM_GBS = 8000.0        # MI355X HBM3E, published
INT8_OPS_PER_RING_MAC = 72   # 36 digit products, 2 ops each

# HBM bytes per ring-GEMM launch (average over the launches of one step) from rocprofv3 --pmc
# runs of this file: FETCH_SIZE and WRITE_SIZE, each scaled by what the same counter reads for
# the copy probe of known size in the same run; the summaries are under profiles/.  None until
# measured for that workload.
GEMM_TRAFFIC_BYTES = {"c3": 199303800, "c4": 987125342}


def log(msg):
    print("[bench] " + msg, file=sys.stderr, flush=True)


def parse_workload(name):
    from workloads import configs
    name = name.lower()
    if name.startswith("c5"):
        dens = 1.0
        if "_d" in name:
            dens = int(name.split("_d")[1]) / 100.0
        return configs.config(5, dens), "c5_d%03d" % round(dens * 100)
    cid = int(name[1:])
    return configs.config(cid), "c%d" % cid


class Layer:
    """Device buffers of one sparse FFN layer and the step that runs the path."""

    def __init__(self, ctx, cfg, seed):
        import numpy as np
        import torch
        from workloads import configs
        self.ctx, self.cfg = ctx, cfg
        dev = torch.device("cuda:0")
        self.mask_np = configs.token_masks(cfg, seed)
        self.mask = torch.from_numpy(self.mask_np).to(dev)
        self.n_blk = int(np.count_nonzero(self.mask_np.max(axis=0)))     # public sparsity level
        self.n_act = self.n_blk * cfg.bs
        self.idx = torch.zeros(cfg.nb, dtype=torch.int32, device=dev)
        self.n_dev = torch.zeros(1, dtype=torch.int32, device=dev)
        gen = torch.Generator(device=dev)

        def words(stream, *shape):
            # additive shares and triple parts are uniform over Z_{2^64} whatever the secrets are
            gen.manual_seed(seed * 1000003 + stream)
            return torch.randint(-(2 ** 63), 2 ** 63 - 1, shape, dtype=torch.int64, device=dev,
                                 generator=gen)

        self.mm = []
        for mm in cfg.matmuls:
            sid = lambda role, party=0: configs.stream_id(cfg, mm.index, role) * 2 + party
            b = dict(mm=mm)
            b["x"] = [words(sid(0, i), mm.m, mm.k) for i in (0, 1)]
            b["y"] = [words(sid(1, i), mm.k, mm.n) for i in (0, 1)]
            b["a"] = [words(sid(4, i), mm.m, mm.k) for i in (0, 1)]
            b["b"] = [words(sid(5, i), mm.k, mm.n) for i in (0, 1)]
            if mm.kind == "somm":
                dshape, gshape, zshape = (mm.m, mm.k), (mm.k, self.n_act), (mm.m, self.n_act)
            else:
                dshape, gshape, zshape = (mm.m, self.n_act), (self.n_act, mm.n), (mm.m, mm.n)
            b["c"] = [words(sid(8, i), *zshape) for i in (0, 1)]
            b["d"] = [torch.empty(dshape, dtype=torch.int64, device=dev) for _ in (0, 1)]
            b["g"] = [torch.empty(gshape, dtype=torch.int64, device=dev) for _ in (0, 1)]
            b["e"] = torch.empty(dshape, dtype=torch.int64, device=dev)
            b["f"] = torch.empty(gshape, dtype=torch.int64, device=dev)
            b["z"] = [torch.empty(zshape, dtype=torch.int64, device=dev) for _ in (0, 1)]
            b["macs_per_launch"] = 2 * mm.m * (mm.k if mm.kind == "somm" else self.n_act) * \
                (self.n_act if mm.kind == "somm" else mm.n)
            self.mm.append(b)
        self.ring_ops_per_step = sum(2 * 2 * b["macs_per_launch"] for b in self.mm)   # 2 parties, 2 ops/MAC

    # ---- the same step with the bandwidth-bound kernels and the ring GEMMs on two streams ----
    def enable_overlap(self, ctx_stream_kernels):
        """Second set of the buffers a step writes (index list, masked and opened operands,
        output shares), two streams of default priority and the events that order them.  The
        masking / opening / compaction kernels of one step then run beside the GEMMs of the
        previous projection or the previous step: consecutive steps alternate between the sets."""
        import torch
        self.ctx_ew = ctx_stream_kernels
        self.s_ew, self.s_gemm = torch.cuda.Stream(), torch.cuda.Stream()
        dev = self.idx.device
        self.sets = []
        for q in (0, 1):
            st = {"idx": self.idx if q == 0 else torch.zeros_like(self.idx),
                  "n_dev": self.n_dev if q == 0 else torch.zeros_like(self.n_dev), "mm": []}
            for b in self.mm:
                if q == 0:
                    st["mm"].append(b)
                else:
                    c2 = dict(b)
                    for key in ("d", "g", "z"):
                        c2[key] = [torch.empty_like(t) for t in b[key]]
                    for key in ("e", "f"):
                        c2[key] = torch.empty_like(b[key])
                    st["mm"].append(c2)
            st["ew_done"] = [torch.cuda.Event() for _ in self.mm]
            st["gemm_done"] = torch.cuda.Event()
            st["gemm_done"].record(torch.cuda.current_stream())
            self.sets.append(st)
        self.parity = 0
        del dev

    def step_overlapped(self):
        import torch
        import paper_2505_07239_amd as comet
        cfg = self.cfg
        st = self.sets[self.parity]
        self.parity ^= 1
        with torch.cuda.stream(self.s_ew):
            self.s_ew.wait_event(st["gemm_done"])          # the GEMMs that last read this set are done
            ctx = self.ctx_ew
            ctx.compact_mask(self.mask, st["idx"], st["n_dev"])
            for j, b in enumerate(st["mm"]):
                mm = b["mm"]
                for i in (0, 1):
                    if mm.kind == "somm":
                        ctx.mask_share(b["x"][i], b["a"][i], out=b["d"][i])
                        ctx.mask_share_gather(b["y"][i], b["b"][i], comet.AXIS_COLS, cfg.bs, st["idx"],
                                              st["n_dev"], self.n_blk, out=b["g"][i])
                    else:
                        ctx.mask_share_gather(b["x"][i], b["a"][i], comet.AXIS_COLS, cfg.bs, st["idx"],
                                              st["n_dev"], self.n_blk, out=b["d"][i])
                        ctx.mask_share_gather(b["y"][i], b["b"][i], comet.AXIS_ROWS, cfg.bs, st["idx"],
                                              st["n_dev"], self.n_blk, out=b["g"][i])
                ctx.open(b["d"][0], b["d"][1], out=b["e"])
                ctx.open(b["g"][0], b["g"][1], out=b["f"])
                st["ew_done"][j].record(self.s_ew)
        with torch.cuda.stream(self.s_gemm):
            ctx = self.ctx
            for j, b in enumerate(st["mm"]):
                mm = b["mm"]
                self.s_gemm.wait_event(st["ew_done"][j])
                for i in (0, 1):
                    if mm.kind == "somm":
                        ctx.somm_share(i, cfg.bs, st["idx"], st["n_dev"], self.n_blk, b["e"], b["f"],
                                       b["a"][i], b["b"][i], b["c"][i], out=b["z"][i])
                    else:
                        ctx.simm_share(i, cfg.bs, st["idx"], st["n_dev"], self.n_blk, b["e"], b["f"],
                                       b["a"][i], b["b"][i], b["c"][i], out=b["z"][i])
            st["gemm_done"].record(self.s_gemm)

    def step(self):
        import paper_2505_07239_amd as comet
        ctx, cfg = self.ctx, self.cfg
        ctx.compact_mask(self.mask, self.idx, self.n_dev)
        for b in self.mm:
            mm = b["mm"]
            for i in (0, 1):
                if mm.kind == "somm":
                    ctx.mask_share(b["x"][i], b["a"][i], out=b["d"][i])
                    ctx.mask_share_gather(b["y"][i], b["b"][i], comet.AXIS_COLS, cfg.bs, self.idx,
                                          self.n_dev, self.n_blk, out=b["g"][i])
                else:
                    ctx.mask_share_gather(b["x"][i], b["a"][i], comet.AXIS_COLS, cfg.bs, self.idx,
                                          self.n_dev, self.n_blk, out=b["d"][i])
                    ctx.mask_share_gather(b["y"][i], b["b"][i], comet.AXIS_ROWS, cfg.bs, self.idx,
                                          self.n_dev, self.n_blk, out=b["g"][i])
            ctx.open(b["d"][0], b["d"][1], out=b["e"])
            ctx.open(b["g"][0], b["g"][1], out=b["f"])
            for i in (0, 1):
                if mm.kind == "somm":
                    ctx.somm_share(i, cfg.bs, self.idx, self.n_dev, self.n_blk, b["e"], b["f"],
                                   b["a"][i], b["b"][i], b["c"][i], out=b["z"][i])
                else:
                    ctx.simm_share(i, cfg.bs, self.idx, self.n_dev, self.n_blk, b["e"], b["f"],
                                   b["a"][i], b["b"][i], b["c"][i], out=b["z"][i])


def cpu_baseline(layer, budget_s=20.0):
    """The CPU oracle, as it stands, on a bounded sample of the same workload:
    both parties' output shares (the oracle's three-product Eq. 1 loops) of
    every projection of the layer, on all output rows when that fits the time
    budget and on a leading block of rows otherwise.  The sampled rows are also
    compared with the GPU's result."""
    import numpy as np
    import oracle as co
    cfg = layer.cfg
    host = lambda t: t.cpu().numpy().view(np.uint64)
    idx = layer.idx[:layer.n_blk].cpu().numpy()
    cores = co.num_threads()
    per_proj = budget_s / len(layer.mm)
    total_ops, total_s, ok, notes = 0.0, 0.0, True, []
    one_ops, one_s = 0.0, 0.0                 # the one-row trials: one output row, so one thread
    for b in layer.mm:
        mm = b["mm"]
        e, f = host(b["e"]), host(b["f"])
        k_eff, n_eff = e.shape[1], f.shape[1]
        a_sel, b_sel = [], []
        for i in (0, 1):
            a_i, b_i = host(b["a"][i]), host(b["b"][i])
            if mm.kind == "somm":
                a_sel.append(a_i)
                b_sel.append(co.index_cols(b_i, idx, cfg.bs))
            else:
                a_sel.append(co.index_cols(a_i, idx, cfg.bs))
                b_sel.append(co.index_rows(b_i, idx, cfg.bs))
        c = [host(b["c"][i]) for i in (0, 1)]
        # size the sample from a one-row trial
        t0 = time.perf_counter()
        co.beaver_share_rows(0, e, f, a_sel[0], b_sel[0], c[0], 0, 1)
        t_row = max(time.perf_counter() - t0, 1e-6)
        one_ops += 2 * (2.0 * k_eff * n_eff)                       # party 0: two products, 2 ops/MAC
        one_s += t_row
        rows = int(max(1, min(mm.m, per_proj / (2.0 * t_row) * min(cores, 8))))
        t0 = time.perf_counter()
        z = [co.beaver_share_rows(i, e, f, a_sel[i], b_sel[i], c[i], 0, rows) for i in (0, 1)]
        dt = time.perf_counter() - t0
        ok = ok and all(np.array_equal(z[i], host(b["z"][i])[:rows]) for i in (0, 1))
        total_ops += 2 * 2 * (2.0 * rows * k_eff * n_eff)         # 2 parties, 2 ops/MAC, 2 products
        total_s += dt
        notes.append("%s rows 0..%d of %d" % (mm.name, rows, mm.m))
    return {"value": total_ops / total_s / 1e9, "unit": "Gop/s", "cores": cores, "kind": "oracle",
            "value_1core": one_ops / one_s / 1e9,
            "sample": "both parties' shares, %s; oracle's 3-product Eq. 1 loops counted as the "
                      "2-product minimum; %.1f s of wall time on %d threads (%.0f thread-seconds)" %
                      ("; ".join(notes), total_s, cores, total_s * cores),
            "matches_gpu": bool(ok)}


def general_forms(ctx, timed):
    """Protocols 2 and 3 with per-token masks on a batch of four unrelated requests (256 tokens,
    LLaMA-7B gate projection, 15 % of the blocks per token): component search, the share
    restricted to the result blocks against the same call on the union of all masks, and the
    down projection with per-token row sets."""
    import numpy as np
    import torch
    from workloads import masks, rng
    m, k, nb, bs, groups = 256, 4096, 344, 32, 4
    dev = torch.device("cuda:0")
    mk = masks.grouped_token_masks(rng.BASE_SEED, 9000, m, nb, groups, 0.15)
    tm = torch.from_numpy(mk).to(dev)
    comp = ctx.components(tm)
    torch.cuda.synchronize()
    n_row, n_blk, n_comp = (int(comp[q].item()) for q in ("n_row", "n_blk", "n_comp"))
    gen = torch.Generator(device=dev)
    gen.manual_seed(77)
    words = lambda *shape: torch.randint(-(2 ** 63), 2 ** 63 - 1, shape, dtype=torch.int64, device=dev,
                                         generator=gen)
    n_act = n_blk * bs
    e, a, f, b, c = words(m, k), words(m, k), words(k, n_act), words(k, nb * bs), words(m, n_act)
    z = torch.empty_like(c)
    out = {"general_n_components": n_comp, "general_rows": n_row, "general_blocks": n_blk}
    out["components_us"] = timed(lambda: ctx.components(tm), reps=20) * 1e6
    t_blocks = timed(lambda: ctx.somm_share_blocks(1, bs, comp["blk_idx"], comp["blk_comp"], comp["n_blk"],
                                                   n_blk, comp["row_comp"], comp["n_row"], e, f, a, b, c,
                                                   out=z), reps=10)
    t_union = timed(lambda: ctx.somm_share(1, bs, comp["blk_idx"], comp["n_blk"], n_blk, e, f, a, b, c,
                                           out=z), reps=10)
    out["somm_result_blocks_us"] = t_blocks * 1e6
    out["somm_union_of_masks_us"] = t_union * 1e6
    # ring MACs on the result blocks only: sum over components of rows x columns x 2k
    rc = comp["row_comp"][:n_row].cpu().numpy()
    bc = comp["blk_comp"][:n_blk].cpu().numpy()
    macs = sum(int((rc == q).sum()) * int((bc == q).sum()) * bs for q in range(n_comp)) * 2 * k
    out["somm_result_blocks_Gops"] = 2.0 * macs / t_blocks / 1e9
    # down projection with per-token row sets (same masks, union of the blocks contracted)
    idx, n_dev = ctx.compact_mask(tm)
    kc = n_blk * bs
    e2, a2, f2, b2, c2 = words(m, kc), words(m, nb * bs), words(kc, k), words(nb * bs, k), words(m, k)
    z2 = torch.empty_like(c2)
    t_rows = timed(lambda: ctx.simm_share_masked(1, bs, idx, n_dev, n_blk, tm, e2, f2, a2, b2, c2, out=z2),
                   reps=10)
    t_plain = timed(lambda: ctx.simm_share(1, bs, idx, n_dev, n_blk, e2, f2, a2, b2, c2, out=z2), reps=10)
    out["simm_row_sets_us"] = t_rows * 1e6
    out["simm_union_of_masks_us"] = t_plain * 1e6
    return out


def weight_layouts(ctx, timed):
    """SOMM of the LLaMA-7B gate projection (256 tokens, 52 of 344 blocks) with the weight side
    stored row-major (d x f, kept neurons are 256-byte segments of every row) and neuron-major
    (f x d, a kept neuron is one contiguous row): the indexed masking of the weights and the
    share call, each with the full-size triple part indexed in the kernel."""
    import torch
    import paper_2505_07239_amd as comet
    from workloads import masks, rng
    m, k, nb, bs = 256, 4096, 344, 32
    dev = torch.device("cuda:0")
    mask = masks.clustered_block_mask(rng.BASE_SEED, 9100, nb, 0.15, 4.0)[None, :]
    idx, n_dev = ctx.compact_mask(torch.from_numpy(mask).to(dev))
    t_blk = int(n_dev.item())
    n_act = t_blk * bs
    gen = torch.Generator(device=dev)
    gen.manual_seed(79)
    words = lambda *shape: torch.randint(-(2 ** 63), 2 ** 63 - 1, shape, dtype=torch.int64, device=dev,
                                         generator=gen)
    e, a, c = words(m, k), words(m, k), words(m, n_act)
    z = torch.empty_like(c)
    out = {}
    for name, tr in (("row_major", False), ("neuron_major", True)):
        y, b = (words(nb * bs, k), words(nb * bs, k)) if tr else (words(k, nb * bs), words(k, nb * bs))
        g = torch.empty((n_act, k) if tr else (k, n_act), dtype=torch.int64, device=dev)
        axis = comet.AXIS_ROWS if tr else comet.AXIS_COLS
        t = timed(lambda: ctx.mask_share_gather(y, b, axis, bs, idx, n_dev, t_blk, out=g), reps=20)
        out["somm_weights_%s_mask_GBs" % name] = 24.0 * k * n_act / t / 1e9
        t = timed(lambda: ctx.somm_share(1, bs, idx, n_dev, t_blk, e, g, a, b, c, neuron_major=tr, out=z),
                  reps=10)
        out["somm_weights_%s_share_us" % name] = t * 1e6
    return out


def glue_steps(ctx, timed):
    """Shuffle steps, merge to full width and rescaling on a 4096 x 11008 matrix of words (the
    activations of 4096 tokens at the FFN width): achieved GB/s of algorithmic bytes."""
    import torch
    import paper_2505_07239_amd as comet
    rows, cols, bs = 4096, 11008, 32
    dev = torch.device("cuda:0")
    gen = torch.Generator(device=dev)
    gen.manual_seed(78)
    words = lambda *shape: torch.randint(-(2 ** 63), 2 ** 63 - 1, shape, dtype=torch.int64, device=dev,
                                         generator=gen)
    x, mk, o = words(rows, cols), words(rows, cols), torch.empty((rows, cols), dtype=torch.int64, device=dev)
    pc = torch.randperm(cols, device=dev, generator=gen).to(torch.int32)
    pr = torch.randperm(rows, device=dev, generator=gen).to(torch.int32)
    n = rows * cols
    out = {}
    t = timed(lambda: ctx.permute_mask(x, pc, mk, comet.AXIS_COLS, +1, out=o), reps=10)
    out["shuffle_cols_GBs"] = 24.0 * n / t / 1e9
    t = timed(lambda: ctx.permute_mask(x, pr, mk, comet.AXIS_ROWS, -1, out=o), reps=10)
    out["shuffle_rows_GBs"] = 24.0 * n / t / 1e9
    t = timed(lambda: ctx.truncate_share(1, x, 16, out=o), reps=10)
    out["truncate_GBs"] = 16.0 * n / t / 1e9
    keep = 52
    idx = (torch.arange(keep, device=dev, dtype=torch.int32) * 6).contiguous()
    nd = torch.tensor([keep], dtype=torch.int32, device=dev)
    c = words(rows, keep * bs)
    t = timed(lambda: ctx.scatter_cols(c, bs, idx, nd, keep, cols, out=o), reps=10)
    out["scatter_GBs"] = (8.0 * n + 16.0 * rows * keep * bs) / t / 1e9   # zero fill + kept blocks read and written
    return out


def micro(ctx, layer):
    """Per-kernel yardsticks on the same device (stderr + returned dict)."""
    import torch
    from workloads import masks
    out = {}

    def timed(fn, reps=20):
        fn()
        torch.cuda.synchronize()
        s, e = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        s.record()
        for _ in range(reps):
            fn()
        e.record()
        torch.cuda.synchronize()
        return s.elapsed_time(e) / reps * 1e-3

    n = 11008 * 4096                                  # weight side of the dense down projection
    a = torch.randint(-(2 ** 63), 2 ** 63 - 1, (n,), dtype=torch.int64, device="cuda")
    b = torch.randint(-(2 ** 63), 2 ** 63 - 1, (n,), dtype=torch.int64, device="cuda")
    o = torch.empty_like(a)
    t = timed(lambda: ctx.open(a, b, out=o))
    out["open_GBs"] = 24.0 * n / t / 1e9
    t = timed(lambda: ctx.mask_share(a, b, out=o))
    out["mask_share_GBs"] = 24.0 * n / t / 1e9
    t = timed(lambda: ctx.probe_copy(a, o))
    out["copy_GBs"] = 16.0 * n / t / 1e9
    del a, b, o
    flags = 1 << 28
    m = masks.stress_mask_device(7, flags, torch.device("cuda:0"), 0.15)
    idx = torch.empty(flags, dtype=torch.int32, device="cuda")
    nd = torch.empty(1, dtype=torch.int32, device="cuda")
    t = timed(lambda: ctx.compact_mask(m, idx, nd), reps=10)
    kept = int(nd.item())
    out["compact_stress_GBs"] = (flags + 4.0 * kept) / t / 1e9
    out["compact_stress_kept"] = kept
    del m, idx
    t = timed(lambda: ctx.compact_mask(layer.mask, layer.idx, layer.n_dev), reps=50)
    out["compact_layer_mask_us"] = t * 1e6
    out.update(general_forms(ctx, timed))
    out.update(glue_steps(ctx, timed))
    out.update(weight_layouts(ctx, timed))
    macs = ctx.probe_mfma_i8(1024, 2000)
    t = timed(lambda: ctx.probe_mfma_i8(1024, 2000), reps=5)
    out["mfma_i8_issue_TOPs"] = 2.0 * macs / t / 1e12
    # same instruction stream on uniformly random operand bytes (what share digits look like):
    # the chip clocks down under the extra switching power
    t = timed(lambda: ctx.probe_mfma_i8(1024, 2000, True), reps=10)
    out["mfma_i8_issue_random_operands_TOPs"] = 2.0 * macs / t / 1e12
    macs = ctx.probe_valu_mac64(2048, 2000)
    t = timed(lambda: ctx.probe_valu_mac64(2048, 2000), reps=5)
    out["valu_mac64_Gops"] = 2.0 * macs / t / 1e9
    out["integer_roofline_Gops"] = max(out["valu_mac64_Gops"],
                                       out["mfma_i8_issue_TOPs"] * 1e3 / 36.0)
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="c3",
                    help="c1..c4, c5_d100 / c5_d050 / c5_d025 / c5_d010 / c5_d005")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-micro", action="store_true")
    ap.add_argument("--overlap", action="store_true",
                    help="run the bandwidth-bound kernels and the ring GEMMs on two streams")
    ap.add_argument("--graph", action="store_true",
                    help="time replays of one step captured in a HIP graph instead of eager calls")
    ap.add_argument("--gemm-chunk", type=int, default=0, help="tuning sweep: scheduling slice length")
    ap.add_argument("--gemm-grid", type=int, default=0, help="tuning sweep: workgroups per launch")
    ap.add_argument("--gemm-tile", type=int, default=0, help="tuning sweep: 2 = 64x64 tile")
    ap.add_argument("--skinny", type=int, default=0, help="tuning sweep: 1 = matrix cores even for m <= 8")
    ap.add_argument("--skinny-slices", type=int, default=0, help="tuning sweep: contraction slices of the m <= 8 kernel")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build measures one GPU only (both parties are simulated on it); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    import paper_2505_07239_amd as comet
    from workloads import rng
    if not os.path.exists(comet.binding.LIB_PATH):
        from paper_2505_07239_amd import build
        build.build()

    cfg, wname = parse_workload(args.workload)
    ctx = comet.Context(0)
    ctx.set_tuning(comet.TUNE_GEMM_CHUNK, args.gemm_chunk)
    ctx.set_tuning(comet.TUNE_GEMM_GRID, args.gemm_grid)
    ctx.set_tuning(comet.TUNE_GEMM_TILE, args.gemm_tile)
    ctx.set_tuning(comet.TUNE_SKINNY, args.skinny)
    ctx.set_tuning(comet.TUNE_SKINNY_SLICES, args.skinny_slices)
    layer = Layer(ctx, cfg, rng.BASE_SEED)
    log("workload %s: %s, m=%d d=%d f=%d bs=%d kept blocks %d/%d (n_act=%d), %.2f G ring ops/step" %
        (wname, cfg.name, cfg.tokens, cfg.d_model, cfg.d_ff, cfg.bs, layer.n_blk, cfg.nb,
         layer.n_act, layer.ring_ops_per_step / 1e9))

    run_step = layer.step
    if args.overlap:
        ctx_ew = comet.Context(0)
        layer.enable_overlap(ctx_ew)
        run_step = layer.step_overlapped
    for _ in range(args.warmup):
        run_step()
    torch.cuda.synchronize()
    launches = 2 * len(layer.mm) * args.steps
    if args.graph:
        # One step captured in a HIP graph (every call only enqueues kernels) and replayed: the
        # launch gaps between the thirty-odd kernels of a step go away.  The share kernel is timed
        # with HIP events in an eager pass first, since events do not work inside a replay.
        ctx.timing_begin(launches)
        for _ in range(args.steps):
            layer.step()
        torch.cuda.synchronize()
        gemm_ms, n_timed = ctx.timing_end()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            layer.step()
        graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            graph.replay()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
    else:
        ctx.timing_begin(launches)
        t0 = time.perf_counter()
        for _ in range(args.steps):
            run_step()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        gemm_ms, n_timed = ctx.timing_end()

    ms_per_step = (t1 - t0) * 1e3 / args.steps
    value = layer.ring_ops_per_step / (ms_per_step * 1e-3) / 1e9
    macs_per_launch = sum(b["macs_per_launch"] for b in layer.mm) / len(layer.mm)
    gemm_ms_avg = gemm_ms / max(n_timed, 1)
    achieved = INT8_OPS_PER_RING_MAC * macs_per_launch / (gemm_ms_avg * 1e-3) / 1e12
    result = {
        "metric": METRIC, "value": value, "unit": "Gop/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "u64", "data": "synthetic",
        "config": {"workload": "%s: %s FFN, %d tokens, d_model %d, d_ff %d, block %d, %d of %d blocks "
                               "kept (%s mask); projections %s; both parties" %
                               (wname, cfg.name, cfg.tokens, cfg.d_model, cfg.d_ff, cfg.bs,
                                layer.n_blk, cfg.nb, cfg.mask_kind,
                                "+".join(m.name for m in cfg.matmuls)),
                   "ring_ops_per_step": layer.ring_ops_per_step,
                   "launches_per_step": 2 * len(layer.mm),
                   "submission": "hip graph replay" if args.graph else
                                 ("eager, two streams" if args.overlap else "eager")},
        "roofline": {"bound": "mfma", "kernel": "ring_gemm_kernel",
                     "achieved": achieved, "peak": PEAK_INT8_TOPS, "unit": "TOP/s",
                     "frac": achieved / PEAK_INT8_TOPS,
                     "traffic": GEMM_TRAFFIC_BYTES.get(wname),
                     "avg_launch_ms": gemm_ms_avg, "launches_timed": n_timed,
                     "ring_macs_per_launch": macs_per_launch,
                     "gemm_share_of_step": gemm_ms / max(n_timed, 1) * launches / ((t1 - t0) * 1e3),
                     "note": "algorithmic int8 ops: 36 digit products x 2 ops per ring MAC, two "
                             "products per party (2*m*k*n_act ring MACs per launch)"},
    }
    if cfg.tokens <= 8 and not args.skinny:
        # a few activation rows: the share calls take the vector-ALU kernel, bound by reading the
        # two weight-side operands (B_i and F, kc x n words each) once per launch
        wbytes = sum(b["macs_per_launch"] for b in layer.mm) / len(layer.mm) / cfg.tokens * 8.0
        ach = wbytes / (gemm_ms_avg * 1e-3) / 1e9
        result["roofline"] = {"bound": "hbm", "kernel": "ring_skinny_kernel", "achieved": ach,
                              "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": ach / PEAK_HBM_GBS,
                              "traffic": GEMM_TRAFFIC_BYTES.get(wname),
                              "avg_launch_ms": gemm_ms_avg, "launches_timed": n_timed,
                              "ring_macs_per_launch": macs_per_launch,
                              "gemm_share_of_step": gemm_ms / max(n_timed, 1) * launches / ((t1 - t0) * 1e3),
                              "note": "algorithmic bytes: the weight-side operands B_i and F of "
                                      "one launch, 8 bytes per word, read once"}
    if not args.no_micro:
        result["kernels"] = micro(ctx, layer)
        for k, v in result["kernels"].items():
            log("%s = %.4g" % (k, v))
        if result["roofline"]["bound"] == "mfma":
            result["roofline"]["frac_of_measured_mfma_issue"] = achieved / result["kernels"]["mfma_i8_issue_TOPs"]
            result["roofline"]["frac_of_measured_mfma_issue_random_operands"] = \
                achieved / result["kernels"]["mfma_i8_issue_random_operands_TOPs"]
        else:
            result["roofline"]["frac_of_measured_copy"] = result["roofline"]["achieved"] / result["kernels"]["copy_GBs"]
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(layer)
        log("cpu oracle: %.2f Gop/s on %d threads; rows match GPU: %s" %
            (result["cpu_baseline"]["value"], result["cpu_baseline"]["cores"],
             result["cpu_baseline"]["matches_gpu"]))
        if not result["cpu_baseline"]["matches_gpu"]:
            log("ERROR: GPU result differs from the oracle on the sampled rows")
            print(json.dumps(result))
            sys.exit(3)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
