#!/usr/bin/env python3
"""Benchmark of the hot path on one MI355X.

One *step* is one pass of the whole local path of a sparse FFN layer over one
batch of synthetic input: compact the predicted block mask, then for every
projection of the layer (gate / up: SOMM, down: SIMM) mask both parties'
shares, open them, and compute both parties' output shares.  The share products
that are ready together go into one grouped call (gate and up of both parties,
then down of both parties; the library runs them as one launch when the single
launches would be short); ``--per-call`` makes one call per product and party,
and the default line carries that run too (``per_call``).  All inputs are
resident in HBM before the timed region starts.

Prints ONE JSON line.  ``value`` is ring-GEMM throughput of the headline
workload (config 3 unless ``--workload`` says otherwise): algorithmic ring
operations (1 multiply-accumulate mod 2^64 = 2 ops, two products per party per
projection -- the minimum for Eq. 1) of one step divided by the step time.
Both simulated parties run on the same GPU one after the other, so this is the
rate one party's GPU sustains.  ``configs`` holds the same measurement, with
fewer steps, for every configuration (c1 .. c5 at all five densities), each with
the roofline that bounds it, the bytes the two parties would exchange (cost
model of the optimality appendix) and a check of a block of output rows against
the CPU oracle.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c3] [--configs all]
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
NEURON_MAJOR_SOMM = True     # SOMM weights stored one row per neuron when they travel as planes (--row-major-weights: off)
UNOPENED_FEW_ROWS = True     # decoding workloads: fold the opening of F into the share kernel (--opened-few-rows: off)
ALL_CONFIGS = ["c1", "c2", "c3", "c4", "c5_d100", "c5_d050", "c5_d025", "c5_d010", "c5_d005"]

# HBM bytes per share-kernel launch (average over the launches of one step) from rocprofv3 --pmc
# runs of this file: FETCH_SIZE and WRITE_SIZE, each scaled by what the same counter reads for
# the copy probe of known size in the same run.  The summaries, with the commands, are the
# files named here under profiles/.  None until measured for that workload and operand format.
GEMM_TRAFFIC = {
    ("c2", "planes", "single"): (13393313, "profiles/bench_c2_kernel_trace_and_hbm_counters.md"),
    ("c3", "planes", "grouped"): (611880557, "profiles/bench_c3_kernel_trace_and_hbm_counters.md"),
    ("c3", "planes", "single"): (197516269, "profiles/bench_c3_kernel_trace_and_hbm_counters.md"),
    ("c4", "words", "single"): (1456341918, "profiles/bench_c4_kernel_trace_and_hbm_counters.md"),
    ("c5_d100", "planes", "single"): (1549274757, "profiles/bench_c5_d100_kernel_trace_and_hbm_counters.md"),
    ("c5_d050", "planes", "single"): (792771729, "profiles/bench_c5_d050_kernel_trace_and_hbm_counters.md"),
    ("c5_d025", "planes", "single"): (396956726, "profiles/bench_c5_d025_kernel_trace_and_hbm_counters.md"),
    ("c5_d010", "planes", "grouped"): (358220326, "profiles/bench_c5_d010_kernel_trace_and_hbm_counters.md"),
    ("c5_d010", "planes", "single"): (178866692, "profiles/bench_c5_d010_kernel_trace_and_hbm_counters.md"),
    ("c5_d005", "planes", "grouped"): (215621442, "profiles/bench_c5_d005_kernel_trace_and_hbm_counters.md"),
    ("c5_d005", "planes", "single"): (107567254, "profiles/bench_c5_d005_kernel_trace_and_hbm_counters.md"),
}


PAPER_CONTEXT = {
    3: "Llama2-7B (ReLU) local computation, dense -> sparse: gate 66.4 -> 21.6 s, up 66.3 -> 19.9 s, down 64.5 -> "
       "8.9 s; communication 345 -> 36.1 GB (gate, up), 346 -> 35.4 GB (down) (Sec. 7, Performance Breakdown, per-layer table)",
    5: "SOMM / SIMM communication against a dense GEMM: 1.41x to 95.3x over the sparsity sweep, 8.1x at 90 % "
       "sparsity; computation is about 15 % of the matmul time on the paper's platform (Sec. 7, Component-wise Analysis)",
}


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
    """Device buffers of one sparse FFN layer and the step that runs the path.

    Shares and triple parts are the words of the seeded streams the GPU tests draw on the host
    (``workloads.rng``, same seed, stream and index), generated on the device; the mask comes
    from ``workloads.configs``.  ``planes``: the weight-side operands of the share calls travel
    as digit planes -- F is opened directly in that format (``comet_open_weight_planes``), the
    triple shares B_i are packed once, outside the step (offline material, Sec. 3.2)."""

    def __init__(self, ctx, cfg, seed, planes, unopened=True, neuron_major=True):
        import numpy as np
        import torch
        from workloads import configs, rng
        self.ctx, self.cfg = ctx, cfg
        self.planes = bool(planes) and cfg.tokens > 8      # the few-row kernel reads words
        # a few rows: the share kernel takes the two masked weight shares and forms F as it reads
        # them (comet_*_share_unopened); F is then never written to memory
        self.unopened = bool(unopened) and not self.planes and cfg.tokens <= 8
        # SOMM weights (and their triple shares) stored one row per neuron: a kept neuron is one
        # contiguous run in both projections of the layer (the weights are permuted and stored
        # once, offline, so their layout is free); the planes the share calls read are the same
        self.neuron_major = bool(neuron_major) and self.planes
        dev = torch.device("cuda:0")
        self.mask_np = configs.token_masks(cfg, seed)
        self.mask = torch.from_numpy(self.mask_np).to(dev)
        self.n_blk = int(np.count_nonzero(self.mask_np.max(axis=0)))     # public sparsity level
        self.n_act = self.n_blk * cfg.bs
        self.idx = torch.zeros(cfg.nb, dtype=torch.int32, device=dev)
        self.n_dev = torch.zeros(1, dtype=torch.int32, device=dev)

        def words(mm, role, *shape, shift=0):
            n = 1
            for v in shape:
                n *= v
            return rng.uniform_u64_torch(seed, configs.stream_id(cfg, mm.index, role) + shift, n, dev).view(*shape)

        self.mm = []
        for mm in cfg.matmuls:
            b = dict(mm=mm)
            # additive shares and triple shares are uniform over Z_{2^64} whatever the secrets are
            b["x"] = [words(mm, configs.R_XSPLIT, mm.m, mm.k), words(mm, configs.R_X, mm.m, mm.k)]
            wshape = (mm.n, mm.k) if (self.neuron_major and mm.kind == "somm") else (mm.k, mm.n)
            b["y"] = [words(mm, configs.R_YSPLIT, *wshape), words(mm, configs.R_Y, *wshape)]
            b["a"] = [words(mm, configs.R_ASPLIT, mm.m, mm.k), words(mm, configs.R_A, mm.m, mm.k)]
            b["b"] = [words(mm, configs.R_BSPLIT, *wshape), words(mm, configs.R_B, *wshape)]
            b["nm"] = self.neuron_major and mm.kind == "somm"
            if mm.kind == "somm":
                dshape, zshape = (mm.m, mm.k), (mm.m, self.n_act)
                gshape = (self.n_act, mm.k) if b["nm"] else (mm.k, self.n_act)
            else:
                dshape, gshape, zshape = (mm.m, self.n_act), (self.n_act, mm.n), (mm.m, mm.n)
            b["c"] = [words(mm, configs.R_CSPLIT, *zshape, shift=50 * i) for i in (0, 1)]
            b["d"] = [torch.empty(dshape, dtype=torch.int64, device=dev) for _ in (0, 1)]
            b["g"] = [torch.empty(gshape, dtype=torch.int64, device=dev) for _ in (0, 1)]
            b["e"] = torch.empty(dshape, dtype=torch.int64, device=dev)
            b["z"] = [torch.empty(zshape, dtype=torch.int64, device=dev) for _ in (0, 1)]
            if self.planes:
                b["bw"] = [ctx.open_weight_planes(b["b"][i], neuron_major=b["nm"]) for i in (0, 1)]   # offline
                b["f"] = ctx.open_weight_planes(b["g"][0], b["g"][1], neuron_major=b["nm"])   # buffer of the right size
            else:
                b["bw"] = b["b"]
                b["f"] = torch.empty(gshape, dtype=torch.int64, device=dev)
            k_eff, n_eff = (mm.k, self.n_act) if mm.kind == "somm" else (self.n_act, mm.n)
            b["macs_per_launch"] = 2 * mm.m * k_eff * n_eff
            # ring elements one party sends for this product (its masked shares of both operands)
            b["sent_elems"] = mm.m * k_eff + k_eff * n_eff
            b["sent_elems_dense"] = mm.m * mm.k + mm.k * mm.n
            self.mm.append(b)
        self.ring_ops_per_step = sum(2 * 2 * b["macs_per_launch"] for b in self.mm)   # 2 parties, 2 ops/MAC

    def _mask_and_open(self, ctx, b, idx, n_dev):
        import paper_2505_07239_amd as comet
        cfg, mm = self.cfg, b["mm"]
        for i in (0, 1):
            if mm.kind == "somm":
                ctx.mask_share(b["x"][i], b["a"][i], out=b["d"][i])
                ctx.mask_share_gather(b["y"][i], b["b"][i], comet.AXIS_ROWS if b["nm"] else comet.AXIS_COLS,
                                      cfg.bs, idx, n_dev, self.n_blk, out=b["g"][i])
            else:
                ctx.mask_share_gather(b["x"][i], b["a"][i], comet.AXIS_COLS, cfg.bs, idx, n_dev, self.n_blk,
                                      out=b["d"][i])
                ctx.mask_share_gather(b["y"][i], b["b"][i], comet.AXIS_ROWS, cfg.bs, idx, n_dev, self.n_blk,
                                      out=b["g"][i])
        ctx.open(b["d"][0], b["d"][1], out=b["e"])
        if self.unopened:
            pass                                            # F = g_0 + g_1 is formed inside the share kernel
        elif self.planes:
            ctx.open_weight_planes(b["g"][0], b["g"][1], out=b["f"].buf, neuron_major=b["nm"])
        else:
            ctx.open(b["g"][0], b["g"][1], out=b["f"])

    def _shares(self, ctx, b, idx, n_dev):
        cfg, mm = self.cfg, b["mm"]
        for i in (0, 1):
            if self.unopened:
                call = ctx.somm_share_unopened if mm.kind == "somm" else ctx.simm_share_unopened
                call(i, cfg.bs, idx, n_dev, self.n_blk, b["e"], b["g"][0], b["g"][1], b["a"][i], b["bw"][i],
                     b["c"][i], out=b["z"][i])
            elif mm.kind == "somm":
                ctx.somm_share(i, cfg.bs, idx, n_dev, self.n_blk, b["e"], b["f"], b["a"][i], b["bw"][i],
                               b["c"][i], out=b["z"][i])
            else:
                ctx.simm_share(i, cfg.bs, idx, n_dev, self.n_blk, b["e"], b["f"], b["a"][i], b["bw"][i],
                               b["c"][i], out=b["z"][i])

    def step(self):
        ctx = self.ctx
        ctx.compact_mask(self.mask, self.idx, self.n_dev)
        for b in self.mm:
            self._mask_and_open(ctx, b, self.idx, self.n_dev)
            self._shares(ctx, b, self.idx, self.n_dev)

    def step_grouped(self):
        """The same step with the share products that are ready together in one call each
        (``comet_share_group``): both parties' shares of the projections of the preceding layer
        (gate and up wait for nothing but their own openings), then both parties' shares of the
        subsequent layer."""
        ctx, cfg = self.ctx, self.cfg
        ctx.compact_mask(self.mask, self.idx, self.n_dev)
        for kind in ("somm", "simm"):
            group = [b for b in self.mm if b["mm"].kind == kind]
            if not group:
                continue
            for b in group:
                self._mask_and_open(ctx, b, self.idx, self.n_dev)
            if self.unopened:                               # (one call per product and party)
                for b in group:
                    self._shares(ctx, b, self.idx, self.n_dev)
                continue
            members = [(i, b["e"], b["f"], b["a"][i], b["bw"][i], b["c"][i]) for b in group for i in (0, 1)]
            outs = [b["z"][i] for b in group for i in (0, 1)]
            ctx.share_group(kind, cfg.bs, self.idx, self.n_dev, self.n_blk, members, out=outs)

    # ---- the same step with the bandwidth-bound kernels and the ring GEMMs on two streams ----
    def enable_overlap(self, ctx_stream_kernels):
        """Second set of the buffers a step writes (index list, masked and opened operands,
        output shares), two streams of default priority and the events that order them.  The
        masking / opening / compaction kernels of one step then run beside the GEMMs of the
        previous projection or the previous step: consecutive steps alternate between the sets."""
        import torch
        self.ctx_ew = ctx_stream_kernels
        self.s_ew, self.s_gemm = torch.cuda.Stream(), torch.cuda.Stream()
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
                    c2["e"] = torch.empty_like(b["e"])
                    c2["f"] = self.ctx.open_weight_planes(b["g"][0], b["g"][1], neuron_major=b["nm"]) if self.planes \
                        else torch.empty_like(b["f"])
                    st["mm"].append(c2)
            st["ew_done"] = [torch.cuda.Event() for _ in self.mm]
            st["gemm_done"] = torch.cuda.Event()
            st["gemm_done"].record(torch.cuda.current_stream())
            self.sets.append(st)
        self.parity = 0

    def step_overlapped(self):
        import torch
        st = self.sets[self.parity]
        self.parity ^= 1
        with torch.cuda.stream(self.s_ew):
            self.s_ew.wait_event(st["gemm_done"])          # the GEMMs that last read this set are done
            self.ctx_ew.compact_mask(self.mask, st["idx"], st["n_dev"])
            for j, b in enumerate(st["mm"]):
                self._mask_and_open(self.ctx_ew, b, st["idx"], st["n_dev"])
                st["ew_done"][j].record(self.s_ew)
        with torch.cuda.stream(self.s_gemm):
            for j, b in enumerate(st["mm"]):
                self.s_gemm.wait_event(st["ew_done"][j])
                self._shares(self.ctx, b, st["idx"], st["n_dev"])
            st["gemm_done"].record(self.s_gemm)


def run_timed(ctx, layer, steps, warmup, run_step=None):
    """W untimed steps, then exactly K timed ones between two synchronisations; the share kernel
    alone is timed with HIP events inside the library.  Returns a dict: ms per step, summed time
    and number of the share launches that were timed, share launches per step."""
    import torch
    import paper_2505_07239_amd as comet
    run_step = run_step or layer.step_grouped
    # share launches per step (the library decides which products of a grouped call share a
    # launch): counted on the last warm-up step
    per_step = 0
    for w in range(max(warmup, 1)):
        last = w == max(warmup, 1) - 1
        if last:
            ctx.set_tuning(comet.TUNE_TIMING_STRIDE, 1)
            ctx.timing_begin(4 * len(layer.mm))
        run_step()
        if last:
            torch.cuda.synchronize()
            _, per_step = ctx.timing_end()
    torch.cuda.synchronize()
    # A timed launch idles the stream for about ten microseconds around the kernel, so only every
    # n-th share launch of the timed region carries an event pair, n coprime to the launches per
    # step: every projection and party is sampled equally often.
    stride = 5 if per_step % 5 else 7
    if per_step * steps < 4 * stride:
        stride = 1
    ctx.set_tuning(comet.TUNE_TIMING_STRIDE, stride)
    ctx.timing_begin(per_step * steps)
    t0 = time.perf_counter()
    for _ in range(steps):
        run_step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    gemm_ms, n_timed = ctx.timing_end()
    ctx.set_tuning(comet.TUNE_TIMING_STRIDE, 0)
    return {"ms_per_step": (t1 - t0) * 1e3 / steps, "gemm_ms": gemm_ms, "n_timed": n_timed,
            "launches_per_step": per_step, "timing_stride": stride}


def roofline_of(layer, wname, timing, skinny_forced, probes):
    """The roofline object of the dominant kernel of a workload."""
    cfg = layer.cfg
    fmt = "planes" if layer.planes else "words"
    ms_per_step, gemm_ms, n_timed = timing["ms_per_step"], timing["gemm_ms"], timing["n_timed"]
    per_step = max(timing["launches_per_step"], 1)
    grouped = per_step < 2 * len(layer.mm)
    traffic, source = GEMM_TRAFFIC.get((wname, fmt, "grouped" if grouped else "single"), (None, None))
    # both parties' shares of every projection, over the share launches of a step (a grouped
    # launch computes several of them)
    macs_per_launch = 2 * sum(b["macs_per_launch"] for b in layer.mm) / per_step
    avg_ms = gemm_ms / max(n_timed, 1)
    share = avg_ms * per_step / ms_per_step
    common = {"traffic": traffic, "traffic_source": source, "avg_launch_ms": avg_ms, "launches_timed": n_timed,
              "launches_per_step": per_step, "timing_stride": timing["timing_stride"],
              "ring_macs_per_launch": macs_per_launch, "gemm_share_of_step": share, "weight_operands": fmt}
    if cfg.tokens <= 8 and not skinny_forced:
        # a few activation rows: the share calls take the vector-ALU kernel, bound by reading the
        # weight-side operands once per launch: B_i and F (kc x n words each), or B_i and the two
        # masked shares F is the sum of when the opening is folded into the kernel
        wbytes = macs_per_launch / cfg.tokens * 8.0 * (1.5 if layer.unopened else 1.0)
        ach = wbytes / (avg_ms * 1e-3) / 1e9
        r = {"bound": "hbm", "kernel": "ring_skinny_kernel", "achieved": ach, "peak": PEAK_HBM_GBS,
             "unit": "GB/s", "frac": ach / PEAK_HBM_GBS,
             "note": "algorithmic bytes: the weight-side operands of one launch, 8 bytes per word, read once: "
                     + ("B_i and the two masked shares [G]_0, [G]_1 whose sum F is (the opening is folded "
                        "into the share kernel)" if layer.unopened else "B_i and F")}
        if probes:
            r["frac_of_measured_copy"] = ach / probes["copy_GBs"]
    else:
        ach = INT8_OPS_PER_RING_MAC * macs_per_launch / (avg_ms * 1e-3) / 1e12
        r = {"bound": "mfma", "kernel": "ring_gemm_group_kernel" if grouped else "ring_gemm_kernel",
             "achieved": ach, "peak": PEAK_INT8_TOPS,
             "unit": "TOP/s", "frac": ach / PEAK_INT8_TOPS,
             "note": "algorithmic int8 ops: 36 digit products x 2 ops per ring MAC, two products per "
                     "party (2*m*k*n_act ring MACs per share product; a grouped launch computes "
                     "several products)"}
        if probes:
            r["frac_of_measured_mfma_issue"] = ach / probes["mfma_i8_issue_TOPs"]
            r["frac_of_measured_mfma_issue_random_operands"] = ach / probes["mfma_i8_issue_random_operands_TOPs"]
    r.update(common)
    return r


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
        # the opened operands as words: E as the GPU wrote it, F from the two masked shares
        # (the GPU path may hold F only as digit planes)
        e, f = host(b["e"]), co.open_(host(b["g"][0]), host(b["g"][1]))
        if b["nm"]:
            f = np.ascontiguousarray(f.T)                 # stored one row per neuron
        k_eff, n_eff = e.shape[1], f.shape[1]
        a_sel, b_sel = [], []
        for i in (0, 1):
            a_i, b_i = host(b["a"][i]), host(b["b"][i])
            if b["nm"]:
                b_i = np.ascontiguousarray(b_i.T)
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


def graph_replay_ms(layer, steps):
    """One step captured in a HIP graph (every call only enqueues kernels) and replayed: the time
    per step without the host-side launch cost of its thirty-odd kernels."""
    import torch
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):               # warm-up outside the capture (workspace allocation)
        layer.step_grouped()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        layer.step_grouped()
    graph.replay()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        graph.replay()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) * 1e3 / steps


def config_entry(ctx, name, probes, planes, skinny_forced, steps=10, warmup=3, layer=None, timing=None,
                 check=None):
    """One configuration: short timed run, roofline, exchanged bytes, oracle check of a row block."""
    import torch
    from workloads import rng
    cfg, wname = parse_workload(name)
    own = layer is None
    if own:
        layer = Layer(ctx, cfg, rng.BASE_SEED, planes, UNOPENED_FEW_ROWS, NEURON_MAJOR_SOMM)
        timing = run_timed(ctx, layer, steps, warmup)
    ms, gemm_ms, n_timed = timing["ms_per_step"], timing["gemm_ms"], timing["n_timed"]
    roof = roofline_of(layer, wname, timing, skinny_forced, probes)
    if cfg.cid == 1:
        # a few microseconds of arithmetic per launch: launch latency decides, no roofline applies
        roof = {"bound": "latency", "kernel": roof["kernel"], "achieved": None, "peak": None, "unit": None,
                "frac": None, "avg_launch_ms": roof["avg_launch_ms"], "weight_operands": roof["weight_operands"],
                "ring_macs_per_launch": roof["ring_macs_per_launch"], "launches_per_step": roof["launches_per_step"]}
    if check is None:
        check = cpu_baseline(layer, budget_s=1.0)
    sent = sum(b["sent_elems"] for b in layer.mm)
    dense = sum(b["sent_elems_dense"] for b in layer.mm)
    entry = {
        "workload": "%s, %d tokens, d_model %d, d_ff %d, block %d, %d of %d blocks kept; %s" %
                    (cfg.name, cfg.tokens, cfg.d_model, cfg.d_ff, cfg.bs, layer.n_blk, cfg.nb,
                     "+".join(m.name for m in cfg.matmuls)),
        "ms_per_step": ms, "steps": steps if own else None,
        "gops_per_party": layer.ring_ops_per_step / (ms * 1e-3) / 1e9,
        "share_kernel_us": gemm_ms / max(n_timed, 1) * 1e3,
        "ring_macs_per_launch": roof["ring_macs_per_launch"],
        "launches_per_step": roof["launches_per_step"],
        "roofline": {k: roof.get(k) for k in ("bound", "kernel", "achieved", "peak", "unit", "frac", "traffic")},
        "frac_of_measured_mfma_issue": roof.get("frac_of_measured_mfma_issue"),
        "frac_of_measured_copy": roof.get("frac_of_measured_copy"),
        "weight_operands": roof["weight_operands"],
        # cost model of the optimality appendix: every party sends its masked shares of both
        # operands of every product once, 8 bytes per ring element, two directions
        "exchanged_bytes_both_directions": 8 * sent * 2,
        "exchanged_bytes_dense_layer": 8 * dense * 2,
        "exchange_reduction": dense / sent,
        "oracle_check": check["sample"],
        "matches_gpu": check["matches_gpu"],
        # the CPU oracle on the sampled rows, same run, same box (a reported baseline, not a target)
        "cpu_oracle_gops": check["value"], "cpu_oracle_cores": check["cores"],
        "cpu_oracle_gops_1core": check.get("value_1core"),
        # what the paper reports for the corresponding layer (its own platform: two servers with
        # A100 + Xeon 8458P, 5 Gbps links, CrypTen; whole-inference sums) -- context only
        "paper_context": PAPER_CONTEXT.get(cfg.cid),
    }
    if cfg.cid <= 2:
        # launch-bound configurations: the same step replayed from a HIP graph
        try:
            entry["ms_per_step_graph_replay"] = graph_replay_ms(layer, 4 * steps)
        except Exception as exc:          # an extra figure: never at the cost of the whole line
            log("graph replay of %s failed: %s" % (name, exc))
            entry["ms_per_step_graph_replay"] = None
    if own:
        del layer
        torch.cuda.empty_cache()
    return entry


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
    words = lambda st, *shape: rng.uniform_u64_torch(rng.BASE_SEED, 9000 + st, int(np.prod(shape)), dev).view(*shape)
    n_act = n_blk * bs
    e, a, f, b, c = words(1, m, k), words(2, m, k), words(3, k, n_act), words(4, k, nb * bs), words(5, m, n_act)
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
    e2, a2, f2, b2, c2 = words(6, m, kc), words(7, m, nb * bs), words(8, kc, k), words(9, nb * bs, k), words(10, m, k)
    z2 = torch.empty_like(c2)
    t_rows = timed(lambda: ctx.simm_share_masked(1, bs, idx, n_dev, n_blk, tm, e2, f2, a2, b2, c2, out=z2),
                   reps=10)
    t_plain = timed(lambda: ctx.simm_share(1, bs, idx, n_dev, n_blk, e2, f2, a2, b2, c2, out=z2), reps=10)
    out["simm_row_sets_us"] = t_rows * 1e6
    out["simm_union_of_masks_us"] = t_plain * 1e6
    # component search on an element-granular mask at FFN width (bs = 1): 512 tokens of six
    # unrelated requests by 13824 neurons, beyond the one-workgroup limits
    em = torch.from_numpy(masks.grouped_token_masks(rng.BASE_SEED, 9050, 512, 13824, 6, 0.02)).to(dev)
    out["components_512x13824_us"] = timed(lambda: ctx.components(em), reps=20) * 1e6
    ctx.set_tuning(5, 1)          # the same multi-workgroup search on the small block-granular mask
    out["components_multi_workgroup_us"] = timed(lambda: ctx.components(tm), reps=20) * 1e6
    ctx.set_tuning(5, 0)
    return out


def mha_layers(ctx, timed):
    """The MHA-shaped workload (LLaMA-2-7B attention, block = one head of 128): sparse QKV layer
    with merged cache-refill rows (Protocol 2 on the result blocks of the head-granular mask, 8
    current tokens + 56 refill rows) and sparse output layer (Protocol 3 with per-token head
    sets), against the same calls on the union of all masks."""
    import numpy as np
    import torch
    from workloads import configs, rng
    cfg = configs.mha_config()
    qkv_mask, out_mask = configs.mha_head_masks(cfg)
    d, h, bs = cfg.d_model, cfg.n_heads, cfg.head_dim
    dev = torch.device("cuda:0")
    words = lambda st, *shape: rng.uniform_u64_torch(rng.BASE_SEED, 9600 + st, int(np.prod(shape)), dev).view(*shape)
    tm = torch.from_numpy(qkv_mask).to(dev)
    comp = ctx.components(tm)
    torch.cuda.synchronize()
    n_row, n_blk, n_comp = (int(comp[q].item()) for q in ("n_row", "n_blk", "n_comp"))
    n_act = n_blk * bs
    out = {"mha_qkv_rows": n_row, "mha_qkv_head_blocks": n_blk, "mha_qkv_components": n_comp}
    e, a, f = words(1, n_row, d), words(2, n_row, d), words(3, d, n_act)
    b, c = words(4, d, 3 * h * bs), words(5, n_row, n_act)
    z = torch.empty_like(c)
    out["mha_components_us"] = timed(lambda: ctx.components(tm), reps=20) * 1e6
    out["mha_qkv_result_blocks_us"] = timed(
        lambda: ctx.somm_share_blocks(1, bs, comp["blk_idx"], comp["blk_comp"], comp["n_blk"], n_blk, comp["row_comp"],
                                      comp["n_row"], e, f, a, b, c, out=z), reps=10) * 1e6
    out["mha_qkv_union_of_masks_us"] = timed(
        lambda: ctx.somm_share(1, bs, comp["blk_idx"], comp["n_blk"], n_blk, e, f, a, b, c, out=z), reps=10) * 1e6
    om = torch.from_numpy(out_mask).to(dev)
    idx, n_dev = ctx.compact_mask(om)
    torch.cuda.synchronize()
    t = int(n_dev.item())
    m, kc = cfg.tokens, t * bs
    e2, a2, f2 = words(6, m, kc), words(7, m, h * bs), words(8, kc, d)
    b2, c2 = words(9, h * bs, d), words(10, m, d)
    z2 = torch.empty_like(c2)
    out["mha_output_heads_in_union"] = t
    out["mha_output_head_sets_us"] = timed(
        lambda: ctx.simm_share_masked(1, bs, idx, n_dev, t, om, e2, f2, a2, b2, c2, out=z2), reps=10) * 1e6
    out["mha_output_union_of_masks_us"] = timed(
        lambda: ctx.simm_share(1, bs, idx, n_dev, t, e2, f2, a2, b2, c2, out=z2), reps=10) * 1e6
    return out


def weight_side_masking(ctx, timed_rotating):
    """Indexed masking of the weight side of the LLaMA-7B gate projection (4096 x 11008 words,
    52 of 344 blocks of 32): row-major weights (kept neurons are 256-byte segments of every row)
    and neuron-major weights (a kept neuron is one contiguous row), each repeated on ONE pair of
    input buffers (the kept part, 109 MB, then stays in the last-level cache) and on FOUR pairs
    in rotation (2.9 GB: every call reads from HBM, which is what a layer step sees)."""
    import numpy as np
    import torch
    import paper_2505_07239_amd as comet
    from workloads import masks, rng
    k, nb, bs = 4096, 344, 32
    dev = torch.device("cuda:0")
    mask = masks.clustered_block_mask(rng.BASE_SEED, 9100, nb, 0.15, 4.0)[None, :]
    idx, n_dev = ctx.compact_mask(torch.from_numpy(mask).to(dev))
    t_blk = int(n_dev.item())
    n_act = t_blk * bs
    sets = [(rng.uniform_u64_torch(rng.BASE_SEED, 9100 + 2 * q, k * nb * bs, dev),
             rng.uniform_u64_torch(rng.BASE_SEED, 9101 + 2 * q, k * nb * bs, dev)) for q in range(4)]
    out = {}
    for name, tr in (("row_major", False), ("neuron_major", True)):
        shape = (nb * bs, k) if tr else (k, nb * bs)
        g = torch.empty((n_act, k) if tr else (k, n_act), dtype=torch.int64, device=dev)
        axis = comet.AXIS_ROWS if tr else comet.AXIS_COLS
        call = lambda q: ctx.mask_share_gather(sets[q][0].view(*shape), sets[q][1].view(*shape), axis, bs, idx,
                                               n_dev, t_blk, out=g)
        out["somm_weights_%s_mask_GBs" % name] = 24.0 * k * n_act / timed_rotating(call, 1) / 1e9
        out["somm_weights_%s_mask_from_hbm_GBs" % name] = 24.0 * k * n_act / timed_rotating(call, 4) / 1e9
    # the opening of the masked weights written as digit planes, next to the plain opening
    g0, g1 = sets[0][0][:k * n_act].view(k, n_act), sets[1][0][:k * n_act].view(k, n_act)
    o = torch.empty_like(g0)
    out["open_GBs_gate_weights"] = 24.0 * k * n_act / timed_rotating(lambda q: ctx.open(g0, g1, out=o), 1) / 1e9
    pl = ctx.open_weight_planes(g0, g1)
    out["open_weight_planes_GBs_gate_weights"] = \
        24.0 * k * n_act / timed_rotating(lambda q: ctx.open_weight_planes(g0, g1, out=pl.buf), 1) / 1e9
    return out


def decoding_batches(ctx, timed_rotating):
    """The gate projection of the decoding workload (LLaMA-2-13B, 179 of 216 blocks of 64 kept)
    for batches of 2, 8, 16 and 32 tokens: weight words (vector-ALU kernel up to 8 rows, matrix-core
    tile kernel beyond) and weight planes (the kernel in which every wavefront streams its own
    fragments).  Three weight sets in rotation, so every call reads from HBM; the rate counts
    B_i and F once per call."""
    import numpy as np
    import torch
    from workloads import rng
    k, nb, bs, t = 5120, 216, 64, 179
    dev = torch.device("cuda:0")
    na = t * bs
    words = lambda st, *shape: rng.uniform_u64_torch(rng.BASE_SEED, 9700 + st, int(np.prod(shape)), dev).view(*shape)
    idx = torch.arange(t, dtype=torch.int32, device=dev)
    n_dev = torch.tensor([t], dtype=torch.int32, device=dev)
    sets = []
    for q in range(3):
        f, b = words(10 * q + 1, k, na), words(10 * q + 2, k, nb * bs)
        sets.append((f, b, ctx.open_weight_planes(f), ctx.open_weight_planes(b)))
    out = {}
    for m in (2, 8, 16, 32):
        e, a, c = words(91, m, k), words(92, m, k), words(93, m, na)
        z = torch.empty_like(c)
        for name, off in (("words", 0), ("planes", 2)):
            call = lambda q: ctx.somm_share(1, bs, idx, n_dev, t, e, sets[q][off], a, sets[q][off + 1], c, out=z)
            out["decode_gate_m%d_%s_GBs" % (m, name)] = 16.0 * k * na / timed_rotating(call, 3, reps=12) / 1e9
    return out


def glue_steps(ctx, timed):
    """Shuffle steps, merge to full width and rescaling on a 4096 x 11008 matrix of words (the
    activations of 4096 tokens at the FFN width): achieved GB/s of algorithmic bytes."""
    import torch
    import paper_2505_07239_amd as comet
    from workloads import rng
    rows, cols, bs = 4096, 11008, 32
    dev = torch.device("cuda:0")
    words = lambda st, *shape: rng.uniform_u64_torch(rng.BASE_SEED, 9200 + st, shape[0] * shape[1], dev).view(*shape)
    x, mk, o = words(1, rows, cols), words(2, rows, cols), torch.empty((rows, cols), dtype=torch.int64, device=dev)
    gen = torch.Generator(device=dev)
    gen.manual_seed(78)
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
    c = words(3, rows, keep * bs)
    t = timed(lambda: ctx.scatter_cols(c, bs, idx, nd, keep, cols, out=o), reps=10)
    out["scatter_GBs"] = (8.0 * n + 16.0 * rows * keep * bs) / t / 1e9   # zero fill + kept blocks read and written
    return out


def micro(ctx, layer):
    """Per-kernel yardsticks on the same device (stderr + returned dict)."""
    import torch
    from workloads import masks, rng
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

    def timed_rotating(call, n_sets, reps=24):
        for q in range(n_sets):
            call(q)
        torch.cuda.synchronize()
        s, e = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        s.record()
        for r in range(reps):
            call(r % n_sets)
        e.record()
        torch.cuda.synchronize()
        return s.elapsed_time(e) / reps * 1e-3

    n = 11008 * 4096                                  # weight side of the dense down projection
    a = rng.uniform_u64_torch(rng.BASE_SEED, 9301, n, "cuda")
    b = rng.uniform_u64_torch(rng.BASE_SEED, 9302, n, "cuda")
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
    # the same number of flags as a batch of per-token masks (65536 tokens x 4096 blocks, tokens
    # agree on most of their blocks): the OR over the tokens is a read-only stream
    tall = (masks.stress_mask_device(8, flags, torch.device("cuda:0"), 0.5).view(65536, 4096)
            & masks.stress_mask_device(9, 4096, torch.device("cuda:0"), 0.3).view(1, 4096)).contiguous()
    idx = torch.empty(4096, dtype=torch.int32, device="cuda")
    t = timed(lambda: ctx.compact_mask(tall, idx, nd), reps=10)
    out["compact_token_masks_65536x4096_GBs"] = (flags + 4.0 * int(nd.item())) / t / 1e9
    # per-token masks of one batch at FFN width (LLaMA-7B: 344 blocks of 32; 512 tokens)
    t = timed(lambda: ctx.compact_mask(tall.view(-1)[:512 * 344].view(512, 344), idx, nd), reps=50)
    out["compact_token_masks_512x344_us"] = t * 1e6
    del tall, idx
    t = timed(lambda: ctx.compact_mask(layer.mask, layer.idx, layer.n_dev), reps=50)
    out["compact_layer_mask_us"] = t * 1e6
    out.update(general_forms(ctx, timed))
    out.update(mha_layers(ctx, timed))
    out.update(glue_steps(ctx, timed))
    out.update(weight_side_masking(ctx, timed_rotating))
    out.update(decoding_batches(ctx, timed_rotating))
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
                    help="headline workload: c1..c4, c5_d100 / c5_d050 / c5_d025 / c5_d010 / c5_d005")
    ap.add_argument("--configs", default="all",
                    help="configurations measured besides the headline: all, none, or a comma list")
    ap.add_argument("--weights", default="planes", choices=["planes", "words"],
                    help="format of the weight-side operands of the share calls")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-micro", action="store_true")
    ap.add_argument("--row-major-weights", action="store_true",
                    help="store the SOMM weights k x n (kept neurons are column blocks) instead of one row per neuron")
    ap.add_argument("--opened-few-rows", action="store_true",
                    help="decoding workloads: open F into memory first instead of folding the opening into the share kernel")
    ap.add_argument("--per-call", action="store_true",
                    help="one share call per product and party instead of the grouped calls")
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
    global UNOPENED_FEW_ROWS, NEURON_MAJOR_SOMM
    UNOPENED_FEW_ROWS = not args.opened_few_rows
    NEURON_MAJOR_SOMM = not args.row_major_weights
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
    planes = args.weights == "planes"
    layer = Layer(ctx, cfg, rng.BASE_SEED, planes, UNOPENED_FEW_ROWS, NEURON_MAJOR_SOMM)
    log("workload %s: %s, m=%d d=%d f=%d bs=%d kept blocks %d/%d (n_act=%d), %.2f G ring ops/step, weight "
        "operands as %s" % (wname, cfg.name, cfg.tokens, cfg.d_model, cfg.d_ff, cfg.bs, layer.n_blk, cfg.nb,
                            layer.n_act, layer.ring_ops_per_step / 1e9, "planes" if layer.planes else "words"))

    run_step = layer.step if args.per_call else layer.step_grouped
    if args.overlap:
        ctx_ew = comet.Context(0)
        layer.enable_overlap(ctx_ew)
        run_step = layer.step_overlapped
    if args.graph:
        # One step captured in a HIP graph (every call only enqueues kernels) and replayed: the
        # launch gaps between the thirty-odd kernels of a step go away.  The share kernel is timed
        # with HIP events in an eager pass first, since events do not work inside a replay.
        timing = run_timed(ctx, layer, args.steps, args.warmup, layer.step)
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            layer.step()
        graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            graph.replay()
        torch.cuda.synchronize()
        timing["ms_per_step"] = (time.perf_counter() - t0) * 1e3 / args.steps
    else:
        timing = run_timed(ctx, layer, args.steps, args.warmup, run_step)
    ms_per_step = timing["ms_per_step"]
    t2 = None
    if run_step == layer.step_grouped and not args.graph:
        # the same K steps with one share call per product and party, for comparison
        t2 = run_timed(ctx, layer, args.steps, 2, layer.step)
        run_step()                      # leave the grouped calls' outputs in place for the oracle check
        torch.cuda.synchronize()

    value = layer.ring_ops_per_step / (ms_per_step * 1e-3) / 1e9
    kernels = None
    if not args.no_micro:
        kernels = micro(ctx, layer)
        for k, v in kernels.items():
            log("%s = %.4g" % (k, v))
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
                   "share_products_per_step": 2 * len(layer.mm),
                   "share_launches_per_step": timing["launches_per_step"],
                   "share_calls": "one call per product and party" if (args.per_call or args.graph or args.overlap)
                                  else "comet_share_group: gate+up of both parties, then down of both parties",
                   "weight_operands": "digit planes (F opened in that format, B_i packed offline)"
                                      if layer.planes else "words",
                   "weight_layout": "one row per neuron in both projections (kept neurons are whole rows)"
                                    if layer.neuron_major else
                                    "gate / up: d_model x d_ff (kept neurons are column blocks); down: d_ff x d_model",
                   "few_row_shares": "opening of F folded into the share kernel" if layer.unopened else None,
                   "inputs": "seeded streams of workloads/ (seed %d), drawn on the device" % rng.BASE_SEED,
                   "submission": "hip graph replay" if args.graph else
                                 ("eager, two streams" if args.overlap else "eager")},
        "roofline": roofline_of(layer, wname, timing, bool(args.skinny), kernels),
    }
    if t2 is not None:
        r2 = roofline_of(layer, wname, t2, bool(args.skinny), kernels)
        result["per_call"] = {"ms_per_step": t2["ms_per_step"], "value": layer.ring_ops_per_step / (t2["ms_per_step"] * 1e-3) / 1e9,
                              "share_launches_per_step": t2["launches_per_step"], "avg_launch_ms": r2["avg_launch_ms"],
                              "frac": r2["frac"], "frac_of_measured_mfma_issue": r2.get("frac_of_measured_mfma_issue")}
    if kernels is not None:
        result["kernels"] = kernels
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(layer)
        log("cpu oracle: %.2f Gop/s on %d threads; rows match GPU: %s" %
            (result["cpu_baseline"]["value"], result["cpu_baseline"]["cores"],
             result["cpu_baseline"]["matches_gpu"]))
    names = [] if args.configs == "none" else (ALL_CONFIGS if args.configs == "all" else args.configs.split(","))
    if names and not args.overlap and not args.graph:
        result["configs"] = {}
        for name in names:
            _, canon = parse_workload(name)
            if canon == wname:
                entry = config_entry(ctx, name, kernels, planes, bool(args.skinny), layer=layer,
                                     timing=timing, check=result.get("cpu_baseline"))
                entry["steps"] = args.steps
            else:
                entry = config_entry(ctx, name, kernels, planes, bool(args.skinny))
            result["configs"][canon] = entry
            log("%s: %.3f ms/step, %.0f Gop/s per party, share kernel %.1f us, %s frac %s, oracle rows match: %s" %
                (canon, entry["ms_per_step"], entry["gops_per_party"], entry["share_kernel_us"],
                 entry["roofline"]["bound"],
                 "%.3f" % entry["roofline"]["frac"] if entry["roofline"]["frac"] is not None else "n/a",
                 entry["matches_gpu"]))
    bad = (not args.no_cpu_baseline and not result["cpu_baseline"]["matches_gpu"]) or \
        any(not e["matches_gpu"] for e in result.get("configs", {}).values())
    print(json.dumps(result))
    if bad:
        log("ERROR: GPU result differs from the oracle on the sampled rows")
        sys.exit(3)


if __name__ == "__main__":
    main()
