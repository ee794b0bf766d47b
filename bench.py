#!/usr/bin/env python3
"""Benchmark of the sparse convolution (+ fused pooling) path on one MI355X.

Default run: the VGG-19-shaped layer set at batch 8 (three layers: 256->256 @56x56 and
512->512 @28x28 through sconv_forward with ReLU, 512->512 @14x14 through sconv_pool_forward
with 2x2/2 max pooling).  One step = one pass over all three layers.  Inputs are synthetic,
seeded, and resident in device memory before the timed region; consecutive steps rotate through
several copies of every buffer so that a step does not find its operands in the last-level cache.

Prints ONE JSON line: whole-step dense-equivalent GFLOP/s (the flops a dense convolution of the
same shapes would need, divided by the time), per-layer figures, the roofline position of the
dominant kernel (timed live with events on the launch stream), and the CPU oracle timed on a
bounded sample of the same workload.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--config vgg19] [--batch 8]
  python bench.py --table [--only single]   # every layer of every (or one) config at both batch sizes -> JSON lines
  python bench.py --sweep          # zero-ratio sweep 0.00..0.95 on the RegNetX 896-channel layer
  python bench.py --layer vgg19:0 --batch 8   # one layer alone (profiling)
  python bench.py --shape 32,64,28,28,128,5,5,1,2,1 --zero-ratio 0.7   # any shape alone
  python bench.py --split          # conversion alone vs. the whole kernel; fused vs. unfused pooling
  python bench.py --graph --config resnet50   # a batch-1 step eagerly and as a HIP graph replay
  python bench.py --axis batch | stride       # batch-size / stride sensitivity on one layer shape
  python bench.py --chain [--batch 8]         # VGG-shaped tail, each layer fed by the previous one's output
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import workloads  # noqa: E402

HBM_PEAK_GBS = 8000.0        # MI355X HBM3E, published
FP32_VECTOR_PEAK_TF = 157.3  # 256 CUs x 4 SIMDs x 16 lanes x 2 (packed) x 2 flop x 2.4 GHz
FP32_MFMA_PEAK_TF = 157.3    # dense fp32 matrix instructions, published
MFMA_VARIANTS = ("quad3x3", "quad1x1", "wide3x3", "gen")
# HBM/fabric bytes per launch from rocprofv3 counter runs (FETCH_SIZE x 2 KiB + WRITE_SIZE x 1 KiB, scaled
# by the copy calibration), keyed by (plan name, layer, batch): a figure from profiles/, not something this
# run measures - the line names its source, and prints null when the plan that ran is not in the table.
MEASURED_TRAFFIC = {
    ("quad3x3/q32t7d/8x4", "vgg-256x56", 8): (54.8e6 + 25.9e6, "profiles/quad3x3_vgg-256x56_n8.txt"),
}
# elements per zero test of the kernels that skip whole groups (1: every zero element is skipped)
SKIP_GRANULE = {"rows": 1, "tap3x3": 1, "quad3x3": 6, "quad1x1": 32, "wide3x3": 16, "gen": 16}
FP32_UNPACKED_PEAK_TF = 78.6  # same without packed fp32 instructions (this build keeps them off)
TUNE = True                   # --no-tune: the static dispatch rules and cost models only
HINT = False                  # --hint: no tuning; the density probe's zero ratio is given to the static rules
PREP = False                  # --prepared: every layer's calls bring the filters in the prepared layout
                              # (sconv_filter_prep, written once at set-up as an inference engine would)
CACHE_BYTES = 512 << 20       # rotate buffers until their total passes twice the 256 MiB last-level cache


def sum_count(x: np.ndarray, layer: workloads.Layer) -> int:
    """Total number of stored nonzeros over all window rows (bookkeeping for the flop count):
    every nonzero element counts once per window that contains it."""
    def cover(n_in, k, out, stride, pad):
        c = np.zeros(n_in, np.int64)
        for o in range(out):
            lo = o * stride - pad
            c[max(lo, 0):min(lo + k, n_in)] += 1
        return c
    ch = cover(layer.H, layer.R, layer.OH, layer.stride, layer.pad)
    cw = cover(layer.W, layer.S, layer.OW, layer.stride, layer.pad)
    nz = (x != 0)
    per_h = nz.sum(axis=(0, 1)).astype(np.int64)          # [H, W]
    return int((per_h * np.outer(ch, cw)).sum())


def layer_work(layer: workloads.Layer, N: int, x: np.ndarray) -> dict:
    OH, OW = layer.OH, layer.OW
    if layer.pool:
        ph, pw, ps = layer.pool
        out_elems = N * layer.K * ((OH - ph) // ps + 1) * ((OW - pw) // ps + 1)
    else:
        out_elems = N * layer.K * OH * OW
    dense_flops = 2.0 * N * layer.K * OH * OW * layer.Cg * layer.R * layer.S
    nz_flops = 2.0 * layer.Kg * sum_count(x, layer)
    alg_bytes = 4.0 * (x.size + layer.K * layer.Cg * layer.R * layer.S + out_elems)
    return {"dense_flops": dense_flops, "nz_flops": nz_flops, "alg_bytes": alg_bytes,
            "zero_ratio": float((x == 0).mean())}


def sampled_check(layer, x, w, got, seed: int, npts: int = 4000) -> dict:
    """Compares outputs of one layer (a host copy `got` of what the GPU wrote) with the CPU oracle at
    sampled points: `npts` random ones plus a grid of tile and filter-block boundaries (first and last
    image; filters 0, 63, 64, last; rows and columns around multiples of the kernels' tile sizes and the
    map's edges).  Pooled layers compare with the window maximum of the oracle's ReLU'd convolution.
    Bar: |got - ref| <= 1e-4 * sum|x*w| per element.  Returns counts and the worst ratio."""
    import oracle
    rng = np.random.default_rng(seed)
    N, K, OHp, OWp = got.shape
    pts = [np.stack([rng.integers(0, d, size=npts) for d in got.shape], axis=1)]
    edge = lambda n: sorted({v for v in (0, 1, 3, 4, 5, 6, 7, 13, 14, 15, 27, 28, 29, n - 2, n - 1) if 0 <= v < n})
    ns = sorted({0, N - 1})
    ks = sorted({v for v in (0, 63, 64, 127, 128, K - 1) if v < K})
    grid = np.array([(n, k, a, b) for n in ns for k in ks for a in edge(OHp) for b in edge(OWp)], dtype=np.int64)
    pts.append(grid)
    pts = np.concatenate(pts, axis=0)
    if layer.pool:
        ph, pw, ps = layer.pool
        ref = np.zeros(len(pts))
        scale = np.zeros(len(pts))
        for py in range(ph):
            for px in range(pw):
                q = pts.copy()
                q[:, 2] = pts[:, 2] * ps + py
                q[:, 3] = pts[:, 3] * ps + px
                v, a = oracle.conv_at(x, w, q, layer.stride, layer.pad, layer.groups, relu=True)
                ref = np.maximum(ref, v)
                scale = np.maximum(scale, a)
    else:
        ref, scale = oracle.conv_at(x, w, pts, layer.stride, layer.pad, layer.groups, relu=True)
    err = np.abs(got[tuple(pts.T)].astype(np.float64) - ref)
    ratio = err / np.maximum(scale, 1e-300)
    ratio[(err == 0)] = 0.0
    return {"checked": int(len(pts)), "failed": int((err > 1e-4 * scale).sum()), "worst_ratio": float(ratio.max())}


def whole_check(layer, x, w, got) -> dict:
    """Every output of one layer against the CPU oracle (fp64 on all host cores; seconds for the
    benchmark layers).  Same bar and record as sampled_check."""
    import oracle
    if layer.pool:
        ref, scale = oracle.conv_pool(x, w, layer.pool, layer.stride, layer.pad, layer.groups)
    else:
        ref, scale = oracle.conv(x, w, layer.stride, layer.pad, layer.groups, relu=True)
    err = np.abs(got.astype(np.float64) - ref)
    ratio = np.where(err == 0, 0.0, err / np.maximum(scale, 1e-300))
    return {"checked": int(err.size), "failed": int((err > 1e-4 * scale).sum()), "worst_ratio": float(ratio.max())}


_flush = None


def flush_buffer():
    """Scratch lent to sconv_tune: overwritten before each of its timed launches, so that it ranks
    plans the way the timed region runs them - operands not in the caches."""
    global _flush
    if _flush is None:
        import torch
        _flush = torch.empty(CACHE_BYTES, dtype=torch.uint8, device="cuda")
    return _flush


_workspaces = {}


def lend_workspace() -> None:
    """The optional workspace of the library (sconv_set_workspace), lent once per stream: 64 MiB, the
    most sconv_workspace_size ever asks for.  With it small launches are split across workgroups."""
    import torch
    import paper_1909_09927_amd as sconv
    key = torch.cuda.current_stream().cuda_stream
    if key not in _workspaces:
        _workspaces[key] = torch.empty(64 << 20, dtype=torch.uint8, device="cuda")
        sconv.sconv_set_workspace(_workspaces[key])


class DeviceLayer:
    """One layer's operands on the device, in `copies` rotating sets."""

    def __init__(self, layer, N, x, w, copies, prepared=None):
        import torch
        import paper_1909_09927_amd as sconv
        self.layer, self.N = layer, N
        self.sconv = sconv
        lend_workspace()
        self.prepared = PREP if prepared is None else prepared
        self.workspace = _workspaces[torch.cuda.current_stream().cuda_stream]
        xd = torch.from_numpy(x).cuda()
        wd = torch.from_numpy(w).cuda()
        self.sets = []
        self.preps = []        # per buffer set: the prepared copy of that set's filters (None: no such layout)
        for i in range(copies):
            xs = xd if i == 0 else xd.clone()
            ws = wd if i == 0 else wd.clone()
            if layer.pool:
                y = sconv.sconv_pool_forward(xs, ws, layer.pool, layer.stride, layer.pad, layer.groups)
            else:
                y = sconv.sconv_forward(xs, ws, layer.stride, layer.pad, layer.groups, relu=True)
            self.sets.append((xs, ws, y))
            self.preps.append(sconv.sconv_filter_prep(ws, layer.groups, layer.stride, layer.pad)
                              if self.prepared else None)
        if self.preps[0] is None:
            self.prepared = False
        self.host = (x, w)
        self.tune_wall_s = 0.0
        self.z = None
        if HINT:
            # set-up: one probe of the input (two small kernels, up to 4 Mi elements); every call of this
            # layer then carries the zero ratio in its descriptor
            t0 = time.perf_counter()
            self.z = sconv.zero_ratio_of(sconv.sconv_density(xd))
            self.tune_wall_s = time.perf_counter() - t0
        d = sconv.desc_for(xd, wd, layer.stride, layer.pad, layer.groups, layer.pool, True, self.z, self.prepared)
        if TUNE:
            # set-up, outside every timed region: the library times its variants and decompositions on
            # this layer's operands and remembers the fastest for this descriptor
            xs, ws, y = self.sets[0]
            t0 = time.perf_counter()
            if self.prepared:
                sconv.sconv_tune(xs, ws, layer.stride, layer.pad, layer.groups, layer.pool, relu=True, out=y,
                                 flush=flush_buffer(), wprep=self.preps[0], ws=self.workspace)
            else:
                sconv.sconv_tune(xs, ws, layer.stride, layer.pad, layer.groups, layer.pool, relu=True, out=y,
                                 flush=flush_buffer())
            self.tune_wall_s = time.perf_counter() - t0
        self.variant = sconv.sconv_variant_name(d, bool(layer.pool))
        self.plan = sconv.sconv_plan_name(d, bool(layer.pool))
        self.i = 0

    def parity(self, seed: int) -> dict:
        """The plan that will be timed, on the buffers that will be timed (set 0), against the oracle."""
        import torch
        self.i = 0
        self.run()
        torch.cuda.synchronize()
        self.i = 0
        x, w = self.host
        got = self.sets[0][2].cpu().numpy()
        L = self.layer
        dense_gflop = 2.0 * self.N * L.K * L.OH * L.OW * L.Cg * L.R * L.S / 1e9
        if dense_gflop <= 60.0:      # the whole tensor where the oracle needs a few seconds at most
            return whole_check(L, x, w, got)
        return sampled_check(L, x, w, got, seed)

    def run(self):
        xs, ws, y = self.sets[self.i]
        wp = self.preps[self.i]
        self.i = (self.i + 1) % len(self.sets)
        L = self.layer
        if self.prepared:
            # the ..._prep calls: prepared filters and the workspace as arguments of the call
            if L.pool:
                self.sconv.sconv_pool_forward(xs, ws, L.pool, L.stride, L.pad, L.groups, out=y, zero_ratio=self.z,
                                              wprep=wp, ws=self.workspace)
            else:
                self.sconv.sconv_forward(xs, ws, L.stride, L.pad, L.groups, relu=True, out=y, zero_ratio=self.z,
                                         wprep=wp, ws=self.workspace)
        elif L.pool:
            self.sconv.sconv_pool_forward(xs, ws, L.pool, L.stride, L.pad, L.groups, out=y, zero_ratio=self.z)
        else:
            self.sconv.sconv_forward(xs, ws, L.stride, L.pad, L.groups, relu=True, out=y, zero_ratio=self.z)


def ramp_up(fn, seconds: float = 0.03) -> None:
    """Untimed set-up before a timed region: keeps the GPU busy with the workload itself for
    `seconds`.  An idle GPU runs its first milliseconds at lower clocks - the same 50-us layer measured
    54, 50, 48 us in three successive 2-ms rounds - and a handful of warm-up launches does not get past
    that."""
    import torch
    t0 = time.perf_counter()
    while time.perf_counter() - t0 < seconds:
        for _ in range(10):
            fn()
        torch.cuda.synchronize()


def time_layer(dl: DeviceLayer, iters: int, warmup: int) -> float:
    """Average launch duration in ms, events on the launch stream (torch's current stream): the
    median of five back-to-back rounds of `iters` launches, so that a stall of the machine (seen
    now and then on 20-us layers) does not pass for the kernel's time."""
    import torch
    ramp_up(dl.run)
    for _ in range(warmup):
        dl.run()
    torch.cuda.synchronize()
    rounds = []
    for _ in range(5):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(iters):
            dl.run()
        e1.record()
        e1.synchronize()
        rounds.append(e0.elapsed_time(e1) / iters)
    # one launch on its own (the stream idle before and after): the latency of a single call,
    # median of five
    singles = []
    for _ in range(5):
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        dl.run()
        e1.record()
        e1.synchronize()
        singles.append(e0.elapsed_time(e1))
    dl.single_launch_ms = sorted(singles)[2]
    # the same launches on one buffer set (operands stay in the 256 MB last-level cache): the warm
    # figure beside the cold one, median of three rounds
    warm = []
    saved, dl.sets, dl.i = dl.sets, dl.sets[:1], 0
    for _ in range(3):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(iters):
            dl.run()
        e1.record()
        e1.synchronize()
        warm.append(e0.elapsed_time(e1) / iters)
    dl.sets, dl.i = saved, 0
    dl.warm_ms = sorted(warm)[1]
    dl.round_ms = (min(rounds), max(rounds))
    return sorted(rounds)[2]


def layer_record(dl: DeviceLayer, work: dict, ms: float) -> dict:
    t = ms * 1e-3
    t_hbm = work["alg_bytes"] / (HBM_PEAK_GBS * 1e9)
    t_valu = work["nz_flops"] / (FP32_VECTOR_PEAK_TF * 1e12)
    # what the plan really issues: a kernel that tests groups of g elements multiplies every element of a
    # group that holds a nonzero (independent zeros: a share z^g of the groups is skipped); the forms without
    # any test (geometry names ending in d, "dense") issue everything - the dense fallback on the matrix pipe
    g = SKIP_GRANULE.get(dl.variant, 1)
    geom = dl.plan.split("/")[1] if "/" in dl.plan else ""
    dense_form = dl.variant in MFMA_VARIANTS and (geom == "dense" or (geom.endswith("d") and geom != "kept"))
    z = work["zero_ratio"]
    skipped = 0.0 if dense_form else (z if g == 1 else z ** g)
    issued = work["dense_flops"] * (1.0 - skipped) if g > 1 or dense_form else work["nz_flops"]
    rounds = getattr(dl, "round_ms", (float("nan"), float("nan")))
    return {
        "layer": dl.layer.name, "N": dl.N, "variant": dl.variant, "plan": dl.plan,
        "prepared_filters": bool(getattr(dl, "prepared", False)), "ms": round(ms, 5),
        "ms_min_max_of_5_rounds": [round(rounds[0], 5), round(rounds[1], 5)],
        "pipe": "mfma" if dl.variant in MFMA_VARIANTS else "valu",
        "dense_fallback": dense_form, "skip_granule_elements": g,
        "granules_skipped_est": round(skipped, 4),
        "issued_gflops_est": round(issued / t / 1e9, 1),
        "tune_wall_s": round(getattr(dl, "tune_wall_s", 0.0), 3),
        "single_launch_ms": round(getattr(dl, "single_launch_ms", float("nan")), 5),
        "warm_ms": round(getattr(dl, "warm_ms", float("nan")), 5),
        "zero_ratio": round(work["zero_ratio"], 4),
        "dense_equiv_gflops": round(work["dense_flops"] / t / 1e9, 1),
        "nonzero_mac_gflops": round(work["nz_flops"] / t / 1e9, 1),
        "alg_GBps": round(work["alg_bytes"] / t / 1e9, 1),
        "hbm_frac": round(work["alg_bytes"] / t / 1e9 / HBM_PEAK_GBS, 4),
        "valu_frac": round(work["nz_flops"] / t / 1e12 / FP32_VECTOR_PEAK_TF, 4),
        "frac_of_unpacked_fp32_peak": round(work["nz_flops"] / t / 1e12 / FP32_UNPACKED_PEAK_TF, 4),
        "bound": "hbm" if t_hbm >= t_valu else ("mfma" if dl.variant in MFMA_VARIANTS else "alu"),
        "bound_frac": round(max(t_hbm, t_valu) / t, 4),
    }


def copies_for(work_list) -> int:
    per_set = sum(w["alg_bytes"] for w in work_list)
    return int(max(2, min(16, -(-CACHE_BYTES // int(per_set)))))


def cpu_baseline_one_thread(config_index: int) -> dict:
    """The dense oracle held to one thread, on the config's last layer at batch 1."""
    import oracle
    cfg = workloads.CONFIGS[config_index]
    li = len(cfg["layers"]) - 1
    layer, x, w = workloads.make_layer_inputs(config_index, li, 1)
    with oracle.one_thread():
        t0 = time.perf_counter()
        if layer.pool:
            oracle.conv_pool(x, w, layer.pool, layer.stride, layer.pad, layer.groups)
        else:
            oracle.conv(x, w, layer.stride, layer.pad, layer.groups, relu=True)
        secs = time.perf_counter() - t0
    flops = 2.0 * layer.K * layer.OH * layer.OW * layer.Cg * layer.R * layer.S
    return {"value": round(flops / secs / 1e9, 2), "unit": "GFLOP/s (dense-equivalent)", "cores": 1,
            "kind": "oracle", "sample": f"{layer.name} at batch 1, {secs:.2f} s"}


def cpu_baseline(config_index: int, batch: int = 2) -> dict:
    """The oracle as it stands, on the host cores, on the same layer set at the benchmark's batch."""
    import oracle
    cfg = workloads.CONFIGS[config_index]
    flops, secs = 0.0, 0.0
    for li, _ in enumerate(cfg["layers"]):
        layer, x, w = workloads.make_layer_inputs(config_index, li, batch)
        t0 = time.perf_counter()
        if layer.pool:
            oracle.conv_pool(x, w, layer.pool, layer.stride, layer.pad, layer.groups)
        else:
            oracle.conv(x, w, layer.stride, layer.pad, layer.groups, relu=True)
        secs += time.perf_counter() - t0
        flops += 2.0 * batch * layer.K * layer.OH * layer.OW * layer.Cg * layer.R * layer.S
    return {"value": round(flops / secs / 1e9, 2), "unit": "GFLOP/s (dense-equivalent)",
            "cores": oracle.threads(), "kind": "oracle",
            "sample": f"one pass over the {cfg['name']} layer set at batch {batch} (fp64 dense oracle, "
                      f"{secs:.2f} s wall, about {secs * oracle.threads():.0f} core-seconds)"}


def cpu_sparse_baseline(config_index: int, all_cores: bool = False) -> dict:
    """The oracle's zero-skipping path as it stands (Algorithm 1 into the materialised format, one thread; then
    Algorithm 2 over it, fp64 sums, one thread or the rows over all host cores) on the config's first layer at
    batch 1."""
    import contextlib
    import oracle
    layer, x, w = workloads.make_layer_inputs(config_index, 0, 1)
    with (contextlib.nullcontext() if all_cores else oracle.one_thread()):
        t0 = time.perf_counter()
        values, index, count = oracle.encode(x, w.shape, 0, layer.stride, layer.pad, layer.groups)
        t1 = time.perf_counter()
        oracle.spmv(values, index, count, w, x.shape, layer.stride, layer.pad, layer.groups)
        t2 = time.perf_counter()
    dense = 2.0 * layer.K * layer.OH * layer.OW * layer.Cg * layer.R * layer.S
    nz = 2.0 * float(np.maximum(count, 0).sum()) * (layer.K // layer.groups)
    return {"value": round(dense / (t2 - t0) / 1e9, 2), "unit": "GFLOP/s (dense-equivalent)",
            "nonzero_mac_gflops": round(nz / (t2 - t0) / 1e9, 2), "cores": oracle.threads() if all_cores else 1,
            "kind": "oracle, zero-skipping path",
            "sample": f"{layer.name} at batch 1: encode (one thread) {t1 - t0:.2f} s + sparse products {t2 - t1:.2f} s"}


def paper_context() -> dict:
    return {"hardware": "NVIDIA GeForce RTX 2080Ti, CUDA 10.2, cuDNN 7.6.5 (paper, Table 2)",
            "note": "relative speedups only; context, not a target",
            "vgg19_conv_layers_vs_cudnn_fast": 3.91, "vgg19_whole_net_vs_cudnn_fast": 1.97,
            "vgg19_conv_layers_vs_cusparse": 3.28, "single_layer_vs_cudnn_fast": [2.24, 2.78],
            "single_layer_vs_cusparse": [2.97, 3.99]}


def run_headline(args) -> None:
    import torch
    ci = [c["name"] for c in workloads.CONFIGS].index(args.config)
    cfg = workloads.CONFIGS[ci]
    N = args.batch if args.batch else max(cfg["batches"])
    host = [workloads.make_layer_inputs(ci, li, N) for li in range(len(cfg["layers"]))]
    works = [layer_work(layer, N, x) for layer, x, w in host]
    copies = copies_for(works)
    dls = [DeviceLayer(layer, N, x, w, copies) for layer, x, w in host]
    torch.cuda.synchronize()
    # parity first, on the buffers and with the plans that are timed below
    parity = {"checked": 0, "failed": 0, "worst_ratio": 0.0, "tolerance": "1e-4 * sum|x*w| per element",
              "against": "CPU oracle (fp64): every output of every layer (layers above 60 dense GFLOP: "
                         "4000 random outputs + tile and filter-block boundaries instead)"}
    if not args.no_parity:
        for li, dl in enumerate(dls):
            r = dl.parity(4242 + li)
            parity["checked"] += r["checked"]
            parity["failed"] += r["failed"]
            parity["worst_ratio"] = max(parity["worst_ratio"], r["worst_ratio"])
        if parity["failed"]:
            print(json.dumps({"error": "parity check failed before timing", "parity": parity,
                              "plans": [dl.plan for dl in dls]}), flush=True)
            sys.exit(3)

    def step():
        for dl in dls:
            dl.run()

    ramp_up(step, 0.1)
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps

    # per-kernel durations, events on the launch stream
    recs = []
    for dl, wk in zip(dls, works):
        ms = time_layer(dl, max(200, args.steps), 20)
        recs.append(layer_record(dl, wk, ms))
    dom = max(range(len(recs)), key=lambda i: recs[i]["ms"])
    r, wk = recs[dom], works[dom]
    t = r["ms"] * 1e-3
    if r["bound"] == "hbm":
        roof = {"bound": "hbm", "achieved": round(wk["alg_bytes"] / t / 1e9, 1), "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": round(wk["alg_bytes"] / t / 1e9 / HBM_PEAK_GBS, 4), "traffic": None}
    else:
        ach = wk["nz_flops"] / t / 1e12
        if r["variant"] in MFMA_VARIANTS:
            # products go through the fp32 matrix pipe; algorithmic flops = nonzero multiply-adds
            roof = {"bound": "mfma", "achieved": round(ach, 2), "peak": FP32_MFMA_PEAK_TF, "unit": "TFLOP/s",
                    "frac": round(ach / FP32_MFMA_PEAK_TF, 4), "traffic": None,
                    "issued_dense_equiv_TFLOPs": round(wk["dense_flops"] / t / 1e12, 2)}
        else:
            roof = {"bound": "alu", "achieved": round(ach, 2), "peak": FP32_VECTOR_PEAK_TF, "unit": "TFLOP/s",
                    "frac": round(ach / FP32_VECTOR_PEAK_TF, 4), "traffic": None,
                    "frac_of_unpacked_fp32_peak": round(ach / FP32_UNPACKED_PEAK_TF, 4)}
    traffic = MEASURED_TRAFFIC.get((r["plan"], r["layer"], N))
    roof["traffic"] = traffic[0] if traffic else None
    roof["traffic_source"] = traffic[1] if traffic else "no counter run of this plan in profiles/"
    roof["kernel"] = f"{r['plan']} on {r['layer']} N={N}"
    roof["dense_fallback"] = r["dense_fallback"]
    roof["kernel_ms"] = r["ms"]
    roof["alg_bytes_per_launch"] = wk["alg_bytes"]
    roof["nonzero_flops_per_launch"] = wk["nz_flops"]

    dense_total = sum(w["dense_flops"] for w in works)
    out = {
        "metric": "dense-equiv GFLOP/s + HBM GB/s (% roofline) per sparse conv(+pool) layer",
        "value": round(dense_total / (ms_per_step * 1e-3) / 1e9, 1),
        "unit": "GFLOP/s (dense-equivalent, whole step)",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{cfg['name']}-shaped layer set ({', '.join(l.name for l in cfg['layers'])}), "
                               f"batch {N}; per layer: " + "; ".join(
                                   f"{r['layer']}: {'conv+ReLU+max-pool' if l.pool else 'conv+ReLU'} as {r['plan']}"
                                   for r, (l, _, _) in zip(recs, host)),
                   "batch": N, "buffer_copies_rotated": copies,
                   "tune_wall_s": round(sum(dl.tune_wall_s for dl in dls), 2)},
        "layers": recs,
        "parity": parity,
        "roofline": roof,
        "paper_context": paper_context(),
    }
    if not PREP and not args.no_prepared:
        # The same step with the filters handed over in the prepared layout (written once at set-up, as an
        # inference engine holding constant filters would): saves the per-call transposition of the vector
        # kernel's transposed-filter form.  Reported beside the headline, never as `value`.
        pdls = [DeviceLayer(layer, N, x, w, copies, prepared=True) for layer, x, w in host]
        pfail = 0
        if not args.no_parity:
            for li, dl in enumerate(pdls):
                pfail += dl.parity(5252 + li)["failed"]
        if pfail:
            print(json.dumps({"error": "parity check of the prepared-filter plans failed",
                              "plans": [dl.plan for dl in pdls]}), flush=True)
            sys.exit(3)

        def pstep():
            for dl in pdls:
                dl.run()

        ramp_up(pstep, 0.1)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            pstep()
        torch.cuda.synchronize()
        pms = (time.perf_counter() - t0) * 1e3 / args.steps
        out["prepared_filters"] = {
            "ms_per_step": round(pms, 4), "value": round(dense_total / (pms * 1e-3) / 1e9, 1),
            "plans": [dl.plan for dl in pdls], "parity_failed": pfail,
            "note": "same step, filters passed in the prepared layout (sconv_filter_prep once at set-up); "
                    "not the headline value"}
        del pdls
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(ci, N)
        out["cpu_baseline_one_thread"] = cpu_baseline_one_thread(ci)
        out["cpu_sparse_oracle"] = cpu_sparse_baseline(ci)
        out["cpu_sparse_oracle_all_cores"] = cpu_sparse_baseline(ci, all_cores=True)
    print(json.dumps(out), flush=True)


def run_table(args) -> None:
    """Every layer of every config at each of its batch sizes; one JSON line per layer."""
    import torch
    for ci, cfg in enumerate(workloads.CONFIGS):
        if args.only and cfg["name"] != args.only:
            continue
        for N in cfg["batches"]:
            for li in range(len(cfg["layers"])):
                layer, x, w = workloads.make_layer_inputs(ci, li, N)
                wk = layer_work(layer, N, x)
                dl = DeviceLayer(layer, N, x, w, copies_for([wk]))
                ms = time_layer(dl, args.steps, args.warmup)
                rec = layer_record(dl, wk, ms)
                rec["config"] = cfg["name"]
                print(json.dumps(rec), flush=True)
                del dl
                torch.cuda.empty_cache()


def run_sweep(args) -> None:
    """Zero-ratio sweep 0.00-0.95: on the RegNetX 896-channel grouped layer at batch 32 by default, or on
    --layer CONFIG:INDEX at --batch (default: the config's largest)."""
    import torch
    ci, li = 4, 0
    if args.layer:
        name, li = args.layer.split(":")
        ci, li = [c["name"] for c in workloads.CONFIGS].index(name), int(li)
    base = workloads.CONFIGS[ci]["layers"][li]
    N = args.batch or max(workloads.CONFIGS[ci]["batches"])
    for z in workloads.SWEEP_ZERO_RATIOS:
        layer = base.with_zero_ratio(z)
        if args.structure != "iid":
            layer = layer.with_structure(args.structure)
        layer, x, w = workloads.make_layer_inputs(ci, li, N, layer)
        wk = layer_work(layer, N, x)
        dl = DeviceLayer(layer, N, x, w, copies_for([wk]))
        ms = time_layer(dl, args.steps, args.warmup)
        rec = layer_record(dl, wk, ms)
        rec["config"] = workloads.CONFIGS[ci]["name"] + "-sweep" + ("" if args.structure == "iid" else "-" + args.structure)
        print(json.dumps(rec), flush=True)
        del dl
        torch.cuda.empty_cache()


def run_layer(args) -> None:
    """One layer alone (for profiling): --layer CONFIG:INDEX at --batch."""
    name, li = args.layer.split(":")
    ci = [c["name"] for c in workloads.CONFIGS].index(name)
    N = args.batch or max(workloads.CONFIGS[ci]["batches"])
    layer, x, w = workloads.make_layer_inputs(ci, int(li), N)
    if args.zero_ratio >= 0:
        layer = layer.with_zero_ratio(args.zero_ratio)
    if args.structure != "iid":
        layer = layer.with_structure(args.structure)
    if args.zero_ratio >= 0 or args.structure != "iid":
        layer, x, w = workloads.make_layer_inputs(ci, int(li), N, layer)
    wk = layer_work(layer, N, x)
    dl = DeviceLayer(layer, N, x, w, copies_for([wk]))
    ms = time_layer(dl, args.steps, args.warmup)
    rec = layer_record(dl, wk, ms)
    rec["config"] = name
    rec["alg_bytes"] = wk["alg_bytes"]
    rec["nonzero_flops"] = wk["nz_flops"]
    print(json.dumps(rec), flush=True)


def run_shape(args) -> None:
    """Any layer shape: --shape N,C,H,W,K,R,S,stride,pad,groups[,ph,pw,ps] at --zero-ratio (default 0.7)."""
    v = [int(t) for t in args.shape.split(",")]
    if len(v) not in (10, 13):
        sys.exit("--shape takes N,C,H,W,K,R,S,stride,pad,groups or the same plus ph,pw,ps")
    N, C, H, W, K, R, S, stride, pad, groups = v[:10]
    pool = tuple(v[10:13]) if len(v) == 13 else None
    z = args.zero_ratio if args.zero_ratio >= 0 else 0.7
    layer = workloads.Layer(f"shape-{args.shape}", C=C, H=H, W=W, K=K, R=R, S=S, stride=stride, pad=pad,
                            groups=groups, pool=pool, zero_ratio=z, structure=args.structure)
    rng = np.random.default_rng(workloads.BASE_SEED + 7777)
    x = workloads.make_feature_map(rng, N, layer)
    w = workloads.make_filters(rng, layer)
    wk = layer_work(layer, N, x)
    dl = DeviceLayer(layer, N, x, w, copies_for([wk]))
    ms = time_layer(dl, args.steps, args.warmup)
    rec = layer_record(dl, wk, ms)
    rec["config"] = "shape"
    print(json.dumps(rec), flush=True)


def _time(fn, iters, warmup) -> float:
    """Average duration of fn in ms: the median of five back-to-back rounds of `iters` calls (one round
    now and then catches a stall of the machine several times the kernel's length)."""
    import torch
    ramp_up(fn)
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    rounds = []
    for _ in range(5):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(iters):
            fn()
        e1.record()
        e1.synchronize()
        rounds.append(e0.elapsed_time(e1) / iters)
    return sorted(rounds)[2]


def run_split(args) -> None:
    """Two of the paper's measurements on this hardware, every layer at its largest batch:
    (1) the format conversion alone (sconv_encode, materialised in HBM) next to the whole
    convolution kernel, which converts on chip and never stores the format (the paper reports the
    conversion at 14-50 % of its kernels' time); (2) for the layers followed by pooling, the fused
    call next to convolution + stand-alone pooling kernel (the fused kernel saves the convolution
    tensor's round trip through memory).  Same buffers every launch (warm caches)."""
    import torch
    import paper_1909_09927_amd as sconv
    lend_workspace()
    for ci, cfg in enumerate(workloads.CONFIGS):
        if ci == 0:
            continue
        N = max(cfg["batches"])
        for li in range(len(cfg["layers"])):
            layer, x, w = workloads.make_layer_inputs(ci, li, N)
            xd, wd = torch.from_numpy(x).cuda(), torch.from_numpy(w).cuda()
            L = layer
            fmt = sconv.FMT_PECR if L.pool else sconv.FMT_ECR
            desc = sconv.desc_for(xd, wd, L.stride, L.pad, L.groups, L.pool, True)
            rows, slots = sconv.sconv_encode_sizes(desc, fmt)
            vals = torch.empty((rows, slots), dtype=torch.float32, device="cuda")
            idx = torch.empty((rows, slots), dtype=torch.int32, device="cuda")
            cnt = torch.empty((rows,), dtype=torch.int32, device="cuda")
            t_enc = _time(lambda: sconv.sconv_encode(xd, w.shape, fmt, L.stride, L.pad, L.groups, L.pool,
                                                     out=(vals, idx, cnt)), args.steps, args.warmup)
            y = sconv.sconv_forward(xd, wd, L.stride, L.pad, L.groups, relu=True)
            t_fwd = _time(lambda: sconv.sconv_forward(xd, wd, L.stride, L.pad, L.groups, relu=True, out=y),
                          args.steps, args.warmup)
            rec = {"config": cfg["name"], "layer": L.name, "N": N,
                   "variant": sconv.sconv_variant_name(desc, False),
                   "forward_ms": round(t_fwd, 5), "encode_only_ms": round(t_enc, 5),
                   "format": "PECR" if L.pool else "ECR",
                   "encoded_MB": round(rows * (slots * 8 + 4) / 1e6, 1),
                   "encode_over_forward": round(t_enc / t_fwd, 3)}
            if L.pool:
                z = sconv.sconv_pool_forward(xd, wd, L.pool, L.stride, L.pad, L.groups)
                t_fused = _time(lambda: sconv.sconv_pool_forward(xd, wd, L.pool, L.stride, L.pad, L.groups,
                                                                 out=z), args.steps, args.warmup)
                t_pool = _time(lambda: sconv.sconv_maxpool(y, x.shape, w.shape, L.pool, L.stride, L.pad,
                                                           L.groups, out=z), args.steps, args.warmup)
                rec.update({"fused_ms": round(t_fused, 5), "pool_only_ms": round(t_pool, 5),
                            "unfused_ms": round(t_fwd + t_pool, 5),
                            "fused_speedup": round((t_fwd + t_pool) / t_fused, 3),
                            "conv_tensor_MB": round(y.numel() * 4 / 1e6, 1),
                            "pool_only_GBps": round((y.numel() + z.numel()) * 4 / (t_pool * 1e-3) / 1e9, 1)})
            print(json.dumps(rec), flush=True)
            del vals, idx, cnt, y
            torch.cuda.empty_cache()


def run_axis(args) -> None:
    """The paper's two other sensitivity axes on one layer shape (Sections 8.4 and 8.5): batch size
    1..32 and convolution stride 1..3, on the VGG-shaped 256->256 3x3 layer at 56x56 (pad 1)."""
    import dataclasses
    import torch
    ci, li = 1, 0
    base = workloads.CONFIGS[ci]["layers"][li]
    cases = []
    if args.axis == "batch":
        cases = [(base, n) for n in (1, 2, 4, 8, 16, 32)]
    else:
        cases = [(dataclasses.replace(base, stride=st, name=f"{base.name}-s{st}"), 8) for st in (1, 2, 3)]
    for layer, N in cases:
        layer, x, w = workloads.make_layer_inputs(ci, li, N, layer)
        wk = layer_work(layer, N, x)
        dl = DeviceLayer(layer, N, x, w, copies_for([wk]))
        ms = time_layer(dl, args.steps, args.warmup)
        rec = layer_record(dl, wk, ms)
        rec["config"] = f"vgg19-{args.axis}-sweep"
        rec["stride"] = layer.stride
        print(json.dumps(rec), flush=True)
        del dl
        torch.cuda.empty_cache()


def run_graph(args) -> None:
    """One step (every layer of --config at --batch) captured in a HIP graph and replayed, next to
    the same step launched eagerly: what the launch path costs on the small batch-1 layers.  The
    library only enqueues on the caller's stream, so a capture needs nothing from it; the first
    (uncaptured) calls do the one-time set-up (occupancy queries, LDS opt-in)."""
    import torch
    ci = [c["name"] for c in workloads.CONFIGS].index(args.config)
    cfg = workloads.CONFIGS[ci]
    N = args.batch if args.batch else min(cfg["batches"])
    host = [workloads.make_layer_inputs(ci, li, N) for li in range(len(cfg["layers"]))]
    dls = [DeviceLayer(layer, N, x, w, 1) for layer, x, w in host]

    def step():
        for dl in dls:
            dl.run()

    step()
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        lend_workspace()             # the capture stream's own workspace: split plans in the graph too
        step()                       # warm-up on the capture stream
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.synchronize()
    t_eager = _time(step, args.steps, args.warmup)
    t_graph = _time(graph.replay, args.steps, args.warmup)
    print(json.dumps({"config": cfg["name"], "N": N, "layers": [l.name for l, _, _ in host],
                      "variants": [dl.variant for dl in dls],
                      "eager_ms_per_step": round(t_eager, 5), "graph_ms_per_step": round(t_graph, 5),
                      "same_buffers_every_step": True}), flush=True)


def run_chain(args) -> None:
    """The VGG-19-shaped tail (28x28 stage to the end) as a chain: every layer consumes the previous
    layer's output on the device, so from the second layer on the zeros are the ones ReLU and pooling
    produced.  Each layer is tuned on the input it really gets.  One JSON line per layer (zero ratio
    of its input, plan, time) and one for the whole chain."""
    import torch
    import paper_1909_09927_amd as sconv
    N = args.batch or 8
    x, ws = workloads.make_chain_inputs(N)
    cur = torch.from_numpy(x).cuda()
    wds = [torch.from_numpy(w).cuda() for w in ws]
    outs, recs = [], []
    flush = flush_buffer() if TUNE else None
    lend_workspace()
    wspace = _workspaces[torch.cuda.current_stream().cuda_stream]
    # --prepared: every layer's filters once in the prepared layout, passed with each call (with the workspace)
    preps = [sconv.sconv_filter_prep(wd, l.groups, l.stride, l.pad) if PREP else None
             for l, wd in zip(workloads.CHAIN, wds)]
    extra = [({"wprep": wp, "ws": wspace} if wp is not None else {}) for wp in preps]
    zs = []
    for (layer, wd), kw in zip(zip(workloads.CHAIN, wds), extra):
        # the producer's output is probed once; tuned plans are kept per density class, so two layers of
        # one shape (512 @14x14 twice, at 41 % and 88 % zeros) each keep their own
        z = sconv.zero_ratio_of(sconv.sconv_density(cur)) if (TUNE or HINT) else None
        zs.append(z)
        if TUNE:
            sconv.sconv_tune(cur, wd, layer.stride, layer.pad, layer.groups, layer.pool, relu=True, flush=flush,
                             zero_ratio=z, **kw)
        if layer.pool:
            y = sconv.sconv_pool_forward(cur, wd, layer.pool, layer.stride, layer.pad, layer.groups, zero_ratio=z, **kw)
        else:
            y = sconv.sconv_forward(cur, wd, layer.stride, layer.pad, layer.groups, relu=True, zero_ratio=z, **kw)
        d = sconv.desc_for(cur, wd, layer.stride, layer.pad, layer.groups, layer.pool, True, z, bool(kw))
        recs.append({"layer": layer.name, "N": N, "plan": sconv.sconv_plan_name(d, bool(layer.pool)),
                     "input_zero_ratio": round(float((cur == 0).float().mean()), 4),
                     "dense_flops": 2.0 * N * layer.K * layer.OH * layer.OW * layer.Cg * 9})
        outs.append((cur, wd, y))
        cur = y
    torch.cuda.synchronize()

    def one(i):
        layer = workloads.CHAIN[i]
        xi, wd, y = outs[i]
        if layer.pool:
            sconv.sconv_pool_forward(xi, wd, layer.pool, layer.stride, layer.pad, layer.groups, out=y, zero_ratio=zs[i],
                                     **extra[i])
        else:
            sconv.sconv_forward(xi, wd, layer.stride, layer.pad, layer.groups, relu=True, out=y, zero_ratio=zs[i],
                                **extra[i])

    def step():
        for i in range(len(outs)):
            one(i)

    total = 0.0
    for i, rec in enumerate(recs):
        ms = _time(lambda: one(i), args.steps, args.warmup)
        rec["ms"] = round(ms, 5)
        rec["dense_equiv_gflops"] = round(rec.pop("dense_flops") / ms / 1e6, 1)
        total += rec["dense_equiv_gflops"] * ms
        print(json.dumps(rec), flush=True)
    ms = _time(step, args.steps, args.warmup)
    print(json.dumps({"chain": [l.name for l in workloads.CHAIN], "N": N, "prepared_filters": PREP,
                      "ms_per_pass": round(ms, 5),
                      "dense_equiv_gflops": round(total / ms, 1),
                      "output_zero_ratio": round(float((cur == 0).float().mean()), 4)}), flush=True)


MICRO_MODES = [
    (0, "fma", "8 independent v_fmac_f32 with a scalar operand", 8),
    (1, "salu_dep", "8 dependent s_add_u32", 8),
    (2, "test_not_taken", "s_bitcmp1 + s_cbranch_scc1, not taken", 1),
    (3, "test_taken", "s_bitcmp1 + s_cbranch_scc1, taken to the next instruction", 1),
    (4, "skip5_not_taken", "test + branch not taken + the 5 v_fmac it guards", 1),
    (5, "skip5_taken", "test + branch taken over 5 v_fmac", 1),
    (6, "setpc", "s_getpc + s_add + s_addc + s_setpc to the next instruction", 1),
    (7, "readlane_fma5", "v_readlane + s_nop 1 + 5 v_fmac on the broadcast value", 1),
    (8, "far_taken", "branch ~1.5 KB out of line, 5 v_fmac there, branch back", 1),
    (9, "ff1_setpc", "s_ff1 + s_bitset0 + s_lshl + s_getpc + s_add + s_addc + s_setpc", 1),
    (10, "mfma_4x4x1", "8 independent v_mfma_f32_4x4x1 (256 multiply-adds each; 8 clocks at the published rate)", 8),
    (11, "mfma_16x16x1", "4 independent v_mfma_f32_16x16x1 (1024 multiply-adds each; 32 clocks at the published rate)", 4),
    (12, "vskip5_on", "s_setvskip turning the vector-skip mode on + 5 v_fmac (not issued)", 1),
    (13, "vskip5_off", "s_setvskip leaving the mode off + 5 v_fmac (they run)", 1),
    (14, "vskip_pos_on", "s_setvskip on + v_readlane + s_nop 1 + 5 v_fmac: a zero position without a branch", 1),
    (15, "vskip_pos_off", "the same with the mode off: a nonzero position", 1),
]


def run_micro(args) -> None:
    """Issue-rate microbenchmarks (libsconv_micro.so): clocks per pattern for one wavefront and per
    SIMD at 1, 2, 4 and 8 resident wavefronts per SIMD.  Clocks are event time x 2.4 GHz (the nominal
    clock; the fma row shows what the chip really holds: 4 clocks per v_fmac is the hardware's rate)."""
    import ctypes
    import torch
    from paper_1909_09927_amd import build as hip_build
    if not os.path.exists(hip_build.MICRO_LIB):
        sys.exit("libsconv_micro.so is not built; run python -m paper_1909_09927_amd.build")
    lib = ctypes.CDLL(hip_build.MICRO_LIB)
    lib.sconv_micro_launch.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p]
    lib.sconv_micro_launch.restype = ctypes.c_int
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    out = torch.empty(cus * 8 * 256, dtype=torch.float32, device="cuda")
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    iters = 2000
    for mode, name, what, per_repeat in MICRO_MODES:
        rec = {"micro": name, "pattern": what, "instructions_counted_per_repeat": per_repeat}
        for w in (1, 2, 4, 8):
            blocks = cus * w

            def go():
                rc = lib.sconv_micro_launch(mode, iters, blocks, out.data_ptr(), stream)
                if rc:
                    sys.exit(f"sconv_micro_launch({name}) failed: {rc}")
            ms = _time(go, 5, 2)
            clocks = ms * 1e-3 * 2.4e9 / (iters * 64 * per_repeat)
            rec[f"clocks_per_wavefront_at_{w}_per_simd"] = round(clocks, 2)
            rec[f"clocks_per_simd_at_{w}_per_simd"] = round(clocks / w, 2)
        print(json.dumps(rec), flush=True)
    # streaming read of 1 GiB (past the 256 MiB last-level cache) with 2, 4 and 8 workgroups per compute unit
    lib.sconv_micro_read.argtypes = [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p]
    lib.sconv_micro_read.restype = ctypes.c_int
    src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()
    rec = {"micro": "read_stream", "pattern": "16-byte loads, four in flight per thread, over 1 GiB", "bytes": 1 << 30}
    for wpc in (2, 4, 8):
        def go():
            rc = lib.sconv_micro_read(src.data_ptr(), 1 << 30, cus * wpc, out.data_ptr(), stream)
            if rc:
                sys.exit(f"sconv_micro_read failed: {rc}")
        ms = _time(go, 10, 3)
        rec[f"TBps_at_{wpc}_workgroups_per_cu"] = round((1 << 30) / (ms * 1e-3) / 1e12, 2)
    print(json.dumps(rec), flush=True)


def run_variants(args) -> None:
    """How well the static choice of kernel generalises: --count random 3x3 / stride 1 / pad 1 layers that
    are not benchmark shapes (64-512 channels and filters, maps 7-56 wide, batch 2-32, 40-90 % independent
    zeros, a quarter of them with fused 2x2/2 pooling, 3-120 dense GFLOP), each timed with the static
    choice (zero ratio in the descriptor with --hint, unknown without) and with every 3x3 variant pinned
    (that variant's own static plan).  One JSON line per shape, then a summary of default / best variant."""
    import torch
    import paper_1909_09927_amd as sconv
    global TUNE, HINT
    TUNE = False
    rng = np.random.default_rng(args.seed)
    shapes = []
    while len(shapes) < args.count:
        C = int(rng.choice([64, 96, 128, 192, 256, 384, 512]))
        K = int(rng.choice([64, 128, 192, 256, 384, 512]))
        H = int(rng.choice([7, 10, 14, 20, 28, 40, 56]))
        W = H if rng.random() < 0.7 else int(rng.choice([7, 14, 28, 56]))
        N = int(rng.choice([2, 4, 8, 16, 32]))
        z = float(rng.choice([0.4, 0.5, 0.6, 0.7, 0.8, 0.9]))
        pool = (2, 2, 2) if rng.random() < 0.25 else None
        dense = 2.0 * N * K * H * W * C * 9
        if N * C * H * W * 4 > 400e6 or dense > 1.2e11 or dense < 3e9:
            continue
        shapes.append((N, C, H, W, K, pool, z))
    ratios = []
    for N, C, H, W, K, pool, z in shapes:
        layer = workloads.Layer(f"rand-{C}to{K}x{H}x{W}" + ("-pool" if pool else ""), C=C, H=H, W=W, K=K, R=3, S=3,
                                stride=1, pad=1, groups=1, pool=pool, zero_ratio=z)
        r2 = np.random.default_rng(1234)
        x = workloads.make_feature_map(r2, N, layer)
        w = workloads.make_filters(r2, layer)
        wk = layer_work(layer, N, x)
        rec = {"shape": [N, C, H, W, K], "pool": bool(pool), "zero_ratio": z}
        for var in (None, "tap", "quad", "wide"):
            if var:
                os.environ["SCONV_VARIANT"] = var
            else:
                os.environ.pop("SCONV_VARIANT", None)
            sconv.sconv_env_refresh()
            dl = DeviceLayer(layer, N, x, w, copies_for([wk]))
            if var is None or dl.variant.startswith(var):
                rec[(var or "default") + "_us"] = round(time_layer(dl, 40, 5) * 1e3, 1)
                if var is None:
                    rec["default_plan"] = dl.plan
            del dl
            torch.cuda.empty_cache()
        os.environ.pop("SCONV_VARIANT", None)
        sconv.sconv_env_refresh()
        best = min(rec[k] for k in ("tap_us", "quad_us", "wide_us") if k in rec)
        rec["default_over_best_variant"] = round(rec["default_us"] / best, 3)
        ratios.append(rec["default_over_best_variant"])
        print(json.dumps(rec), flush=True)
    print(json.dumps({"shapes": len(ratios), "hint": HINT, "seed": args.seed,
                      "mean_default_over_best": round(float(np.mean(ratios)), 3),
                      "worst_default_over_best": round(float(np.max(ratios)), 3),
                      "within_1.1": int(sum(r <= 1.1 for r in ratios))}), flush=True)


def run_pair(args) -> None:
    """The single-workgroup hand-off of Section 6.4 on a LeNet-shaped pair (5x5 1->20 on 28x28 + 2x2/2
    pooling, then 5x5 20->50 + pooling): one launch with the intermediate map in LDS, next to the two fused
    calls one after the other (intermediate through device memory).  Parity is checked first."""
    import torch
    import oracle
    import paper_1909_09927_amd as sconv
    lend_workspace()
    rng = np.random.default_rng(workloads.BASE_SEED + 61)
    for N in (1, 8, 64, 256):
        x = np.where(rng.random((N, 1, 28, 28)) < 0.3, np.abs(rng.standard_normal((N, 1, 28, 28))), 0).astype(np.float32)
        w1 = (rng.standard_normal((20, 1, 5, 5)) * np.sqrt(2 / 25)).astype(np.float32)
        w2 = (rng.standard_normal((50, 20, 5, 5)) * np.sqrt(2 / 500)).astype(np.float32)
        xd, w1d, w2d = (torch.from_numpy(t).cuda() for t in (x, w1, w2))
        first = {"pool": (2, 2, 2)}
        y, mid = sconv.sconv_pair_forward(xd, w1d, w2d, first, first, keep_mid=True)
        torch.cuda.synchronize()
        ref, sc = oracle.conv_pool(mid.cpu().numpy(), w2, (2, 2, 2))
        ok = bool((np.abs(y.cpu().numpy() - ref) <= 1e-4 * sc).all())
        m = sconv.sconv_pool_forward(xd, w1d, (2, 2, 2))
        z = sconv.sconv_pool_forward(m, w2d, (2, 2, 2))

        def two():
            sconv.sconv_pool_forward(xd, w1d, (2, 2, 2), out=m)
            sconv.sconv_pool_forward(m, w2d, (2, 2, 2), out=z)
        t_pair = _time(lambda: sconv.sconv_pair_forward(xd, w1d, w2d, first, first), args.steps, args.warmup)
        t_two = _time(two, args.steps, args.warmup)
        print(json.dumps({"pair": "lenet conv1+pool -> conv2+pool", "N": N, "parity_ok": ok,
                          "zero_ratio_in": round(float((x == 0).mean()), 3),
                          "zero_ratio_mid": round(float((mid == 0).float().mean()), 3),
                          "one_launch_ms": round(t_pair, 5), "two_calls_ms": round(t_two, 5)}), flush=True)


def run_copy_calibration(args) -> None:
    """A plain device copy of known size, for scaling the FETCH_SIZE / WRITE_SIZE counters."""
    import torch
    nbytes = 1 << 30
    a = torch.empty(nbytes // 4, dtype=torch.float32, device="cuda").normal_()
    b = torch.empty_like(a)
    for _ in range(5):
        b.copy_(a)
    torch.cuda.synchronize()
    print(json.dumps({"copy_bytes_read": nbytes, "copy_bytes_written": nbytes, "launches": 5}), flush=True)


def main() -> None:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", default="vgg19", choices=[c["name"] for c in workloads.CONFIGS])
    ap.add_argument("--batch", type=int, default=0)
    ap.add_argument("--table", action="store_true")
    ap.add_argument("--only", default="", help="--table: this config only")
    ap.add_argument("--sweep", action="store_true")
    ap.add_argument("--split", action="store_true",
                    help="conversion-only and unfused-pooling timings beside the whole kernels")
    ap.add_argument("--axis", default="", choices=["", "batch", "stride"],
                    help="batch-size or stride sweep on the VGG-shaped 256-channel layer")
    ap.add_argument("--chain", action="store_true",
                    help="the VGG-19-shaped tail as a chain: each layer consumes the previous layer's output")
    ap.add_argument("--graph", action="store_true",
                    help="one step of --config at --batch (default: its smallest) eagerly and as a HIP graph replay")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-parity", action="store_true",
                    help="skip the sampled comparison with the CPU oracle that precedes the timed region")
    ap.add_argument("--no-tune", action="store_true",
                    help="skip sconv_tune at set-up: static dispatch rules and cost models only")
    ap.add_argument("--prepared", action="store_true",
                    help="every layer's calls bring prepared filters (sconv_filter_prep at set-up)")
    ap.add_argument("--no-prepared", action="store_true",
                    help="headline: skip the extra prepared-filter measurement")
    ap.add_argument("--hint", action="store_true",
                    help="no tuning: probe every layer's input once (sconv_density) and give the static rules "
                         "its zero ratio (SCONV_ZERO_RATIO in the descriptor's flags)")
    ap.add_argument("--variants", action="store_true",
                    help="random 3x3 shapes outside the benchmark set: the static choice against every pinned variant")
    ap.add_argument("--seed", type=int, default=23, help="--variants: seed of the shape draw")
    ap.add_argument("--count", type=int, default=40, help="--variants: number of shapes")
    ap.add_argument("--pair", action="store_true",
                    help="two LeNet-shaped layers in one launch (hand-off in LDS) against two calls")
    ap.add_argument("--micro", action="store_true",
                    help="issue-rate microbenchmarks: vector FMAs, scalar tests, branches, computed jumps")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="run a 1 GiB device copy (scales the HBM traffic counters)")
    ap.add_argument("--layer", default="", help="CONFIG:INDEX, time that layer alone")
    ap.add_argument("--shape", default="", help="N,C,H,W,K,R,S,stride,pad,groups[,ph,pw,ps]: time this shape alone")
    ap.add_argument("--zero-ratio", type=float, default=-1.0, help="override the layer's zero ratio (--layer)")
    ap.add_argument("--structure", default="iid", choices=["iid", "clustered"],
                    help="zero pattern of the input for --sweep / --layer: independent zeros, or dead "
                         "planes plus spatial patches at the same overall ratio")
    args = ap.parse_args()
    global TUNE, HINT, PREP
    PREP = args.prepared
    HINT = args.hint
    TUNE = not args.no_tune and not args.hint and not os.environ.get("SCONV_VARIANT")
    if args.gpus != 1:
        sys.exit("bench.py measures one GPU: the path has no multi-GPU part (images or filters would "
                 "simply be split across devices with no exchange); run with --gpus 1")
    import torch
    if not torch.cuda.is_available():
        sys.exit("bench.py needs a GPU")
    import paper_1909_09927_amd as sconv
    if not os.path.exists(sconv.LIB_PATH):
        sys.exit("libsconv.so is not built; run python -m paper_1909_09927_amd.build")
    if args.copy_calibration:
        run_copy_calibration(args)
    elif args.micro:
        run_micro(args)
    elif args.pair:
        run_pair(args)
    elif args.variants:
        run_variants(args)
    elif args.shape:
        run_shape(args)
    elif args.sweep:
        run_sweep(args)
    elif args.layer:
        run_layer(args)
    elif args.table:
        run_table(args)
    elif args.split:
        run_split(args)
    elif args.chain:
        run_chain(args)
    elif args.graph:
        run_graph(args)
    elif args.axis:
        run_axis(args)
    else:
        run_headline(args)


if __name__ == "__main__":
    main()
