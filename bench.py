#!/usr/bin/env python3
"""Benchmark of the MMSE INT4 scale search on one MI355X.

Default (``--part whole --config 5``): a "step" is one pass of the whole hot path over the
VGG-16-shaped configuration of the benchmark spec (configs[4]) -- the largest workload that
the configurations name: per-kernel abs-max, 512-point grid sweep, argmin, 20 golden-section
iterations and packed INT4 codes for all 16 weight tensors (138 M weights), the second
INT4 tensor on the residual of all 16 layers, and search + codes of all 16 calibration
activation tensors (146 M elements) -- first enqueue to last kernel, inputs resident in
HBM before the timed region starts, outputs left on the device.

Prints ONE JSON line.  ``value`` = (element, candidate) evaluations per second of the whole
step.  ``roofline`` describes the kernel with the most time per step, timed by itself between
HIP events on its launch stream (``all_alu_kernels`` lists the others, ``hbm`` the streaming
passes against the 8 TB/s of HBM3E); ``cpu_baseline`` times the CPU oracle on a bounded sample of
the same inputs on the host cores and ``matches_oracle`` compares every output on that sample;
``other_configs`` carries short runs of configurations 1-4.  ``--part weights|activation|dual|
dual-ls|compare`` time single parts (default configuration 2).
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

METRIC = "element x candidate MSE evals/sec + end-to-end whole-net search ms (1 MI355X)"

# VALU issue peak of MI355X: 256 CUs x 4 SIMDs x 32 lanes/clk x 2.4 GHz = 78.6e12 lane-ops/s.
# (A SIMD retires two wave64 fp32 instructions from two different waves every 4 clocks; with
# every one of them an FMA this is the published 157.3 TFLOP/s.)
LANE_OPS_PER_S = 256 * 4 * 32 * 2.4e9
OPS_PER_EVAL = 5          # v_mul, v_rndne, v_med3, v_fma, v_fma(c)
FLOPS_PER_EVAL = 7        # 1 + 1 + 1 + 2 + 2
HBM_GBS = 8000.0          # published HBM3E bandwidth of MI355X


def bench_activation(args, cfg, torch, B) -> int:
    """Per-layer search (Eq. 15) + packed codes for the largest activation tensor of the configuration."""
    if not cfg.act_shapes:
        print(f"bench.py: configuration {cfg.cfg} has no activations", file=sys.stderr)
        return 2
    G = args.grid_points if args.grid_points > 0 else cfg.grid_points
    iters = args.refine_iters if args.refine_iters >= 0 else cfg.refine_iters
    li = max(range(len(cfg.act_shapes)), key=lambda i: cfg.act_shapes[i].per_image)
    x = cfg.act_tensor(li)
    N = x.size
    xd = torch.from_numpy(x).cuda()
    p = B.params(0, 15, G, iters, args.cands_per_lane)
    ws = B.alloc_workspace(B.mmse_workspace_bytes_activation(N, p))
    out = B.SearchResult(torch.empty(1, dtype=torch.float32, device="cuda"),
                         torch.empty(1, dtype=torch.int32, device="cuda"),
                         torch.empty(1, dtype=torch.float64, device="cuda"))
    packed = torch.empty((N + 1) // 2, dtype=torch.uint8, device="cuda")

    variant = args.act_variant
    if variant == "offset":
        x = x - np.float32(0.75)                  # a tensor with a negative floor, so that delta matters
        xd = torch.from_numpy(x).cuda()
    p2 = B.params(-8, 7, G, iters, args.cands_per_lane)
    out2 = B.SearchResult(torch.empty(1, dtype=torch.float32, device="cuda"),
                          torch.empty(1, dtype=torch.int32, device="cuda"),
                          torch.empty(1, dtype=torch.float64, device="cuda"),
                          torch.empty((N + 1) // 2, dtype=torch.uint8, device="cuda") if variant == "residual" else None)
    outo = B.OffsetResult(torch.empty(1, dtype=torch.float32, device="cuda"), out.scale, out.idx, out.sse, packed)

    def step():
        if variant == "offset":
            B.mmse_scale_search_offset(xd, p, ws, outo)
            return
        B.mmse_scale_search_activation(xd, p, ws, out)
        B.quantize_pack_int4(xd, out.scale, 0, 15, packed)
        if variant == "residual":
            B.activation_residual_quantize(xd, out.scale, 0, 15, p2, ws, out2)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps
    evals = N * (G + 2 + iters) * (2 if variant == "residual" else 1)

    # dominant kernel alone: grid sweep (refine_iters = 0 leaves abs-max, sweep, reduction, argmin)
    p0 = B.params(0, 15, G, 0, args.cands_per_lane)
    p20 = B.params(-8, 7, G, 0, args.cands_per_lane)
    step()
    s1 = out.scale.clone()
    outs0 = B.SearchResult(torch.empty(1, dtype=torch.float32, device="cuda"),
                           torch.empty(1, dtype=torch.int32, device="cuda"),
                           torch.empty(1, dtype=torch.float64, device="cuda"))
    outo0 = B.OffsetResult(torch.empty(1, dtype=torch.float32, device="cuda"), outs0.scale, outs0.idx, outs0.sse, None)

    def sweep_only():
        if variant == "offset":
            B.mmse_scale_search_offset(xd, p0, ws, outo0)
        elif variant == "residual":
            B.activation_residual_quantize(xd, s1, 0, 15, p20, ws, outs0)
        else:
            B.mmse_scale_search_activation(xd, p0, ws, outs0)

    sweep_only()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    ev0.record()
    for _ in range(args.steps):
        sweep_only()
    ev1.record()
    torch.cuda.synchronize()
    sweep_ms = ev0.elapsed_time(ev1) / args.steps
    peak_tflops = LANE_OPS_PER_S * FLOPS_PER_EVAL / OPS_PER_EVAL / 1e12
    # the sweep drops the elements that are zero after the variant's pre-operation while staging (they add nothing to
    # a sum at any scale): the roofline counts the others where the bench can count them (the plain variant)
    counted = int(torch.count_nonzero(xd).item()) if variant == "plain" else N
    ach = counted * G * FLOPS_PER_EVAL / (sweep_ms * 1e-3) / 1e12
    roofline = {"bound": "alu", "kernel": "k_act_sweep (+abs-max, block reduction, argmin in the timed region)",
                "achieved": round(ach, 3), "peak": round(peak_tflops, 3), "unit": "TFLOP/s",
                "frac": round(ach / peak_tflops, 4), "traffic": None, "avg_launch_ms": round(sweep_ms, 5),
                "evals_per_s": N * G / (sweep_ms * 1e-3),
                "counted": ("evaluations of non-zero elements" if variant == "plain" else
                            "all elements (dense equivalent: can exceed 1 where the pre-operation leaves zeros)"),
                "nonzero_fraction": round(counted / max(N, 1), 4),
                "dense_equivalent_frac": round(N * G * FLOPS_PER_EVAL / (sweep_ms * 1e-3) / 1e12 / peak_tflops, 4)}
    cpu_baseline, parity = None, None
    if not args.no_cpu_baseline:
        import oracle
        step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        if variant == "offset":
            o = oracle.can_offset_search(x, 15, G, iters)
            ref_packed = o["packed"]
            parity = float(outo.delta[0]) == float(o["delta"])
        else:
            o = oracle.can_search(x, 0, 15, G, iters)
            ref_packed = oracle.can_quantize_pack_int4(x, [o["scale"]], 0, 15)
            parity = True
            if variant == "residual":
                o2 = oracle.can_act_residual_quantize(x, o["scale"], (0, 15), (-8, 7), G, iters)
                parity = (int(out2.idx[0]) == o2["idx"] and float(out2.scale[0]) == float(o2["scale"])
                          and abs(float(out2.sse[0]) - o2["sse"]) <= 1e-4 * o2["sse"]
                          and np.array_equal(out2.packed.cpu().numpy(), o2["packed"]))
        dt = time.perf_counter() - t0
        cpu_baseline = {"value": evals / dt, "unit": "evals/s", "cores": oracle.num_threads(), "kind": "oracle",
                        "sample": f"the full tensor once ({N} elements): search + codes", "seconds": round(dt, 3)}
        parity = bool(parity and int(out.idx[0]) == o["idx"] and float(out.scale[0]) == float(o["scale"])
                      and abs(float(out.sse[0]) - o["sse"]) <= 1e-4 * o["sse"]
                      and np.array_equal(packed.cpu().numpy(), ref_packed))
    print(json.dumps({
        "metric": METRIC, "value": evals / (ms_per_step * 1e-3), "unit": "evals/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"BASELINE.json configs[{cfg.cfg - 1}] largest activation tensor "
                               f"({cfg.act_shapes[li].name}, batch {cfg.act_batch})",
                   "variant": {"plain": "Eq. 15", "residual": "Eq. 15 then the second tensor of Eq. 16 (signed)",
                               "offset": "Eq. 2 with the MMSE scale (tensor shifted by -0.75)"}[variant],
                   "elements": N, "grid_points": G, "refine_iters": iters, "range": "unsigned INT4 (0..15)",
                   "outputs": "scale, argmin index, sse, packed INT4 codes", "evals_per_step": evals},
        "roofline": roofline, "cpu_baseline": cpu_baseline, "matches_oracle": parity}))
    return 0


def bench_dual(args, cfg, torch, B) -> int:
    """Algorithm 1 iterated (two INT4 tensors per kernel, eps 1e-3, at most 4 sweeps) on every weight tensor."""
    G = args.grid_points if args.grid_points > 0 else cfg.grid_points
    iters = args.refine_iters if args.refine_iters >= 0 else cfg.refine_iters
    eps, max_sweeps = 1e-3, 4
    host_w = [cfg.weight_tensor(i) for i in range(len(cfg.weight_shapes))]
    dev_w = [torch.from_numpy(w).cuda() for w in host_w]
    p = B.params(-8, 7, G, iters, args.cands_per_lane)
    plan = B.DualBatchedPlan(dev_w, p, eps, max_sweeps)
    outs = plan.run()
    step = plan.run

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps
    # evaluations of the sweeps whose result was kept (a lower bound of the work done: a last,
    # discarded sweep is not counted)
    evals = sum(int(o.sweeps.sum().item()) * w.shape[1] * 2 * (G + 2 + iters) for o, w in zip(outs, host_w))
    cpu_baseline, parity = None, None
    if not args.no_cpu_baseline:
        import oracle
        t0 = time.perf_counter()
        sample_evals, ok = 0, True
        for w, o in zip(host_w, outs):
            rows = np.unique(np.linspace(0, w.shape[0] - 1, 8).astype(int))
            ref = oracle.can_dual_alternating(np.ascontiguousarray(w[rows]), -8, 7, G, iters, eps, max_sweeps)
            sample_evals += int(ref["sweeps"].sum()) * w.shape[1] * 2 * (G + 2 + iters)
            ok = ok and np.array_equal(o.sweeps.cpu().numpy()[rows], ref["sweeps"]) \
                and np.array_equal(o.scale1.cpu().numpy()[rows], ref["scale1"]) \
                and np.array_equal(o.scale2.cpu().numpy()[rows], ref["scale2"]) \
                and np.allclose(o.sse.cpu().numpy()[rows], ref["sse"], rtol=1e-4, atol=0)
        dt = time.perf_counter() - t0
        cpu_baseline = {"value": sample_evals / dt, "unit": "evals/s", "cores": oracle.num_threads(), "kind": "oracle",
                        "sample": "8 kernels of every tensor", "seconds": round(dt, 3)}
        parity = bool(ok)
    print(json.dumps({
        "metric": METRIC, "value": evals / (ms_per_step * 1e-3), "unit": "evals/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"BASELINE.json configs[{cfg.cfg - 1}] weights, two INT4 tensors per kernel by "
                               f"alternating optimisation (eps {eps}, <= {max_sweeps} sweeps)",
                   "tensors": len(host_w), "weights": sum(w.size for w in host_w), "grid_points": G,
                   "refine_iters": iters, "evals_per_step_kept_sweeps": evals,
                   "mean_sweeps": float(np.mean(np.concatenate([o.sweeps.cpu().numpy() for o in outs])))},
        "roofline": None, "cpu_baseline": cpu_baseline, "matches_oracle": parity}))
    return 0


def bench_dual_linesearch(args, cfg, torch, B) -> int:
    """Dual line search (Eq. 12) over a G1 x G2 grid of scale pairs for every kernel of at most 8192 weights."""
    G1 = G2 = args.pair_grid
    host_w = [w for w in (cfg.weight_tensor(i) for i in range(len(cfg.weight_shapes))) if w.shape[1] <= 8192]
    dev_w = [torch.from_numpy(w).cuda() for w in host_w]
    ws = [B.alloc_workspace(B.mmse_workspace_bytes_dual_linesearch(w.shape[0], w.shape[1], G1, G2)) for w in host_w]
    outs = [B.dual_line_search(d, -8, 7, G1, G2, ws=s) for d, s in zip(dev_w, ws)]

    def step():
        for d, s, o in zip(dev_w, ws, outs):
            B.dual_line_search(d, -8, 7, G1, G2, ws=s, out=o)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for _ in range(args.steps):
        step()
    e1.record()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps
    gpu_ms = e0.elapsed_time(e1) / args.steps
    weights = sum(w.size for w in host_w)
    pair_evals = weights * G1 * G2                    # (element, scale pair) errors, each a minimum over 16 codes
    code_evals = pair_evals * 16
    ops = pair_evals * (16 * 5.5 + 2)                 # VALU instructions per (element, pair)
    roofline = {"bound": "alu", "kernel": "k_dual_ls (+ pick and codes kernels, < 1 % of the time)",
                "achieved": ops / (gpu_ms * 1e-3) / 1e12, "peak": LANE_OPS_PER_S / 1e12,
                "unit": "T lane-instructions/s", "frac": ops / (gpu_ms * 1e-3) / LANE_OPS_PER_S,
                "avg_step_ms_on_stream": gpu_ms, "traffic": None,
                "note": "5.5 VALU instructions per (element, pair, first code): fma, mul, rndne, med3, fma, half a min3; 2 per (element, pair)"}
    cpu_baseline, parity = None, None
    if not args.no_cpu_baseline:
        import oracle
        t0 = time.perf_counter()
        sample, ok = 0, True
        for w, o in zip(host_w, outs):
            rows = np.unique(np.linspace(0, w.shape[0] - 1, 3).astype(int))
            if w.shape[1] > 1200:
                rows = rows[:1]
            ref = oracle.can_dual_linesearch_kernelwise(np.ascontiguousarray(w[rows]), -8, 7, G1, G2)
            sample += len(rows) * w.shape[1] * G1 * G2 * 16
            ok = ok and all(np.array_equal(getattr(o, k).cpu().numpy()[rows], ref[k])
                            for k in ("scale1", "scale2", "idx1", "idx2", "sse"))
        dt = time.perf_counter() - t0
        cpu_baseline = {"value": sample / dt, "unit": "evals/s", "cores": oracle.num_threads(), "kind": "oracle",
                        "sample": "1 to 3 kernels of every tensor", "seconds": round(dt, 3)}
        parity = bool(ok)
    print(json.dumps({
        "metric": METRIC, "value": code_evals / (ms_per_step * 1e-3), "unit": "evals/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"BASELINE.json configs[{cfg.cfg - 1}] weights, dual line search of two INT4 tensors "
                               f"per kernel over a {G1} x {G2} grid of scale pairs",
                   "tensors": len(host_w), "weights": weights, "pair_grid": [G1, G2],
                   "evals_per_step": code_evals, "eval": "one (element, scale pair, first code) squared error"},
        "roofline": roofline, "cpu_baseline": cpu_baseline, "matches_oracle": parity}))
    return 0


def bench_compare(args, cfg, torch, B) -> int:
    """The four optimisers of Section 3.4 (Table 2) on every weight tensor: total squared error and time."""
    host_w = [cfg.weight_tensor(i) for i in range(len(cfg.weight_shapes))]
    dev_w = [torch.from_numpy(w).cuda() for w in host_w]
    G = args.grid_points if args.grid_points > 0 else cfg.grid_points
    iters = args.refine_iters if args.refine_iters >= 0 else cfg.refine_iters
    energy = sum(float(np.sum(w.astype(np.float64) ** 2)) for w in host_w)
    modes = {"uniform": (1, 0), "golden": (1, iters), "omse": (G, iters)}
    rows = {}

    def timed(fn):
        for _ in range(max(1, args.warmup // 5)):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(max(1, args.steps // 5)):
            out = fn()
        torch.cuda.synchronize()
        return out, (time.perf_counter() - t0) * 1e3 / max(1, args.steps // 5)

    for name, (g, it) in modes.items():
        plan = B.BatchedPlan(dev_w, B.params(-8, 7, g, it), want_packed=False)
        res, ms = timed(plan.run)
        rows[name] = {"sse": sum(float(r.sse.sum().item()) for r in res), "ms": ms}
    res, ms = timed(lambda: [B.mmse_scale_alternating_kernelwise(d, -8, 7, 50) for d in dev_w])
    rows["alternating"] = {"sse": sum(float(r[1].sum().item()) for r in res), "ms": ms,
                           "mean_updates": float(np.mean(np.concatenate([r[2].cpu().numpy() for r in res])))}
    for r in rows.values():
        r["normalized_mse"] = r["sse"] / energy
    cpu_baseline, parity = None, None
    if not args.no_cpu_baseline:
        import oracle
        t0 = time.perf_counter()
        ok = True
        for w, r in zip(host_w, res):
            sel = np.unique(np.linspace(0, w.shape[0] - 1, 16).astype(int))
            rs, re, ru = oracle.can_alternating_scale_kernelwise(np.ascontiguousarray(w[sel]), -8, 7, 50)
            ok = ok and np.array_equal(r[0].cpu().numpy()[sel], rs) and np.array_equal(r[2].cpu().numpy()[sel], ru)
        cpu_baseline = {"kind": "oracle", "sample": "16 kernels of every tensor, alternating mode",
                        "seconds": round(time.perf_counter() - t0, 3), "cores": oracle.num_threads(), "value": None,
                        "unit": "evals/s"}
        parity = bool(ok)
    print(json.dumps({
        "metric": METRIC, "value": None, "unit": "evals/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": rows["omse"]["ms"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"BASELINE.json configs[{cfg.cfg - 1}] weights under the four optimisers of Section 3.4",
                   "grid_points": G, "refine_iters": iters, "alternating_max_updates": 50},
        "modes": rows, "roofline": None, "cpu_baseline": cpu_baseline, "matches_oracle": parity}))
    return 0


def _stage_table(rows):
    """Aggregate [(stage, ms)] lists of several traced calls: stage -> (launches per call, ms per call)."""
    agg = {}
    for tr in rows:
        for st, ms in tr:
            c, t = agg.get(st, (0, 0.0))
            agg[st] = (c + 1, t + ms)
    n = max(1, len(rows))
    return {st: (c / n, t / n) for st, (c, t) in agg.items()}


def _traffic_table():
    """profiles/hbm_traffic.txt: kernel, workload, fetched bytes, written bytes per launch (rocprofv3 --pmc
    FETCH_SIZE / WRITE_SIZE, scaled by a device copy of known size in the same run)."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.txt")
    out = {}
    if os.path.exists(path):
        for line in open(path):
            f = line.split("#")[0].split()
            if len(f) == 4:
                out[(f[0], f[1])] = (float(f[2]), float(f[3]))
    return out


def _alu_entry(name, evals, launches, ms_total, traffic=None):
    lane_ops = evals * OPS_PER_EVAL / (ms_total * 1e-3)
    tflops = evals * FLOPS_PER_EVAL / (ms_total * 1e-3) / 1e12
    peak = LANE_OPS_PER_S * FLOPS_PER_EVAL / OPS_PER_EVAL / 1e12
    return {"bound": "alu", "kernel": name, "achieved": round(tflops, 3), "peak": round(peak, 3), "unit": "TFLOP/s",
            "frac": round(lane_ops / LANE_OPS_PER_S, 4), "traffic": traffic,
            "launches_per_step": launches, "avg_launch_ms": round(ms_total / max(launches, 1e-9), 5),
            "evals_per_launch": evals / max(launches, 1e-9), "evals_per_s": evals / (ms_total * 1e-3),
            "frac_of_157.3_tflops": round(tflops / 157.3, 4)}


def _hbm_entry(name, nbytes, launches, ms_total, traffic=None):
    gbs = nbytes / (ms_total * 1e-3) / 1e9
    return {"bound": "hbm", "kernel": name, "achieved": round(gbs, 1), "peak": HBM_GBS, "unit": "GB/s",
            "frac": round(gbs / HBM_GBS, 4), "traffic": traffic, "launches_per_step": launches,
            "avg_launch_ms": round(ms_total / max(launches, 1e-9), 5),
            "algorithmic_bytes_per_launch": nbytes / max(launches, 1e-9)}


def _nibbles(packed: np.ndarray, count: int) -> np.ndarray:
    out = np.empty(packed.size * 2, dtype=np.uint8)
    out[0::2] = packed & 0xF
    out[1::2] = packed >> 4
    return out[:count]


def run_whole(args, cfg, torch, B, detail: bool, steps: int, warmup: int) -> dict:
    """Everything the configuration names, first enqueue to last kernel: weights (search + codes), the second
    tensor on the selected layers, and search + codes of every layer's calibration activations."""
    from paper_1902_06822_amd import select
    G = args.grid_points if args.grid_points > 0 else cfg.grid_points
    iters = args.refine_iters if args.refine_iters >= 0 else cfg.refine_iters
    t_gen = time.perf_counter()
    host_w = [cfg.weight_tensor(i) for i in range(len(cfg.weight_shapes))]
    dev_w = [torch.from_numpy(w).cuda() for w in host_w]
    nlayers = len(dev_w)
    nkey = nlayers if cfg.residual == "all" else (max(1, round(0.10 * nlayers)) if cfg.residual == "top10pct" else 0)
    energy = [float(np.sum(w.astype(np.float64) ** 2)) for w in host_w] if cfg.residual == "top10pct" else []   # constants of the network
    keep_host = detail and not args.no_cpu_baseline
    host_w_shapes = [w.shape for w in host_w]
    if not keep_host:
        host_w = None
    dev_x, host_x = [], []
    for i in range(len(cfg.act_shapes)):
        x = cfg.act_tensor(i)
        dev_x.append(torch.from_numpy(x).cuda())
        host_x.append(x if keep_host else None)
    print(f"bench.py: configuration {cfg.cfg}: inputs generated in {time.perf_counter() - t_gen:.1f} s",
          file=sys.stderr, flush=True)
    pw = B.params(-8, 7, G, iters, args.cands_per_lane)
    pa = B.params(0, 15, G, iters, args.cands_per_lane)
    plan_w = B.BatchedPlan(dev_w, pw, want_packed=True)
    fixed_key = list(range(nlayers)) if cfg.residual == "all" else None
    # second tensor: one plan over all layers, run whole (configuration 5) or, in one call, for the layers the
    # ranking picks (configuration 4); every buffer exists before the timed region
    res_all = B.BatchedPlan(dev_w, pw, want_packed=True, scale1=[r.scale for r in plan_w.results]) if nkey else None
    plan_sums = B.LayerSumsPlan([r.sse for r in plan_w.results]) if (nkey and not fixed_key) else None
    side = torch.cuda.Stream()
    order = sorted(range(len(dev_x)), key=lambda i: -dev_x[i].numel())            # large tensors first
    plan_a, act_out = None, []
    if dev_x:
        plan_a = B.ActBatchedPlan([dev_x[i] for i in order], pa, want_packed=True)
        act_out = [None] * len(dev_x)
        for n_, i in enumerate(order):
            act_out[i] = plan_a.results[n_]
    key_used = []

    def step():
        main = torch.cuda.current_stream()
        if plan_a is not None and not args.serial:
            # activations on a side stream while the weight path runs on the main stream
            start = torch.cuda.Event()
            start.record(main)
            side.wait_event(start)
            with torch.cuda.stream(side):
                plan_a.run()
        elif plan_a is not None:
            plan_a.run()
        plan_w.run()
        if fixed_key:
            res_all.run()
        elif nkey:
            sums = plan_sums.run().cpu().numpy()           # one small kernel, one device-to-host copy; the ranking is host logic
            key = select.select_top_fraction(select.normalized_mse(list(sums), energy), 0.10)
            key_used[:] = key
            res_all.run_subset(key)
        if plan_a is not None and not args.serial:
            main.wait_stream(side)

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / steps
    P = G + 2 + iters
    w_elems = sum(K * n for K, n in host_w_shapes)
    key_elems = w_elems if fixed_key else sum(host_w_shapes[i][0] * host_w_shapes[i][1] for i in key_used)
    a_elems = sum(x.numel() for x in dev_x)
    evals = (w_elems + key_elems + a_elems) * P
    out = {"ms_per_step": ms_per_step, "evals_per_step": evals, "value": evals / (ms_per_step * 1e-3),
           "config": {"workload": f"BASELINE.json configs[{cfg.cfg - 1}] whole network ({cfg.name}): kernel-wise weight "
                                  f"search + codes, second tensor ({cfg.residual}), search + codes of all calibration "
                                  f"activations",
                      "weight_tensors": nlayers, "weights": w_elems,
                      "second_tensor_layers": (nlayers if fixed_key else list(key_used)),
                      "activation_tensors": len(dev_x), "activation_elements": a_elems, "grid_points": G,
                      "refine_iters": iters, "ranges": "weights signed INT4 (-8..7), activations unsigned INT4 (0..15)",
                      "streams": "one" if (args.serial or plan_a is None) else "weights on the main stream, activations on a side stream",
                      "evals_per_step": evals,
                      "evals_counted": "every element x candidate of the definition; the activation sweep does not issue "
                                       "the evaluations of zero elements (their term is zero at every scale)"}}

    # ---- the scales back on the host (not part of a step: the results stay on the device)
    scales = [r.scale for r in plan_w.results] + ([r.scale for r in res_all.results] if res_all is not None else []) \
        + [r.scale for r in act_out]
    d2h = []
    for _ in range(3):
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        host_scales = torch.cat(scales).cpu()
        d2h.append((time.perf_counter() - t1) * 1e3)
    out["d2h_scales_ms"] = {"median_ms": sorted(d2h)[1], "floats": int(host_scales.numel()),
                            "note": "all scales of the network gathered on the device and copied to the host; outside the timed step"}

    # ---- every kernel by itself: the weight path, the second tensor and the activation path one after the other on
    # one stream, HIP events on that stream around every launch (mmse_trace_*)
    reps = max(3, min(10, steps))
    trace = B.StageTrace(512)
    traffic = _traffic_table()
    wl = f"cfg{cfg.cfg}"

    def traced(plan):
        rows = []
        for _ in range(2):                  # untimed: the host work since the timed steps let the clock drop
            plan.run()
        for _ in range(reps):
            plan.run_traced(trace)
            rows.append(trace.read())
        return _stage_table(rows)

    kernels = []
    tw = traced(plan_w)
    sw_l = tw.get(1, (0, 0.0))[0] + tw.get(2, (0, 0.0))[0] + tw.get(6, (0, 0.0))[0]
    sw_ms = tw.get(1, (0, 0.0))[1] + tw.get(2, (0, 0.0))[1] + tw.get(6, (0, 0.0))[1]
    def tr_of(kernel):
        t = traffic.get((kernel, wl))
        return (t[0] + t[1]) if t else None

    e_w = _alu_entry("k_sweep_kernelwise: abs-max, grid sweep, argmin of all weight tensors",
                     w_elems * G, sw_l, sw_ms, tr_of("k_sweep_kernelwise"))
    kernels.append(e_w)
    rf_l = tw.get(3, (0, 0.0))[0] + tw.get(4, (0, 0.0))[0]
    rf_ms = tw.get(3, (0, 0.0))[1] + tw.get(4, (0, 0.0))[1]
    if rf_l:
        kernels.append(_alu_entry("k_refine_kernelwise: golden-section refinement (+ codes) of all weight tensors",
                                  w_elems * (2 + iters), rf_l, rf_ms))
    weights_alone_ms = sum(t for _, t in tw.values())
    second_alone_ms = 0.0
    if fixed_key:
        tr2 = traced(res_all)
        l2 = tr2.get(1, (0, 0.0))[0] + tr2.get(2, (0, 0.0))[0]
        m2 = tr2.get(1, (0, 0.0))[1] + tr2.get(2, (0, 0.0))[1]
        kernels.append(_alu_entry("k_sweep_kernelwise on the residual of the first tensor (second tensor, all layers)",
                                  w_elems * G, l2, m2, tr_of("k_sweep_kernelwise")))
        second_alone_ms = sum(t for _, t in tr2.values())
    acts_alone_ms = 0.0
    hbm = []
    if plan_a is not None:
        ta = traced(plan_a)
        acts_alone_ms = sum(t for _, t in ta.values())
        l, m = ta[12]
        # the sweep drops zero elements while staging (a zero adds nothing to a chunk's sum at any scale), so its
        # roofline counts the evaluations of the non-zero elements; the dense count is given beside it
        a_nonzero = sum(int(torch.count_nonzero(x).item()) for x in dev_x)
        # what a refinement pass reads: the copy the sweep leaves in the workspace, every 64-element chunk's non-zero
        # elements zero-filled to a multiple of eight, 4096-element blocks with 64 words about their chunks each
        a_compact_bytes = 0
        for x in dev_x:
            f = x.reshape(-1)
            pad = (-f.numel()) % 64
            if pad:
                f = torch.cat([f, f.new_zeros(pad)])
            nz = (f.view(-1, 64) != 0).sum(dim=1)
            a_compact_bytes += int((((nz + 7) // 8) * 8).sum().item()) * 4 + ((x.numel() + 4095) // 4096) * 256
        e_a = _alu_entry("k_act_sweep: grid sweep of all activation tensors", a_nonzero * G, l, m, tr_of("k_act_sweep"))
        e_a["counted"] = "evaluations of non-zero elements (zero elements are dropped while staging)"
        issued = (w_elems + key_elems + a_nonzero) * P
        out["issued"] = {"evals_per_step": issued, "evals_per_s": issued / (ms_per_step * 1e-3),
                         "note": "the same step counting only the evaluations the kernels issue: those of zero "
                                 "activation elements left out"}
        e_a["nonzero_fraction"] = round(a_nonzero / max(a_elems, 1), 4)
        e_a["dense_evals_per_launch"] = a_elems * G / max(l, 1e-9)
        e_a["dense_equivalent_frac"] = round(a_elems * G * OPS_PER_EVAL / (m * 1e-3) / LANE_OPS_PER_S, 4)
        kernels.append(e_a)
        l, m = ta[11]
        hbm.append(_hbm_entry("k_act_absmax: max |x| of every activation tensor", 4.0 * a_elems, l, m, tr_of("k_act_absmax")))
        if 15 in ta:
            l, m = ta[15]
            hbm.append(_hbm_entry("k_act_probe: one refinement pass over the compacted copy of every activation tensor "
                                  "(up to 8 scales per non-zero element)",
                                  1.0 * a_compact_bytes * l, l, m, tr_of("k_act_probe")))
            hbm[-1]["dense_bytes_per_launch"] = 4.0 * a_elems
            if iters == 20:      # 2+2+4 scales per element in the first pass, 1+2+4 in each of the others
                ev = (8 + 7 * (l - 1)) * a_nonzero
                hbm[-1]["scales_evaluated_per_element"] = 8 + 7 * (round(l) - 1)
                hbm[-1]["alu_frac"] = round(ev * OPS_PER_EVAL / (m * 1e-3) / LANE_OPS_PER_S, 4)
        l, m = ta[18]
        hbm.append(_hbm_entry("k_act_pack: INT4 codes of every activation tensor", 4.5 * a_elems, l, m, tr_of("k_act_pack")))
    trace.close()
    dominant = max(kernels, key=lambda e: e["avg_launch_ms"] * e["launches_per_step"])
    roofline = dict(dominant)
    roofline["note"] = ("alu peak = 256 CUs x 4 SIMDs x 32 lanes/clk x 2.4 GHz = 78.6e12 VALU lane-ops/s (= 157.3 TFLOP/s fp32 "
                        "vector when every instruction is an FMA); an evaluation is 5 instructions / 7 flops, so the peak in "
                        "flops of this mix is 110.1 TFLOP/s; frac = algorithmic lane-ops/s (5 per evaluation) over 78.6e12.  "
                        "The sweeps leave the saturation (v_med3) out for chunks whose largest magnitude stays inside the "
                        "integer range at the smallest scale of a wave, where it is the identity: they issue 8-13 % fewer "
                        "instructions than 5 per evaluation (counts in profiles/), which frac does not discount.  The activation "
                        "sweep also drops zero elements while staging (they add nothing to a sum at any scale): its frac "
                        "counts the evaluations of non-zero elements only, and dense_equivalent_frac all of them.  Each "
                        "kernel timed by itself between HIP events on its launch stream, after the timed steps.")
    roofline["traffic_note"] = ("fetched + written bytes per launch at the memory side of L2, from rocprofv3 --pmc FETCH_SIZE / "
                                "WRITE_SIZE runs of this command (profiles/hbm_traffic.txt); algorithmic bytes: 4 per element read "
                                "once, plus 8 * grid_points per 4096 elements and the compacted copy written by k_act_sweep; "
                                "k_act_probe reads that copy")
    roofline["all_alu_kernels"] = kernels
    roofline["hbm"] = hbm
    roofline["hbm_note"] = (f"activation set {4 * a_elems / 1e6:.0f} MB, read once per pass (refinement passes: its compacted copy); the chip's last-level cache is 256 MB"
                            if dev_x else "no activation tensors in this configuration")
    out["roofline"] = roofline
    out["alone_ms"] = {"weights": round(weights_alone_ms, 4), "second_tensor": round(second_alone_ms, 4),
                       "activations": round(acts_alone_ms, 4),
                       "note": "each path by itself on one stream (sum of its kernels between events)"}

    # ---- CPU oracle (reported baseline, not the target) on a bounded sample of the same workload, and parity on it
    out["cpu_baseline"], out["matches_oracle"] = None, None
    if keep_host:
        import oracle
        step()
        torch.cuda.synchronize()
        every = max(1, args.cpu_sample_every)
        ok, sample = True, 0
        secs = 0.0
        for i, w in enumerate(host_w):
            K, n = w.shape
            rows = np.arange(i % every, K, every)
            if rows.size == 0:
                continue
            wr = np.ascontiguousarray(w[rows])
            r1 = plan_w.results[i]
            g_s, g_j, g_e = r1.scale.cpu().numpy(), r1.idx.cpu().numpy(), r1.sse.cpu().numpy()
            g_nib = _nibbles(r1.packed.cpu().numpy(), K * n).reshape(K, n)[rows]
            t0 = time.perf_counter()
            s1, j1, e1 = oracle.can_search_kernelwise(wr, -8, 7, G, iters)
            pk = oracle.can_quantize_pack_int4(wr, s1, -8, 7)
            secs += time.perf_counter() - t0
            sample += wr.size * P
            ok = ok and np.array_equal(g_s[rows], s1) and np.array_equal(g_j[rows], j1) \
                and np.allclose(g_e[rows], e1, rtol=1e-4, atol=0) \
                and np.array_equal(g_nib, _nibbles(pk, wr.size).reshape(rows.size, n))
            r2 = res_all.results[i] if (fixed_key or i in key_used) else None
            if r2 is not None:
                g2_nib = _nibbles(r2.packed.cpu().numpy(), K * n).reshape(K, n)[rows]
                t0 = time.perf_counter()
                s2, j2, e2, p2 = oracle.can_residual_quantize(wr, s1, -8, 7, G, iters)
                secs += time.perf_counter() - t0
                sample += wr.size * P
                ok = ok and np.array_equal(r2.scale.cpu().numpy()[rows], s2) and np.array_equal(r2.idx.cpu().numpy()[rows], j2) \
                    and np.allclose(r2.sse.cpu().numpy()[rows], e2, rtol=1e-4, atol=0) \
                    and np.array_equal(g2_nib, _nibbles(p2, wr.size).reshape(rows.size, n))
        act_sampled = []
        for n_, i in enumerate(order):                       # every `every`-th tensor in size order
            if n_ % every != (1 % every):
                continue
            x = host_x[i]
            g = act_out[i]
            t0 = time.perf_counter()
            o = oracle.can_search(x, 0, 15, G, iters)
            pk = oracle.can_quantize_pack_int4(x, [o["scale"]], 0, 15)
            secs += time.perf_counter() - t0
            sample += x.size * P
            act_sampled.append(cfg.act_shapes[i].name)
            ok = ok and (float(g.scale[0]), int(g.idx[0])) == (float(o["scale"]), o["idx"]) \
                and abs(float(g.sse[0]) - o["sse"]) <= 1e-4 * o["sse"] and np.array_equal(g.packed.cpu().numpy(), pk)
        what = "the full workload: first and second tensor of every weight kernel and every activation tensor, search + codes" if every == 1 else \
            (f"every {every}th kernel of every weight tensor (first and second tensor, codes included) and "
             f"{len(act_sampled)} of {len(dev_x)} activation tensors ({', '.join(act_sampled)}; search + codes)")
        out["cpu_baseline"] = {"value": sample / secs, "unit": "evals/s", "cores": oracle.num_threads(), "kind": "oracle",
                               "sample": what, "sample_evals": sample, "seconds": round(secs, 3)}
        out["matches_oracle"] = bool(ok)
    return out


def bench_whole(args, cfg, torch, B) -> int:
    res = run_whole(args, cfg, torch, B, detail=True, steps=args.steps, warmup=args.warmup)
    others = {}
    if not args.headline_only:
        from paper_1902_06822_amd import synth
        import gc
        for c in (1, 2, 3, 4):
            if c == cfg.cfg:
                continue
            gc.collect()
            torch.cuda.empty_cache()
            ocfg = synth.config(c)
            big = c == 4
            r = run_whole(args, ocfg, torch, B, detail=False, steps=(args.steps if big else 10 * args.steps),
                          warmup=(args.warmup if big else 10 * args.warmup))
            alu = r["roofline"]["all_alu_kernels"]
            others[f"configs[{c - 1}]"] = {
                "workload": r["config"]["workload"], "ms_per_step": r["ms_per_step"], "evals_per_s": r["value"],
                "evals_per_step": r["evals_per_step"], "issued": r.get("issued"), "alone_ms": r["alone_ms"],
                "alu_frac_by_kernel": {e["kernel"].split(":")[0]: e["frac"] for e in alu},
                "hbm_frac_by_kernel": {e["kernel"].split(":")[0]: e["frac"] for e in r["roofline"]["hbm"]},
                "second_tensor_layers": r["config"]["second_tensor_layers"]}
    print(json.dumps({
        "metric": METRIC, "value": res["value"], "unit": "evals/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": res["ms_per_step"], "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": res["config"], "issued": res.get("issued"), "alone_ms": res["alone_ms"],
        "d2h_scales_ms": res["d2h_scales_ms"],
        "roofline": res["roofline"],
        "cpu_baseline": res["cpu_baseline"], "matches_oracle": res["matches_oracle"],
        "other_configs": others}))
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10,
                    help="untimed steps; the GPU needs some tens of milliseconds of work to reach its steady clock")
    ap.add_argument("--config", type=int, default=0,
                    help="BASELINE.json configuration, 1..5 (default: 5 for --part whole, 2 for the other parts)")
    ap.add_argument("--headline-only", action="store_true",
                    help="--part whole: skip the short runs of the other configurations (the other_configs key)")
    ap.add_argument("--cpu-sample-every", type=int, default=1,
                    help="--part whole: 1 = the oracle runs on the full workload (about 10 s on 16 host threads); "
                         "n > 1 = on every n-th kernel of every weight tensor and every n-th activation tensor")
    ap.add_argument("--cands-per-lane", type=int, default=0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--part", choices=("weights", "activation", "dual", "dual-ls", "compare", "whole"), default="whole",
                    help="whole (default): everything the configuration names, end to end; weights: the kernel-wise "
                         "path alone; activation: the largest calibration tensor through the per-layer path; "
                         "dual, dual-ls, compare: the two-tensor methods and the comparison optimisers")
    ap.add_argument("--copy-calibration-mib", type=int, default=0,
                    help="also run plain device copies of this many MiB (for scaling FETCH_SIZE/WRITE_SIZE "
                         "counters under rocprofv3 --pmc); not part of any timed region")
    ap.add_argument("--pair-grid", type=int, default=32, help="G1 = G2 of --part dual-ls")
    ap.add_argument("--act-variant", choices=("plain", "residual", "offset"), default="plain",
                    help="--part activation: the per-layer search alone, with the second tensor, or in offset form")
    ap.add_argument("--serial", action="store_true", help="--part whole: activations and weights one after the other on one stream")
    ap.add_argument("--grid-points", type=int, default=0, help="override G of the configuration")
    ap.add_argument("--refine-iters", type=int, default=-1, help="override the refinement iterations")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no sharding, no collectives); "
              f"--gpus {args.gpus} is not supported", file=sys.stderr)
        return 2

    import torch
    from paper_1902_06822_amd import binding as B, synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; there is no CPU fallback", file=sys.stderr)
        return 3
    B.load_library()
    torch.cuda.set_device(0)

    if args.copy_calibration_mib > 0:
        src = torch.ones(args.copy_calibration_mib * (1 << 20) // 4, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    if args.config == 0:
        args.config = 5 if args.part == "whole" else 2
    cfg = synth.config(args.config)
    if args.part == "activation":
        return bench_activation(args, cfg, torch, B)
    if args.part == "dual":
        return bench_dual(args, cfg, torch, B)
    if args.part == "dual-ls":
        return bench_dual_linesearch(args, cfg, torch, B)
    if args.part == "compare":
        return bench_compare(args, cfg, torch, B)
    if args.part == "whole":
        return bench_whole(args, cfg, torch, B)
    G = args.grid_points if args.grid_points > 0 else cfg.grid_points
    iters = args.refine_iters if args.refine_iters >= 0 else cfg.refine_iters
    host_w = [cfg.weight_tensor(i) for i in range(len(cfg.weight_shapes))]
    dev_w = [torch.from_numpy(w).cuda() for w in host_w]
    elements = sum(w.size for w in host_w)
    evals_per_step = elements * (G + 2 + iters)
    p = B.params(-8, 7, G, iters, args.cands_per_lane)
    plan = B.BatchedPlan(dev_w, p, want_packed=True)
    torch.cuda.synchronize()

    # ---- whole path
    for _ in range(args.warmup):
        plan.run()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        plan.run()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    value = evals_per_step / (ms_per_step * 1e-3)

    # ---- the same step, one at a time between HIP events on the launch stream: median and minimum
    nrep = max(20, min(args.steps, 100))
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(nrep)]
    for a, b in evs:
        a.record()
        plan.run()
        b.record()
    torch.cuda.synchronize()
    per_step = sorted(a.elapsed_time(b) for a, b in evs)
    step_stats = {"runs": nrep, "median_ms": per_step[nrep // 2], "min_ms": per_step[0]}
    # outputs stay on the device; what it costs to bring scales, indices and errors to the host, reported apart
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for r in plan.results:
        r.scale.cpu(); r.idx.cpu(); r.sse.cpu()
    step_stats["d2h_scales_idx_sse_ms"] = (time.perf_counter() - t0) * 1e3

    # ---- dominant kernel alone: grid sweep + argmin (refine_iters = 0, no packing => one kernel per launch)
    p_sweep = B.params(-8, 7, G, 0, args.cands_per_lane)
    sweep_plan = B.BatchedPlan(dev_w, p_sweep, want_packed=False)
    trace = B.StageTrace(256)
    sweep_plan.run_traced(trace)
    nlaunch = len(trace.read())                 # sweep launches of one call (general and small-kernel passes)
    trace.close()
    for _ in range(max(1, args.warmup)):
        sweep_plan.run()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    ev0.record()
    for _ in range(args.steps):
        sweep_plan.run()
    ev1.record()
    torch.cuda.synchronize()
    sweep_ms = ev0.elapsed_time(ev1) / args.steps          # per step = nlaunch launches
    sweep_evals = elements * G
    lane_ops = sweep_evals * OPS_PER_EVAL / (sweep_ms * 1e-3)
    achieved_tflops = sweep_evals * FLOPS_PER_EVAL / (sweep_ms * 1e-3) / 1e12
    peak_tflops = LANE_OPS_PER_S * FLOPS_PER_EVAL / OPS_PER_EVAL / 1e12
    roofline = {
        "bound": "alu",
        "kernel": "k_sweep_kernelwise",
        "achieved": round(achieved_tflops, 3),
        "peak": round(peak_tflops, 3),
        "unit": "TFLOP/s",
        "frac": round(achieved_tflops / peak_tflops, 4),
        # HBM-side bytes per step from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs (profiles/hbm_traffic.txt)
        "traffic": (lambda t: (t[0] + t[1]) if t else None)(_traffic_table().get(("k_sweep_kernelwise", f"cfg{args.config}"))
                                                            if args.grid_points == 0 else None),
        "traffic_note": "fetched + written bytes per launch at the memory side of L2 (profiles/hbm_traffic.txt)",
        "algorithmic_bytes": 4 * elements,
        "avg_launch_ms": round(sweep_ms / nlaunch, 5),
        "launches_per_step": nlaunch,
        "evals_per_s": sweep_evals / (sweep_ms * 1e-3),
        "lane_ops_per_s": lane_ops,
        "peak_lane_ops_per_s": LANE_OPS_PER_S,
        "note": "peak = 157.3 TFLOP/s fp32 vector (78.6e12 VALU lane-ops/s) x 7 flops per 10 flop-slots of the "
                "5-instruction eval (mul, rndne, med3, fma, fma); frac = lane-ops/s over 78.6e12",
        "frac_of_157.3_tflops": round(achieved_tflops / 157.3, 4),
    }

    # ---- CPU oracle on the same inputs (reported baseline, not the target)
    cpu_baseline = None
    parity = None
    if not args.no_cpu_baseline:
        import oracle
        res = plan.run()
        torch.cuda.synchronize()
        times = []
        for _ in range(3 if elements < 50_000_000 else 1):            # a fraction of a second per run: take the median
            t0 = time.perf_counter()
            ref = [oracle.can_search_kernelwise(w, -8, 7, G, iters) for w in host_w]
            ref_packed = [oracle.can_quantize_pack_int4(w, r[0], -8, 7) for w, r in zip(host_w, ref)]
            times.append(time.perf_counter() - t0)
        dt = sorted(times)[len(times) // 2]
        cpu_baseline = {
            "value": evals_per_step / dt,
            "unit": "evals/s",
            "cores": oracle.num_threads(),
            "kind": "oracle",
            "sample": f"the full workload ({len(host_w)} tensors, {elements} weights): search + codes, "
                      f"median of {len(times)} run(s)",
            "seconds": round(dt, 3),
        }
        parity = all(
            np.array_equal(g.idx.cpu().numpy(), r[1]) and np.array_equal(g.scale.cpu().numpy(), r[0])
            and np.allclose(g.sse.cpu().numpy(), r[2], rtol=1e-4, atol=0)
            and np.array_equal(g.packed.cpu().numpy(), pk)
            for g, r, pk in zip(res, ref, ref_packed))

    out = {
        "metric": METRIC,
        "value": value,
        "unit": "evals/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {
            "workload": f"BASELINE.json configs[{args.config - 1}]: {cfg.name}",
            "tensors": len(host_w), "weights": elements, "grid_points": G, "refine_iters": iters,
            "range": "signed INT4 (-8..7)", "outputs": "scale, argmin index, sse, packed INT4 codes",
            "evals_per_step": evals_per_step, "cands_per_lane": args.cands_per_lane,
        },
        "step_ms_by_events": step_stats,
        "roofline": roofline,
        "cpu_baseline": cpu_baseline,
        "matches_oracle": parity,
    }
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
