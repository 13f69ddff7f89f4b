#!/usr/bin/env python3
"""Benchmark of the MMSE INT4 scale search on one MI355X.

A "step" is one pass of the whole hot path over one network's weights: per-kernel
abs-max, G-point grid sweep, argmin, golden-section refinement and packed INT4
codes for every tensor of the configuration (default: the ResNet-18-shaped
configuration 2 of the benchmark spec; 11.7 M weights, G = 256, 20 refinement
iterations), through ``mmse_scale_search_batched``.  Inputs are resident in HBM
before the timed region starts.

Prints ONE JSON line (see the keys below).  ``roofline`` times the dominant
kernel (the grid sweep) by itself with HIP events on the launch stream;
``cpu_baseline`` times the CPU oracle on the same inputs on the host cores.
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


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=2, help="BASELINE.json configuration (weights part)")
    ap.add_argument("--cands-per-lane", type=int, default=0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
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

    cfg = synth.config(args.config)
    G, iters = cfg.grid_points, cfg.refine_iters
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

    # ---- dominant kernel alone: grid sweep + argmin (refine_iters = 0, no packing => one kernel per launch)
    p_sweep = B.params(-8, 7, G, 0, args.cands_per_lane)
    sweep_plan = B.BatchedPlan(dev_w, p_sweep, want_packed=False)
    nlaunch = (len(dev_w) + 31) // 32
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
        "traffic": None,
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
        t0 = time.perf_counter()
        ref = [oracle.can_search_kernelwise(w, -8, 7, G, iters) for w in host_w]
        ref_packed = [oracle.can_quantize_pack_int4(w, r[0], -8, 7) for w, r in zip(host_w, ref)]
        dt = time.perf_counter() - t0
        cpu_baseline = {
            "value": evals_per_step / dt,
            "unit": "evals/s",
            "cores": oracle.num_threads(),
            "kind": "oracle",
            "sample": f"the full workload once ({len(host_w)} tensors, {elements} weights): search + codes",
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
        "roofline": roofline,
        "cpu_baseline": cpu_baseline,
        "matches_oracle": parity,
    }
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
