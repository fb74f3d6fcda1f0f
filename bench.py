#!/usr/bin/env python3
"""Benchmark of the AAAC hot path on one MI355X.

A step is one pass of the whole path over one synthetic layer that is already
resident in HBM: aaac_act_stats (importance from the calibration activations),
aaac_fit (scales + all Lloyd iterations), aaac_encode, aaac_dequant.  The
workload at --gpus 1 is the Llama-2-7B-shaped q_proj setting (4096x4096 bf16,
65,536 calibration tokens, INT4 group 128, 20 iterations).

Prints one JSON line.  `value` is weight-iterations per second over the whole
step (N*K*iterations / step time).  `roofline` describes the Lloyd-iteration
kernel: its average duration is measured with HIP events on the launch stream
around every aaac_fit call inside the timed region (fit time / iterations, so
launch gaps and the small scale / table kernels count against it).
`cpu_baseline` is the CPU oracle, single-threaded, on the same layer.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

# Algorithmic cost of one Lloyd iteration per weight: 2 bytes of bf16 weight plus
# the group's reciprocal scale (4 bytes per group), and 33 vector-ALU lane
# operations (unpack 1, normalise 1, two 4-level searches 16, two table look-ups 2,
# two error chains 8, selection/bin 1, fp64 accumulate 4).
LANE_OPS_PER_WEIGHT = 33.0
ALU_PEAK_TLANEOPS = 256 * 64 * 2.4e9 / 1e12  # 256 CUs x 64 lanes x 2.4 GHz, one op per lane-clock
HBM_PEAK_GBS = 8000.0


def bytes_per_weight(g):
    return 2.0 + 4.0 / g


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=1, help="index into the benchmark settings (single-layer ones)")
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip the oracle timing (profiling runs)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one plain 1 GiB device copy (reference for HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (the path has no multi-GPU part); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import paper_2605_08692_amd as A
    from paper_2605_08692_amd import inputs

    A.library()  # no fallback: fails here if the HIP library is missing
    dev = "cuda:0"
    torch.cuda.set_device(0)
    cfg = inputs.CONFIGS[args.config]
    assert len(cfg["layers"]) == 1, "bench.py times the single-layer settings"
    layer = cfg["layers"][0]
    g, fmt, iters = cfg["g"], cfg["fmt"], cfg["iters"]
    N, K = layer["N"], layer["K"]
    W = inputs.layer_weights(layer, dev)
    X = inputs.activations(cfg["xs"][layer["x"]], dev)
    grid = inputs.format_grid(fmt)

    # every buffer is allocated once, outside the timed region
    I = torch.empty(K, dtype=torch.float32, device=dev)
    ws_stats = torch.empty(max(A.aaac_act_stats_workspace(X.shape[0], K), 256), dtype=torch.uint8, device=dev)
    ws_fit = torch.empty(A.aaac_fit_workspace(N, K, g, fmt), dtype=torch.uint8, device=dev)
    tf = torch.empty(32, dtype=torch.float32, device=dev)
    tb = torch.empty(32, dtype=torch.int16, device=dev)
    obj = torch.empty(iters, dtype=torch.float64, device=dev)
    codes = torch.empty((N, K // 2), dtype=torch.uint8, device=dev)
    scales = torch.empty((N, K // g), dtype=torch.uint8 if fmt == A.NVFP4 else torch.int16, device=dev)
    What = torch.empty((N, K), dtype=torch.bfloat16, device=dev)
    stream = torch.cuda.current_stream()

    def step(events=None):
        def mark(i):
            if events is not None:
                events[i].record(stream)
        mark(0)
        A.aaac_act_stats(X, I, ws_stats, stream)
        mark(1)
        A.aaac_fit(W, g, fmt, I, grid, iters, tf, tb, obj, ws_fit, stream)
        mark(2)
        A.aaac_encode(W, g, fmt, I, tb, codes, scales, stream)
        mark(3)
        A.aaac_dequant(codes, scales, tb, g, fmt, What, stream)
        mark(4)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(5)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(args.steps):
        step(evs[s])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / args.steps

    def stage(i):
        return float(np.mean([e[i].elapsed_time(e[i + 1]) for e in evs]))
    stats_ms, fit_ms, enc_ms, deq_ms = stage(0), stage(1), stage(2), stage(3)
    iter_us = fit_ms * 1e3 / iters
    n_w = N * K
    weights_per_s_iter = n_w / (iter_us * 1e-6)
    value = n_w * iters / (ms_per_step * 1e-3)

    if args.copy_calibration:
        a = torch.empty(1 << 28, dtype=torch.float32, device=dev)
        b = torch.empty_like(a)
        b.copy_(a)
        torch.cuda.synchronize()

    traffic = None
    tpath = os.path.join(ROOT, "profiles", f"traffic_lloyd_iter_cfg{args.config}.json")
    if os.path.exists(tpath):
        traffic = json.load(open(tpath)).get("hbm_bytes_per_launch")

    achieved = LANE_OPS_PER_WEIGHT * weights_per_s_iter / 1e12
    out = {
        "metric": "weights/s per Lloyd iteration (E+M), whole hot path",
        "value": value,
        "unit": "weights/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": cfg["name"], "layer": f"{N}x{K} bf16", "tokens": int(X.shape[0]),
                   "group_size": g, "format": "nvfp4" if fmt == A.NVFP4 else "int4", "iterations": iters},
        "layer_fit_ms": fit_ms + enc_ms,
        "stage_ms": {"act_stats": stats_ms, "fit": fit_ms, "encode": enc_ms, "dequant": deq_ms},
        "act_stats_GBs": X.numel() * 2 / (stats_ms * 1e-3) / 1e9,
        "lloyd_iteration_us": iter_us,
        "lloyd_weights_per_s": weights_per_s_iter,
        "roofline": {"bound": "alu", "kernel": "lloyd_iter_kernel", "achieved": achieved,
                     "peak": ALU_PEAK_TLANEOPS, "unit": "Tlane-op/s", "frac": achieved / ALU_PEAK_TLANEOPS,
                     "traffic": traffic,
                     "hbm_achieved_GBs": bytes_per_weight(g) * weights_per_s_iter / 1e9,
                     "hbm_frac": bytes_per_weight(g) * weights_per_s_iter / 1e9 / HBM_PEAK_GBS},
    }

    if not args.no_cpu_baseline:
        import oracle
        Wb = inputs.bits(W)
        Ih = I.cpu().numpy()
        t1 = time.perf_counter()
        oracle.fit(Wb, g, fmt, Ih, grid, iters)
        dt = time.perf_counter() - t1
        out["cpu_baseline"] = {"value": n_w * iters / dt, "unit": "weights/s", "cores": 1, "kind": "oracle",
                               "sample": f"oracle fit of the same {N}x{K} layer, all {iters} iterations, "
                                         f"{dt:.1f} s on one host core"}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
