#!/usr/bin/env python3
"""Benchmark of the AAAC hot path on one MI355X.

A step is one pass of the whole path over synthetic layers that are already
resident in HBM: aaac_act_stats (importance from the calibration activations,
once per distinct input width), aaac_fit / aaac_fit_batch (scales + all Lloyd
iterations), aaac_encode and aaac_dequant for every layer.  The default workload
is the largest of the five benchmark settings, the Llama-3-70B-shaped MLP pair
(gate 28672x8192 and down 8192x28672 bf16, 131,072 calibration tokens per input
width, NVFP4 group 16, 30 iterations, one layer fitted after the other);
--config selects another setting.  The default run also measures the four
smaller settings, each with its own inputs and a step of the same kind, and
reports them under `per_config`.

Prints one JSON line.  `value` is weight-iterations per second over the whole
step (sum of N*K over the layers * passes over the weights / step time).
`roofline` describes the Lloyd-iteration kernel: its average duration is measured
with HIP events on the launch stream around every fit call inside the timed
region (fit time / iterations, so launch gaps and the small scale / init /
final-table kernels count against it).  `achieved` prices every weight at the
33 vector-ALU lane operations of the algorithmic model (a count of what the
method needs, not of what the kernel executes); `counters` holds what the
hardware counters read for the same kernel (executed lane operations per weight,
vector-ALU and LDS busy fractions, HBM bytes per launch), taken from
profiles/counters_lloyd_iter.json when that file was measured on the kernel
sources as they are now (it carries their hash), else null.  `cpu_baseline` is
the CPU oracle, single-threaded.

Options beyond the default path (each adds its own object to the line):
--n-inner / --n-outer run both loops of the learning algorithm (refine_roofline:
the refinement pass), --sel-size one table choice per that many weights with
separate selection bits, --quantile-init the quantile tables as the start
(quantile_init), --gemv-rows / --gemm-rows the quantised layers applied to
activation rows (gemv_w4a16, gemm_w4a16).
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
# the group's stored scale (1 byte per group of an FP8 scale, 2 of a bf16 scale), and 33
# vector-ALU lane operations (unpack 1, normalise 1, two 4-level searches 16, two table
# look-ups 2, two error chains 8, selection/bin 1, fp64 accumulate 4).  The kernel itself
# reads the group's reciprocal scale as an fp32 (4 bytes per group).
LANE_OPS_PER_WEIGHT = 33.0
# A refinement pass (choice frozen) searches one table and needs no errors: unpack 1,
# normalise 1, one search 8, bin 1, fp64 accumulate 4.
LANE_OPS_PER_WEIGHT_REFINE = 15.0
ALU_PEAK_TLANEOPS = 256 * 64 * 2.4e9 / 1e12  # 256 CUs x 64 lanes x 2.4 GHz, one op per lane-clock
HBM_PEAK_GBS = 8000.0
MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense bf16 matrix-core peak


def bytes_per_weight(g):
    """What the Lloyd kernel reads per weight: the bf16 weight and the group's fp32 reciprocal scale."""
    return 2.0 + 4.0 / g


def algorithmic_bytes_per_weight(g, fmt_is_nvfp4):
    """What the method needs per weight: the bf16 weight and the group's stored scale."""
    return 2.0 + (1.0 if fmt_is_nvfp4 else 2.0) / g


def kernel_source_hash():
    """Hash of the sources of the Lloyd-iteration kernel (counter summaries carry it)."""
    import hashlib
    h = hashlib.sha256()
    for name in ("aaac_lloyd.hip", "aaac_search.h", "aaac_device.h", "aaac_internal.h"):
        with open(os.path.join(ROOT, "paper_2605_08692_amd", "csrc", name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]


def measured_counters(workload):
    """Hardware-counter figures of the Lloyd kernel on `workload`, or None when there are none for the
    kernel as it is now."""
    path = os.path.join(ROOT, "profiles", "counters_lloyd_iter.json")
    if not os.path.exists(path):
        return None
    with open(path) as f:
        data = json.load(f)
    if data.get("kernel_source_hash") != kernel_source_hash():
        return None
    w = data.get("workloads", {}).get(workload)
    if w is None:
        return None
    keep = ("kernel", "launches_averaged", "weights_per_launch", "executed_lane_ops_per_weight", "valu_busy", "lds_busy",
            "lds_instructions_per_weight", "hbm_bytes_per_launch", "algorithmic_bytes_per_launch")
    return {k: w[k] for k in keep if k in w}


def measure(args, cfg_id, steps_arg, warmup_arg, cpu_baseline, extras):
    """One setting: inputs, buffers, warm-up, timed steps; returns the JSON object of that setting.
    extras: also run what the options ask for beyond the timed steps (products, copy calibration)."""
    import numpy as np
    import torch

    import paper_2605_08692_amd as A
    from paper_2605_08692_amd import inputs

    A.library()  # no fallback: fails here if the HIP library is missing
    dev = "cuda:0"
    torch.cuda.set_device(0)
    cfg = inputs.CONFIGS[cfg_id]
    default_steps = {0: 50, 1: 20, 2: 20, 3: 10, 4: 25}[cfg_id]  # cfg4: 25 x 14.5 ms, a timed region of about a third of a second
    steps = steps_arg if steps_arg is not None else default_steps
    warmup = warmup_arg if warmup_arg is not None else (2 if cfg_id >= 3 else 3)
    g, fmt, iters = cfg["g"], cfg["fmt"], cfg["iters"]
    grid = inputs.format_grid(fmt)
    fit_grid = None if args.quantile_init else grid   # None: quantile tables, taken on the GPU inside the fit
    S = args.sel_size if args.sel_size is not None else g
    nested = args.n_inner > 1 or S != g or args.quantile_init
    n_outer = args.n_outer if args.n_outer is not None else (3 if args.n_inner > 1 else iters)
    n_inner = args.n_inner
    iters = n_outer  # length of the objective trace
    passes = n_outer * n_inner  # passes over the weights per fit
    batch = len(cfg["layers"]) > 2 or nested  # the decoder block goes through aaac_fit_batch

    # inputs and every buffer are created once, outside the timed region
    Xs = {k: inputs.activations(r, dev) for k, r in cfg["xs"].items()}
    Is = {k: torch.empty(X.shape[1], dtype=torch.float32, device=dev) for k, X in Xs.items()}
    ws_stats = {k: torch.empty(max(A.aaac_act_stats_workspace(*X.shape), 256), dtype=torch.uint8, device=dev)
                for k, X in Xs.items()}
    layers = []
    for l in cfg["layers"]:
        N, K = l["N"], l["K"]
        layers.append(dict(
            name=l["name"], N=N, K=K, x=l["x"], W=inputs.layer_weights(l, dev),
            tf=torch.empty(32, dtype=torch.float32, device=dev), tb=torch.empty(32, dtype=torch.int16, device=dev),
            obj=torch.empty(iters, dtype=torch.float64, device=dev),
            codes=torch.empty((N, K // 2), dtype=torch.uint8, device=dev),
            scales=torch.empty((N, K // g), dtype=torch.uint8 if fmt == A.NVFP4 else torch.int16, device=dev),
            What=torch.empty((N, K), dtype=torch.bfloat16, device=dev),
            bits=torch.empty((N, A.sel_stride(K, S)), dtype=torch.uint8, device=dev) if S < g else None,
            ws=torch.empty(A.aaac_fit_workspace(N, K, g, fmt), dtype=torch.uint8, device=dev)))
    if batch:
        import ctypes
        arr = (A.binding.aaac_layer_t * len(layers))()
        for i, L in enumerate(layers):
            arr[i] = A.binding.aaac_layer_t(L["W"].data_ptr(), L["N"], L["K"], L["W"].stride(0), Is[L["x"]].data_ptr(),
                                            L["tf"].data_ptr(), L["tb"].data_ptr(), L["obj"].data_ptr())
        ws_batch = torch.empty(A.aaac_fit_nested_workspace(arr, g, fmt, sel_size=S), dtype=torch.uint8, device=dev)
    stream = torch.cuda.current_stream()
    n_w = sum(L["N"] * L["K"] for L in layers)

    def step(events=None):
        def mark(i):
            if events is not None:
                events[i].record(stream)
        mark(0)
        for k, X in Xs.items():
            A.aaac_act_stats(X, Is[k], ws_stats[k], stream)
        mark(1)
        if nested:
            A.aaac_fit_nested(arr, g, fmt, fit_grid, n_outer, n_inner, ws_batch, stream, sel_size=S)
        elif batch:
            A.aaac_fit_batch(arr, g, fmt, grid, iters, ws_batch, stream)
        else:
            for L in layers:
                A.aaac_fit(L["W"], g, fmt, Is[L["x"]], grid, iters, L["tf"], L["tb"], L["obj"], L["ws"], stream)
        mark(2)
        for L in layers:
            if S < g:
                A.aaac_encode_sel(L["W"], g, S, fmt, Is[L["x"]], L["tb"], L["codes"], L["scales"], L["bits"], stream)
            else:
                A.aaac_encode(L["W"], g, fmt, Is[L["x"]], L["tb"], L["codes"], L["scales"], stream)
        mark(3)
        for L in layers:
            if S < g:
                A.aaac_dequant_sel(L["codes"], L["scales"], L["bits"], L["tb"], g, S, fmt, L["What"], stream)
            else:
                A.aaac_dequant(L["codes"], L["scales"], L["tb"], g, fmt, L["What"], stream)
        mark(4)

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(5)] for _ in range(steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(steps):
        step(evs[s])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / steps

    def stage(i):
        return float(np.mean([e[i].elapsed_time(e[i + 1]) for e in evs]))
    stats_ms, fit_ms, enc_ms, deq_ms = stage(0), stage(1), stage(2), stage(3)
    iter_us = fit_ms * 1e3 / passes
    weights_per_s_iter = n_w / (iter_us * 1e-6)
    value = n_w * passes / (ms_per_step * 1e-3)

    q_ms, quant = 0.0, None
    if args.quantile_init:
        # the initialisation alone (it is inside `fit` above): four histogram passes over the weights
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        qg = torch.empty(32, dtype=torch.float32, device=dev)
        for L in layers:
            A.aaac_quantile_init(L["W"], g, fmt, qg, L["ws"], stream)
        e0.record(stream)
        for _ in range(5):
            for L in layers:
                A.aaac_quantile_init(L["W"], g, fmt, qg, L["ws"], stream)
        e1.record(stream)
        torch.cuda.synchronize()
        q_ms = e0.elapsed_time(e1) / 5
        # the scale kernel (reads W, writes one fp32 per group) and three histogram passes (read both) touch the
        # weights; the fourth pass of the radix select reads the short candidate list
        q_gbs = 4 * bytes_per_weight(g) * n_w / (q_ms * 1e-3) / 1e9
        quant = {"ms": q_ms, "passes_over_weights": 4, "of_which_scale_kernel": 1, "hbm_achieved_GBs": q_gbs,
                 "hbm_frac": q_gbs / HBM_PEAK_GBS}
        iter_us = (fit_ms - q_ms) * 1e3 / passes
        weights_per_s_iter = n_w / (iter_us * 1e-6)

    refine = None
    if n_inner > 1:
        # refinement pass alone: the same fit with one inner step costs n_outer assignment passes
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        reps = max(steps, 3)
        A.aaac_fit_nested(arr, g, fmt, fit_grid, n_outer, 1, ws_batch, stream, sel_size=S)
        e0.record(stream)
        for _ in range(reps):
            A.aaac_fit_nested(arr, g, fmt, fit_grid, n_outer, 1, ws_batch, stream, sel_size=S)
        e1.record(stream)
        torch.cuda.synchronize()
        assign_ms = e0.elapsed_time(e1) / reps - q_ms   # these fits include the initialisation
        refine_us = (fit_ms - q_ms - assign_ms) * 1e3 / (n_outer * (n_inner - 1))
        ops = LANE_OPS_PER_WEIGHT_REFINE * n_w / (refine_us * 1e-6) / 1e12
        refine = {"kernel": "lloyd_iter_kernel (choice frozen)", "assign_pass_us": assign_ms * 1e3 / n_outer,
                  "refine_pass_us": refine_us, "weights_per_s": n_w / (refine_us * 1e-6), "bound": "alu",
                  "achieved": ops, "peak": ALU_PEAK_TLANEOPS, "unit": "Tlane-op/s", "frac": ops / ALU_PEAK_TLANEOPS}
        # `roofline` below stays the assignment pass
        iter_us = assign_ms * 1e3 / n_outer
        weights_per_s_iter = n_w / (iter_us * 1e-6)

    def time_product(Mx, matrix_cores):
        # The quantised layers of the last step applied to Mx activation rows; 20 calls per layer are
        # captured in a HIP graph so that the host's call overhead does not hide the kernel.  The calls
        # cycle through copies of the layer that together exceed the 256 MB cache behind L2, so that
        # `us` is the time with the codes coming from HBM, as in decoding, where a token reads every
        # layer once; `us_cached` repeats one copy, which that cache then holds when it is small enough.
        side = torch.cuda.Stream()
        per_layer = []
        for L in layers:
            xs = torch.randn((Mx, L["K"]), device=dev).to(torch.bfloat16)
            ys = torch.empty((Mx, L["N"]), dtype=torch.float32, device=dev)
            nbytes = L["N"] * L["K"] * (0.5 + (1 if fmt == A.NVFP4 else 2) / g + (1 / (8 * S) if S < g else 0))
            ncopy = int(min(16, max(1, -(-600e6 // nbytes))))
            copies = [(L["codes"], L["scales"], L["bits"])] + [
                (L["codes"].clone(), L["scales"].clone(), None if L["bits"] is None else L["bits"].clone())
                for _ in range(ncopy - 1)]
            wsx = torch.empty(max(A.aaac_gemm_w4a16_workspace(Mx, L["K"]), 256), dtype=torch.uint8, device=dev) \
                if matrix_cores else None

            def call(st, c):
                codes, scales, bits = copies[c % len(copies)]
                if matrix_cores:
                    A.aaac_gemm_w4a16(xs, codes, scales, bits, L["tb"], g, S, fmt, y=ys, ws=wsx, stream=st)
                else:
                    A.aaac_gemv_w4a16(xs, codes, scales, bits, L["tb"], g, S, fmt, y=ys, stream=st)

            def timed(cycle):
                side.wait_stream(torch.cuda.current_stream())
                with torch.cuda.stream(side):
                    call(side, 0)
                    torch.cuda.synchronize()
                    graph = torch.cuda.CUDAGraph()
                    with torch.cuda.graph(graph, stream=side):
                        for i in range(20):
                            call(side, i if cycle else 0)
                    graph.replay()
                    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                    e0.record(side)
                    graph.replay()
                    e1.record(side)
                torch.cuda.synchronize()
                return e0.elapsed_time(e1) * 1e3 / 20
            us, us_cached = timed(True), timed(False)
            del copies
            per_layer.append({"layer": L["name"], "us": us, "us_cached": us_cached, "copies_cycled": ncopy,
                              "weights_per_s": L["N"] * L["K"] / (us * 1e-6),
                              "hbm_GBs": nbytes / (us * 1e-6) / 1e9, "hbm_frac": nbytes / (us * 1e-6) / 1e9 / HBM_PEAK_GBS,
                              "TFLOPs": 2.0 * Mx * L["N"] * L["K"] / (us * 1e-6) / 1e12,
                              "mfma_frac": 2.0 * Mx * L["N"] * L["K"] / (us * 1e-6) / 1e12 / MFMA_BF16_PEAK_TFLOPS})
        # a few rows of x: bound by reading the codes once (HBM); many rows: by the matrix cores
        bound = "mfma" if matrix_cores and Mx > 64 else "hbm"
        return {"rows_of_x": Mx, "bound": bound, "peak_GBs": HBM_PEAK_GBS, "peak_TFLOPs": MFMA_BF16_PEAK_TFLOPS,
                "layers": per_layer}

    gemv = time_product(args.gemv_rows, False) if extras and args.gemv_rows > 0 else None
    gemm = time_product(args.gemm_rows, True) if extras and args.gemm_rows > 0 else None

    if extras and args.copy_calibration:
        a = torch.empty(1 << 28, dtype=torch.float32, device=dev)
        b = torch.empty_like(a)
        b.copy_(a)
        torch.cuda.synchronize()

    counters = measured_counters(cfg["name"]) if not nested else None
    traffic = counters.get("hbm_bytes_per_launch") if counters else None

    x_bytes = sum(X.numel() * 2 for X in Xs.values())
    achieved = LANE_OPS_PER_WEIGHT * weights_per_s_iter / 1e12
    out = {
        "metric": "weights/s per Lloyd iteration (E+M), whole hot path",
        "value": value,
        "unit": "weights/s",
        "n_gpus": 1,
        "steps": steps,
        "warmup": warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": cfg["name"], "layers": [f'{L["name"]} {L["N"]}x{L["K"]} bf16' for L in layers],
                   "tokens": int(next(iter(Xs.values())).shape[0]), "group_size": g,
                   "format": "nvfp4" if fmt == A.NVFP4 else "int4", "iterations": iters,
                   "n_inner": n_inner, "passes_per_fit": passes, "sel_size": S},
        "layer_fit_ms": fit_ms + enc_ms,
        "stage_ms": {"act_stats": stats_ms, "fit": fit_ms, "encode": enc_ms, "dequant": deq_ms},
        "act_stats_GBs": x_bytes / (stats_ms * 1e-3) / 1e9,
        "lloyd_iteration_us": iter_us,
        "lloyd_weights_per_s": weights_per_s_iter,
        "roofline": {"bound": "alu", "kernel": "lloyd_iter_kernel", "achieved": achieved,
                     "peak": ALU_PEAK_TLANEOPS, "unit": "Tlane-op/s", "frac": achieved / ALU_PEAK_TLANEOPS,
                     "traffic": traffic,
                     "model_lane_ops_per_weight": LANE_OPS_PER_WEIGHT,
                     "counters": counters,
                     "algorithmic_bytes_per_weight": algorithmic_bytes_per_weight(g, fmt == A.NVFP4),
                     "bytes_read_per_weight": bytes_per_weight(g),
                     "hbm_achieved_GBs": algorithmic_bytes_per_weight(g, fmt == A.NVFP4) * weights_per_s_iter / 1e9,
                     "hbm_frac": algorithmic_bytes_per_weight(g, fmt == A.NVFP4) * weights_per_s_iter / 1e9
                     / HBM_PEAK_GBS},
        "weights": n_w,
    }

    if refine is not None:
        out["refine_roofline"] = refine
    if gemv is not None:
        out["gemv_w4a16"] = gemv
    if gemm is not None:
        out["gemm_w4a16"] = gemm
    if quant is not None:
        out["quantile_init"] = quant
        out["config"]["init"] = "quantile"

    if cpu_baseline:
        import oracle
        # bounded sample: the oracle's fit of (a row slice of) the first layer, all iterations
        L = layers[0]
        rows = min(L["N"], max(1, int(8.0e8 / (L["K"] * passes))))  # 10-20 s at 15-25 ns per weight-iteration
        Wb = inputs.bits(L["W"][:rows])
        Ih = Is[L["x"]].cpu().numpy()
        t1 = time.perf_counter()
        if nested:
            g0 = oracle.quantile_init(Wb, g, fmt) if args.quantile_init else grid
            oracle.fit_sel(Wb, g, S, fmt, Ih, g0, n_outer, n_inner)
        else:
            oracle.fit(Wb, g, fmt, Ih, grid, iters)
        dt = time.perf_counter() - t1
        out["cpu_baseline"] = {"value": rows * L["K"] * passes / dt, "unit": "weights/s", "cores": 1,
                               "kind": "oracle",
                               "sample": f'oracle fit of {rows} of the {L["N"]} rows of {L["name"]} '
                                         f'({rows}x{L["K"]}), all {passes} passes, {dt:.1f} s on one host core'}
    return out



def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--config", type=int, default=None,
                    help="index into the five benchmark settings (default: 4, the largest, with the smaller ones "
                         "measured too and reported as per_config)")
    ap.add_argument("--no-per-config", action="store_true",
                    help="skip the measurement of the smaller settings that the default run adds as per_config")
    ap.add_argument("--n-inner", type=int, default=1,
                    help="k-means steps per assignment step (Alg. 1's inner loop); above 1 the fit goes through "
                         "aaac_fit_nested with --n-outer assignment steps")
    ap.add_argument("--n-outer", type=int, default=None, help="assignment steps when --n-inner > 1 (default 3)")
    ap.add_argument("--sel-size", type=int, default=None,
                    help="weights per table choice when smaller than the scale group (selection bits stored "
                         "separately); the fit then goes through aaac_fit_nested")
    ap.add_argument("--quantile-init", action="store_true",
                    help="start from the quantile tables of Alg. 1 (computed on the GPU inside the fit) instead of "
                         "the format grid; the fit then goes through aaac_fit_nested")
    ap.add_argument("--gemv-rows", type=int, default=0,
                    help="after the timed steps, also time aaac_gemv_w4a16 (the quantised layers applied to this many "
                         "rows of activations) and report it as gemv_w4a16")
    ap.add_argument("--gemm-rows", type=int, default=0,
                    help="the same for aaac_gemm_w4a16 (matrix cores, weights rounded to bf16), reported as gemm_w4a16")
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip the oracle timing (profiling runs)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one plain 1 GiB device copy (reference for HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (the path has no multi-GPU part); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    config = 4 if args.config is None else args.config
    out = measure(args, config, args.steps, args.warmup, cpu_baseline=not args.no_cpu_baseline, extras=True)
    plain = (args.config is None and args.n_inner == 1 and args.sel_size is None and not args.quantile_init
             and args.gemv_rows == 0 and args.gemm_rows == 0)
    if plain and not args.no_per_config:
        # the smaller settings in the same run: same kind of step, their own inputs, fewer details
        per = {}
        for c in range(4):
            r = measure(args, c, None, None, cpu_baseline=False, extras=False)
            per[r["config"]["workload"]] = {
                "weights": r["weights"], "steps": r["steps"], "ms_per_step": r["ms_per_step"],
                "stage_ms": r["stage_ms"], "act_stats_GBs": r["act_stats_GBs"],
                "lloyd_iteration_us": r["lloyd_iteration_us"], "lloyd_weights_per_s": r["lloyd_weights_per_s"],
                "frac": r["roofline"]["frac"], "counters": r["roofline"]["counters"],
                "note": ("launch-bound: 131,072 weights are two per resident lane" if c == 0 else None)}
        out["per_config"] = per
    print(json.dumps(out))


if __name__ == "__main__":
    main()
