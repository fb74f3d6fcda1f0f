"""GPU parity at the five benchmark settings, full size and full iteration count, in the launch
configuration bench.py times: importance from the setting's own calibration activations, then
aaac_fit / aaac_fit_batch, aaac_encode and aaac_dequant against the CPU oracle, layer by layer.

Bars as in test_gpu_parity.py: codes, scales with their selection bits, bf16 tables and
dequantised weights bit-exact; fp32 tables within 1e-5 relative; objective within 1e-9 relative;
importance within 1e-6 relative on sampled columns.

The oracle needs about 17 ns per weight and iteration on one core (two minutes for a 235 M-weight
layer at 30 iterations), so the layers of a setting run in one thread each (the oracle itself
stays single-threaded; ctypes releases the interpreter lock), and each thread takes the
iterations five at a time, continuing from the tables of the previous five (the oracle's resume
is bit-exact, pinned in test_oracle_method.py) and noting its progress in a log file.
"""
import concurrent.futures
import os
import threading
import time

import numpy as np
import pytest
import torch

import oracle
import paper_2605_08692_amd as A
from paper_2605_08692_amd import inputs
from test_gpu_parity import DEV, host, say, tables_close, u16

pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
_log_lock = threading.Lock()


def progress(line):
    """One line per finished piece of work, on stdout and in gpurun_out/full_configs_progress.log
    (pytest holds stdout back until the test ends; the file shows a long test is alive)."""
    say(line)
    try:
        d = os.path.join(ROOT, "gpurun_out")
        os.makedirs(d, exist_ok=True)
        with _log_lock, open(os.path.join(d, "full_configs_progress.log"), "a") as f:
            f.write(f"{time.strftime('%H:%M:%S')} {line}\n")
    except OSError:
        pass


def oracle_fit_in_steps(Wb, g, fmt, I, grid, iters, label, step=5):
    """oracle.fit over `iters` iterations, `step` at a time; returns what oracle.fit(trace=True) returns."""
    tables = np.asarray(grid, np.float32)
    obj, trace, done = [], [], 0
    ref = oracle.fit(Wb, g, fmt, I, tables, 0)
    while done < iters:
        n = min(step, iters - done)
        t0 = time.time()
        ref = oracle.fit(Wb, g, fmt, I, tables, n, trace=True)
        tables = ref["tables_f32"]
        obj.append(ref["objective"])
        trace.append(ref["tables_trace"])
        done += n
        progress(f"[full] {label}: oracle iterations {done}/{iters} ({time.time() - t0:.1f}s for {n})")
    ref = dict(ref)
    ref["objective"] = np.concatenate(obj) if obj else np.empty(0)
    ref["tables_trace"] = np.concatenate(trace) if trace else np.empty((0, 32), np.float32)
    return ref


def sampled_importance_check(X, I, n=24):
    """Oracle importance for a sample of columns of a large X."""
    K = X.shape[1]
    cols = np.unique(np.concatenate([[0, K - 1], np.random.default_rng(0).integers(0, K, n)]))
    sub = X[:, torch.from_numpy(cols).to(X.device)].contiguous()
    ref = oracle.act_stats(inputs.bits(sub))
    got = host(I)[cols]
    assert np.allclose(got, ref, rtol=1e-6, atol=0), (got, ref)


def check_config(cfg, iters, batch, workers):
    """Every layer of a setting at full size: importance, fit (one aaac_fit_batch call over all layers
    when `batch`, else one aaac_fit per layer), encode, dequant; each layer against the oracle."""
    g, fmt = cfg["g"], cfg["fmt"]
    grid = inputs.format_grid(fmt)
    Is = {}
    for key, recipe in cfg["xs"].items():
        X = inputs.activations(recipe, DEV)
        Is[key] = A.aaac_act_stats(X)
        torch.cuda.synchronize()
        sampled_importance_check(X, Is[key], n=24 if X.shape[1] <= 16384 else 8)
        progress(f"[full] {cfg['name']}: importance {tuple(X.shape)} ok")
        del X
        torch.cuda.empty_cache()
    Ws = [inputs.layer_weights(l, DEV) for l in cfg["layers"]]
    Il = [Is[l["x"]] for l in cfg["layers"]]
    # the fit on both sides is fed the library's importance: a rounding difference in the
    # importance step cannot leak into code parity
    if batch:
        layers, outs = A.make_layers(Ws, Il, iters)
        ws = torch.empty(A.aaac_fit_batch_workspace(layers, g, fmt), dtype=torch.uint8, device=DEV)
        A.aaac_fit_batch(layers, g, fmt, grid, iters, ws)
    else:
        outs = [A.aaac_fit(W, g, fmt, I, grid, iters) for W, I in zip(Ws, Il)]
    torch.cuda.synchronize()
    progress(f"[full] {cfg['name']}: GPU fit of {len(Ws)} layer(s), {iters} iterations done")

    def one_layer(i):
        l, W, I, (tf, tb, ob) = cfg["layers"][i], Ws[i], Il[i], outs[i]
        label = f'{cfg["name"]}/{l["name"]}'
        Wb, Ih = inputs.bits(W), host(I)
        ref = oracle_fit_in_steps(Wb, g, fmt, Ih, grid, iters, label)
        tfh, tbh = host(tf), u16(tb)
        if not (tbh == ref["tables_bf16"]).all() or not tables_close(tfh, ref["tables_f32"]):
            # the first iteration whose fp32 tables differ tells a one-ulp flip from a bug
            for t in range(1, iters + 1):
                tft, _, _ = A.aaac_fit(W, g, fmt, I, grid, t)
                torch.cuda.synchronize()
                d = host(tft) != ref["tables_trace"][t - 1]
                if d.any():
                    progress(f"[full] {label}: first table difference at iteration {t}: entries "
                             f"{np.nonzero(d)[0]} {host(tft)[d]} {ref['tables_trace'][t - 1][d]}")
                    break
        assert tables_close(tfh, ref["tables_f32"]), (label, tfh, ref["tables_f32"])
        assert (tbh == ref["tables_bf16"]).all(), label
        o = host(ob)[:iters]
        assert np.allclose(o, ref["objective"], rtol=1e-9, atol=0), (label, o, ref["objective"])
        t0 = time.time()
        rc, rs = oracle.encode(Wb, g, fmt, Ih, ref["tables_bf16"])
        rd = oracle.dequant(rc, rs, ref["tables_bf16"], g, fmt)
        progress(f"[full] {label}: oracle encode + dequant {time.time() - t0:.1f}s")
        return rc, rs, rd

    # the GPU calls of the comparison run in this thread, layer by layer, as the oracle results arrive
    with concurrent.futures.ThreadPoolExecutor(max_workers=workers) as pool:
        futures = [pool.submit(one_layer, i) for i in range(len(Ws))]
        for i, fut in enumerate(futures):
            rc, rs, rd = fut.result()
            l, W, I, (tf, tb, ob) = cfg["layers"][i], Ws[i], Il[i], outs[i]
            codes, scales = A.aaac_encode(W, g, fmt, I, tb)
            What = A.aaac_dequant(codes, scales, tb, g, fmt)
            torch.cuda.synchronize()
            sc = host(scales).view(rs.dtype)
            assert (sc == rs).all(), f'{l["name"]}: {(sc != rs).sum()} scale/selection mismatches'
            ch = host(codes)
            assert (ch == rc).all(), f'{l["name"]}: {(ch != rc).sum()} code byte mismatches'
            assert (u16(What) == rd).all(), l["name"]
            progress(f'[full] {cfg["name"]}/{l["name"]}: tables, objective, codes, scales, dequant match '
                     f'(sigma = 1 in {(rs >> (7 if fmt == A.NVFP4 else 15)).mean():.3f} of groups)')
            del codes, scales, What, rc, rs, rd


def test_cfg0_small_nvfp4_10_iterations():
    check_config(inputs.CONFIGS[0], inputs.CONFIGS[0]["iters"], batch=False, workers=1)


def test_cfg1_llama2_7b_qproj_int4_20_iterations():
    check_config(inputs.CONFIGS[1], inputs.CONFIGS[1]["iters"], batch=False, workers=1)


def test_cfg2_down_proj_nvfp4_20_iterations():
    check_config(inputs.CONFIGS[2], inputs.CONFIGS[2]["iters"], batch=False, workers=1)


def test_cfg3_llama3_8b_block_int4_one_batch_call_20_iterations():
    """All seven linears of the decoder block through ONE aaac_fit_batch call."""
    check_config(inputs.CONFIGS[3], inputs.CONFIGS[3]["iters"], batch=True, workers=4)


def test_cfg4_llama3_70b_mlp_nvfp4_both_layers_30_iterations():
    """gate_proj 28672x8192 and down_proj 8192x28672, one aaac_fit call each."""
    check_config(inputs.CONFIGS[4], inputs.CONFIGS[4]["iters"], batch=False, workers=2)
