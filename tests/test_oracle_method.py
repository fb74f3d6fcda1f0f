"""Pins for the oracle's whole-method behaviour: hand-derived worked vectors,
the reduction to plain round-to-nearest, monotone objective, invariances and the
textbook 1-D Lloyd special case.
"""
import json
import os

import numpy as np
import pytest
import torch

import oracle
from paper_2605_08692_amd import inputs

from test_oracle_steps import bf16_bits, bf16_vals, random_layer

GOLD = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "worked_vectors.json")))
E2M1 = inputs.E2M1_GRID
INT4G = inputs.INT4_GRID
FMT = {"nvfp4": oracle.NVFP4, "int4": oracle.INT4}


def unpack(codes):
    out = np.empty((codes.shape[0], codes.shape[1] * 2), np.uint8)
    out[:, 0::2] = codes & 15
    out[:, 1::2] = codes >> 4
    return out


def case_arrays(case):
    if "W" in case:
        W = np.array(case["W"], np.float32)[None, :]
        codes = np.array(case["codes"], np.uint8)[None, :]
    else:
        p = case["W_pattern"]
        W = (np.tile(np.array(p["values_over_64"], np.float32), p["repeat"]) / np.float32(64))[None, :]
        q = case["codes_pattern"]
        codes = np.tile(np.array(q["values"], np.uint8), q["repeat"])[None, :]
    return W, codes


@pytest.mark.parametrize("case", GOLD["cases"], ids=lambda c: c["name"])
def test_worked_vectors(case):
    fmt, g = FMT[case["fmt"]], case["g"]
    W, codes_ref = case_arrays(case)
    Wb = bf16_bits(W)
    assert (bf16_vals(Wb) == W).all()  # the vectors are exact in bf16
    tables = np.array(case["T0"] + case["T1"], np.float32)
    tb = bf16_bits(tables)
    I = (np.arange(W.shape[1]) % 5 + 1).astype(np.float32)
    codes, scales = oracle.encode(Wb, g, fmt, I, tb)
    assert (unpack(codes) == codes_ref).all()
    if "packed" in case:
        assert codes.tolist() == [case["packed"]]
    assert scales.tolist() == [[case["scale"]]]
    sign_bit = 7 if fmt == oracle.NVFP4 else 15
    assert scales[0, 0] >> sign_bit == case["sigma"]
    assert (oracle.dequant(codes, scales, tb, g, fmt) == Wb).all()
    if case["tables_fixed_point"]:
        res = oracle.fit(Wb, g, fmt, I, tables, 5)
        assert (res["tables_f32"] == tables).all() and (res["objective"] == 0).all()


@pytest.mark.parametrize("g,fmt,grid,qmax", [(16, oracle.NVFP4, E2M1, 6), (128, oracle.INT4, INT4G, 7),
                                             (64, oracle.INT4, INT4G, 7)])
def test_zero_iterations_with_the_format_grid_is_round_to_nearest(g, fmt, grid, qmax):
    W, I = random_layer(20 + g, 8, 512)
    res = oracle.fit(W, g, fmt, I, np.concatenate([grid, grid]), 0)
    assert (res["tables_f32"] == np.concatenate([grid, grid])).all()
    codes, scales = oracle.encode(W, g, fmt, I, res["tables_bf16"])
    # independent round-to-nearest in numpy: scale from torch's casts, fp32
    # normalisation, brute-force argmin over the grid
    Wf = bf16_vals(W)
    a = np.abs(Wf).reshape(8, 512 // g, g).max(axis=2) / np.float32(qmax)
    if fmt == oracle.NVFP4:
        s8 = np.maximum(torch.from_numpy(a).to(torch.float8_e4m3fn).view(torch.uint8).numpy(), 1)
        s = torch.from_numpy(s8).view(torch.float8_e4m3fn).float().numpy()
        assert (scales == s8).all()
    else:
        sb = torch.from_numpy(a).to(torch.bfloat16)
        s = sb.float().numpy()
        assert (scales == sb.view(torch.int16).numpy().view(np.uint16)).all()
    wn = Wf * np.repeat(np.float32(1) / s, g, axis=1)
    rtn = np.abs(wn.astype(np.float64)[:, :, None] - grid.astype(np.float64)[None, None, :]).argmin(axis=2)
    assert (grid[unpack(codes)] == grid[rtn]).all()
    # every selection bit is 0 and dequantisation is grid value times scale
    What = oracle.dequant(codes, scales, res["tables_bf16"], g, fmt)
    expect = torch.from_numpy(grid[rtn] * np.repeat(s, g, axis=1)).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert (What == expect).all()


@pytest.mark.parametrize("cfg_id", [0])
def test_objective_never_increases_and_both_tables_get_used(cfg_id):
    cfg = inputs.CONFIGS[cfg_id]
    layer = cfg["layers"][0]
    W = inputs.bits(inputs.layer_weights(layer))
    I = oracle.act_stats(inputs.bits(inputs.activations(cfg["xs"][layer["x"]])))
    res = oracle.fit(W, cfg["g"], cfg["fmt"], I, inputs.format_grid(cfg["fmt"]), cfg["iters"], trace=True)
    J = res["objective"]
    assert (J[1:] <= J[:-1] * (1 + 1e-6)).all() and J[-1] < 0.9 * J[0]
    # T0 = T1 at the start: the first step ties everywhere, so T1 keeps the grid
    assert (res["tables_trace"][0, 16:] == inputs.E2M1_GRID).all()
    assert (res["tables_trace"][1, 16:] != inputs.E2M1_GRID).any()
    for t in res["tables_trace"]:
        assert (np.diff(t[:16]) >= 0).all() and (np.diff(t[16:]) >= 0).all()
    codes, scales = oracle.encode(W, cfg["g"], cfg["fmt"], I, res["tables_bf16"])
    assert 0.05 < (scales >> 7).mean() < 0.95
    assert res["tables_bf16"].nbytes == 64 and codes.nbytes == W.size // 2 and scales.nbytes == W.size // 16


def test_int4_objective_monotone_and_resume_is_exact():
    W, I = random_layer(31, 64, 1024)
    grid = inputs.format_grid(oracle.INT4)
    full = oracle.fit(W, 128, oracle.INT4, I, grid, 8, trace=True)
    J = full["objective"]
    assert (J[1:] <= J[:-1] * (1 + 1e-6)).all()
    half = oracle.fit(W, 128, oracle.INT4, I, grid, 4)
    rest = oracle.fit(W, 128, oracle.INT4, I, half["tables_f32"], 4)
    assert (rest["tables_f32"] == full["tables_f32"]).all()
    assert (rest["objective"] == J[4:]).all()


def test_sign_bit_round_trip_and_recon_consistency():
    W, I = random_layer(33, 16, 512)
    for g, fmt, bit in ((16, oracle.NVFP4, 7), (128, oracle.INT4, 15)):
        res = oracle.fit(W, g, fmt, I, inputs.format_grid(fmt), 4)
        tb = res["tables_bf16"]
        codes, scales = oracle.encode(W, g, fmt, I, tb)
        unsigned, vals, wn = oracle.normalise(W, g, fmt)
        sigma = scales >> bit
        assert ((scales & ((1 << bit) - 1)) == unsigned).all() and (unsigned > 0).all()
        # sigma and the error it implies agree with an assignment under the bf16 tables
        Tb = bf16_vals(tb)
        a = oracle.assign(wn, g, I, Tb)
        assert (a["sigma"] == sigma).all()
        idx = np.where(np.repeat(sigma, g, axis=1) == 1, a["idx1"], a["idx0"])
        assert (unpack(codes) == idx).all()
        # dequantised weights reproduce the selected error: sum I (w~ - T[c])^2 = min(e0, e1)
        What = bf16_vals(oracle.dequant(codes, scales, tb, g, fmt)).astype(np.float64)
        recon = Tb[16 * np.repeat(sigma, g, axis=1) + unpack(codes)].astype(np.float64)
        s = np.repeat(vals, g, axis=1).astype(np.float64)
        assert np.allclose(What, recon * s, rtol=2 ** -8)
        err = (I.astype(np.float64) * (wn - recon) ** 2).reshape(16, 512 // g, g).sum(axis=2)
        assert np.allclose(err, np.minimum(a["e0"], a["e1"]), rtol=1e-5)


def test_invariance_to_importance_scaling_and_row_permutation():
    W, I = random_layer(35, 32, 256)
    grid = inputs.format_grid(oracle.NVFP4)
    base = oracle.fit(W, 16, oracle.NVFP4, I, grid, 5)
    scaled = oracle.fit(W, 16, oracle.NVFP4, I * np.float32(2 ** 7), grid, 5)
    assert (scaled["tables_f32"] == base["tables_f32"]).all()
    c0, s0 = oracle.encode(W, 16, oracle.NVFP4, I, base["tables_bf16"])
    c1, s1 = oracle.encode(W, 16, oracle.NVFP4, I * np.float32(2 ** 7), base["tables_bf16"])
    assert (c0 == c1).all() and (s0 == s1).all()
    perm = np.random.default_rng(0).permutation(32)
    permuted = oracle.fit(W[perm], 16, oracle.NVFP4, I, grid, 5)
    assert np.allclose(permuted["tables_f32"], base["tables_f32"], rtol=1e-6, atol=1e-7)
    cp, sp = oracle.encode(W[perm], 16, oracle.NVFP4, I, base["tables_bf16"])
    assert (cp == c0[perm]).all() and (sp == s0[perm]).all()
    # a more important channel pulls the selection: doubling I on half the columns changes something
    I2 = I.copy()
    I2[::2] *= np.float32(64)
    other = oracle.fit(W, 16, oracle.NVFP4, I2, grid, 5)
    assert (other["tables_f32"] != base["tables_f32"]).any()


def lloyd_1d(x, T, iters):
    """Textbook unweighted 1-D Lloyd (float64): nearest centre by distance, mean of each cell."""
    T = T.astype(np.float64).copy()
    for _ in range(iters):
        cell = np.abs(x[:, None] - T[None, :]).argmin(axis=1)
        for i in range(16):
            if (cell == i).any():
                T[i] = x[cell == i].mean()
        T.sort()
    return T


def test_unit_importance_single_table_is_textbook_lloyd():
    W, _ = random_layer(37, 32, 256)
    I = np.ones(256, np.float32)
    far = np.arange(1000, 1016, dtype=np.float32)  # never selected
    start = np.linspace(-5.5, 5.7, 16).astype(np.float32)
    res = oracle.fit(W, 16, oracle.NVFP4, I, np.concatenate([start, far]), 6)
    _, _, wn = oracle.normalise(W, 16, oracle.NVFP4)
    ref = lloyd_1d(wn.astype(np.float64).ravel(), start, 6)
    assert (res["tables_f32"][16:] == far).all()
    assert np.allclose(res["tables_f32"][:16], ref, rtol=1e-5, atol=1e-6)


def test_rejects_bad_shapes():
    W, I = random_layer(39, 2, 64)
    with pytest.raises(ValueError):
        oracle.fit(W, 24, oracle.NVFP4, I, inputs.format_grid(0), 1)
    with pytest.raises(ValueError):
        oracle.fit(W[:, :40], 16, oracle.NVFP4, I[:40], inputs.format_grid(0), 1)
    with pytest.raises(ValueError):
        oracle.fit(W, 16, oracle.NVFP4, I, inputs.format_grid(0), -1)
