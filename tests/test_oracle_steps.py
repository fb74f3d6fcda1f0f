"""Pins for the oracle's individual steps: scales, nearest entry, assignment
and the weighted-centroid update.  Expected values come from brute force, exact
rational arithmetic and hand-derived vectors, never from the oracle itself.
"""
import json
import os
from fractions import Fraction

import numpy as np
import pytest
import torch

import oracle
from paper_2605_08692_amd import inputs

GOLD = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "worked_vectors.json")))
E2M1 = inputs.E2M1_GRID
INT4G = inputs.INT4_GRID


def bf16_bits(a):
    return torch.from_numpy(np.asarray(a, np.float32)).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)


def bf16_vals(b):
    return torch.from_numpy(b.view(np.int16)).view(torch.bfloat16).float().numpy()


def random_layer(seed, N, K, scale=0.02):
    rng = np.random.default_rng(seed)
    W = bf16_bits(rng.standard_normal((N, K)) * scale)
    I = (rng.random(K).astype(np.float32) + np.float32(0.05)) * np.float32(100)
    I[rng.integers(0, K, 3)] *= np.float32(400)  # outlier channels
    return W, I


# ---------------------------------------------------------------- scales

def test_scales_against_library_conversions():
    # absmax/6 -> torch's float8_e4m3fn cast; absmax/7 -> torch's bf16 cast
    W, _ = random_layer(3, 8, 256)
    Wf = bf16_vals(W)
    a16 = np.abs(Wf).reshape(8, 16, 16).max(axis=2)
    ref8 = torch.from_numpy(a16 / np.float32(6)).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    ref8 = np.maximum(ref8, 1)
    codes, vals, wn = oracle.normalise(W, 16, oracle.NVFP4)
    assert (codes == ref8).all()
    assert (vals == torch.from_numpy(ref8).view(torch.float8_e4m3fn).float().numpy()).all()
    r = np.float32(1) / vals
    assert (wn == Wf * np.repeat(r, 16, axis=1)).all()

    a128 = np.abs(Wf).reshape(8, 2, 128).max(axis=2)
    ref16 = torch.from_numpy(a128 / np.float32(7)).to(torch.bfloat16)
    codes, vals, wn = oracle.normalise(W, 128, oracle.INT4)
    assert (codes == ref16.view(torch.int16).numpy().view(np.uint16)).all()
    assert (vals == ref16.float().numpy()).all()
    assert (wn == Wf * np.repeat(np.float32(1) / vals, 128, axis=1)).all()
    # the largest normalised magnitude of a group is about 6 (resp. 7)
    assert np.abs(wn).reshape(8, 2, 128).max(axis=2).max() < 7.1


def test_scale_of_zero_and_tiny_groups_stays_positive():
    W = np.zeros((2, 128), np.uint16)
    W[1, :] = bf16_bits(np.full(128, 1e-30))
    c8, v8, wn8 = oracle.normalise(W, 16, oracle.NVFP4)
    assert (c8 == 1).all() and (v8 == 2.0 ** -9).all() and np.isfinite(wn8).all()
    c16, v16, wn16 = oracle.normalise(W, 128, oracle.INT4)
    assert c16[0, 0] == 0x0080 and v16[0, 0] == 2.0 ** -126
    assert c16[1, 0] == bf16_bits([np.float32(bf16_vals(W[1, :1])[0]) / np.float32(7)])[0]
    assert np.isfinite(wn16).all()
    # huge group: FP8 scale saturates at 448
    W[0, :16] = bf16_bits(np.full(16, 1e6))
    c8, v8, _ = oracle.normalise(W, 16, oracle.NVFP4)
    assert c8[0, 0] == 0x7E and v8[0, 0] == 448.0


def test_groups_run_along_the_input_dimension():
    # one large weight at (row 1, column 40): only group (1, 40 // 16) sees it
    W = bf16_bits(np.full((3, 64), 0.5))
    W[1, 40] = bf16_bits([48.0])[0]
    codes, vals, _ = oracle.normalise(W, 16, oracle.NVFP4)
    assert vals[1, 2] == 8.0
    mask = np.ones_like(vals, bool)
    mask[1, 2] = False
    assert (vals[mask] == oracle.e4m3_to_f32(oracle.f32_to_e4m3(0.5 / 6))).all()


# --------------------------------------------------------- nearest entry

@pytest.mark.parametrize("grid", [E2M1, INT4G])
def test_nearest_entry_is_round_to_nearest_on_format_grids(grid):
    # midpoints of both format grids are exact, so the index must be that of a
    # brute-force argmin (first minimum = lower entry on ties) - by value,
    # because the E2M1 grid holds 0 twice
    xs = np.concatenate([np.linspace(-9, 9, 2001), grid, (grid[:-1] + grid[1:]) / 2]).astype(np.float32)
    for x in xs:
        idx = oracle.nearest_index(x, grid)
        brute = int(np.argmin(np.abs(np.float64(x) - grid.astype(np.float64))))
        assert grid[idx] == grid[brute], (x, idx, brute)
    assert oracle.nearest_index(0.0, E2M1) == 7 and oracle.nearest_index(1e-30, E2M1) == 8
    assert oracle.nearest_index(0.25, E2M1) == 8 and oracle.nearest_index(-0.25, E2M1) == 6
    assert oracle.nearest_index(-100, INT4G) == 0 and oracle.nearest_index(100, INT4G) == 15
    assert oracle.nearest_index(2.5, INT4G) == 10  # tie between 2 and 3 goes down


def test_nearest_entry_brute_force_on_random_tables():
    rng = np.random.default_rng(4)
    for _ in range(30):
        T = np.sort(rng.standard_normal(16) * 3).astype(np.float32)
        if rng.random() < 0.5:
            T[5] = T[6] = T[7]  # a triple: equal midpoints, an empty cell
        xs = np.concatenate([rng.standard_normal(300) * 4, T]).astype(np.float32)
        for x in xs:
            idx = oracle.nearest_index(x, T)
            dist = np.abs(np.float64(x) - T.astype(np.float64))
            # optimal up to the fp32 rounding of one midpoint
            assert dist[idx] <= dist.min() + 4e-7 * max(1.0, abs(float(x))), (x, idx)


def test_nearest_entry_uses_both_halves_of_the_table():
    T = np.arange(16, dtype=np.float32)
    assert [oracle.nearest_index(v, T) for v in np.arange(16)] == list(range(16))


# ------------------------------------------------------------ assignment

def brute_assign(wn, g, I, tables):
    """float64 brute force over all 16 entries: errors and indices."""
    N, K = wn.shape
    out = []
    for r in range(2):
        T = tables[16 * r:16 * r + 16].astype(np.float64)
        d = np.abs(wn.astype(np.float64)[:, :, None] - T[None, None, :])
        idx = d.argmin(axis=2)
        err = (I.astype(np.float64)[None, :] * d.min(axis=2) ** 2).reshape(N, K // g, g).sum(axis=2)
        out.append((idx, err))
    return out


@pytest.mark.parametrize("g,fmt", [(16, oracle.NVFP4), (128, oracle.INT4), (32, oracle.INT4)])
def test_assignment_matches_brute_force(g, fmt):
    W, I = random_layer(5 + g, 6, 256)
    _, _, wn = oracle.normalise(W, g, fmt)
    rng = np.random.default_rng(g)
    tables = np.concatenate([np.sort(rng.standard_normal(16) * 3), np.sort(rng.standard_normal(16) * 3 + 0.2)]).astype(np.float32)
    res = oracle.assign(wn, g, I, tables)
    (i0, e0), (i1, e1) = brute_assign(wn, g, I, tables)
    assert np.allclose(res["e0"], e0, rtol=2e-5) and np.allclose(res["e1"], e1, rtol=2e-5)
    # indices agree except within rounding of a midpoint
    for got, ref, T in ((res["idx0"], i0, tables[:16]), (res["idx1"], i1, tables[16:])):
        bad = got != ref
        assert bad.mean() < 1e-3
        assert np.allclose(T[got[bad]].astype(np.float64) - wn[bad], wn[bad] - T[ref[bad]].astype(np.float64), atol=1e-5) or not bad.any()
    clear = np.abs(e0 - e1) > 1e-5 * np.maximum(e0, e1)
    assert clear.mean() > 0.9
    assert (res["sigma"][clear] == (e1 < e0)[clear]).all()
    assert abs(res["objective"] - np.minimum(e0, e1).sum()) < 1e-5 * np.minimum(e0, e1).sum()


def test_assignment_ties_pick_table_zero_and_group_error_is_a_pairwise_tree():
    W, I = random_layer(9, 4, 64)
    _, _, wn = oracle.normalise(W, 16, oracle.NVFP4)
    res = oracle.assign(wn, 16, I, np.concatenate([E2M1, E2M1]))
    assert (res["sigma"] == 0).all() and (res["e0"] == res["e1"]).all()
    # fp32 pairwise tree, spelled out for one group
    T = E2M1
    x = wn[2, 16:32]
    idx = res["idx0"][2, 16:32]
    u = (I[16:32] * ((x - T[idx]) * (x - T[idx]))).astype(np.float32)
    while u.size > 1:
        u = (u[0::2] + u[1::2]).astype(np.float32)
    assert res["e0"][2, 1] == u[0]


# ---------------------------------------------------------- centroid step

def exact_centroids(wn, g, I, tables, sigma, idx):
    """Exact rational weighted means per (table, entry); None for empty cells."""
    num = [Fraction(0)] * 32
    den = [Fraction(0)] * 32
    N, K = wn.shape
    for n in range(N):
        for k in range(K):
            b = 16 * int(sigma[n, k // g]) + int(idx[n, k])
            num[b] += Fraction(float(I[k])) * Fraction(float(wn[n, k]))
            den[b] += Fraction(float(I[k]))
    return [None if d == 0 else n_ / d for n_, d in zip(num, den)], num, den


@pytest.mark.parametrize("g,fmt", [(16, oracle.NVFP4), (128, oracle.INT4)])
def test_centroid_update_equals_exact_weighted_mean(g, fmt):
    W, I = random_layer(11 + g, 6, 256)
    _, _, wn = oracle.normalise(W, g, fmt)
    grid = E2M1 if fmt == oracle.NVFP4 else INT4G
    tables = np.concatenate([grid, grid + np.float32(0.25)]).astype(np.float32)
    # selection and cells from float64 brute force (independent of the oracle);
    # the grids' midpoints are exact, so nothing is ambiguous except exact ties,
    # which take the lower entry = argmin's first minimum
    (i0, e0), (i1, e1) = brute_assign(wn, g, I, tables)
    res = oracle.assign(wn, g, I, tables)
    sigma = res["sigma"]
    assert ((e1 < e0) == sigma.astype(bool))[np.abs(e0 - e1) > 1e-5 * np.maximum(e0, e1)].all()
    idx = np.where(np.repeat(sigma, g, axis=1) == 1, i1, i0)
    # duplicate zero of E2M1: positive values belong to entry 8, not argmin's 7
    if fmt == oracle.NVFP4:
        rep = np.repeat(sigma, g, axis=1)
        idx = np.where((rep == 0) & (idx == 7) & (wn > 0), 8, idx)
        idx = np.where((rep == 1) & (idx == 7) & (wn > 0.25), 8, idx)
    exact, num, den = exact_centroids(wn, g, I, tables, sigma, idx)
    newT, sums, J = oracle.lloyd_iteration(wn, g, I, tables)
    expect = tables.copy()
    for b in range(32):
        if exact[b] is not None:
            expect[b] = np.float32(float(exact[b]))
            assert sums[b] == float(num[b]) and sums[32 + b] == float(den[b])
        else:
            assert sums[32 + b] == 0.0
    expect = np.concatenate([np.sort(expect[:16]), np.sort(expect[16:])])
    ulp = np.spacing(np.abs(expect))
    assert (np.abs(newT - expect) <= ulp).all()
    assert (newT == expect).mean() > 0.9
    assert both_used(sigma)


def both_used(sigma):
    return 0 < sigma.mean() < 1


def test_empty_cells_keep_their_entry_and_zero_importance_counts_as_empty():
    # all weights positive: entries 0..6 of the E2M1 grid get nothing
    rng = np.random.default_rng(13)
    W = bf16_bits(np.abs(rng.standard_normal((4, 64))) * 0.02 + 0.001)
    I = np.ones(64, np.float32)
    _, _, wn = oracle.normalise(W, 16, oracle.NVFP4)
    far = np.arange(100, 116, dtype=np.float32)
    T, sums, _ = oracle.lloyd_iteration(wn, 16, I, np.concatenate([E2M1, far]))
    assert (T[:7] == E2M1[:7]).all() and (T[16:] == far).all()
    assert (sums[32:39] == 0).all() and (sums[48:] == 0).all()
    assert (T[8:16] != E2M1[8:16]).any()
    # zero importance everywhere: every cell is empty, nothing moves
    T0, sums0, J0 = oracle.lloyd_iteration(wn, 16, np.zeros(64, np.float32), np.concatenate([E2M1, far]))
    assert (T0 == np.concatenate([E2M1, far])).all() and J0 == 0.0


def test_centroid_weights_are_importances_not_counts():
    # two weights in one cell, importances 1 and 3: mean = (1*a + 3*b)/4
    W = np.zeros((1, 16), np.float32)
    W[0, 0], W[0, 1], W[0, 15] = 0.875, 1.125, 6.0  # both nearest to entry 1.0; 6.0 fixes the scale at 1
    I = np.ones(16, np.float32)
    I[1] = 3.0
    _, vals, wn = oracle.normalise(bf16_bits(W), 16, oracle.NVFP4)
    assert vals[0, 0] == 1.0
    T, _, _ = oracle.lloyd_iteration(wn, 16, I, np.concatenate([E2M1, np.arange(100, 116, dtype=np.float32)]))
    assert T[10] == np.float32((0.875 + 3 * 1.125) / 4)
