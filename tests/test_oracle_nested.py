"""Pins for the oracle's two-level loop (n_outer assignment steps, each followed
by n_inner k-means steps with the table choice frozen; paper Alg. 1)."""
from fractions import Fraction

import numpy as np
import pytest

import oracle
from paper_2605_08692_amd import inputs

from test_oracle_method import lloyd_1d
from test_oracle_steps import brute_assign, random_layer

E2M1 = inputs.E2M1_GRID
INT4G = inputs.INT4_GRID


def test_one_inner_step_is_the_plain_lloyd_iteration():
    W, I = random_layer(51, 48, 512)
    for g, fmt in ((16, oracle.NVFP4), (128, oracle.INT4)):
        grid = inputs.format_grid(fmt)
        a = oracle.fit(W, g, fmt, I, grid, 5, trace=True)
        b = oracle.fit_nested(W, g, fmt, I, grid, 5, 1, trace=True)
        assert (a["tables_f32"] == b["tables_f32"]).all() and (a["objective"] == b["objective"]).all()
        assert (a["tables_trace"] == b["tables_trace"]).all()


def weighted_distortion(wn, g, I, tables, sigma):
    """sum I (w~ - nearest entry of the chosen table)^2 in fp64, brute force."""
    (_, e0), (_, e1) = brute_assign(wn, g, I, tables)
    return np.where(sigma == 1, e1, e0).sum()


def test_inner_steps_lower_the_distortion_of_the_frozen_assignment():
    W, I = random_layer(53, 32, 512)
    g, fmt = 16, oracle.NVFP4
    _, _, wn = oracle.normalise(W, g, fmt)
    tables = np.concatenate([E2M1, E2M1 + np.float32(0.25)]).astype(np.float32)
    sigma = oracle.assign(wn, g, I, tables)["sigma"]
    assert 0.05 < sigma.mean() < 0.95
    d = [weighted_distortion(wn, g, I, tables, sigma)]
    T = tables
    for _ in range(6):
        T = oracle.kmeans_step(wn, g, I, sigma, T)
        assert (np.diff(T[:16]) >= 0).all() and (np.diff(T[16:]) >= 0).all()
        d.append(weighted_distortion(wn, g, I, T, sigma))
    d = np.array(d)
    assert (d[1:] <= d[:-1] * (1 + 1e-6)).all() and d[-1] < 0.8 * d[0]


def test_second_inner_step_equals_exact_centroids_of_the_new_cells():
    W, I = random_layer(55, 6, 256)
    g, fmt = 16, oracle.NVFP4
    _, _, wn = oracle.normalise(W, g, fmt)
    tables = np.concatenate([np.linspace(-6, 6.3, 16), np.linspace(-5.6, 5.9, 16)]).astype(np.float32)
    sigma = oracle.assign(wn, g, I, tables)["sigma"]
    T1 = oracle.kmeans_step(wn, g, I, sigma, tables)
    T2 = oracle.kmeans_step(wn, g, I, sigma, T1)
    # cells of the second step by brute force under T1 (fp64 argmin; random data, no exact ties)
    (i0, _), (i1, _) = brute_assign(wn, g, I, T1)
    rep = np.repeat(sigma, g, axis=1)
    idx = np.where(rep == 1, i1, i0)
    num = [Fraction(0)] * 32
    den = [Fraction(0)] * 32
    for n in range(wn.shape[0]):
        for k in range(wn.shape[1]):
            b = 16 * int(rep[n, k]) + int(idx[n, k])
            num[b] += Fraction(float(I[k])) * Fraction(float(wn[n, k]))
            den[b] += Fraction(float(I[k]))
    expect = T1.copy()
    for b in range(32):
        if den[b] != 0:
            expect[b] = np.float32(float(num[b] / den[b]))
    expect = np.concatenate([np.sort(expect[:16]), np.sort(expect[16:])])
    assert (np.abs(T2 - expect) <= np.spacing(np.abs(expect))).all()
    assert (T2 == expect).mean() > 0.9


def test_only_groups_assigned_to_a_table_move_it():
    # all groups on table 0: table 1 must stay where it is through every inner step
    W, I = random_layer(57, 16, 256)
    far = np.arange(1000, 1016, dtype=np.float32)
    res = oracle.fit_nested(W, 16, oracle.NVFP4, I, np.concatenate([E2M1, far]), 2, 4, trace=True)
    assert (res["tables_trace"][:, 16:] == far).all()
    assert (res["tables_trace"][0, :16] != res["tables_trace"][3, :16]).any()


def test_unit_importance_single_table_is_textbook_lloyd_over_the_inner_loop():
    W, _ = random_layer(59, 32, 256)
    I = np.ones(256, np.float32)
    far = np.arange(1000, 1016, dtype=np.float32)
    start = np.linspace(-5.5, 5.7, 16).astype(np.float32)
    res = oracle.fit_nested(W, 16, oracle.NVFP4, I, np.concatenate([start, far]), 1, 7)
    _, _, wn = oracle.normalise(W, 16, oracle.NVFP4)
    ref = lloyd_1d(wn.astype(np.float64).ravel(), start, 7)
    assert np.allclose(res["tables_f32"][:16], ref, rtol=1e-5, atol=1e-6)


def test_objective_of_outer_steps_never_increases():
    cfg = inputs.CONFIGS[0]
    layer = cfg["layers"][0]
    W = inputs.bits(inputs.layer_weights(layer))
    I = oracle.act_stats(inputs.bits(inputs.activations(cfg["xs"][layer["x"]])))
    res = oracle.fit_nested(W, cfg["g"], cfg["fmt"], I, inputs.format_grid(cfg["fmt"]), 4, 5)
    J = res["objective"]
    assert (J[1:] <= J[:-1] * (1 + 1e-6)).all()
    plain = oracle.fit(W, cfg["g"], cfg["fmt"], I, inputs.format_grid(cfg["fmt"]), 4)
    assert (res["tables_f32"] != plain["tables_f32"]).any()
    with pytest.raises(ValueError):
        oracle.fit_nested(W, cfg["g"], cfg["fmt"], I, inputs.format_grid(cfg["fmt"]), 2, 0)
