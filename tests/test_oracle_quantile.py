"""Pins for the quantile initialisation (paper Eq. init_t0, Eq. init_t1; Alg. 1
steps 4-5): library quantiles, exact rational interpolation, closed forms."""
from fractions import Fraction

import numpy as np
import pytest

import oracle
from paper_2605_08692_amd import inputs

from test_oracle_steps import bf16_bits, random_layer

Q0 = [Fraction(i, 15) for i in range(16)]
Q1 = [Fraction(1, 30) + Fraction(29, 30) * Fraction(i, 15) for i in range(16)]


def test_levels_are_the_papers():
    # delta = 1 / (2 (M - 1)) with M = 16; T1 starts half a step in and ends at the maximum
    assert Q1[0] == Fraction(1, 2 * 15) and Q1[15] == 1 and Q0[15] == 1 and Q0[0] == 0
    assert all(a < b for a, b in zip(Q0, Q1[:15] + [2]))
    assert Q1[1] - Q1[0] == Fraction(29, 30) * (Q0[1] - Q0[0])


@pytest.mark.parametrize("g,fmt,N,K", [(16, oracle.NVFP4, 64, 512), (128, oracle.INT4, 33, 1024), (32, oracle.INT4, 7, 96)])
def test_against_numpy_quantiles(g, fmt, N, K):
    W, _ = random_layer(80 + g, N, K)
    _, _, wn = oracle.normalise(W, g, fmt)
    grid = oracle.quantile_init(W, g, fmt)
    x = wn.astype(np.float64).ravel()
    ref = np.quantile(x, [float(q) for q in Q0 + Q1], method="linear")
    assert np.allclose(grid, ref, rtol=2e-6, atol=1e-7)
    assert grid[0] == wn.min() and grid[15] == wn.max() and grid[31] == wn.max()
    assert (np.diff(grid[:16]) >= 0).all() and (np.diff(grid[16:]) >= 0).all()
    assert (grid[16:31] >= grid[:15]).all() and (grid[16:31] <= grid[1:16]).all()  # half a step further


def exact_quantiles(x):
    xs = sorted(Fraction(float(v)) for v in x)
    out = []
    for q in Q0 + Q1:
        pos = q * (len(xs) - 1)
        lo = pos.numerator // pos.denominator
        frac = pos - lo
        out.append(xs[lo] if frac == 0 else xs[lo] + frac * (xs[lo + 1] - xs[lo]))
    return out


def test_against_exact_rational_interpolation():
    W, _ = random_layer(83, 5, 128)
    g, fmt = 16, oracle.NVFP4
    _, _, wn = oracle.normalise(W, g, fmt)
    grid = oracle.quantile_init(W, g, fmt)
    ref = exact_quantiles(wn.ravel())
    near = np.array([np.float32(float(r)) for r in ref])
    assert (np.abs(grid - near) <= np.spacing(np.abs(near))).all()
    assert (grid == near).mean() > 0.9


def test_closed_form_on_integer_ramp():
    # one group with absmax 7/64: the scale is 1/64 and the normalised weights are these integers
    ramp = np.array([-7, -6, -5, -4, -3, -2, -1, 0, 1, 2, 3, 4, 5, 6, 7, 7], np.float32) / np.float32(64)
    W = bf16_bits(ramp[None, :])
    _, _, wn = oracle.normalise(W, 16, oracle.INT4)
    assert (np.sort(wn.ravel()) == [-7, -6, -5, -4, -3, -2, -1, 0, 1, 2, 3, 4, 5, 6, 7, 7]).all()
    grid = oracle.quantile_init(W, 16, oracle.INT4)
    # n = 16: position of level i/15 is i -> the i-th smallest value itself
    assert grid[:16].tolist() == [-7, -6, -5, -4, -3, -2, -1, 0, 1, 2, 3, 4, 5, 6, 7, 7]
    # T1: position (15 + 29 i)/30 = 0.5 + 29 i / 30 on the sequence x_j = j - 7 (j <= 14), x_15 = 7
    want = []
    xs = [-7, -6, -5, -4, -3, -2, -1, 0, 1, 2, 3, 4, 5, 6, 7, 7]
    for i in range(16):
        pos = Fraction(15 + 29 * i, 30)
        lo = pos.numerator // pos.denominator
        fr = pos - lo
        want.append(float(xs[lo] + fr * (xs[min(lo + 1, 15)] - xs[lo])))
    assert np.allclose(grid[16:], want, rtol=1e-7, atol=0)
    assert grid[16] == np.float32(-6.5) and grid[31] == 7


def test_invariant_to_the_order_of_rows_and_uses_every_weight():
    W, _ = random_layer(85, 12, 256)
    a = oracle.quantile_init(W, 16, oracle.NVFP4)
    b = oracle.quantile_init(W[::-1].copy(), 16, oracle.NVFP4)
    assert (a == b).all()
    # one huge weight moves only the top quantile of its own group's normalisation, but the maximum
    # of the normalised weights is at most 6 * (1 + rounding of the scale): the top entry sees it
    _, _, wn = oracle.normalise(W, 16, oracle.NVFP4)
    assert a[15] == wn.max()


def test_single_weight_group_and_rejects_empty():
    W = bf16_bits(np.full((1, 16), 0.25, np.float32))
    grid = oracle.quantile_init(W, 16, oracle.NVFP4)
    _, _, wn = oracle.normalise(W, 16, oracle.NVFP4)
    assert (grid == wn[0, 0]).all()
    with pytest.raises(ValueError):
        oracle.quantile_init(np.zeros((0, 16), np.uint16), 16, oracle.NVFP4)


def test_quantile_tables_differ_so_both_are_used_from_the_first_assignment():
    W, I = random_layer(87, 64, 512)
    g, fmt = 16, oracle.NVFP4
    q = oracle.quantile_init(W, g, fmt)
    assert (q[:16] != q[16:]).sum() >= 15          # "distinct but nearby starting points"
    _, _, wn = oracle.normalise(W, g, fmt)
    first = oracle.assign(wn, g, I, q)["sigma"]
    assert 0.05 < first.mean() < 0.95                # with T0 == T1 the first assignment is all zeros
    same = oracle.assign(wn, g, I, inputs.format_grid(fmt))["sigma"]
    assert same.sum() == 0
    a = oracle.fit_nested(W, g, fmt, I, q, 4, 2)
    assert (np.diff(a["objective"]) <= 0).all()


def test_zero_results_are_positive_zero():
    # every weight is -0.0: the normalised weights are -0.0, the tables must hold +0.0
    W = np.full((2, 16), 0x8000, np.uint16)
    grid = oracle.quantile_init(W, 16, oracle.NVFP4)
    assert (grid.view(np.uint32) == 0).all()
