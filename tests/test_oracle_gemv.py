"""Pins for the oracle's W4A16 product y = x W^^T with w^ = T_sigma[code] * s
(paper Eq. pipeline / Eq. aaac_dequant): library conversions + numpy matmul,
unit vectors against the pinned dequantisation, a hand-worked case."""
import numpy as np
import pytest
import torch

import oracle
from paper_2605_08692_amd import inputs

from test_oracle_method import unpack
from test_oracle_steps import bf16_bits, bf16_vals, random_layer


def quantised_layer(seed, N, K, g, S, fmt):
    W, I = random_layer(seed, N, K)
    grid = inputs.format_grid(fmt)
    res = oracle.fit_sel(W, g, S, fmt, I, grid, 2, 2)
    codes, scales, bits = oracle.encode_sel(W, g, S, fmt, I, res["tables_bf16"])
    return W, res["tables_bf16"], codes, scales, bits


def reference_weights(codes, scales, bits, tb, g, S, fmt):
    """Dequantised weights in fp64, rebuilt with torch's conversions (no oracle code)."""
    N, K = codes.shape[0], codes.shape[1] * 2
    c = unpack(codes).astype(np.int64)
    T = torch.from_numpy(tb.view(np.int16)).view(torch.bfloat16).double().numpy()
    if fmt == oracle.NVFP4:
        sign = scales >> 7
        sval = torch.from_numpy((scales & 0x7F).astype(np.uint8)).view(torch.float8_e4m3fn).double().numpy()
    else:
        sign = scales >> 15
        sval = torch.from_numpy((scales & 0x7FFF).astype(np.uint16).view(np.int16)).view(torch.bfloat16).double().numpy()
    if S < g:
        sigma = np.unpackbits(bits, axis=1, bitorder="little")[:, :K // S]
        sigma = np.repeat(sigma, S, axis=1).astype(np.int64)
    else:
        sigma = np.repeat(sign, g, axis=1).astype(np.int64)
    return T[16 * sigma + c] * np.repeat(sval, g, axis=1)


@pytest.mark.parametrize("g,S,fmt,N,K,M", [(16, 16, oracle.NVFP4, 24, 256, 3), (128, 128, oracle.INT4, 17, 512, 1),
                                           (128, 16, oracle.INT4, 9, 256, 2), (64, 32, oracle.NVFP4, 5, 128, 4)])
def test_against_numpy_matmul_of_rebuilt_weights(g, S, fmt, N, K, M):
    W, tb, codes, scales, bits = quantised_layer(90 + g + S, N, K, g, S, fmt)
    rng = np.random.default_rng(g)
    x = bf16_bits(rng.standard_normal((M, K)) * 3)
    y, mag = oracle.gemv_w4a16(x, codes, scales, bits, tb, g, S, fmt)
    What = reference_weights(codes, scales, bits, tb, g, S, fmt)
    xr = bf16_vals(x).astype(np.float64)
    ref = xr @ What.T
    assert np.allclose(y, ref, rtol=1e-6, atol=1e-6 * np.abs(ref).max())
    assert np.allclose(mag, (np.abs(xr)[:, None, :] * np.abs(What)[None, :, :]).sum(axis=2), rtol=1e-12)
    # the product tracks the original layer: quantisation error is small against the signal
    exact = xr @ bf16_vals(W).astype(np.float64).T
    assert np.abs(ref - exact).mean() < 0.2 * np.abs(exact).mean()


@pytest.mark.parametrize("g,S,fmt", [(16, 16, oracle.NVFP4), (128, 16, oracle.INT4), (128, 128, oracle.INT4)])
def test_unit_vectors_return_the_dequantised_columns(g, S, fmt):
    # x = e_k: y[n] = T * s exactly (24 significant bits), and its bf16 rounding is oracle.dequant_sel
    N, K = 12, 256
    _, tb, codes, scales, bits = quantised_layer(95 + g + S, N, K, g, S, fmt)
    x = np.zeros((K, K), np.float32)
    np.fill_diagonal(x, 1.0)
    y, mag = oracle.gemv_w4a16(bf16_bits(x), codes, scales, bits, tb, g, S, fmt)   # [K, N]
    deq = oracle.dequant_sel(codes, scales, bits, tb, g, S, fmt)                   # [N, K] bf16 bits
    assert (bf16_bits(y.T) == deq).all()
    assert (mag == np.abs(y.astype(np.float64))).all()


def test_hand_worked_product():
    # INT4, g = S = 16: tables T0 = -8..7, T1 = T0 + 0.5; one row.  Codes 0..15 on table 1
    # (scale sign set) with scale 2^-6 -> w^ = (c - 7.5) / 64; x = 1 for even k, 2 for odd k.
    tb = bf16_bits(np.concatenate([np.arange(-8, 8), np.arange(-8, 8) + 0.5]).astype(np.float32))
    codes = np.array([[(2 * i) | ((2 * i + 1) << 4) for i in range(8)]], np.uint8)
    scales = np.array([[0x3C80 | 0x8000]], np.uint16)
    x = bf16_bits(np.array([[1, 2] * 8], np.float32))
    y, mag = oracle.gemv_w4a16(x, codes, scales, None, tb, 16, 16, oracle.INT4)
    want = sum((1 if k % 2 == 0 else 2) * (k - 7.5) / 64 for k in range(16))
    assert y[0, 0] == np.float32(want) and want == 0.0625   # (56 - 60 + 2 * (64 - 60)) / 64
    assert mag[0, 0] == sum((1 if k % 2 == 0 else 2) * abs(k - 7.5) / 64 for k in range(16))
    # the same codes on table 0 (sign clear): w^ = (c - 8) / 64
    scales0 = np.array([[0x3C80]], np.uint16)
    y0, _ = oracle.gemv_w4a16(x, codes, scales0, None, tb, 16, 16, oracle.INT4)
    assert y0[0, 0] == np.float32(sum((1 if k % 2 == 0 else 2) * (k - 8) / 64 for k in range(16)))


def test_linear_in_x_and_rejects_bad_shapes():
    N, K, g, fmt = 6, 128, 16, oracle.NVFP4
    _, tb, codes, scales, bits = quantised_layer(99, N, K, g, g, fmt)
    rng = np.random.default_rng(1)
    a = bf16_bits(rng.integers(-4, 5, (1, K)).astype(np.float32))
    b = bf16_bits(rng.integers(-4, 5, (1, K)).astype(np.float32))
    ab = bf16_bits(bf16_vals(a) + bf16_vals(b))       # small integers: the sum is exact in bf16
    ya, _ = oracle.gemv_w4a16(a, codes, scales, None, tb, g, g, fmt)
    yb, _ = oracle.gemv_w4a16(b, codes, scales, None, tb, g, g, fmt)
    yab, _ = oracle.gemv_w4a16(ab, codes, scales, None, tb, g, g, fmt)
    assert np.allclose(yab, ya.astype(np.float64) + yb, rtol=1e-6, atol=1e-7)
    with pytest.raises(ValueError):
        oracle.gemv_w4a16(a, codes, scales, None, tb, 128, 16, fmt)   # S < g without selection bits


@pytest.mark.parametrize("g,S,fmt", [(16, 16, oracle.NVFP4), (128, 16, oracle.INT4)])
def test_rounded_weight_product_is_the_matmul_with_the_dequantised_layer(g, S, fmt):
    # oracle.gemm_w4a16 = x times exactly the bf16 weights that the pinned dequantisation returns
    N, K, M = 10, 256, 3
    _, tb, codes, scales, bits = quantised_layer(101 + g, N, K, g, S, fmt)
    rng = np.random.default_rng(g + 1)
    x = bf16_bits(rng.standard_normal((M, K)))
    y, mag = oracle.gemm_w4a16(x, codes, scales, bits, tb, g, S, fmt)
    What = bf16_vals(oracle.dequant_sel(codes, scales, bits, tb, g, S, fmt)).astype(np.float64)
    xr = bf16_vals(x).astype(np.float64)
    assert np.allclose(y, xr @ What.T, rtol=1e-6, atol=1e-6 * np.abs(xr @ What.T).max())
    assert np.allclose(mag, (np.abs(xr)[:, None, :] * np.abs(What)[None, :, :]).sum(axis=2), rtol=1e-12)
    # it differs from the unrounded product by at most the bf16 rounding of each weight
    y0, mag0 = oracle.gemv_w4a16(x, codes, scales, bits, tb, g, S, fmt)
    assert (np.abs(y.astype(np.float64) - y0) <= 2.0 ** -8 * mag0).all() and (y != y0).any()
