"""Randomised parity sweep (GPU): the whole path against the CPU oracle on seeded random shapes and
settings inside the documented limits of every entry point - group and selection sizes, both scale
formats, both loops, quantile or format-grid start, padded strides, zero groups, ties, extreme
ranges, zero importances; and both W4A16 products on random quantised layers.  The fixed cases of
test_gpu_parity.py are chosen by hand; these are not."""
import numpy as np
import pytest
import torch

import paper_2605_08692_amd as A
from paper_2605_08692_amd import inputs
import oracle
import test_gpu_parity as T

pytestmark = pytest.mark.gpu
DEV = T.DEV


def rand_weight(rng, N, K, seed):
    kind = int(rng.integers(0, 5))
    W = inputs.make_weight(N, K, "gauss_outlier" if kind % 2 == 0 else "student5", seed, DEV)
    if kind == 2:    # all-zero rows and leading groups
        W[int(rng.integers(0, N))] = 0
        W[:, : 16 * int(rng.integers(1, max(2, K // 32)))] *= (torch.rand(N, 1, device=DEV, generator=T.seeded(10 * seed + 1)) < 0.7).to(torch.bfloat16)
    elif kind == 3:  # rows of very different magnitude
        W = (W.float() * torch.exp(torch.randn(N, 1, device=DEV, generator=T.seeded(10 * seed + 2)) * 4)).to(torch.bfloat16)
    elif kind == 4:  # few distinct values: ties in every search
        W = (torch.round(W.float() * 200) / 200).to(torch.bfloat16)
    return W


def rand_importance(rng, K, seed):
    I = torch.rand(K, device=DEV, generator=T.seeded(10 * seed + 3)) * float(10 ** rng.uniform(-3, 3)) + 1e-6
    k = int(rng.integers(0, 3))
    if k == 1:
        I[torch.rand(K, device=DEV, generator=T.seeded(10 * seed + 4)) < 0.2] = 0
    elif k == 2:
        I[torch.rand(K, device=DEV, generator=T.seeded(10 * seed + 5)) < 0.02] *= 1e4
    return I


@pytest.mark.parametrize("seed", range(40))
def test_random_fit_encode_dequant(seed):
    rng = np.random.default_rng(1000 + seed)
    fmt = int(rng.integers(0, 2))
    g = int(rng.choice([16, 32, 64, 128]))
    S = int(rng.choice([s for s in (16, 32, 64, 128) if s <= g]))
    K = g * int(rng.integers(1, max(2, 2304 // g)))
    N = int(rng.integers(1, 160))
    n_outer, n_inner = int(rng.integers(0, 4)), int(rng.integers(1, 4))
    while N * K * max(1, n_outer * n_inner) > 3.0e6:
        N = max(1, N // 2)
    pad = int(rng.integers(0, 3))
    quantile = bool(rng.integers(0, 3) == 0)
    T.say(f"[sweep {seed}] N={N} K={K} g={g} S={S} fmt={fmt} outer={n_outer} inner={n_inner} pad={pad} quantile={quantile}")
    W, I = rand_weight(rng, N, K, 5000 + seed), rand_importance(rng, K, 5000 + seed)
    grid = None
    if quantile:
        grid = oracle.quantile_init(inputs.bits(W), g, fmt)
        qg = A.aaac_quantile_init(W, g, fmt)
        torch.cuda.synchronize()
        assert (T.u32(T.host(qg)) == T.u32(grid)).all()
    T.check_sel_layer(W, I, g, S, fmt, n_outer, n_inner, grid=grid, pad_stride=pad)


@pytest.mark.parametrize("seed", range(40))
def test_random_w4a16_products(seed):
    rng = np.random.default_rng(2000 + seed)
    fmt = int(rng.integers(0, 2))
    g = int(rng.choice([16, 32, 64, 128]))
    S = int(rng.choice([s for s in (16, 32, 64, 128) if s <= g]))
    matrix_cores = bool(seed % 2)
    unit = max(g, 64 if matrix_cores else 32)
    K = unit * int(rng.integers(1, max(2, 4608 // unit)))
    N = int(rng.integers(1, 400))
    M = int(rng.choice([1, 2, 3, 4, 5, 8, 9, 16, 17, 32, 33, 48, 64, 65, 100, 129, 200, 257, 300])) if matrix_cores \
        else int(rng.integers(1, 20))
    if matrix_cores and seed % 8 == 7:  # long rows, few of them: K split over several blocks
        K, N, M = int(rng.choice([6144, 8192, 12288, 16384])), int(rng.integers(1, 130)), int(rng.integers(1, 41))
    while N * K * M > 6.0e7:
        N = max(1, N // 2)
    T.say(f"[sweep {seed}] {'gemm' if matrix_cores else 'gemv'} N={N} K={K} g={g} S={S} fmt={fmt} M={M}")
    tb, codes, scales, bits = T.synthetic_quantised_layer(N, K, g, S, fmt, 7000 + seed)
    x = (torch.randn((M, K), device=DEV, generator=T.seeded(70000 + seed)) * 2).to(torch.bfloat16)
    if matrix_cores:
        y = A.aaac_gemm_w4a16(x, codes, scales, bits, tb, g, S, fmt)
        torch.cuda.synchronize()
        ref, mag = oracle.gemm_w4a16(*T.oracle_args(x, codes, scales, bits, tb, fmt), g, S, fmt)
        err = np.abs(T.host(y).astype(np.float64) - ref)
        assert (err <= (K + 8) * 2.0 ** -24 * mag + np.spacing(np.abs(ref))).all()
        assert np.median(err / (mag + 1e-30)) < 16 * 2.0 ** -24
    else:
        y = A.aaac_gemv_w4a16(x, codes, scales, bits, tb, g, S, fmt)
        torch.cuda.synchronize()
        ref, mag = oracle.gemv_w4a16(*T.oracle_args(x, codes, scales, bits, tb, fmt), g, S, fmt)
        err = np.abs(T.host(y).astype(np.float64) - ref)
        assert (err <= T.gemv_tolerance(K, mag) + np.spacing(np.abs(ref))).all()
