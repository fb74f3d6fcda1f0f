"""Pins for the oracle's number formats and for its importance step.

The bf16 and FP8-E4M3 rounders are checked against PyTorch's own conversions
(a library routine the oracle does not use), exhaustively over the FP8 codes,
and against hand-derived values; importance against closed forms.
"""
import json
import os

import numpy as np
import torch

import oracle

GOLD = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "worked_vectors.json")))


def test_bf16_widening_matches_torch():
    h = np.arange(0, 1 << 16, 7, dtype=np.uint16)
    ref = torch.from_numpy(h.view(np.int16)).view(torch.bfloat16).float().numpy()
    got = np.array([oracle.bf16_to_f32(int(x)) for x in h], np.float32)
    ok = (got == ref) | (np.isnan(got) & np.isnan(ref))
    assert ok.all()


def test_bf16_rounding_matches_torch_and_ties_to_even():
    rng = np.random.default_rng(0)
    x = np.concatenate([
        rng.standard_normal(4000).astype(np.float32) * np.float32(0.02),
        rng.standard_normal(1000).astype(np.float32) * np.float32(1e-38),  # fp32 subnormals
        np.array([0.0, -0.0, 1.0, 1.00390625, 1.01171875, -1.00390625, 3.3895e38, 65504.0], np.float32),
    ])
    # exact ties: bf16 value + half a bf16 ulp
    base = (rng.integers(0x0080, 0x7F00, 2000).astype(np.uint32) << 16) | 0x8000
    x = np.concatenate([x, base.view(np.float32)])
    ref = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    got = np.array([oracle.f32_to_bf16(v) for v in x], np.uint16)
    assert (got == ref).all()
    # 1 + 2^-8 is a tie between 0x3F80 (even) and 0x3F81: even wins; 1 + 3*2^-8 goes up to 0x3F82
    assert oracle.f32_to_bf16(1.00390625) == 0x3F80
    assert oracle.f32_to_bf16(1.01171875) == 0x3F82


def test_e4m3_decode_all_codes_matches_torch():
    codes = np.arange(256, dtype=np.uint8)
    ref = torch.from_numpy(codes).view(torch.float8_e4m3fn).float().numpy()
    got = np.array([oracle.e4m3_to_f32(int(c)) for c in codes], np.float32)
    ok = (got == ref) | (np.isnan(got) & np.isnan(ref))
    assert ok.all()
    assert oracle.e4m3_to_f32(0x7E) == 448.0 and oracle.e4m3_to_f32(0x01) == 2.0 ** -9


def test_e4m3_round_trip_midpoints_and_neighbours():
    vals = [oracle.e4m3_to_f32(c) for c in range(0x7F)]
    assert all(b > a for a, b in zip(vals, vals[1:]))  # strictly ascending magnitudes
    for c in range(0x7F):
        assert oracle.f32_to_e4m3(vals[c]) == c
        assert oracle.f32_to_e4m3(-vals[c]) == (c | 0x80) or c == 0
    for c in range(0x7E):
        mid = np.float32((np.float64(vals[c]) + np.float64(vals[c + 1])) / 2)  # exact in fp32
        even = c if c % 2 == 0 else c + 1
        assert oracle.f32_to_e4m3(mid) == even
        below = np.nextafter(mid, np.float32(0), dtype=np.float32)
        above = np.nextafter(mid, np.float32(1e9), dtype=np.float32)
        assert oracle.f32_to_e4m3(below) == c
        assert oracle.f32_to_e4m3(above) == c + 1


def test_e4m3_rounding_matches_torch_in_range():
    rng = np.random.default_rng(1)
    x = np.abs(rng.standard_normal(5000)).astype(np.float32) * np.float32(0.01)
    x = np.concatenate([x, np.abs(rng.standard_normal(2000)).astype(np.float32) * np.float32(50)])
    x = x[x < 440]
    ref = torch.from_numpy(x).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    got = np.array([oracle.f32_to_e4m3(v) for v in x], np.uint8)
    assert (got == ref).all()


def test_e4m3_hand_values():
    for value, code in GOLD["e4m3_hand_values"]["pairs"]:
        assert oracle.f32_to_e4m3(value) == code, (value, code)


def _bf16_bits(a):
    return torch.from_numpy(np.asarray(a, np.float32)).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)


def test_importance_closed_form_powers_of_two():
    # X[t,k] = 2^(k mod 8)  =>  I_k = tokens * 4^(k mod 8), exactly
    tokens, K = 37, 24
    X = np.tile(2.0 ** (np.arange(K) % 8), (tokens, 1)).astype(np.float32)
    I = oracle.act_stats(_bf16_bits(X))
    assert (I == (tokens * 4.0 ** (np.arange(K) % 8)).astype(np.float32)).all()


def test_importance_is_per_column_sum_over_tokens():
    # distinct columns and more tokens than columns: a transposed or row-wise sum fails
    rng = np.random.default_rng(2)
    tokens, K = 50, 8
    Xb = _bf16_bits(rng.standard_normal((tokens, K)) * (1 + np.arange(K)))
    Xf = torch.from_numpy(Xb.view(np.int16)).view(torch.bfloat16).double().numpy()
    ref = (Xf ** 2).sum(axis=0)
    I = oracle.act_stats(Xb)
    assert I.shape == (K,)
    assert np.allclose(I, ref, rtol=1e-7, atol=0)
    # sign of the activations cannot matter, an extra token adds its square
    assert (oracle.act_stats(_bf16_bits(-Xf)) == I).all()
    extra = np.vstack([Xf, np.full((1, K), 3.0)])
    assert np.allclose(oracle.act_stats(_bf16_bits(extra)), ref + 9.0, rtol=1e-7)


def test_importance_long_sum_is_accurate():
    # 2^20 tokens of alternating large / tiny squares: a plain fp32 running sum
    # would lose the small terms; the result must be the exact sum rounded once
    tokens = 1 << 16
    col = np.where(np.arange(tokens) % 2 == 0, 256.0, 2.0 ** -4).astype(np.float32)
    X = np.stack([col, np.ones(tokens, np.float32)], axis=1)
    I = oracle.act_stats(_bf16_bits(X))
    exact0 = (tokens // 2) * (65536.0 + 2.0 ** -8)
    assert I[0] == np.float32(exact0) and I[1] == np.float32(tokens)
