"""Pins for selection groups smaller than scale groups (S < g; paper "Granularity
parameters", Alg. 1 last step): every g weights share a scale, every S weights a
table choice, and the choices are stored as separate bits."""
import json
import os

import numpy as np
import pytest

import oracle
from paper_2605_08692_amd import inputs

from test_oracle_method import unpack
from test_oracle_steps import bf16_bits, bf16_vals, brute_assign, random_layer

GOLD = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "worked_vectors.json")))
FMT = {"nvfp4": oracle.NVFP4, "int4": oracle.INT4}


def unpack_bits(bits, n_groups):
    return np.unpackbits(bits, axis=1, bitorder="little")[:, :n_groups]


@pytest.mark.parametrize("case", GOLD["sel_cases"], ids=lambda c: c["name"])
def test_worked_vector_with_two_selection_groups(case):
    fmt, g, S = FMT[case["fmt"]], case["g"], case["S"]
    W = np.array(case["W"], np.float32)[None, :]
    Wb = bf16_bits(W)
    assert (bf16_vals(Wb) == W).all()
    tb = bf16_bits(np.array(case["T0"] + case["T1"], np.float32))
    I = (np.arange(W.shape[1]) % 5 + 1).astype(np.float32)
    codes, scales, bits = oracle.encode_sel(Wb, g, S, fmt, I, tb)
    assert (unpack(codes) == np.array(case["codes"], np.uint8)[None, :]).all()
    assert scales.tolist() == [[case["scale"]]]          # unsigned: sigma is not in the scale
    assert bits.tolist() == [case["sel_bits"]]
    assert unpack_bits(bits, len(case["sigma"])).tolist() == [case["sigma"]]
    assert (oracle.dequant_sel(codes, scales, bits, tb, g, S, fmt) == Wb).all()
    # with one choice for the whole scale group neither table fits all 32 weights exactly
    c1, s1 = oracle.encode(Wb, g, fmt, I, tb)
    assert (oracle.dequant(c1, s1, tb, g, fmt) != Wb).any()


def test_equal_sizes_reduce_to_the_sign_bit_path():
    W, I = random_layer(61, 24, 512)
    for g, fmt in ((16, oracle.NVFP4), (128, oracle.INT4), (64, oracle.INT4)):
        grid = inputs.format_grid(fmt)
        a = oracle.fit_nested(W, g, fmt, I, grid, 2, 3, trace=True)
        b = oracle.fit_sel(W, g, g, fmt, I, grid, 2, 3, trace=True)
        assert (a["tables_trace"] == b["tables_trace"]).all() and (a["objective"] == b["objective"]).all()
        c0, s0 = oracle.encode(W, g, fmt, I, a["tables_bf16"])
        c1, s1, bits = oracle.encode_sel(W, g, g, fmt, I, a["tables_bf16"])
        assert bits is None and (c0 == c1).all() and (s0 == s1).all()
        assert (oracle.dequant(c0, s0, a["tables_bf16"], g, fmt)
                == oracle.dequant_sel(c1, s1, None, a["tables_bf16"], g, g, fmt)).all()


@pytest.mark.parametrize("g,S,fmt", [(128, 16, oracle.INT4), (128, 64, oracle.INT4), (64, 32, oracle.INT4),
                                     (32, 16, oracle.NVFP4)])
def test_selection_bits_follow_brute_force_errors_of_the_small_groups(g, S, fmt):
    W, I = random_layer(63 + S, 10, 512)
    codes_s, vals, wn = oracle.normalise(W, g, fmt)
    rng = np.random.default_rng(S)
    tables = np.concatenate([np.sort(rng.standard_normal(16) * 3), np.sort(rng.standard_normal(16) * 3 + 0.2)])
    tb = bf16_bits(tables.astype(np.float32))
    T = bf16_vals(tb)
    codes, scales, bits = oracle.encode_sel(W, g, S, fmt, I, tb)
    assert (scales == codes_s).all()                     # scales of the g-groups, no sign
    (i0, e0), (i1, e1) = brute_assign(wn, S, I, T)      # fp64 brute force per S weights
    sigma = unpack_bits(bits, 512 // S)
    clear = np.abs(e0 - e1) > 1e-5 * np.maximum(e0, e1)
    assert clear.mean() > 0.9 and (sigma[clear] == (e1 < e0)[clear]).all()
    assert 0.1 < sigma.mean() < 0.9
    # codes index the table each small group chose
    rep = np.repeat(sigma, S, axis=1)
    want = np.where(rep == 1, i1, i0)
    assert (unpack(codes) != want).mean() < 1e-3
    # dequantised value = chosen entry times the scale of the enclosing g-group
    ent = np.where(rep == 1, T[16 + unpack(codes).astype(int)], T[unpack(codes).astype(int)])
    ref = bf16_bits(ent * np.repeat(vals, g, axis=1))
    assert (oracle.dequant_sel(codes, scales, bits, tb, g, S, fmt) == ref).all()
    # padding bits of each row's last byte are zero and the bit count is K/S per row
    assert bits.shape == (10, (512 // S + 7) // 8)
    assert (np.unpackbits(bits, axis=1, bitorder="little")[:, 512 // S:] == 0).all()


def test_finer_selection_never_raises_the_objective_of_given_tables():
    # sum over small groups of min(e0, e1) <= min over tables of the sums; the pairwise tree makes
    # the error of a 128-group the tree sum of its eight 16-group errors, so this holds in fp32 too
    W, I = random_layer(67, 16, 1024)
    _, _, wn = oracle.normalise(W, 128, oracle.INT4)
    tables = np.concatenate([inputs.INT4_GRID, inputs.INT4_GRID + np.float32(0.4)]).astype(np.float32)
    J = [oracle.assign(wn, S, I, tables)["objective"] for S in (128, 64, 32, 16)]
    assert all(b <= a * (1 + 1e-6) for a, b in zip(J, J[1:])) and J[-1] < 0.99 * J[0]
    a128 = oracle.assign(wn, 128, I, tables)
    a16 = oracle.assign(wn, 16, I, tables)
    for r in ("e0", "e1"):
        tree = a16[r].reshape(16, 8, 8).copy()
        tree = tree[:, :, 0::2] + tree[:, :, 1::2]
        tree = tree[:, :, 0::2] + tree[:, :, 1::2]
        tree = tree[:, :, 0] + tree[:, :, 1]
        assert (tree == a128[r]).all()


def test_learning_with_small_selection_groups_composes_the_pinned_steps():
    # fit_sel = normalise with g, then the assignment and k-means steps with S
    W, I = random_layer(69, 20, 512)
    g, S, fmt = 128, 16, oracle.INT4
    grid = inputs.format_grid(fmt)
    res = oracle.fit_sel(W, g, S, fmt, I, grid, 3, 2, trace=True)
    _, _, wn = oracle.normalise(W, g, fmt)
    T = grid.copy()
    trace, obj = [], []
    for _ in range(3):
        a = oracle.assign(wn, S, I, T)
        obj.append(a["objective"])
        for _ in range(2):
            T = oracle.kmeans_step(wn, S, I, a["sigma"], T)
            trace.append(T.copy())
    assert (np.array(trace) == res["tables_trace"]).all() and (np.array(obj) == res["objective"]).all()
    # finer selection ends at a lower objective than one choice per scale group on the same data
    coarse = oracle.fit_sel(W, g, g, fmt, I, grid, 3, 2)
    assert res["objective"][-1] < coarse["objective"][-1]
    assert (np.diff(res["objective"]) <= 1e-9 * res["objective"][0]).all()


def test_rejects_bad_group_sizes():
    W, I = random_layer(71, 4, 256)
    grid = inputs.format_grid(oracle.INT4)
    with pytest.raises(ValueError):
        oracle.fit_sel(W, 64, 128, oracle.INT4, I, grid, 1, 1)   # S > g
    with pytest.raises(ValueError):
        oracle.fit_sel(W, 128, 24, oracle.INT4, I, grid, 1, 1)   # S not a supported size
