"""GPU parity: the HIP library (through its C ABI) against the CPU oracle,
element by element on the same seeded inputs.

Bars: scale codes, 4-bit codes, selection bits, bf16 tables and dequantised
weights bit-exact; fp32 tables within 1e-5 relative (+1e-6 of the table's range
near zero); importance within 1e-6 relative; objective within 1e-9 relative.
"""
import contextlib
import json
import os
import time

import numpy as np
import pytest
import torch

import oracle
import paper_2605_08692_amd as A
from paper_2605_08692_amd import inputs

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
GOLD = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "worked_vectors.json")))


def say(*a):
    print(*a, flush=True)


def seeded(seed):
    """A generator on the test device with a fixed seed: every random draw of these tests names one."""
    return torch.Generator(device=DEV).manual_seed(int(seed))


@contextlib.contextmanager
def fit_path(name):
    """Route the fits inside the block through one of the library's two paths: "launches" (one launch
    per pass over the weights) or "persistent" (all passes of a small layer in one launch); layers
    the persistent path does not take go through launches either way."""
    old = os.environ.get("AAAC_FIT_PATH")
    os.environ["AAAC_FIT_PATH"] = name
    try:
        yield
    finally:
        if old is None:
            del os.environ["AAAC_FIT_PATH"]
        else:
            os.environ["AAAC_FIT_PATH"] = old


FIT_PATHS = ("launches", "persistent")


def tables_close(gpu, ref):
    gpu, ref = np.asarray(gpu, np.float64), np.asarray(ref, np.float64)
    tol = 1e-5 * np.maximum(np.abs(gpu), np.abs(ref)) + 1e-6 * np.abs(ref).max()
    return (np.abs(gpu - ref) <= tol).all()


def host(t):
    return t.detach().cpu().numpy()


def u16(t):
    if t.dtype == torch.bfloat16:
        t = t.contiguous().view(torch.int16)
    return host(t).view(np.uint16)


def check_layer(Wt, I_host, g, fmt, grid, iters, label, check_dequant=True):
    """fit + encode + dequant on the GPU vs the oracle for one layer."""
    say(f"[parity] {label}: N={Wt.shape[0]} K={Wt.shape[1]} g={g} fmt={fmt} iters={iters}")
    Wb = inputs.bits(Wt)
    It = torch.from_numpy(I_host).to(DEV)
    t0 = time.time()
    ref = oracle.fit(Wb, g, fmt, I_host, grid, iters, trace=True)
    rc, rs = oracle.encode(Wb, g, fmt, I_host, ref["tables_bf16"])
    say(f"[parity] {label}: oracle {time.time() - t0:.1f}s")
    for path in FIT_PATHS:  # both ways through the library (the same one for layers too large for "persistent")
        with fit_path(path):
            tf, tb, obj = A.aaac_fit(Wt, g, fmt, It, grid, iters)
            torch.cuda.synchronize()
            tfh, tbh = host(tf), u16(tb)
            if not (tbh == ref["tables_bf16"]).all() or not tables_close(tfh, ref["tables_f32"]):
                # locate the first iteration whose tables differ, to tell a 1-ulp flip from a bug
                for t in range(1, iters + 1):
                    tft, _, _ = A.aaac_fit(Wt, g, fmt, It, grid, t)
                    torch.cuda.synchronize()
                    d = host(tft) != ref["tables_trace"][t - 1]
                    if d.any():
                        say(f"[parity] {label} ({path}): first table difference at iteration {t}: entries "
                            f"{np.nonzero(d)[0]}", host(tft)[d], ref["tables_trace"][t - 1][d])
                        break
        assert tables_close(tfh, ref["tables_f32"]), (path, tfh, ref["tables_f32"])
        assert (tbh == ref["tables_bf16"]).all(), path
        if iters:
            o = host(obj)[:iters]
            assert np.allclose(o, ref["objective"], rtol=1e-9, atol=0), (path, o, ref["objective"])
    codes, scales = A.aaac_encode(Wt, g, fmt, It, tb)
    What = A.aaac_dequant(codes, scales, tb, g, fmt)
    torch.cuda.synchronize()
    sc = host(scales).view(rs.dtype)
    assert (sc == rs).all(), f"{(sc != rs).sum()} scale/selection mismatches"
    ch = host(codes)
    assert (ch == rc).all(), f"{(ch != rc).sum()} code byte mismatches"
    if check_dequant:
        rd = oracle.dequant(rc, rs, ref["tables_bf16"], g, fmt)
        assert (u16(What) == rd).all()
    return ref


def importance_for(cfg, key):
    X = inputs.activations(cfg["xs"][key], DEV)
    I = A.aaac_act_stats(X)
    torch.cuda.synchronize()
    return X, I


# ------------------------------------------------------------- importance

@pytest.mark.parametrize("tokens,K,pad", [(256, 512, 0), (37, 520, 8), (1, 8, 0), (1000, 1032, 24), (4096, 4096, 0),
                                          (700, 28672, 0),     # 7 column groups of 4096
                                          (5000, 11008, 0),    # 3 column groups x 85 token chunks, ragged last group
                                          (300, 12000, 16)])
def test_act_stats_matches_oracle(tokens, K, pad):
    say(f"[act_stats] tokens={tokens} K={K} pad={pad}")
    X = inputs.make_activations(tokens, K + pad, ("gauss", 3, "x20"), 7, DEV)[:, :K]
    I = A.aaac_act_stats(X)
    torch.cuda.synchronize()
    ref = oracle.act_stats(inputs.bits(X))
    assert np.allclose(host(I), ref, rtol=1e-6, atol=0)
    assert (host(I) == ref).mean() > 0.999


def test_act_stats_empty_and_exact():
    I = A.aaac_act_stats(torch.empty((0, 64), dtype=torch.bfloat16, device=DEV))
    torch.cuda.synchronize()
    assert (host(I) == 0).all()
    X = torch.full((300, 16), 3.0, dtype=torch.bfloat16, device=DEV)
    I = A.aaac_act_stats(X)
    torch.cuda.synchronize()
    assert (host(I) == 2700.0).all()


# ------------------------------------------------------- formats and scales

def test_scale_codes_cover_every_e4m3_boundary():
    # one group per candidate absmax: 6 * (each E4M3 value, each midpoint, and the
    # bf16 neighbours of those), so every rounding boundary of the FP8 scale is hit
    vals = np.array([oracle.e4m3_to_f32(c) for c in range(0x7F)], np.float64)
    cand = np.concatenate([vals, (vals[:-1] + vals[1:]) / 2, [0.0, 1e-30, 500.0, 1e5]]) * 6.0
    b = torch.from_numpy(cand.astype(np.float32)).to(torch.bfloat16).view(torch.int16).numpy().astype(np.int32)
    b = np.unique(np.concatenate([b - 1, b, b + 1]).clip(0, 0x7F7F)).astype(np.uint16)
    W = np.zeros((b.size, 16), np.uint16)
    W[:, 3] = b
    W[::2, 3] |= 0x8000  # sign must not matter
    Wt = inputs.from_bits(W, DEV)
    I = torch.ones(16, device=DEV)
    tb = torch.from_numpy(oracle.fit(W, 16, 0, np.ones(16, np.float32), inputs.format_grid(0), 0)["tables_bf16"].view(np.int16)).to(DEV)
    codes, scales = A.aaac_encode(Wt, 16, A.NVFP4, I, tb)
    torch.cuda.synchronize()
    rc, rs = oracle.encode(W, 16, 0, np.ones(16, np.float32), host(tb).view(np.uint16))
    assert (host(scales) == rs).all() and (host(codes) == rc).all()
    assert len(np.unique(rs & 0x7F)) > 120
    # bf16 scales: absmax/7 over many magnitudes, including tiny ones
    rng = np.random.default_rng(5)
    Wf = (rng.standard_normal((512, 128)) * np.exp(rng.uniform(-60, 10, (512, 1)))).astype(np.float32)
    Wf[0] = 0
    Wt = torch.from_numpy(Wf).to(torch.bfloat16).to(DEV)
    I = torch.ones(128, device=DEV)
    tb = torch.from_numpy(oracle.fit(inputs.bits(Wt), 128, 1, np.ones(128, np.float32), inputs.format_grid(1), 0)["tables_bf16"].view(np.int16)).to(DEV)
    codes, scales = A.aaac_encode(Wt, 128, A.INT4, I, tb)
    torch.cuda.synchronize()
    rc, rs = oracle.encode(inputs.bits(Wt), 128, 1, np.ones(128, np.float32), host(tb).view(np.uint16))
    assert (host(scales).view(np.uint16) == rs).all() and (host(codes) == rc).all()



@pytest.mark.parametrize("fmt,g", [(A.NVFP4, 16), (A.INT4, 128), (A.INT4, 32)])
def test_scales_and_codes_for_every_bf16_absmax(fmt, g):
    """A group's absmax is a bf16 value, so these 32,639 groups are every finite input that the
    scale's division (absmax / 6, absmax / 7) and the reciprocal 1 / s can meet; the other weights
    of a group are fractions of the absmax, so their codes depend on the rounded reciprocal."""
    say(f"[scales] every bf16 absmax, fmt={fmt} g={g}")
    amax = np.arange(1, 0x7F80, dtype=np.uint16)                       # all positive finite bf16 values
    n = amax.size
    rng = np.random.default_rng(31 + g)
    frac = rng.uniform(-1.0, 1.0, (n, g)).astype(np.float32)
    Wf = frac * (amax.astype(np.uint32) << 16).view(np.float32)[:, None]
    Wt = torch.from_numpy(Wf).to(torch.bfloat16)
    Wb = Wt.view(torch.int16).numpy().view(np.uint16).copy()
    pos = rng.integers(0, g, n)
    Wb[np.arange(n), pos] = amax | (rng.integers(0, 2, n).astype(np.uint16) << 15)   # the absmax itself, either sign
    rows = 128                                                          # groups per row: K = 128 g
    pad = (-n) % rows
    Wb = np.concatenate([Wb, np.zeros((pad, g), np.uint16)]).reshape(-1, rows * g)
    Wt = inputs.from_bits(Wb, DEV)
    K = Wb.shape[1]
    I = torch.rand(K, device=DEV, generator=seeded(977 + g)) + 0.1
    tb = torch.from_numpy(oracle.fit(Wb[:4], g, fmt, np.ones(K, np.float32), inputs.format_grid(fmt), 0)["tables_bf16"].view(np.int16)).to(DEV)
    codes, scales = A.aaac_encode(Wt, g, fmt, I, tb)
    What = A.aaac_dequant(codes, scales, tb, g, fmt)
    torch.cuda.synchronize()
    rc, rs = oracle.encode(Wb, g, fmt, host(I), host(tb).view(np.uint16))
    sc = host(scales) if fmt == A.NVFP4 else host(scales).view(np.uint16)
    assert (sc == rs).all()
    assert (host(codes) == rc).all()
    assert (u16(What) == oracle.dequant(rc, rs, host(tb).view(np.uint16), g, fmt)).all()

@pytest.mark.parametrize("case", GOLD["cases"], ids=lambda c: c["name"])
def test_worked_vectors_on_gpu(case):
    from test_oracle_method import FMT, case_arrays, unpack
    fmt, g = FMT[case["fmt"]], case["g"]
    W, codes_ref = case_arrays(case)
    Wt = torch.from_numpy(W).to(torch.bfloat16).to(DEV)
    tables = np.array(case["T0"] + case["T1"], np.float32)
    I = torch.from_numpy((np.arange(W.shape[1]) % 5 + 1).astype(np.float32)).to(DEV)
    tf, tb, _ = A.aaac_fit(Wt, g, fmt, I, tables, 0)
    codes, scales = A.aaac_encode(Wt, g, fmt, I, tb)
    What = A.aaac_dequant(codes, scales, tb, g, fmt)
    torch.cuda.synchronize()
    assert (host(tf) == tables).all()
    assert (unpack(host(codes)) == codes_ref).all()
    assert host(scales).view(np.uint8 if fmt == 0 else np.uint16).tolist() == [[case["scale"]]]
    assert (u16(What) == inputs.bits(Wt)).all()
    if case["tables_fixed_point"]:
        tf5, _, obj = A.aaac_fit(Wt, g, fmt, I, tables, 5)
        torch.cuda.synchronize()
        assert (host(tf5) == tables).all() and (host(obj)[:5] == 0).all()


# ------------------------------------------------- fit / encode / dequant

@pytest.mark.parametrize("N,K,g,fmt,iters", [
    (256, 512, 16, 0, 10),     # the small benchmark shape
    (37, 1040, 16, 0, 4),      # ragged: K spans two strips plus a tail, odd row count
    (5, 128, 128, 1, 3),       # a single group per row
    (130, 1536, 128, 1, 5),
    (64, 640, 32, 1, 4),
    (64, 704, 64, 0, 4),
    (1, 16, 16, 0, 2),         # smallest possible layer
    (3000, 512, 16, 0, 3),     # several rows per wavefront
])
def test_fit_encode_dequant_match_oracle(N, K, g, fmt, iters):
    Wt = inputs.make_weight(N, K, "gauss_outlier", 50 + N + K, DEV)
    X = inputs.make_activations(64, K, ("gauss", 0.01, "u10_50"), 60 + K, DEV)
    I = oracle.act_stats(inputs.bits(X))
    check_layer(Wt, I, g, fmt, inputs.format_grid(fmt), iters, f"small{N}x{K}")


def test_distinct_initial_tables_and_padded_rows():
    # T0 != T1 from the start, leading dimension larger than K
    N, K, g = 96, 1024, 16
    full = inputs.make_weight(N, K + 64, "student5", 77, DEV)
    Wt = full[:, :K]
    I = oracle.act_stats(inputs.bits(inputs.make_activations(128, K, ("silu_gate", 0.005, "x30"), 78, DEV)))
    grid = np.concatenate([inputs.E2M1_GRID, inputs.E2M1_GRID + np.float32(0.25)]).astype(np.float32)
    Wc = Wt.contiguous()
    ref = check_layer(Wc, I, g, 0, grid, 4, "distinct_init")
    It = torch.from_numpy(I).to(DEV)
    tf, tb, _ = A.aaac_fit(Wt, g, 0, It, grid, 4)
    codes, scales = A.aaac_encode(Wt, g, 0, It, tb)
    out = torch.zeros((N, K + 64), dtype=torch.bfloat16, device=DEV)
    A.aaac_dequant(codes, scales, tb, g, 0, W_hat=out[:, :K])
    torch.cuda.synchronize()
    assert (u16(tb) == ref["tables_bf16"]).all()
    rc, rs = oracle.encode(inputs.bits(Wc), g, 0, I, ref["tables_bf16"])
    assert (host(codes) == rc).all() and (host(scales) == rs).all()
    assert (u16(out[:, :K].contiguous()) == oracle.dequant(rc, rs, ref["tables_bf16"], g, 0)).all()
    assert (out[:, K:] == 0).all()


@pytest.mark.parametrize("fmt,g", [(0, 16), (1, 128)])
def test_clustered_and_duplicate_table_entries(fmt, g):
    """Entries closer together than a search bucket, triples of equal entries and a
    whole table collapsed to one value: the bucket search must fall back to the
    plain count and still agree with the oracle."""
    Wt = inputs.make_weight(96, 1024, "gauss_outlier", 91, DEV)
    I = oracle.act_stats(inputs.bits(inputs.make_activations(64, 1024, ("gauss", 0.01, "u10_50"), 92, DEV)))
    base = inputs.E2M1_GRID if fmt == 0 else inputs.INT4_GRID
    t0 = base.copy()
    t0[7:10] = [0.0, 0.004, 0.009]          # two midpoints inside one bucket, where the weights are dense
    t1 = base.copy()
    t1[4:7] = t1[5]                          # a triple: equal midpoints, an empty cell
    t1[11:13] = t1[11] + np.float32([0.0, 1e-6])
    check_layer(Wt, I, g, fmt, np.concatenate([t0, t1]).astype(np.float32), 3, "clustered")
    flat = np.concatenate([base, np.full(16, 0.5, np.float32)]).astype(np.float32)
    check_layer(Wt, I, g, fmt, flat, 2, "collapsed_table")
    both_flat = np.concatenate([np.full(16, -0.25, np.float32), np.full(16, 0.5, np.float32)])
    check_layer(Wt, I, g, fmt, both_flat, 2, "both_collapsed")


def test_degenerate_inputs():
    # all-zero weights, zero importance, empty layer, zero iterations
    g = 16
    Wz = torch.zeros((8, 64), dtype=torch.bfloat16, device=DEV)
    I1 = np.ones(64, np.float32)
    check_layer(Wz, I1, g, 0, inputs.format_grid(0), 2, "all_zero_weights")
    Wt = inputs.make_weight(8, 64, "gauss_outlier", 3, DEV)
    check_layer(Wt, np.zeros(64, np.float32), g, 0, inputs.format_grid(0), 2, "zero_importance")
    check_layer(Wt, I1, g, 0, inputs.format_grid(0), 0, "zero_iterations")
    We = torch.empty((0, 64), dtype=torch.bfloat16, device=DEV)
    tf, tb, _ = A.aaac_fit(We, g, 0, torch.ones(64, device=DEV), inputs.format_grid(0), 3)
    torch.cuda.synchronize()
    assert (host(tf) == inputs.format_grid(0)).all()
    codes, scales = A.aaac_encode(We, g, 0, torch.ones(64, device=DEV), tb)
    assert codes.shape == (0, 32) and scales.shape == (0, 4)


def test_fit_is_repeatable_and_resumable():
    Wt = inputs.make_weight(512, 1024, "gauss_outlier", 11, DEV)
    I = torch.rand(1024, device=DEV, generator=seeded(11001)) + 0.1
    grid = inputs.format_grid(1)
    a = A.aaac_fit(Wt, 128, 1, I, grid, 6)
    b = A.aaac_fit(Wt, 128, 1, I, grid, 6)
    h = A.aaac_fit(Wt, 128, 1, I, grid, 3)
    torch.cuda.synchronize()
    r = A.aaac_fit(Wt, 128, 1, I, host(h[0]), 3)
    torch.cuda.synchronize()
    assert (u16(a[1]) == u16(b[1])).all() and np.allclose(host(a[0]), host(b[0]), rtol=1e-12)
    assert (u16(a[1]) == u16(r[1])).all() and np.allclose(host(a[0]), host(r[0]), rtol=1e-6)


def test_one_launch_fit_is_the_same_bit_for_bit_on_every_run():
    """The one-launch path adds the blocks' partial sums in block order, whatever the timing: fp32 tables
    and the objective trace repeat exactly (the launch-per-pass path only promises the last bits of an
    fp64 sum away)."""
    Wt = inputs.make_weight(200, 512, "gauss_outlier", 12, DEV)
    I = torch.rand(512, device=DEV, generator=seeded(11030)) + 0.1
    with fit_path("persistent"):
        runs = [A.aaac_fit(Wt, 16, 0, I, inputs.format_grid(0), 7) for _ in range(4)]
        torch.cuda.synchronize()
    for tf, tb, ob in runs[1:]:
        assert torch.equal(tf, runs[0][0]) and torch.equal(tb, runs[0][1]) and torch.equal(ob, runs[0][2])


@pytest.mark.parametrize("path", FIT_PATHS)
def test_whole_path_can_be_captured_in_a_graph_and_replayed(path):
    """The library only launches kernels (no memset or memcpy nodes), so a caller may
    capture it; every replay must give the eager result, also after other work.  With
    "persistent" the captured fit is the one-launch kernel whose blocks wait for each other."""
    with fit_path(path):   # read by the library when the calls are made, i.e. at capture
        whole_path_in_a_graph(*((512, 1024, 16, 0, 4) if path == "launches" else (256, 512, 16, 0, 4)))


def whole_path_in_a_graph(N, K, g, fmt, iters):
    Wt = inputs.make_weight(N, K, "gauss_outlier", 21, DEV)
    X = inputs.make_activations(256, K, ("gauss", 0.01, "u10_50"), 22, DEV)
    grid = inputs.format_grid(fmt)
    I = torch.empty(K, device=DEV)
    ws_s = torch.empty(max(A.aaac_act_stats_workspace(256, K), 256), dtype=torch.uint8, device=DEV)
    ws_f = torch.empty(A.aaac_fit_workspace(N, K, g, fmt), dtype=torch.uint8, device=DEV)
    tf = torch.empty(32, device=DEV)
    tb = torch.empty(32, dtype=torch.int16, device=DEV)
    obj = torch.empty(iters, dtype=torch.float64, device=DEV)
    codes = torch.empty((N, K // 2), dtype=torch.uint8, device=DEV)
    scales = torch.empty((N, K // g), dtype=torch.uint8, device=DEV)
    What = torch.empty((N, K), dtype=torch.bfloat16, device=DEV)

    def run():
        A.aaac_act_stats(X, I, ws_s)
        A.aaac_fit(Wt, g, fmt, I, grid, iters, tf, tb, obj, ws_f)
        A.aaac_encode(Wt, g, fmt, I, tb, codes, scales)
        A.aaac_dequant(codes, scales, tb, g, fmt, What)

    run()
    torch.cuda.synchronize()
    want = [t.clone() for t in (I, tb, codes, scales, What)]
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        run()  # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        run()
    for rep in range(3):
        for t in (I, tb, codes, scales, What, tf):
            t.zero_()  # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for got, ref in zip((I, tb, codes, scales, What), want):
            assert torch.equal(got.view(torch.uint8) if got.dtype == torch.bfloat16 else got,
                               ref.view(torch.uint8) if ref.dtype == torch.bfloat16 else ref), rep


def test_alg1_in_full_and_both_products_can_be_captured_in_a_graph():
    """Quantile initialisation, both loops, small selection groups, encode with selection bits and
    the two W4A16 products: kernels only, so a graph replay must reproduce the eager results."""
    N, K, g, S, fmt = 300, 1024, 128, 16, 1
    Wt = inputs.make_weight(N, K, "gauss_outlier", 23, DEV)
    I = torch.rand(K, device=DEV, generator=seeded(11002)) + 0.05
    x1 = torch.randn((1, K), device=DEV, generator=seeded(11003)).to(torch.bfloat16)
    x9 = torch.randn((9, K), device=DEV, generator=seeded(11004)).to(torch.bfloat16)
    layers, ((tf, tb, ob),) = A.make_layers([Wt], [I], 2)
    ws = torch.empty(A.aaac_fit_nested_workspace(layers, g, fmt, sel_size=S), dtype=torch.uint8, device=DEV)
    codes = torch.empty((N, K // 2), dtype=torch.uint8, device=DEV)
    scales = torch.empty((N, K // g), dtype=torch.int16, device=DEV)
    bits = torch.empty((N, A.sel_stride(K, S)), dtype=torch.uint8, device=DEV)
    y1 = torch.empty((1, N), device=DEV)
    y9 = torch.empty((9, N), device=DEV)
    wsx = torch.empty(A.aaac_gemm_w4a16_workspace(9, K), dtype=torch.uint8, device=DEV)

    def run():
        A.aaac_fit_nested(layers, g, fmt, None, 2, 3, ws, sel_size=S)
        A.aaac_encode_sel(Wt, g, S, fmt, I, tb, codes, scales, bits)
        A.aaac_gemv_w4a16(x1, codes, scales, bits, tb, g, S, fmt, y=y1)
        A.aaac_gemm_w4a16(x9, codes, scales, bits, tb, g, S, fmt, y=y9, ws=wsx)

    run()
    torch.cuda.synchronize()
    outs = (tb, codes, scales, bits, y9)
    want = [t.clone() for t in outs]
    want_y1 = y1.clone()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        run()
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        run()
    for rep in range(3):
        for t in outs + (y1, tf):
            t.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for got, ref in zip(outs[:4], want[:4]):
            assert torch.equal(got, ref), rep
        # the products add in an order that may differ between runs (LDS atomics): compare closely
        assert torch.allclose(y9, want[4], rtol=1e-4, atol=1e-5) and torch.allclose(y1, want_y1, rtol=1e-4, atol=1e-5)


def test_batch_matches_single_calls():
    cfg = inputs.scaled_config(inputs.CONFIGS[3], rows_div=64, tokens_div=512)
    Ws = [inputs.layer_weights(l, DEV) for l in cfg["layers"]]
    Is = {}
    for k in cfg["xs"]:
        Is[k] = importance_for(cfg, k)[1]
    Il = [Is[l["x"]] for l in cfg["layers"]]
    layers, outs = A.make_layers(Ws, Il, 4)
    ws = torch.empty(A.aaac_fit_batch_workspace(layers, cfg["g"], cfg["fmt"]), dtype=torch.uint8, device=DEV)
    A.aaac_fit_batch(layers, cfg["g"], cfg["fmt"], inputs.format_grid(cfg["fmt"]), 4, ws)
    torch.cuda.synchronize()
    for W, I, (tf, tb, ob), l in zip(Ws, Il, outs, cfg["layers"]):
        ref = oracle.fit(inputs.bits(W), cfg["g"], cfg["fmt"], host(I), inputs.format_grid(cfg["fmt"]), 4)
        assert (u16(tb) == ref["tables_bf16"]).all(), l["name"]
        assert tables_close(host(tf), ref["tables_f32"])
        assert np.allclose(host(ob)[:4], ref["objective"], rtol=1e-9)


def test_batch_of_more_layers_than_one_launch_group_and_an_empty_layer():
    shapes = [(64, 512), (8, 1024), (0, 512), (200, 512), (33, 1536), (16, 512), (128, 1024), (5, 512), (77, 2048),
              (40, 512), (256, 512)]
    g, fmt, iters = 16, 0, 3
    Ws = [inputs.make_weight(N, K, "gauss_outlier", 700 + i, DEV) if N else
          torch.empty((0, K), dtype=torch.bfloat16, device=DEV) for i, (N, K) in enumerate(shapes)]
    Is = [torch.rand(K, device=DEV, generator=seeded(11005 + 100 * i)) + 0.05 for i, (_, K) in enumerate(shapes)]
    layers, outs = A.make_layers(Ws, Is, iters)
    ws = torch.empty(A.aaac_fit_batch_workspace(layers, g, fmt), dtype=torch.uint8, device=DEV)
    A.aaac_fit_batch(layers, g, fmt, inputs.format_grid(fmt), iters, ws)
    torch.cuda.synchronize()
    for (N, K), W, I, (tf, tb, ob) in zip(shapes, Ws, Is, outs):
        if N == 0:
            assert (host(tf) == inputs.format_grid(fmt)).all() and (host(ob)[:iters] == 0).all()
            continue
        ref = oracle.fit(inputs.bits(W), g, fmt, host(I), inputs.format_grid(fmt), iters)
        assert (u16(tb) == ref["tables_bf16"]).all(), (N, K)
        assert tables_close(host(tf), ref["tables_f32"])
        assert np.allclose(host(ob)[:iters], ref["objective"], rtol=1e-9)


def nested_on_gpu(Ws, Is, g, fmt, grid, n_outer, n_inner, S=None):
    """aaac_fit_nested through both of the library's paths; the two must agree (bf16 tables bit for
    bit), and the callers compare the returned one with the oracle."""
    results = []
    for path in FIT_PATHS:
        layers, outs = A.make_layers(Ws, Is, n_outer)
        ws = torch.empty(A.aaac_fit_nested_workspace(layers, g, fmt, sel_size=S), dtype=torch.uint8, device=DEV)
        with fit_path(path):
            A.aaac_fit_nested(layers, g, fmt, grid, n_outer, n_inner, ws, sel_size=S)
            torch.cuda.synchronize()
        results.append(outs)
    for (tf0, tb0, ob0), (tf1, tb1, ob1) in zip(*results):
        assert (u16(tb0) == u16(tb1)).all(), "the two fit paths give different bf16 tables"
        assert np.allclose(host(tf0), host(tf1), rtol=1e-6, atol=0)
        if n_outer:
            assert np.allclose(host(ob0)[:n_outer], host(ob1)[:n_outer], rtol=1e-9, atol=0)
    return results[1]


@pytest.mark.parametrize("N,K,g,fmt,n_outer,n_inner", [
    (256, 512, 16, 0, 3, 10),    # the paper's default loop counts on the small benchmark shape
    (130, 1536, 128, 1, 2, 4),
    (37, 1040, 16, 0, 2, 3),
    (64, 640, 32, 1, 3, 2),
    (96, 1024, 16, 0, 0, 5),     # no outer step: the grid comes back
])
def test_nested_loops_match_oracle(N, K, g, fmt, n_outer, n_inner):
    say(f"[nested] N={N} K={K} g={g} fmt={fmt} outer={n_outer} inner={n_inner}")
    Wt = inputs.make_weight(N, K, "gauss_outlier", 300 + N + K, DEV)
    I = oracle.act_stats(inputs.bits(inputs.make_activations(64, K, ("gauss", 0.01, "u10_50"), 310 + K, DEV)))
    grid = inputs.format_grid(fmt)
    ref = oracle.fit_nested(inputs.bits(Wt), g, fmt, I, grid, n_outer, n_inner)
    (tf, tb, ob), = nested_on_gpu([Wt], [torch.from_numpy(I).to(DEV)], g, fmt, grid, n_outer, n_inner)
    assert (u16(tb) == ref["tables_bf16"]).all()
    assert tables_close(host(tf), ref["tables_f32"])
    if n_outer:
        assert np.allclose(host(ob)[:n_outer], ref["objective"], rtol=1e-9)
    # and the codes that follow from these tables
    It = torch.from_numpy(I).to(DEV)
    codes, scales = A.aaac_encode(Wt, g, fmt, It, tb)
    torch.cuda.synchronize()
    rc, rs = oracle.encode(inputs.bits(Wt), g, fmt, I, ref["tables_bf16"])
    assert (host(codes) == rc).all() and (host(scales).view(rs.dtype) == rs).all()


def test_nested_loops_clustered_tables_and_batch():
    # refinement passes through poisoned buckets, several layers at once, one inner step == plain fit
    shapes = [(96, 1024), (40, 512), (200, 1536)]
    g, fmt = 16, 0
    Ws = [inputs.make_weight(N, K, "student5", 400 + i, DEV) for i, (N, K) in enumerate(shapes)]
    Is = [torch.rand(K, device=DEV, generator=seeded(11006 + 100 * i)) + 0.05 for i, (_, K) in enumerate(shapes)]
    t0 = inputs.E2M1_GRID.copy()
    t0[7:10] = [0.0, 0.004, 0.009]
    t1 = inputs.E2M1_GRID + np.float32(0.25)
    t1[4:7] = t1[5]
    grid = np.concatenate([t0, t1]).astype(np.float32)
    outs = nested_on_gpu(Ws, Is, g, fmt, grid, 2, 3)
    for W, I, (tf, tb, ob) in zip(Ws, Is, outs):
        ref = oracle.fit_nested(inputs.bits(W), g, fmt, host(I), grid, 2, 3)
        assert (u16(tb) == ref["tables_bf16"]).all()
        assert tables_close(host(tf), ref["tables_f32"])
        assert np.allclose(host(ob)[:2], ref["objective"], rtol=1e-9)
    plain = [A.aaac_fit(W, g, fmt, I, inputs.format_grid(fmt), 3) for W, I in zip(Ws, Is)]
    one = nested_on_gpu(Ws, Is, g, fmt, inputs.format_grid(fmt), 3, 1)
    torch.cuda.synchronize()
    for (tf, tb, ob), (pf, pb, po) in zip(one, plain):
        assert (u16(tb) == u16(pb)).all() and np.allclose(host(tf), host(pf), rtol=1e-6)


def test_nested_loops_cfg1_full_size():
    """The Llama-2-7B-shaped q_proj with the paper's default loop counts (3, 10)."""
    cfg = inputs.CONFIGS[1]
    l = cfg["layers"][0]
    Wt = inputs.layer_weights(l, DEV)
    I = torch.rand(l["K"], device=DEV, generator=seeded(11007)) * 100 + 1
    grid = inputs.format_grid(cfg["fmt"])
    t0 = time.time()
    ref = oracle.fit_nested(inputs.bits(Wt), cfg["g"], cfg["fmt"], host(I), grid, 3, 10)
    say(f"[nested] cfg1 oracle {time.time() - t0:.1f}s")
    (tf, tb, ob), = nested_on_gpu([Wt], [I], cfg["g"], cfg["fmt"], grid, 3, 10)
    assert (u16(tb) == ref["tables_bf16"]).all()
    assert tables_close(host(tf), ref["tables_f32"])
    assert np.allclose(host(ob)[:3], ref["objective"], rtol=1e-9)


# ------------------------------------------ selection groups smaller than scale groups

def check_sel_layer(Wt, I, g, S, fmt, n_outer, n_inner, grid=None, pad_stride=0):
    """Fit, encode and dequantise with S < g on the GPU and compare everything with the oracle."""
    grid = inputs.format_grid(fmt) if grid is None else grid
    Ih = host(I)
    ref = oracle.fit_sel(inputs.bits(Wt), g, S, fmt, Ih, grid, n_outer, n_inner)
    (tf, tb, ob), = nested_on_gpu([Wt], [I], g, fmt, grid, n_outer, n_inner, S=S)
    assert (u16(tb) == ref["tables_bf16"]).all()
    assert tables_close(host(tf), ref["tables_f32"])
    if n_outer:
        assert np.allclose(host(ob)[:n_outer], ref["objective"], rtol=1e-9)
    N, K = Wt.shape
    stride = A.sel_stride(K, S) + pad_stride
    bits = torch.full((N, stride), 0xFF, dtype=torch.uint8, device=DEV) if S < g else None
    codes, scales, bits = A.aaac_encode_sel(Wt, g, S, fmt, I, tb, sel_bits=bits)
    What = A.aaac_dequant_sel(codes, scales, bits, tb, g, S, fmt)
    torch.cuda.synchronize()
    rc, rs, rb = oracle.encode_sel(inputs.bits(Wt), g, S, fmt, Ih, ref["tables_bf16"])
    assert (host(codes) == rc).all()
    assert (host(scales).view(rs.dtype) == rs).all()
    if S < g:
        used = A.sel_stride(K, S)
        assert (host(bits)[:, :used] == rb).all()
        assert (host(bits)[:, used:] == 0xFF).all()          # bytes past the row's bits are not touched
        assert (host(scales).view(rs.dtype) >> (7 if fmt == A.NVFP4 else 15) == 0).all()
    assert (u16(What) == oracle.dequant_sel(rc, rs, rb, ref["tables_bf16"], g, S, fmt)).all()
    return ref


@pytest.mark.parametrize("N,K,g,S,fmt,n_outer,n_inner,pad", [
    (128, 4096, 128, 16, 1, 3, 4, 0),    # the paper's INT4 setting with S = 16
    (37, 1152, 128, 16, 1, 2, 1, 3),     # ragged: 2.25 strips, 9 selection bytes per row, padded stride
    (64, 640, 64, 32, 1, 2, 2, 0),
    (50, 1536, 128, 64, 1, 2, 2, 1),
    (96, 1056, 32, 16, 0, 2, 2, 0),      # 66 selection groups: the last byte of a row holds two bits
    (33, 512, 128, 32, 0, 1, 3, 0),
    (40, 2048, 64, 64, 1, 2, 2, 0),      # S == g through the same entry points: sign-bit path
])
def test_selection_groups_smaller_than_scale_groups(N, K, g, S, fmt, n_outer, n_inner, pad):
    say(f"[sel] N={N} K={K} g={g} S={S} fmt={fmt} outer={n_outer} inner={n_inner}")
    Wt = inputs.make_weight(N, K, "gauss_outlier", 500 + N + K, DEV)
    I = torch.from_numpy(oracle.act_stats(inputs.bits(
        inputs.make_activations(64, K, ("gauss", 0.01, "u10_50"), 510 + K, DEV)))).to(DEV)
    check_sel_layer(Wt, I, g, S, fmt, n_outer, n_inner, pad_stride=pad)


def test_selection_groups_worked_vector():
    case = GOLD["sel_cases"][0]
    g, S, fmt = case["g"], case["S"], A.INT4
    Wt = torch.tensor(case["W"], dtype=torch.float32, device=DEV).to(torch.bfloat16)[None, :]
    tb = torch.tensor(case["T0"] + case["T1"], dtype=torch.float32, device=DEV).to(torch.bfloat16).view(torch.int16)
    I = (torch.arange(Wt.shape[1], device=DEV) % 5 + 1).float()
    codes, scales, bits = A.aaac_encode_sel(Wt, g, S, fmt, I, tb)
    What = A.aaac_dequant_sel(codes, scales, bits, tb, g, S, fmt)
    torch.cuda.synchronize()
    c = host(codes)[0]
    assert np.stack([c & 15, c >> 4], axis=1).reshape(-1).tolist() == case["codes"]
    assert host(scales).view(np.uint16).tolist() == [[case["scale"]]]
    assert host(bits).tolist() == [case["sel_bits"]]
    assert (What == Wt).all()


def test_selection_groups_cfg1_shape_full_size():
    """4096x4096, INT4 g=128 with one choice per 16 weights (+1/16 bit per weight)."""
    cfg = inputs.CONFIGS[1]
    l = cfg["layers"][0]
    Wt = inputs.layer_weights(l, DEV)
    I = torch.rand(l["K"], device=DEV, generator=seeded(11008)) * 100 + 1
    t0 = time.time()
    ref = check_sel_layer(Wt, I, cfg["g"], 16, cfg["fmt"], 2, 3)
    coarse = oracle.fit_sel(inputs.bits(Wt), cfg["g"], cfg["g"], cfg["fmt"], host(I), inputs.format_grid(cfg["fmt"]), 2, 3)
    say(f"[sel] cfg1 S=16 {time.time() - t0:.1f}s, objective {ref['objective'][-1]:.4e} vs S=128 {coarse['objective'][-1]:.4e}")
    assert ref["objective"][-1] < coarse["objective"][-1]


# ------------------------------------------ quantile initialisation

def u32(a):
    return np.ascontiguousarray(a, np.float32).view(np.uint32)


@pytest.mark.parametrize("N,K,g,fmt,kind", [
    (64, 512, 16, 0, "gauss_outlier"),
    (130, 1536, 128, 1, "gauss_outlier"),
    (37, 1040, 16, 0, "student5"),
    (1, 16, 16, 0, "gauss_outlier"),        # 16 weights: every level falls between two of them
    (3, 32, 32, 1, "gauss_outlier"),
    (200, 4096, 128, 1, "gauss_outlier"),
    (1030, 2048, 64, 1, "student5"),        # more chunks than one block takes
])
def test_quantile_init_matches_oracle(N, K, g, fmt, kind):
    say(f"[quantile] N={N} K={K} g={g} fmt={fmt} {kind}")
    Wt = inputs.make_weight(N, K, kind, 600 + N + K, DEV)
    grid = A.aaac_quantile_init(Wt, g, fmt)
    torch.cuda.synchronize()
    ref = oracle.quantile_init(inputs.bits(Wt), g, fmt)
    assert (u32(host(grid)) == u32(ref)).all()


def test_quantile_init_degenerate_weights_and_padded_rows():
    # all weights zero, some of them -0.0: every normalised weight is a zero, the tables are +0
    Wz = torch.zeros((40, 256), dtype=torch.bfloat16, device=DEV)
    Wz[::3] = -0.0
    grid = A.aaac_quantile_init(Wz, 16, A.NVFP4)
    torch.cuda.synchronize()
    assert (u32(host(grid)) == 0).all()
    assert (u32(oracle.quantile_init(inputs.bits(Wz), 16, A.NVFP4)) == 0).all()
    # two distinct values only: long runs of equal keys
    Wt = torch.where(torch.rand((64, 512), device=DEV, generator=seeded(11009)) < 0.3, 0.05, -0.02).to(torch.bfloat16)
    grid = A.aaac_quantile_init(Wt, 128, A.INT4)
    torch.cuda.synchronize()
    assert (u32(host(grid)) == u32(oracle.quantile_init(inputs.bits(Wt), 128, A.INT4))).all()
    # a few distinct values in a layer of half a million weights: far more keys share the followed
    # prefixes than the candidate list of the radix select holds, so its last pass reads the weights
    vals = torch.tensor([-0.07, -0.02, 0.0, 0.013, 0.05], device=DEV)
    for g, fmt in ((16, A.NVFP4), (128, A.INT4)):
        pick = torch.randint(0, 5, (512, 1024), device=DEV, generator=seeded(11011 + g))
        Wt = vals[pick].to(torch.bfloat16)
        grid = A.aaac_quantile_init(Wt, g, fmt)
        torch.cuda.synchronize()
        assert (u32(host(grid)) == u32(oracle.quantile_init(inputs.bits(Wt), g, fmt))).all()
    # rows with a padded leading dimension; the padding holds large values that must not be read
    big = torch.full((50, 768), 100.0, dtype=torch.bfloat16, device=DEV)
    Wp = big[:, :640]
    Wp.copy_(inputs.make_weight(50, 640, "gauss_outlier", 77, DEV))
    grid = A.aaac_quantile_init(Wp, 64, A.INT4)
    torch.cuda.synchronize()
    assert (u32(host(grid)) == u32(oracle.quantile_init(inputs.bits(Wp.contiguous()), 64, A.INT4))).all()


def test_fit_from_quantile_tables_matches_oracle():
    # init_grid = NULL: Alg. 1 as printed, quantile tables then both loops, also with S < g and in a batch
    shapes = [(96, 1024), (40, 512), (128, 1536)]
    g, S, fmt = 128, 16, A.INT4
    Ws = [inputs.make_weight(N, K, "gauss_outlier", 700 + i, DEV) for i, (N, K) in enumerate(shapes)]
    Is = [torch.rand(K, device=DEV, generator=seeded(11010 + 100 * i)) * 10 + 0.05 for i, (_, K) in enumerate(shapes)]
    outs = nested_on_gpu(Ws, Is, g, fmt, None, 3, 2, S=S)
    for W, I, (tf, tb, ob) in zip(Ws, Is, outs):
        q = oracle.quantile_init(inputs.bits(W), g, fmt)
        ref = oracle.fit_sel(inputs.bits(W), g, S, fmt, host(I), q, 3, 2)
        assert (u16(tb) == ref["tables_bf16"]).all()
        assert tables_close(host(tf), ref["tables_f32"])
        assert np.allclose(host(ob)[:3], ref["objective"], rtol=1e-9)
    # zero outer steps: the tables that come back are the quantile tables themselves
    (tf, tb, ob), = nested_on_gpu(Ws[:1], Is[:1], g, fmt, None, 0, 1)
    assert (u32(host(tf)) == u32(oracle.quantile_init(inputs.bits(Ws[0]), g, fmt))).all()


@pytest.mark.parametrize("cfg_id", [1, 2])
def test_quantile_init_full_size(cfg_id):
    cfg = inputs.CONFIGS[cfg_id]
    l = cfg["layers"][0]
    Wt = inputs.layer_weights(l, DEV)
    grid = A.aaac_quantile_init(Wt, cfg["g"], cfg["fmt"])
    torch.cuda.synchronize()
    t0 = time.time()
    ref = oracle.quantile_init(inputs.bits(Wt), cfg["g"], cfg["fmt"])
    say(f"[quantile] cfg{cfg_id} oracle {time.time() - t0:.1f}s")
    assert (u32(host(grid)) == u32(ref)).all()


# ------------------------------------------ the quantised layer applied to activations (W4A16)

def gemv_tolerance(K, mag):
    """First-order bound on the fp32 summation error: roundings on the path of one term
    (16 FMAs of the half-group sum, 2 for the scale, 4 lane-exchange adds, 4 adds per slab of 2048
    columns into the row sum) times the unit roundoff times sum |terms|."""
    return (22 + 4 * -(-K // 2048)) * 2.0 ** -24 * mag + 1e-30


def quantise_on_gpu(Wt, I, g, S, fmt, iters=2):
    (tf, tb, ob), = nested_on_gpu([Wt], [I], g, fmt, inputs.format_grid(fmt), iters, 1, S=S)
    codes, scales, bits = A.aaac_encode_sel(Wt, g, S, fmt, I, tb)
    torch.cuda.synchronize()
    return tb, codes, scales, bits


@pytest.mark.parametrize("N,K,g,S,fmt,M", [
    (256, 512, 16, 16, 0, 1),       # a quarter slab
    (130, 4096, 128, 128, 1, 1),    # two slabs, odd row count
    (77, 2080, 16, 16, 0, 3),       # ragged last slab, three rows of x (four held, one zero)
    (64, 4096, 128, 16, 1, 2),      # selection bits read from the bit array
    (40, 6144, 64, 32, 1, 4),       # three slabs: two wavefronts of the block stay idle
    (300, 18432, 32, 32, 0, 5),     # nine slabs (wavefronts take a second slab), x in two batches
    (9, 1024, 16, 16, 1, 7),        # bf16 scales with groups of 16 (two per lane)
])
def test_gemv_w4a16_matches_oracle(N, K, g, S, fmt, M):
    say(f"[gemv] N={N} K={K} g={g} S={S} fmt={fmt} M={M}")
    Wt = inputs.make_weight(N, K, "gauss_outlier", 800 + N + K, DEV)
    I = torch.rand(K, device=DEV, generator=seeded(11011 + N + K)) + 0.05
    tb, codes, scales, bits = quantise_on_gpu(Wt, I, g, S, fmt)
    x = (torch.randn((M, K), device=DEV, generator=seeded(11012 + N + K + M)) * 2).to(torch.bfloat16)
    y = A.aaac_gemv_w4a16(x, codes, scales, bits, tb, g, S, fmt)
    torch.cuda.synchronize()
    ref, mag = oracle.gemv_w4a16(inputs.bits(x), host(codes), host(scales).view(np.uint8 if fmt == 0 else np.uint16),
                                 None if bits is None else host(bits), u16(tb), g, S, fmt)
    err = np.abs(host(y).astype(np.float64) - ref)
    assert (err <= gemv_tolerance(K, mag) + np.spacing(np.abs(ref))).all(), float((err / (mag + 1e-30)).max())
    # and it is the product with the dequantised layer, up to the bf16 rounding of the stored weights
    What = A.aaac_dequant_sel(codes, scales, bits, tb, g, S, fmt).double()
    torch.cuda.synchronize()
    assert np.abs(host(y) - host(x.double() @ What.T)).max() <= 2.0 ** -8 * mag.max()


def test_gemv_w4a16_unit_vectors_and_strides():
    # x = e_k returns column k of the dequantised layer exactly; padded x and y rows
    N, K, g, fmt = 48, 256, 16, 0
    Wt = inputs.make_weight(N, K, "student5", 31, DEV)
    I = torch.rand(K, device=DEV, generator=seeded(11013)) + 0.05
    tb, codes, scales, bits = quantise_on_gpu(Wt, I, g, g, fmt)
    xbig = torch.zeros((4, K + 64), dtype=torch.bfloat16, device=DEV)
    xbig[:, K:] = 100.0                       # padding that must not be read
    x = xbig[:, :K]
    for m, k in enumerate((0, 17, 130, 255)):
        x[m, k] = 1.0
    ybig = torch.full((4, N + 8), -7.0, dtype=torch.float32, device=DEV)
    y = A.aaac_gemv_w4a16(x, codes, scales, bits, tb, g, g, fmt, y=ybig[:, :N])
    What = A.aaac_dequant(codes, scales, tb, g, fmt)
    torch.cuda.synchronize()
    for m, k in enumerate((0, 17, 130, 255)):
        assert (y[m].to(torch.bfloat16) == What[:, k]).all()
    assert (ybig[:, N:] == -7.0).all()


def test_w4a16_every_e4m3_scale_code():
    # hand-made codes and scales: every storable E4M3 scale (0x00..0x7E, both values of the selection
    # bit on top) appears in every row, so the hardware FP8 conversion the products use is compared
    # with the oracle's E4M3 decoding code by code (subnormals included)
    N, K, g, fmt = 24, 4096, 16, 0
    rng = np.random.default_rng(77)
    sc = np.arange(256, dtype=np.uint8)
    sc[sc == 0x7F] = 0x7E
    sc[sc == 0xFF] = 0xFE
    scales_h = np.stack([np.roll(sc, 11 * n) for n in range(N)])
    codes_h = rng.integers(0, 256, (N, K // 2), dtype=np.uint8)
    tabs = np.sort(rng.normal(0, 3, (2, 16)).astype(np.float32), axis=1).reshape(32)
    tb = torch.from_numpy(tabs).to(DEV).to(torch.bfloat16)
    codes, scales = torch.from_numpy(codes_h).to(DEV), torch.from_numpy(scales_h).to(DEV)
    x = (torch.randn((3, K), device=DEV, generator=seeded(11014)) * 2).to(torch.bfloat16)
    y = A.aaac_gemv_w4a16(x, codes, scales, None, tb.view(torch.int16), g, g, fmt)
    torch.cuda.synchronize()
    ref, mag = oracle.gemv_w4a16(inputs.bits(x), codes_h, scales_h, None, u16(tb.view(torch.int16)), g, g, fmt)
    err = np.abs(host(y).astype(np.float64) - ref)
    assert (err <= gemv_tolerance(K, mag) + np.spacing(np.abs(ref))).all(), float((err / (mag + 1e-30)).max())
    # unit vectors pick single dequantised weights: exact, scale by scale
    cols = [0, 16 * 1 + 3, 16 * 7 + 9, 16 * 8, 16 * 126 + 15, 16 * 129, 16 * 254 + 1, K - 1]
    xe = torch.zeros((len(cols), K), dtype=torch.bfloat16, device=DEV)
    for m, k in enumerate(cols):
        xe[m, k] = 1.0
    ye = A.aaac_gemv_w4a16(xe, codes, scales, None, tb.view(torch.int16), g, g, fmt)
    torch.cuda.synchronize()
    refe, _ = oracle.gemv_w4a16(inputs.bits(xe), codes_h, scales_h, None, u16(tb.view(torch.int16)), g, g, fmt)
    assert (host(ye).astype(np.float64) == refe).all()
    # the matrix-core product sees the same scales
    ws = torch.empty(max(A.aaac_gemm_w4a16_workspace(3, K), 256), dtype=torch.uint8, device=DEV)
    yg = A.aaac_gemm_w4a16(x, codes, scales, None, tb.view(torch.int16), g, g, fmt, ws=ws)
    torch.cuda.synchronize()
    refg, magg = oracle.gemm_w4a16(inputs.bits(x), codes_h, scales_h, None, u16(tb.view(torch.int16)), g, g, fmt)
    assert (np.abs(host(yg).astype(np.float64) - refg) <= (K + 8) * 2.0 ** -24 * magg + np.spacing(np.abs(refg))).all()


def test_gemv_w4a16_cfg1_full_size():
    cfg = inputs.CONFIGS[1]
    l = cfg["layers"][0]
    g, fmt = cfg["g"], cfg["fmt"]
    Wt = inputs.layer_weights(l, DEV)
    I = torch.rand(l["K"], device=DEV, generator=seeded(11015)) * 100 + 1
    tb, codes, scales, bits = quantise_on_gpu(Wt, I, g, g, fmt)
    x = torch.randn((1, l["K"]), device=DEV, generator=seeded(11016)).to(torch.bfloat16)
    y = A.aaac_gemv_w4a16(x, codes, scales, bits, tb, g, g, fmt)
    torch.cuda.synchronize()
    # the oracle on a sample of rows (every 37th)
    rows = np.arange(0, l["N"], 37)
    ref, mag = oracle.gemv_w4a16(inputs.bits(x), host(codes)[rows], host(scales).view(np.uint16)[rows], None, u16(tb),
                                 g, g, fmt)
    err = np.abs(host(y)[:, rows].astype(np.float64) - ref)
    assert (err <= gemv_tolerance(l["K"], mag) + np.spacing(np.abs(ref))).all()
    # every output against the original layer: quantisation error only
    exact = host(x.double() @ Wt.double().T)
    assert np.abs(host(y) - exact).mean() < 0.2 * np.abs(exact).mean()


# ------------------------------------------ the W4A16 product on the matrix cores

def synthetic_quantised_layer(N, K, g, S, fmt, seed, exact=False):
    """Codes, scales, selection bits and tables drawn directly (no fit).  exact: integer tables and
    power-of-two scales, so that with small integer activations every sum is exact in fp32."""
    gen = torch.Generator(device=DEV).manual_seed(seed)
    codes = torch.randint(0, 256, (N, K // 2), dtype=torch.uint8, device=DEV, generator=gen)
    sign = torch.randint(0, 2, (N, K // g), device=DEV, generator=gen)
    if S < g:
        bits = torch.randint(0, 256, (N, A.sel_stride(K, S)), dtype=torch.uint8, device=DEV, generator=gen)
        sign = torch.zeros_like(sign)
    else:
        bits = None
    if fmt == A.NVFP4:
        mag = torch.full((N, K // g), 0x38, device=DEV) if exact else torch.randint(1, 0x60, (N, K // g), device=DEV, generator=gen)
        scales = (mag | (sign << 7)).to(torch.uint8)
    else:
        if exact:
            mag = torch.full((N, K // g), 0x3F80, device=DEV)
        else:
            mag = (torch.rand((N, K // g), device=DEV, generator=gen) * 0.02 + 1e-3).to(torch.bfloat16).view(torch.int16).int() & 0x7FFF
        scales = (mag | (sign << 15)).to(torch.int32).to(torch.int16)
    if exact:
        t = torch.cat([torch.arange(-8, 8, device=DEV).float(), torch.arange(-7, 9, device=DEV).float() * 2])
    else:
        t = torch.sort(torch.randn((2, 16), device=DEV, generator=gen) * 3, dim=1)[0].reshape(32)
    tb = t.to(torch.bfloat16).view(torch.int16)
    return tb, codes, scales, bits


def oracle_args(x, codes, scales, bits, tb, fmt):
    return (inputs.bits(x), host(codes), host(scales).view(np.uint8 if fmt == 0 else np.uint16),
            None if bits is None else host(bits), u16(tb))


@pytest.mark.parametrize("N,K,g,S,fmt,M", [
    (64, 256, 16, 16, 0, 16),
    (100, 320, 16, 16, 0, 5),       # ragged rows and a partial chunk of 64 columns
    (33, 64, 64, 64, 1, 1),         # one lane quarter of columns
    (200, 1024, 128, 16, 1, 33),    # selection bits from the bit array, three tiles of x rows
    (48, 2048, 32, 32, 0, 64),
    (130, 4096, 128, 128, 1, 70),   # x in three batches: 32, 32 and 6 rows, K split over two blocks
    (20, 512, 16, 16, 1, 17),       # bf16 scales with groups of 16
    (5000, 512, 64, 32, 1, 8),      # many rows: several row tiles per block
    (70, 8192, 16, 16, 0, 16),      # few layer rows: K split over four blocks whose parts are added in y
    (200, 6144, 128, 16, 1, 32),    # two tiles of x rows in registers, K split in three, selection bits
    (1000, 512, 16, 16, 0, 24),     # two tiles of x rows, ragged last block of layer rows
    (90, 2560, 32, 32, 0, 96),      # three batches of 32 rows of x
    (300, 320, 16, 16, 0, 130),     # more than 64 rows of x: the tiled kernel, ragged tiles in both directions
    (128, 1024, 128, 16, 1, 256),   # tiled, selection bits from the bit array
    (77, 640, 32, 32, 1, 65),       # tiled, one partial tile each way
    (260, 2048, 16, 16, 1, 200),    # tiled, bf16 scales with groups of 16
    (256, 8192, 16, 16, 0, 256),    # tiled, two tiles only: K split over 16 blocks each, parts added in y
    (200, 4096, 128, 32, 1, 100),   # tiled, ragged tiles with K split over 8 blocks, selection bits
])
def test_gemm_w4a16_exact_on_integer_data_and_bounded_on_real_data(N, K, g, S, fmt, M):
    say(f"[gemm] N={N} K={K} g={g} S={S} fmt={fmt} M={M}")
    # integer tables, unit scales, small integer activations: every partial sum is an integer
    # below 2^24, so the result is exact whatever the order of the additions
    tb, codes, scales, bits = synthetic_quantised_layer(N, K, g, S, fmt, 900 + N, exact=True)
    x = torch.randint(-4, 5, (M, K), device=DEV, generator=seeded(11017 + N + K + M)).to(torch.bfloat16)
    y = A.aaac_gemm_w4a16(x, codes, scales, bits, tb, g, S, fmt)
    torch.cuda.synchronize()
    ref, mag = oracle.gemm_w4a16(*oracle_args(x, codes, scales, bits, tb, fmt), g, S, fmt)
    assert mag.max() < 2 ** 24 and (host(y) == ref).all()
    # real-valued tables, scales and activations: any summation order of K exact products stays within
    # (K - 1) roundings, plus the 8 adds of the cross-wavefront reduction
    tb, codes, scales, bits = synthetic_quantised_layer(N, K, g, S, fmt, 950 + N)
    x = torch.randn((M, K), device=DEV, generator=seeded(11018 + N + K + M)).to(torch.bfloat16)
    y = A.aaac_gemm_w4a16(x, codes, scales, bits, tb, g, S, fmt)
    torch.cuda.synchronize()
    ref, mag = oracle.gemm_w4a16(*oracle_args(x, codes, scales, bits, tb, fmt), g, S, fmt)
    err = np.abs(host(y).astype(np.float64) - ref)
    assert (err <= (K + 8) * 2.0 ** -24 * mag + np.spacing(np.abs(ref))).all()
    assert np.median(err / (mag + 1e-30)) < 16 * 2.0 ** -24      # and far inside it for the typical output


def test_gemm_w4a16_unit_vectors_return_the_stored_dequantised_weights():
    # x = e_k: y[m, n] is the bf16 weight aaac_dequant stores, exactly (rounding of T * s included)
    N, K, g, fmt = 70, 576, 16, 0
    Wt = inputs.make_weight(N, K, "student5", 41, DEV)
    I = torch.rand(K, device=DEV, generator=seeded(11019)) + 0.05
    tb, codes, scales, bits = quantise_on_gpu(Wt, I, g, g, fmt)
    ks = [0, 1, 7, 8, 63, 64, 100, 255, 256, 300, 511, 512, 575]
    x = torch.zeros((len(ks), K), dtype=torch.bfloat16, device=DEV)
    for m, k in enumerate(ks):
        x[m, k] = 1.0
    y = A.aaac_gemm_w4a16(x, codes, scales, bits, tb, g, g, fmt)
    What = A.aaac_dequant(codes, scales, tb, g, fmt)
    torch.cuda.synchronize()
    for m, k in enumerate(ks):
        assert (y[m] == What[:, k].float()).all(), k


def test_gemm_w4a16_cfg1_full_size_matches_the_product_with_the_dequantised_layer():
    cfg = inputs.CONFIGS[1]
    l = cfg["layers"][0]
    g, fmt = cfg["g"], cfg["fmt"]
    Wt = inputs.layer_weights(l, DEV)
    I = torch.rand(l["K"], device=DEV, generator=seeded(11020)) * 100 + 1
    tb, codes, scales, bits = quantise_on_gpu(Wt, I, g, g, fmt)
    x = torch.randn((32, l["K"]), device=DEV, generator=seeded(11021)).to(torch.bfloat16)
    y = A.aaac_gemm_w4a16(x, codes, scales, bits, tb, g, g, fmt)
    torch.cuda.synchronize()
    rows = np.arange(0, l["N"], 97)
    ref, mag = oracle.gemm_w4a16(inputs.bits(x), host(codes)[rows], host(scales).view(np.uint16)[rows], None, u16(tb),
                                 g, g, fmt)
    err = np.abs(host(y)[:, rows].astype(np.float64) - ref)
    assert (err <= (l["K"] + 8) * 2.0 ** -24 * mag + np.spacing(np.abs(ref))).all()
    assert np.median(err / (mag + 1e-30)) < 16 * 2.0 ** -24      # the typical output lies far inside the any-order bound
    # all outputs against torch's fp64 product with the stored dequantised weights
    What = A.aaac_dequant(codes, scales, tb, g, fmt).double()
    full = host(x.double() @ What.T)
    assert np.abs(host(y) - full).max() <= 1e-4 * np.abs(full).max()


@pytest.mark.parametrize("layer", [0, 1])
def test_w4a16_products_cfg4_full_size_on_sampled_layer_rows(layer):
    """The launch configurations that bench.py times on the largest workload: one row (vector ALUs),
    16 rows (x in registers; down_proj splits K over four blocks) and a ragged 300-row batch (tiles),
    each checked on every 449th layer row against the oracle."""
    cfg = inputs.CONFIGS[4]
    l = cfg["layers"][layer]
    N, K, g, fmt = l["N"], l["K"], cfg["g"], cfg["fmt"]
    say(f"[cfg4 products] {l['name']} N={N} K={K}")
    tb, codes, scales, bits = synthetic_quantised_layer(N, K, g, g, fmt, 9100 + layer)
    rows = np.arange(0, N, 449)
    codes_h, scales_h = host(codes)[rows], host(scales).view(np.uint8)[rows]
    for M in (1, 16, 300):
        x = (torch.randn((M, K), device=DEV, generator=seeded(11022 + 10 * layer + M)) * 2).to(torch.bfloat16)
        if M == 1:
            y = A.aaac_gemv_w4a16(x, codes, scales, bits, tb, g, g, fmt)
            torch.cuda.synchronize()
            ref, mag = oracle.gemv_w4a16(inputs.bits(x), codes_h, scales_h, None, u16(tb), g, g, fmt)
            tol = gemv_tolerance(K, mag)
        else:
            y = A.aaac_gemm_w4a16(x, codes, scales, bits, tb, g, g, fmt)
            torch.cuda.synchronize()
            ref, mag = oracle.gemm_w4a16(inputs.bits(x), codes_h, scales_h, None, u16(tb), g, g, fmt)
            tol = (K + 8) * 2.0 ** -24 * mag
        err = np.abs(host(y)[:, rows].astype(np.float64) - ref)
        assert (err <= tol + np.spacing(np.abs(ref))).all(), M
        assert np.median(err / (mag + 1e-30)) < 16 * 2.0 ** -24, M   # typical error: a few roundings, whatever K
        del x, y


def torch_quantile_tables(Wt, g, fmt):
    """The quantile tables from torch's own sort and casts (no library code, no oracle): scales by
    torch's float8 / bf16 conversions, reciprocal through fp64, one fp32 multiply, torch.sort, then
    the exact integer positions and fp64 interpolation of the reading.  Only for layers whose groups
    all have absmax / 6 <= 448: torch's float8 cast does not saturate where the scale format does."""
    N, K = Wt.shape
    a = Wt.float().abs().reshape(N, K // g, g).amax(dim=2)
    if fmt == A.NVFP4:
        code = (a / 6.0).to(torch.float8_e4m3fn).view(torch.uint8).clamp_(min=1)
        s = code.view(torch.float8_e4m3fn).float()
    else:
        s = (a / 7.0).to(torch.bfloat16).float().clamp_(min=2.0 ** -126)
    r = (1.0 / s.double()).float()
    x = (Wt.float().reshape(N, K // g, g) * r[:, :, None]).reshape(-1)
    x = torch.sort(x)[0]
    n = x.numel()
    out = []
    for t in range(2):
        for i in range(16):
            num, den = (i, 15) if t == 0 else (15 + 29 * i, 450)
            lo, rem = divmod(num * (n - 1), den)
            v = x[lo].double()
            if rem:
                v = v + (torch.tensor(float(rem), dtype=torch.float64, device=DEV) / den) * (x[lo + 1].double() - v)
            out.append(v.float() + 0.0)
    return torch.stack(out)


@pytest.mark.parametrize("cfg_id,layer", [(4, 0), (3, 6)])
def test_quantile_init_largest_layers_against_torch_sort(cfg_id, layer):
    """At the benchmark's largest sizes the CPU oracle's sort is too slow; torch's sort of the
    normalised weights (built with torch's own casts) gives the same order statistics."""
    cfg = inputs.CONFIGS[cfg_id]
    l = cfg["layers"][layer]
    Wt = inputs.layer_weights(l, DEV)
    grid = A.aaac_quantile_init(Wt, cfg["g"], cfg["fmt"])
    ref = torch_quantile_tables(Wt, cfg["g"], cfg["fmt"])
    torch.cuda.synchronize()
    assert (u32(host(grid)) == u32(host(ref))).all()
    # the same helper against the oracle on a slice, so that the helper itself is checked
    small = Wt[:64].contiguous()
    assert (u32(host(torch_quantile_tables(small, cfg["g"], cfg["fmt"]))) ==
            u32(oracle.quantile_init(inputs.bits(small), cfg["g"], cfg["fmt"]))).all()
