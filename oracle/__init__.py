"""ctypes front end of the CPU oracle (oracle/aaac_oracle.cpp).

Test infrastructure only: imported by tests/, by ``__graft_entry__.smoke`` and
by the ``cpu_baseline`` leg of ``bench.py``.  Nothing in the product package
imports it.  All arguments are host numpy arrays; bf16 data travels as uint16
bit patterns.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "aaac_oracle.cpp")
_LIB = os.path.join(_HERE, "liboracle.so")

NVFP4, INT4 = 0, 1


def build(force=False):
    """Compile the oracle with g++ (plain IEEE arithmetic, no contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["g++", "-O2", "-std=c++17", "-ffp-contract=off", "-fno-fast-math", "-Wall",
               "-Wextra", "-shared", "-fPIC", "-o", _LIB, _SRC]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None
_P = ctypes.c_void_p
_I64 = ctypes.c_int64
_INT = ctypes.c_int


def lib():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        L = _lib
        L.oracle_bf16_to_f32.restype = ctypes.c_float
        L.oracle_bf16_to_f32.argtypes = [ctypes.c_uint16]
        L.oracle_f32_to_bf16.restype = ctypes.c_uint16
        L.oracle_f32_to_bf16.argtypes = [ctypes.c_float]
        L.oracle_e4m3_to_f32.restype = ctypes.c_float
        L.oracle_e4m3_to_f32.argtypes = [ctypes.c_uint8]
        L.oracle_f32_to_e4m3.restype = ctypes.c_uint8
        L.oracle_f32_to_e4m3.argtypes = [ctypes.c_float]
        L.oracle_nearest_index.restype = _INT
        L.oracle_nearest_index.argtypes = [ctypes.c_float, _P]
        L.oracle_act_stats.restype = None
        L.oracle_act_stats.argtypes = [_P, _I64, _I64, _I64, _P]
        L.oracle_normalise.restype = _INT
        L.oracle_normalise.argtypes = [_P, _I64, _I64, _I64, _INT, _INT, _P, _P, _P]
        L.oracle_assign.restype = _INT
        L.oracle_assign.argtypes = [_P, _I64, _I64, _INT, _P, _P, _P, _P, _P, _P, _P, _P]
        L.oracle_lloyd_iteration.restype = _INT
        L.oracle_lloyd_iteration.argtypes = [_P, _I64, _I64, _INT, _P, _P, _P, _P]
        L.oracle_fit.restype = _INT
        L.oracle_fit.argtypes = [_P, _I64, _I64, _I64, _INT, _INT, _P, _P, _INT, _P, _P, _P, _P]
        L.oracle_kmeans_step.restype = _INT
        L.oracle_kmeans_step.argtypes = [_P, _I64, _I64, _INT, _P, _P, _P]
        L.oracle_fit_nested.restype = _INT
        L.oracle_fit_nested.argtypes = [_P, _I64, _I64, _I64, _INT, _INT, _P, _P, _INT, _INT, _P, _P, _P, _P]
        L.oracle_fit_sel.restype = _INT
        L.oracle_fit_sel.argtypes = [_P, _I64, _I64, _I64, _INT, _INT, _INT, _P, _P, _INT, _INT, _P, _P, _P, _P]
        L.oracle_encode_sel.restype = _INT
        L.oracle_encode_sel.argtypes = [_P, _I64, _I64, _I64, _INT, _INT, _INT, _P, _P, _P, _P, _P, _I64]
        L.oracle_dequant_sel.restype = _INT
        L.oracle_dequant_sel.argtypes = [_P, _P, _P, _I64, _P, _I64, _I64, _INT, _INT, _INT, _P, _I64]
        L.oracle_quantile_init.restype = _INT
        L.oracle_quantile_init.argtypes = [_P, _I64, _I64, _I64, _INT, _INT, _P]
        L.oracle_gemv_w4a16.restype = _INT
        L.oracle_gemv_w4a16.argtypes = [_P, _I64, _I64, _P, _P, _P, _I64, _P, _I64, _I64, _INT, _INT, _INT, _P, _P]
        L.oracle_gemm_w4a16.restype = _INT
        L.oracle_gemm_w4a16.argtypes = L.oracle_gemv_w4a16.argtypes
        L.oracle_encode.restype = _INT
        L.oracle_encode.argtypes = [_P, _I64, _I64, _I64, _INT, _INT, _P, _P, _P, _P]
        L.oracle_dequant.restype = _INT
        L.oracle_dequant.argtypes = [_P, _P, _P, _I64, _I64, _INT, _INT, _P, _I64]
    return _lib


def _ptr(a):
    return None if a is None else a.ctypes.data_as(_P)


def _c(a, dtype):
    a = np.ascontiguousarray(a, dtype=dtype)
    return a


def _check(rc, what):
    if rc != 0:
        raise ValueError(f"oracle {what}: invalid arguments (rc={rc})")


def _scale_dtype(fmt):
    return np.uint8 if fmt == NVFP4 else np.uint16


# ---------------------------------------------------------------- scalars

def bf16_to_f32(h):
    return lib().oracle_bf16_to_f32(int(h))


def f32_to_bf16(f):
    return lib().oracle_f32_to_bf16(float(np.float32(f)))


def e4m3_to_f32(c):
    return lib().oracle_e4m3_to_f32(int(c))


def f32_to_e4m3(f):
    return lib().oracle_f32_to_e4m3(float(np.float32(f)))


def nearest_index(x, table16):
    t = _c(table16, np.float32)
    assert t.shape == (16,)
    return lib().oracle_nearest_index(float(np.float32(x)), _ptr(t))


# ------------------------------------------------------------------ steps

def act_stats(X_bits):
    """X_bits: uint16 [tokens, K] (bf16 bit patterns) -> float32 [K]."""
    X = _c(X_bits, np.uint16)
    tokens, K = X.shape
    out = np.empty(K, np.float32)
    lib().oracle_act_stats(_ptr(X), tokens, K, K, _ptr(out))
    return out


def normalise(W_bits, g, fmt):
    """-> (unsigned scale codes [N, K/g], scale values f32 [N, K/g], w~ f32 [N, K])."""
    W = _c(W_bits, np.uint16)
    N, K = W.shape
    codes = np.empty((N, K // g), _scale_dtype(fmt))
    vals = np.empty((N, K // g), np.float32)
    wn = np.empty((N, K), np.float32)
    _check(lib().oracle_normalise(_ptr(W), N, K, K, g, fmt, _ptr(codes), _ptr(vals), _ptr(wn)),
           "normalise")
    return codes, vals, wn


def assign(wn, g, importance, tables):
    """One assignment step -> dict(e0, e1, sigma, idx0, idx1, objective)."""
    wn = _c(wn, np.float32)
    N, K = wn.shape
    I = _c(importance, np.float32)
    T = _c(tables, np.float32).reshape(32)
    G = K // g
    e0 = np.empty((N, G), np.float32)
    e1 = np.empty((N, G), np.float32)
    sigma = np.empty((N, G), np.uint8)
    idx0 = np.empty((N, K), np.uint8)
    idx1 = np.empty((N, K), np.uint8)
    J = ctypes.c_double()
    _check(lib().oracle_assign(_ptr(wn), N, K, g, _ptr(I), _ptr(T), _ptr(e0), _ptr(e1),
                               _ptr(sigma), _ptr(idx0), _ptr(idx1), ctypes.byref(J)), "assign")
    return dict(e0=e0, e1=e1, sigma=sigma, idx0=idx0, idx1=idx1, objective=J.value)


def lloyd_iteration(wn, g, importance, tables):
    """-> (new tables f32 [32], sums f64 [64] = Swx then Sw, objective)."""
    wn = _c(wn, np.float32)
    N, K = wn.shape
    I = _c(importance, np.float32)
    T = _c(tables, np.float32).reshape(32).copy()
    sums = np.empty(64, np.float64)
    J = ctypes.c_double()
    _check(lib().oracle_lloyd_iteration(_ptr(wn), N, K, g, _ptr(I), _ptr(T), _ptr(sums),
                                        ctypes.byref(J)), "lloyd_iteration")
    return T, sums, J.value


def fit(W_bits, g, fmt, importance, init_grid, iterations, trace=False):
    """-> dict(tables_f32 [32], tables_bf16 uint16 [32], objective [iters], tables_trace)."""
    W = _c(W_bits, np.uint16)
    N, K = W.shape
    I = _c(importance, np.float32)
    G0 = _c(init_grid, np.float32).reshape(32)
    tf = np.empty(32, np.float32)
    tb = np.empty(32, np.uint16)
    obj = np.empty(max(iterations, 0), np.float64)
    tt = np.empty((max(iterations, 0), 32), np.float32) if trace else None
    _check(lib().oracle_fit(_ptr(W), N, K, K, g, fmt, _ptr(I), _ptr(G0), iterations, _ptr(tf),
                            _ptr(tb), _ptr(obj), _ptr(tt)), "fit")
    return dict(tables_f32=tf, tables_bf16=tb, objective=obj, tables_trace=tt)


def kmeans_step(wn, g, importance, sigma, tables):
    """One inner k-means step with the table choice frozen -> new tables f32 [32]."""
    wn = _c(wn, np.float32)
    N, K = wn.shape
    I = _c(importance, np.float32)
    sg = _c(sigma, np.uint8).reshape(N, K // g)
    T = _c(tables, np.float32).reshape(32).copy()
    _check(lib().oracle_kmeans_step(_ptr(wn), N, K, g, _ptr(I), _ptr(sg), _ptr(T)), "kmeans_step")
    return T


def fit_nested(W_bits, g, fmt, importance, init_grid, n_outer, n_inner, trace=False):
    """Alg. 1 with both loops -> dict(tables_f32, tables_bf16, objective [n_outer], tables_trace)."""
    W = _c(W_bits, np.uint16)
    N, K = W.shape
    I = _c(importance, np.float32)
    G0 = _c(init_grid, np.float32).reshape(32)
    tf = np.empty(32, np.float32)
    tb = np.empty(32, np.uint16)
    obj = np.empty(max(n_outer, 0), np.float64)
    tt = np.empty((max(n_outer * n_inner, 0), 32), np.float32) if trace else None
    _check(lib().oracle_fit_nested(_ptr(W), N, K, K, g, fmt, _ptr(I), _ptr(G0), n_outer, n_inner, _ptr(tf),
                                   _ptr(tb), _ptr(obj), _ptr(tt)), "fit_nested")
    return dict(tables_f32=tf, tables_bf16=tb, objective=obj, tables_trace=tt)


def encode(W_bits, g, fmt, importance, tables_bf16):
    """-> (codes uint8 [N, K/2], signed scales [N, K/g])."""
    W = _c(W_bits, np.uint16)
    N, K = W.shape
    I = _c(importance, np.float32)
    tb = _c(tables_bf16, np.uint16).reshape(32)
    codes = np.empty((N, K // 2), np.uint8)
    scales = np.empty((N, K // g), _scale_dtype(fmt))
    _check(lib().oracle_encode(_ptr(W), N, K, K, g, fmt, _ptr(I), _ptr(tb), _ptr(codes),
                               _ptr(scales)), "encode")
    return codes, scales


def dequant(codes, scales, tables_bf16, g, fmt):
    """-> W_hat uint16 [N, K] (bf16 bit patterns)."""
    codes = _c(codes, np.uint8)
    N, K = codes.shape[0], codes.shape[1] * 2
    scales = _c(scales, _scale_dtype(fmt))
    tb = _c(tables_bf16, np.uint16).reshape(32)
    out = np.empty((N, K), np.uint16)
    _check(lib().oracle_dequant(_ptr(codes), _ptr(scales), _ptr(tb), N, K, g, fmt, _ptr(out), K),
           "dequant")
    return out


# ------------------------------------------- selection groups smaller than scale groups

def fit_sel(W_bits, g, S, fmt, importance, init_grid, n_outer, n_inner, trace=False):
    """Alg. 1 with scale groups of g and selection groups of S <= g weights."""
    W = _c(W_bits, np.uint16)
    N, K = W.shape
    I = _c(importance, np.float32)
    G0 = _c(init_grid, np.float32).reshape(32)
    tf = np.empty(32, np.float32)
    tb = np.empty(32, np.uint16)
    obj = np.empty(max(n_outer, 0), np.float64)
    tt = np.empty((max(n_outer * n_inner, 0), 32), np.float32) if trace else None
    _check(lib().oracle_fit_sel(_ptr(W), N, K, K, g, S, fmt, _ptr(I), _ptr(G0), n_outer, n_inner, _ptr(tf),
                                _ptr(tb), _ptr(obj), _ptr(tt)), "fit_sel")
    return dict(tables_f32=tf, tables_bf16=tb, objective=obj, tables_trace=tt)


def sel_stride(K, S):
    return (K // S + 7) // 8


def encode_sel(W_bits, g, S, fmt, importance, tables_bf16):
    """-> (codes uint8 [N, K/2], scales [N, K/g], sel_bits uint8 [N, ceil(K/S/8)] or None if S == g)."""
    W = _c(W_bits, np.uint16)
    N, K = W.shape
    I = _c(importance, np.float32)
    tb = _c(tables_bf16, np.uint16).reshape(32)
    codes = np.empty((N, K // 2), np.uint8)
    scales = np.empty((N, K // g), _scale_dtype(fmt))
    bits = np.full((N, sel_stride(K, S)), 0xFF, np.uint8) if S < g else None
    _check(lib().oracle_encode_sel(_ptr(W), N, K, K, g, S, fmt, _ptr(I), _ptr(tb), _ptr(codes), _ptr(scales),
                                   _ptr(bits), sel_stride(K, S)), "encode_sel")
    return codes, scales, bits


def dequant_sel(codes, scales, sel_bits, tables_bf16, g, S, fmt):
    codes = _c(codes, np.uint8)
    N, K = codes.shape[0], codes.shape[1] * 2
    scales = _c(scales, _scale_dtype(fmt))
    tb = _c(tables_bf16, np.uint16).reshape(32)
    bits = None if sel_bits is None else _c(sel_bits, np.uint8)
    out = np.empty((N, K), np.uint16)
    _check(lib().oracle_dequant_sel(_ptr(codes), _ptr(scales), _ptr(bits), 0 if bits is None else bits.shape[1],
                                    _ptr(tb), N, K, g, S, fmt, _ptr(out), K), "dequant_sel")
    return out


def quantile_init(W_bits, g, fmt):
    """Initial tables from quantiles of the normalised weights -> float32 [32] (T0 then T1)."""
    W = _c(W_bits, np.uint16)
    N, K = W.shape
    grid = np.empty(32, np.float32)
    _check(lib().oracle_quantile_init(_ptr(W), N, K, K, g, fmt, _ptr(grid)), "quantile_init")
    return grid


def gemv_w4a16(x_bits, codes, scales, sel_bits, tables_bf16, g, S, fmt, round_weights=False):
    """y = x W^^T with the quantised layer: x_bits uint16 [M, K] (bf16) -> (y float32 [M, N],
    abs_sum float64 [M, N] = sum_k |x * w^|).  round_weights: w^ rounded to bf16 first."""
    x = _c(x_bits, np.uint16)
    M, K = x.shape
    codes = _c(codes, np.uint8)
    N = codes.shape[0]
    assert codes.shape[1] * 2 == K
    scales = _c(scales, _scale_dtype(fmt))
    tb = _c(tables_bf16, np.uint16).reshape(32)
    bits = None if sel_bits is None else _c(sel_bits, np.uint8)
    y = np.empty((M, N), np.float32)
    mag = np.empty((M, N), np.float64)
    fn = lib().oracle_gemm_w4a16 if round_weights else lib().oracle_gemv_w4a16
    _check(fn(_ptr(x), M, K, _ptr(codes), _ptr(scales), _ptr(bits),
              0 if bits is None else bits.shape[1], _ptr(tb), N, K, g, S, fmt, _ptr(y), _ptr(mag)), "gemv_w4a16")
    return y, mag


def gemm_w4a16(x_bits, codes, scales, sel_bits, tables_bf16, g, S, fmt):
    """The product with the dequantised weights rounded to bf16 (those dequant_sel returns)."""
    return gemv_w4a16(x_bits, codes, scales, sel_bits, tables_bf16, g, S, fmt, round_weights=True)
