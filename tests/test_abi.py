"""Host-side checks of the C ABI that need no GPU: the library loads, exports
every function include/aaac.h declares, and rejects bad arguments before any
HIP call."""
import ctypes
import os
import re

import numpy as np
import pytest

import paper_2605_08692_amd as A

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = open(os.path.join(ROOT, "include", "aaac.h")).read()

OK, E_NULL, E_SHAPE, E_ARG, E_WS = 0, -1, -2, -3, -4


def declared_functions():
    body = re.sub(r"/\*.*?\*/", "", HEADER, flags=re.S)
    return sorted(set(re.findall(r"\b(aaac_[a-z_0-9]+)\s*\(", body)))


def test_header_functions_are_exported():
    names = declared_functions()
    assert {"aaac_act_stats", "aaac_fit", "aaac_encode", "aaac_dequant", "aaac_fit_batch",
            "aaac_act_stats_workspace", "aaac_fit_workspace", "aaac_fit_batch_workspace",
            "aaac_status_string"} <= set(names)
    L = A.library()
    for n in names:
        assert hasattr(L, n), n


def test_status_strings():
    L = A.library()
    for code in (0, -1, -2, -3, -4, -5):
        assert len(L.aaac_status_string(code)) > 1


def test_workspace_queries():
    assert A.aaac_fit_workspace(4096, 4096, 128, A.INT4) > 4096 * 32 * 4
    assert A.aaac_fit_workspace(4096, 4096, 24, A.INT4) == 0
    assert A.aaac_fit_workspace(4096, 4100, 128, A.INT4) == 0
    assert A.aaac_fit_workspace(0, 4096, 128, A.INT4) > 0
    assert A.aaac_act_stats_workspace(65536, 4096) >= 4096 * 8
    assert A.aaac_act_stats_workspace(10, 0) == 0


FAKE = ctypes.c_void_p(0x10000)  # aligned non-null stand-in; never dereferenced on the error paths


def fit_rc(W=FAKE, N=8, K=64, ldw=64, g=16, fmt=0, I=FAKE, grid="ok", iters=1, tb=FAKE, ws=FAKE, ws_bytes=1 << 30):
    if isinstance(grid, str):
        gr = np.concatenate([np.arange(16), np.arange(16)]).astype(np.float32)
    else:
        gr = grid
    gp = None if gr is None else gr.ctypes.data_as(ctypes.c_void_p)
    return A.library().aaac_fit(W, N, K, ldw, g, fmt, I, gp, iters, None, tb, None, ws, ws_bytes, None)


def test_fit_argument_validation():
    assert fit_rc(W=None) == E_NULL
    assert fit_rc(I=None) == E_NULL
    assert fit_rc(tb=None) == E_NULL
    assert fit_rc(grid=None) == E_NULL
    assert fit_rc(g=24) == E_SHAPE
    assert fit_rc(K=72) == E_SHAPE          # not a multiple of the group size
    assert fit_rc(ldw=60) == E_SHAPE        # leading dimension below K
    assert fit_rc(ldw=68) == E_SHAPE        # leading dimension not a multiple of 8
    assert fit_rc(N=-1) == E_SHAPE
    assert fit_rc(W=ctypes.c_void_p(0x10002)) == E_SHAPE  # misaligned
    assert fit_rc(fmt=2) == E_ARG
    assert fit_rc(iters=-1) == E_ARG
    bad = np.concatenate([np.arange(16), np.arange(16)]).astype(np.float32)
    bad[3] = 10
    assert fit_rc(grid=bad) == E_ARG
    nan = np.concatenate([np.arange(16), np.arange(16)]).astype(np.float32)
    nan[20] = np.nan
    assert fit_rc(grid=nan) == E_ARG
    assert fit_rc(ws=None) == E_WS
    assert fit_rc(ws_bytes=16) == E_WS
    assert fit_rc(ws=ctypes.c_void_p(0x10010)) == E_WS  # not 256-byte aligned


def test_other_entry_points_validate():
    L = A.library()
    assert L.aaac_act_stats(None, 4, 64, 64, FAKE, FAKE, 1 << 20, None) == E_NULL
    assert L.aaac_act_stats(FAKE, 4, 64, 64, None, FAKE, 1 << 20, None) == E_NULL
    assert L.aaac_act_stats(FAKE, 4, 60, 64, FAKE, FAKE, 1 << 20, None) == E_SHAPE
    assert L.aaac_act_stats(FAKE, 4, 64, 32, FAKE, FAKE, 1 << 20, None) == E_SHAPE
    assert L.aaac_act_stats(FAKE, -4, 64, 64, FAKE, FAKE, 1 << 20, None) == E_SHAPE
    assert L.aaac_act_stats(FAKE, 4, 64, 64, FAKE, FAKE, 8, None) == E_WS
    # the variant without a workspace: same checks, and a K beyond what its own array holds
    assert L.aaac_act_stats_static(None, 4, 64, 64, FAKE, None) == E_NULL
    assert L.aaac_act_stats_static(FAKE, 4, 64, 64, None, None) == E_NULL
    assert L.aaac_act_stats_static(FAKE, 4, 60, 64, FAKE, None) == E_SHAPE
    assert L.aaac_act_stats_static(FAKE, 4, 64, 32, FAKE, None) == E_SHAPE
    assert L.aaac_act_stats_static(FAKE, 4, (1 << 20) + 4096, (1 << 20) + 4096, FAKE, None) == E_WS
    assert L.aaac_encode(FAKE, 8, 64, 64, 16, 0, FAKE, FAKE, None, FAKE, None) == E_NULL
    assert L.aaac_encode(FAKE, 8, 64, 64, 48, 0, FAKE, FAKE, FAKE, FAKE, None) == E_SHAPE
    assert L.aaac_encode(FAKE, 8, 64, 64, 16, 7, FAKE, FAKE, FAKE, FAKE, None) == E_ARG
    assert L.aaac_dequant(FAKE, None, FAKE, 8, 64, 16, 0, FAKE, 64, None) == E_NULL
    assert L.aaac_dequant(FAKE, FAKE, FAKE, 8, 64, 16, 0, FAKE, 63, None) == E_SHAPE
    assert L.aaac_dequant(FAKE, FAKE, FAKE, 8, 64, 16, 3, FAKE, 64, None) == E_ARG
    assert L.aaac_fit_batch(None, 1, 16, 0, FAKE, 1, FAKE, 1 << 20, None) == E_NULL
    assert L.aaac_fit_nested(None, 1, 16, 16, 0, FAKE, 1, 1, FAKE, 1 << 20, None) == E_NULL
    layer = A.binding.aaac_layer_t(0x10000, 8, 64, 64, 0x10000, None, 0x10000, None)
    arr = (A.binding.aaac_layer_t * 1)(layer)
    grid = np.concatenate([np.arange(16), np.arange(16)]).astype(np.float32)
    gp = grid.ctypes.data_as(ctypes.c_void_p)
    assert L.aaac_fit_nested(arr, 1, 16, 16, 0, gp, 1, 0, FAKE, 1 << 20, None) == E_ARG    # no inner step
    assert L.aaac_fit_nested(arr, 1, 16, 16, 0, gp, -1, 2, FAKE, 1 << 20, None) == E_ARG
    assert L.aaac_fit_nested(arr, 1, 16, 16, 0, gp, 1 << 20, 1 << 20, FAKE, 1 << 20, None) == E_ARG  # pass count overflows
    assert L.aaac_fit_nested(arr, 1, 16, 16, 0, gp, 2, 2, FAKE, 16, None) == E_WS
    assert L.aaac_fit_nested_workspace(arr, 1, 16, 16, 0) == L.aaac_fit_batch_workspace(arr, 1, 16, 0) > 0
    # quantile initialisation
    assert L.aaac_quantile_init(None, 8, 64, 64, 16, 0, FAKE, FAKE, 1 << 22, None) == E_NULL
    assert L.aaac_quantile_init(FAKE, 8, 64, 64, 16, 0, None, FAKE, 1 << 22, None) == E_NULL
    assert L.aaac_quantile_init(FAKE, 0, 64, 64, 16, 0, FAKE, FAKE, 1 << 22, None) == E_SHAPE   # no weights
    assert L.aaac_quantile_init(FAKE, 8, 72, 72, 16, 0, FAKE, FAKE, 1 << 22, None) == E_SHAPE
    assert L.aaac_quantile_init(FAKE, 8, 64, 64, 16, 4, FAKE, FAKE, 1 << 22, None) == E_ARG
    assert L.aaac_quantile_init(FAKE, 8, 64, 64, 16, 0, FAKE, FAKE, 64, None) == E_WS
    assert L.aaac_quantile_init_workspace(8, 64, 16, 0) == L.aaac_fit_workspace(8, 64, 16, 0)
    empty = (A.binding.aaac_layer_t * 1)(A.binding.aaac_layer_t(None, 0, 64, 64, 0x10000, None, 0x10000, None))
    assert L.aaac_fit_nested(empty, 1, 16, 16, 0, None, 1, 1, FAKE, 1 << 22, None) == E_SHAPE  # quantiles of nothing
    assert L.aaac_fit_batch(arr, 1, 16, 0, None, 1, FAKE, 1 << 22, None) == E_NULL
    # the quantised layer applied to activations
    gemv = lambda **kw: L.aaac_gemv_w4a16(*[kw.get(k, d) for k, d in (
        ("x", FAKE), ("M", 2), ("ldx", 128), ("codes", FAKE), ("scales", FAKE), ("bits", None), ("stride", 0),
        ("tb", FAKE), ("N", 8), ("K", 128), ("g", 16), ("S", 16), ("fmt", 0), ("y", FAKE), ("ldy", 8), ("st", None))])
    assert gemv(x=None) == E_NULL and gemv(y=None) == E_NULL and gemv(tb=None) == E_NULL
    assert gemv(K=144, ldx=144) == E_SHAPE            # a multiple of the group size but not of 32
    assert gemv(ldx=120) == E_SHAPE and gemv(ldy=4) == E_SHAPE
    assert gemv(g=64, S=16) == E_NULL                 # selection bits needed
    assert gemv(g=64, S=16, bits=FAKE, stride=0) == E_SHAPE
    assert gemv(fmt=9) == E_ARG
    assert gemv(codes=ctypes.c_void_p(0x10008)) == E_SHAPE   # codes not 16-byte aligned
    W = ctypes.c_void_p(0x20000)
    assert L.aaac_gemm_w4a16(FAKE, 2, 128, FAKE, FAKE, None, 0, FAKE, 8, 96, 16, 16, 0, FAKE, 8, W, 1 << 20, None) == E_SHAPE  # K % 64
    assert L.aaac_gemm_w4a16(FAKE, 2, 128, FAKE, ctypes.c_void_p(0x10004), None, 0, FAKE, 8, 128, 16, 16, 0, FAKE, 8, W, 1 << 20, None) == E_SHAPE
    assert L.aaac_gemm_w4a16(FAKE, 2, 128, FAKE, FAKE, None, 0, FAKE, 8, 128, 64, 16, 0, FAKE, 8, W, 1 << 20, None) == E_NULL
    assert L.aaac_gemm_w4a16(FAKE, 2, 128, FAKE, FAKE, None, 0, FAKE, 8, 128, 16, 16, 0, FAKE, 8, W, 64, None) == E_WS
    assert L.aaac_gemm_w4a16(FAKE, 2, 128, FAKE, FAKE, None, 0, FAKE, 8, 128, 16, 16, 0, FAKE, 8, None, 0, None) == E_WS
    assert L.aaac_gemm_w4a16_workspace(2, 128) == 8 * 64 * 16 and L.aaac_gemm_w4a16_workspace(64, 8192) == 32 * 8 * 4 * 64 * 16
    # selection groups: a size that divides the scale group, 16..128
    assert L.aaac_fit_nested(arr, 1, 16, 32, 0, gp, 1, 1, FAKE, 1 << 20, None) == E_SHAPE  # larger than the scale group
    assert L.aaac_fit_nested(arr, 1, 64, 8, 1, gp, 1, 1, FAKE, 1 << 20, None) == E_SHAPE
    assert L.aaac_fit_nested(arr, 1, 64, 24, 1, gp, 1, 1, FAKE, 1 << 20, None) == E_SHAPE
    assert L.aaac_fit_nested_workspace(arr, 1, 64, 24, 1) == 0
    assert L.aaac_fit_nested_workspace(arr, 1, 64, 16, 1) >= L.aaac_fit_nested_workspace(arr, 1, 64, 64, 1) > 0
    assert L.aaac_encode_sel(FAKE, 8, 128, 128, 64, 16, 1, FAKE, FAKE, FAKE, FAKE, None, 1, None) == E_NULL
    assert L.aaac_encode_sel(FAKE, 8, 128, 128, 64, 16, 1, FAKE, FAKE, FAKE, FAKE, FAKE, 0, None) == E_SHAPE  # stride < 1
    assert L.aaac_encode_sel(FAKE, 8, 128, 128, 64, 128, 1, FAKE, FAKE, FAKE, FAKE, FAKE, 1, None) == E_SHAPE
    assert L.aaac_encode_sel(FAKE, 8, 128, 128, 64, 16, 5, FAKE, FAKE, FAKE, FAKE, FAKE, 1, None) == E_ARG
    assert L.aaac_dequant_sel(FAKE, FAKE, None, 1, FAKE, 8, 128, 64, 16, 1, FAKE, 128, None) == E_NULL
    assert L.aaac_dequant_sel(FAKE, FAKE, FAKE, 0, FAKE, 8, 128, 64, 16, 1, FAKE, 128, None) == E_SHAPE
    assert L.aaac_dequant_sel(FAKE, FAKE, FAKE, 1, FAKE, 8, 128, 64, 48, 1, FAKE, 128, None) == E_SHAPE


def test_binding_raises_with_message():
    import torch
    W = torch.zeros((8, 72), dtype=torch.bfloat16)
    with pytest.raises(A.AaacError) as e:
        A.aaac_fit(W, 16, A.NVFP4, torch.ones(72), np.zeros(32, np.float32), 1,
                   tables_f32=torch.zeros(32), tables_bf16=torch.zeros(32, dtype=torch.int16),
                   objective_trace=torch.zeros(1, dtype=torch.float64), ws=torch.zeros(4096, dtype=torch.uint8))
    assert e.value.status == E_SHAPE and "shape" in str(e.value)
