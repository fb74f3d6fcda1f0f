"""ctypes binding of libaaac.so: same names as the C ABI in include/aaac.h.

Argument marshalling only.  Tensors are torch tensors on the GPU (torch is used
for device memory and streams); every step runs in the library's kernels.  There
is no fallback: if the library is missing, every call raises.
"""
import ctypes
import os

import torch

NVFP4, INT4 = 0, 1

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libaaac.so")
_lib = None

_P = ctypes.c_void_p
_I64 = ctypes.c_int64
_INT = ctypes.c_int
_SZ = ctypes.c_size_t


class AaacError(RuntimeError):
    def __init__(self, status, what):
        self.status = status
        msg = library().aaac_status_string(status).decode() if _lib is not None else str(status)
        super().__init__(f"{what}: {msg} ({status})")


class aaac_layer_t(ctypes.Structure):
    _fields_ = [("W", _P), ("N", _I64), ("K", _I64), ("ldw", _I64), ("importance", _P),
                ("tables_f32", _P), ("tables_bf16", _P), ("objective_trace", _P)]


def library_path():
    return _LIB_PATH


def library():
    """The loaded C library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise RuntimeError(f"{_LIB_PATH} not found: build it with `python -m paper_2605_08692_amd.build`")
        L = ctypes.CDLL(_LIB_PATH)
        L.aaac_status_string.restype = ctypes.c_char_p
        L.aaac_status_string.argtypes = [_INT]
        L.aaac_act_stats_workspace.restype = _SZ
        L.aaac_act_stats_workspace.argtypes = [_I64, _I64]
        L.aaac_act_stats.restype = _INT
        L.aaac_act_stats.argtypes = [_P, _I64, _I64, _I64, _P, _P, _SZ, _P]
        L.aaac_act_stats_static.restype = _INT
        L.aaac_act_stats_static.argtypes = [_P, _I64, _I64, _I64, _P, _P]
        L.aaac_fit_workspace.restype = _SZ
        L.aaac_fit_workspace.argtypes = [_I64, _I64, _INT, _INT]
        L.aaac_fit.restype = _INT
        L.aaac_fit.argtypes = [_P, _I64, _I64, _I64, _INT, _INT, _P, _P, _INT, _P, _P, _P, _P, _SZ, _P]
        L.aaac_fit_batch_workspace.restype = _SZ
        L.aaac_fit_batch_workspace.argtypes = [_P, _INT, _INT, _INT]
        L.aaac_fit_batch.restype = _INT
        L.aaac_fit_batch.argtypes = [_P, _INT, _INT, _INT, _P, _INT, _P, _SZ, _P]
        L.aaac_fit_nested_workspace.restype = _SZ
        L.aaac_fit_nested_workspace.argtypes = [_P, _INT, _INT, _INT, _INT]
        L.aaac_fit_nested.restype = _INT
        L.aaac_fit_nested.argtypes = [_P, _INT, _INT, _INT, _INT, _P, _INT, _INT, _P, _SZ, _P]
        L.aaac_quantile_init_workspace.restype = _SZ
        L.aaac_quantile_init_workspace.argtypes = [_I64, _I64, _INT, _INT]
        L.aaac_quantile_init.restype = _INT
        L.aaac_quantile_init.argtypes = [_P, _I64, _I64, _I64, _INT, _INT, _P, _P, _SZ, _P]
        L.aaac_gemv_w4a16.restype = _INT
        L.aaac_gemv_w4a16.argtypes = [_P, _I64, _I64, _P, _P, _P, _I64, _P, _I64, _I64, _INT, _INT, _INT, _P, _I64, _P]
        L.aaac_gemm_w4a16_workspace.restype = _SZ
        L.aaac_gemm_w4a16_workspace.argtypes = [_I64, _I64]
        L.aaac_gemm_w4a16.restype = _INT
        L.aaac_gemm_w4a16.argtypes = [_P, _I64, _I64, _P, _P, _P, _I64, _P, _I64, _I64, _INT, _INT, _INT, _P, _I64, _P,
                                      _SZ, _P]
        L.aaac_encode_sel.restype = _INT
        L.aaac_encode_sel.argtypes = [_P, _I64, _I64, _I64, _INT, _INT, _INT, _P, _P, _P, _P, _P, _I64, _P]
        L.aaac_dequant_sel.restype = _INT
        L.aaac_dequant_sel.argtypes = [_P, _P, _P, _I64, _P, _I64, _I64, _INT, _INT, _INT, _P, _I64, _P]
        L.aaac_encode.restype = _INT
        L.aaac_encode.argtypes = [_P, _I64, _I64, _I64, _INT, _INT, _P, _P, _P, _P, _P]
        L.aaac_dequant.restype = _INT
        L.aaac_dequant.argtypes = [_P, _P, _P, _I64, _I64, _INT, _INT, _P, _I64, _P]
        _lib = L
    return _lib


def _stream(stream):
    if stream is None:
        if not torch.cuda.is_available():  # argument errors can still be reported without a device
            return None
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def _dp(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _check(rc, what):
    if rc != 0:
        raise AaacError(rc, what)


def _grid(init_grid):
    g = torch.as_tensor(init_grid, dtype=torch.float32, device="cpu").contiguous()
    if g.numel() != 32:
        raise ValueError("init_grid must hold 32 floats")
    return g


def _scale_dtype(fmt):
    return torch.uint8 if fmt == NVFP4 else torch.int16


def _workspace(nbytes, device):
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)


def aaac_act_stats_workspace(tokens, K):
    return library().aaac_act_stats_workspace(tokens, K)


def aaac_act_stats(X, importance=None, ws=None, stream=None):
    """X: bf16 [tokens, K] (row stride allowed) -> importance fp32 [K]."""
    assert X.dtype == torch.bfloat16 and X.dim() == 2 and X.stride(1) == 1
    tokens, K = X.shape
    if importance is None:
        importance = torch.empty(K, dtype=torch.float32, device=X.device)
    need = aaac_act_stats_workspace(tokens, K)
    if ws is None:
        ws = _workspace(need, X.device)
    ldx = X.stride(0) if tokens > 1 else max(X.stride(0), K)
    _check(library().aaac_act_stats(_dp(X), tokens, K, ldx, _dp(importance), _dp(ws), ws.numel(),
                                    _stream(stream)), "aaac_act_stats")
    return importance


def aaac_act_stats_static(X, importance, stream=None):
    """aaac_act_stats with the partial sums in the library's own device array: no workspace, and
    `importance` must be given (nothing is allocated here either)."""
    assert X.dtype == torch.bfloat16 and X.dim() == 2 and X.stride(1) == 1
    tokens, K = X.shape
    ldx = X.stride(0) if tokens > 1 else max(X.stride(0), K)
    _check(library().aaac_act_stats_static(_dp(X), tokens, K, ldx, _dp(importance), _stream(stream)),
           "aaac_act_stats_static")
    return importance


def aaac_fit_workspace(N, K, group_size, fmt):
    return library().aaac_fit_workspace(N, K, group_size, fmt)


def aaac_fit(W, group_size, fmt, importance, init_grid, iterations, tables_f32=None,
             tables_bf16=None, objective_trace=None, ws=None, stream=None, want_objective=True):
    """W: bf16 [N, K].  Returns (tables_f32 [32], tables_bf16 int16 [32], objective f64 [iters])."""
    assert W.dtype == torch.bfloat16 and W.dim() == 2 and W.stride(1) == 1
    N, K = W.shape
    dev = W.device
    if tables_f32 is None:
        tables_f32 = torch.empty(32, dtype=torch.float32, device=dev)
    if tables_bf16 is None:
        tables_bf16 = torch.empty(32, dtype=torch.int16, device=dev)
    if objective_trace is None and want_objective:
        objective_trace = torch.empty(max(iterations, 1), dtype=torch.float64, device=dev)
    if ws is None:
        ws = _workspace(aaac_fit_workspace(N, K, group_size, fmt), dev)
    g = _grid(init_grid)
    ldw = W.stride(0) if N > 1 else max(W.stride(0), K)
    _check(library().aaac_fit(_dp(W), N, K, ldw, group_size, fmt, _dp(importance),
                              ctypes.c_void_p(g.data_ptr()), iterations, _dp(tables_f32),
                              _dp(tables_bf16), _dp(objective_trace), _dp(ws), ws.numel(),
                              _stream(stream)), "aaac_fit")
    return tables_f32, tables_bf16, objective_trace


def make_layers(Ws, importances, iterations, want_objective=True):
    """Descriptor array + output tensors for aaac_fit_batch."""
    n = len(Ws)
    arr = (aaac_layer_t * n)()
    outs = []
    for i, (W, I) in enumerate(zip(Ws, importances)):
        assert W.dtype == torch.bfloat16 and W.dim() == 2 and W.stride(1) == 1
        N, K = W.shape
        tf = torch.empty(32, dtype=torch.float32, device=W.device)
        tb = torch.empty(32, dtype=torch.int16, device=W.device)
        ob = torch.empty(max(iterations, 1), dtype=torch.float64, device=W.device) if want_objective else None
        arr[i] = aaac_layer_t(W.data_ptr(), N, K, W.stride(0) if N > 1 else max(W.stride(0), K),
                              I.data_ptr(), tf.data_ptr(), tb.data_ptr(),
                              ob.data_ptr() if ob is not None else None)
        outs.append((tf, tb, ob))
    return arr, outs


def aaac_fit_batch_workspace(layers, group_size, fmt):
    return library().aaac_fit_batch_workspace(layers, len(layers), group_size, fmt)


def aaac_fit_batch(layers, group_size, fmt, init_grid, iterations, ws, stream=None):
    """layers: array from make_layers.  Outputs land in the tensors make_layers returned."""
    g = _grid(init_grid)
    _check(library().aaac_fit_batch(layers, len(layers), group_size, fmt, ctypes.c_void_p(g.data_ptr()),
                                    iterations, _dp(ws), ws.numel(), _stream(stream)), "aaac_fit_batch")


def aaac_fit_nested_workspace(layers, group_size, fmt, sel_size=None):
    return library().aaac_fit_nested_workspace(layers, len(layers), group_size, sel_size or group_size, fmt)


def aaac_fit_nested(layers, group_size, fmt, init_grid, n_outer, n_inner, ws, stream=None, sel_size=None):
    """Both loops of the learning algorithm, one table choice per sel_size weights (default: per
    scale group); layers: array from make_layers (objective: n_outer values).  init_grid None:
    the tables start from the quantiles of each layer's normalised weights."""
    g = None if init_grid is None else _grid(init_grid)
    _check(library().aaac_fit_nested(layers, len(layers), group_size, sel_size or group_size, fmt,
                                     None if g is None else ctypes.c_void_p(g.data_ptr()), n_outer, n_inner,
                                     _dp(ws), ws.numel(), _stream(stream)), "aaac_fit_nested")


def aaac_encode(W, group_size, fmt, importance, tables_bf16, codes=None, scales=None, stream=None):
    """-> (codes uint8 [N, K/2], scales uint8|int16 [N, K/group_size] with sigma in the top bit)."""
    assert W.dtype == torch.bfloat16 and W.dim() == 2 and W.stride(1) == 1
    N, K = W.shape
    if codes is None:
        codes = torch.empty((N, K // 2), dtype=torch.uint8, device=W.device)
    if scales is None:
        scales = torch.empty((N, K // group_size), dtype=_scale_dtype(fmt), device=W.device)
    ldw = W.stride(0) if N > 1 else max(W.stride(0), K)
    _check(library().aaac_encode(_dp(W), N, K, ldw, group_size, fmt, _dp(importance), _dp(tables_bf16),
                                 _dp(codes), _dp(scales), _stream(stream)), "aaac_encode")
    return codes, scales


def aaac_dequant(codes, scales, tables_bf16, group_size, fmt, W_hat=None, stream=None):
    """-> W_hat bf16 [N, K]."""
    N, K = codes.shape[0], codes.shape[1] * 2
    if W_hat is None:
        W_hat = torch.empty((N, K), dtype=torch.bfloat16, device=codes.device)
    ldo = W_hat.stride(0) if N > 1 else max(W_hat.stride(0), K)
    _check(library().aaac_dequant(_dp(codes), _dp(scales), _dp(tables_bf16), N, K, group_size, fmt,
                                  _dp(W_hat), ldo, _stream(stream)), "aaac_dequant")
    return W_hat


def sel_stride(K, sel_size):
    """Bytes per row of the separate selection bits."""
    return (K // sel_size + 7) // 8


def aaac_encode_sel(W, group_size, sel_size, fmt, importance, tables_bf16, codes=None, scales=None,
                    sel_bits=None, stream=None):
    """-> (codes, scales, sel_bits uint8 [N, ceil(K/sel_size/8)] or None when sel_size == group_size)."""
    assert W.dtype == torch.bfloat16 and W.dim() == 2 and W.stride(1) == 1
    N, K = W.shape
    if codes is None:
        codes = torch.empty((N, K // 2), dtype=torch.uint8, device=W.device)
    if scales is None:
        scales = torch.empty((N, K // group_size), dtype=_scale_dtype(fmt), device=W.device)
    if sel_bits is None and sel_size < group_size:
        sel_bits = torch.empty((N, sel_stride(K, sel_size)), dtype=torch.uint8, device=W.device)
    ldw = W.stride(0) if N > 1 else max(W.stride(0), K)
    stride = 0 if sel_bits is None else (sel_bits.stride(0) if N > 1 else max(sel_bits.stride(0), sel_bits.shape[1]))
    _check(library().aaac_encode_sel(_dp(W), N, K, ldw, group_size, sel_size, fmt, _dp(importance),
                                     _dp(tables_bf16), _dp(codes), _dp(scales), _dp(sel_bits), stride,
                                     _stream(stream)), "aaac_encode_sel")
    return codes, scales, sel_bits


def aaac_dequant_sel(codes, scales, sel_bits, tables_bf16, group_size, sel_size, fmt, W_hat=None, stream=None):
    """-> W_hat bf16 [N, K]."""
    N, K = codes.shape[0], codes.shape[1] * 2
    if W_hat is None:
        W_hat = torch.empty((N, K), dtype=torch.bfloat16, device=codes.device)
    ldo = W_hat.stride(0) if N > 1 else max(W_hat.stride(0), K)
    stride = 0 if sel_bits is None else (sel_bits.stride(0) if N > 1 else max(sel_bits.stride(0), sel_bits.shape[1]))
    _check(library().aaac_dequant_sel(_dp(codes), _dp(scales), _dp(sel_bits), stride, _dp(tables_bf16), N, K,
                                      group_size, sel_size, fmt, _dp(W_hat), ldo, _stream(stream)),
           "aaac_dequant_sel")
    return W_hat


def aaac_quantile_init_workspace(N, K, group_size, fmt):
    return library().aaac_quantile_init_workspace(N, K, group_size, fmt)


def aaac_quantile_init(W, group_size, fmt, grid=None, ws=None, stream=None):
    """Initial tables from quantiles of the normalised weights -> fp32 [32] on W's device."""
    assert W.dtype == torch.bfloat16 and W.dim() == 2 and W.stride(1) == 1
    N, K = W.shape
    if grid is None:
        grid = torch.empty(32, dtype=torch.float32, device=W.device)
    if ws is None:
        ws = _workspace(aaac_quantile_init_workspace(N, K, group_size, fmt), W.device)
    ldw = W.stride(0) if N > 1 else max(W.stride(0), K)
    _check(library().aaac_quantile_init(_dp(W), N, K, ldw, group_size, fmt, _dp(grid), _dp(ws), ws.numel(),
                                        _stream(stream)), "aaac_quantile_init")
    return grid


def aaac_gemv_w4a16(x, codes, scales, sel_bits, tables_bf16, group_size, sel_size, fmt, y=None, stream=None):
    """x bf16 [M, K] times the quantised layer -> y fp32 [M, N]."""
    assert x.dtype == torch.bfloat16 and x.dim() == 2 and x.stride(1) == 1
    M, K = x.shape
    N = codes.shape[0]
    if y is None:
        y = torch.empty((M, N), dtype=torch.float32, device=x.device)
    ldx = x.stride(0) if M > 1 else max(x.stride(0), K)
    ldy = y.stride(0) if M > 1 else max(y.stride(0), N)
    stride = 0 if sel_bits is None else (sel_bits.stride(0) if N > 1 else max(sel_bits.stride(0), sel_bits.shape[1]))
    _check(library().aaac_gemv_w4a16(_dp(x), M, ldx, _dp(codes), _dp(scales), _dp(sel_bits), stride,
                                     _dp(tables_bf16), N, K, group_size, sel_size, fmt, _dp(y), ldy,
                                     _stream(stream)), "aaac_gemv_w4a16")
    return y


def aaac_gemm_w4a16_workspace(M, K):
    return library().aaac_gemm_w4a16_workspace(M, K)


def aaac_gemm_w4a16(x, codes, scales, sel_bits, tables_bf16, group_size, sel_size, fmt, y=None, ws=None, stream=None):
    """x bf16 [M, K] times the quantised layer on the matrix cores (weights rounded to bf16) -> y fp32 [M, N]."""
    assert x.dtype == torch.bfloat16 and x.dim() == 2 and x.stride(1) == 1
    M, K = x.shape
    N = codes.shape[0]
    if y is None:
        y = torch.empty((M, N), dtype=torch.float32, device=x.device)
    if ws is None:
        ws = _workspace(aaac_gemm_w4a16_workspace(M, K), x.device)
    ldx = x.stride(0) if M > 1 else max(x.stride(0), K)
    ldy = y.stride(0) if M > 1 else max(y.stride(0), N)
    stride = 0 if sel_bits is None else (sel_bits.stride(0) if N > 1 else max(sel_bits.stride(0), sel_bits.shape[1]))
    _check(library().aaac_gemm_w4a16(_dp(x), M, ldx, _dp(codes), _dp(scales), _dp(sel_bits), stride,
                                     _dp(tables_bf16), N, K, group_size, sel_size, fmt, _dp(y), ldy, _dp(ws),
                                     ws.numel(), _stream(stream)), "aaac_gemm_w4a16")
    return y
