"""aaac_act_stats_static (the entry point that allocates nothing: its partial sums live in an
array inside the library's device code) against aaac_act_stats, through the C ABI.  Both run the
same kernels with the same split of the tokens, so the importances must agree bit for bit; two
calls in a row, the second on a smaller input, share the array."""
import ctypes

import numpy as np
import pytest
import torch

import paper_2605_08692_amd as A
from paper_2605_08692_amd import inputs

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def raw_static(X, out):
    L = A.library()
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    return L.aaac_act_stats_static(ctypes.c_void_p(X.data_ptr()), X.shape[0], X.shape[1], X.stride(0),
                                   ctypes.c_void_p(out.data_ptr()), stream)


def raw_with_workspace(X, out):
    L = A.library()
    need = L.aaac_act_stats_workspace(X.shape[0], X.shape[1])
    ws = torch.empty(max(need, 256), dtype=torch.uint8, device=DEV)
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    rc = L.aaac_act_stats(ctypes.c_void_p(X.data_ptr()), X.shape[0], X.shape[1], X.stride(0),
                          ctypes.c_void_p(out.data_ptr()), ctypes.c_void_p(ws.data_ptr()), ws.numel(), stream)
    torch.cuda.synchronize()
    return rc


def test_two_calls_in_a_row_match_the_entry_point_with_a_workspace():
    big = inputs.make_activations(5000, 11008, ("gauss", 0.01, "u10_50"), 31, DEV)     # 3 column groups x 85 chunks
    small = inputs.make_activations(37, 520, ("gauss", 3, "x20"), 32, DEV)             # one ragged column group
    outs = [torch.full((X.shape[1],), -1.0, device=DEV) for X in (big, small)]
    torch.cuda.synchronize()
    # back to back on one stream, nothing in between: the second call reuses the array the first one filled
    assert raw_static(big, outs[0]) == 0
    assert raw_static(small, outs[1]) == 0
    torch.cuda.synchronize()
    for X, got in zip((big, small), outs):
        want = torch.empty(X.shape[1], device=DEV)
        assert raw_with_workspace(X, want) == 0
        assert torch.equal(got, want), (X.shape, (got != want).sum().item())
        assert (got > 0).all()
    # and once more in the other order, with an empty input in between (zeros, no kernel touches the array)
    again = [torch.empty_like(o) for o in outs]
    empty = torch.full((64,), -1.0, device=DEV)
    assert raw_static(small, again[1]) == 0
    assert raw_static(torch.empty((0, 64), dtype=torch.bfloat16, device=DEV), empty) == 0
    assert raw_static(big, again[0]) == 0
    torch.cuda.synchronize()
    assert torch.equal(again[0], outs[0]) and torch.equal(again[1], outs[1]) and (empty == 0).all()


def test_widest_input_the_array_holds_and_the_first_one_it_does_not():
    K = 1 << 20                                   # 256 column groups of 4096: exactly 8 MiB of partial sums
    X = torch.zeros((3, K), dtype=torch.bfloat16, device=DEV)
    X[:, ::4097] = 2.0
    out = torch.empty(K, device=DEV)
    assert raw_static(X, out) == 0
    torch.cuda.synchronize()
    want = torch.zeros(K, device=DEV)
    want[::4097] = 12.0
    assert torch.equal(out, want)
    wide = torch.zeros((1, K + 4096), dtype=torch.bfloat16, device=DEV)
    assert raw_static(wide, torch.empty(K + 4096, device=DEV)) == -4   # AAAC_ERR_WORKSPACE, nothing launched
