"""The selection entry point that allocates nothing (its workspace is an array inside the
library's device image), called through the C ABI with raw pointers and compared with
cs_heavy_hitters_topk on the same estimates: index for index and value for value, since the
selection is integer work.  Two calls in a row on the one shared array, the second on a
smaller input, then a third with other sizes; the file is collected last so that a failure here
hides no other test."""
import ctypes

import numpy as np
import pytest
import torch

import paper_1903_04488_amd as cs

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _estimates(d, seed):
    gen = torch.Generator(device=DEV)
    gen.manual_seed(seed)
    est = torch.empty(d, dtype=torch.float32, device=DEV)
    est.normal_(0.0, 0.01, generator=gen)
    # ties at the threshold, signed zeros and a few large values
    est[::97] = 0.0125
    est[5::1013] = -0.0125
    est[3::50_021] = -3.0
    est[min(7, d - 1)] = -0.0
    return est


def _reference(est, k):
    ws = torch.empty(cs.cs_topk_workspace_bytes(est.numel(), k), dtype=torch.uint8, device=DEV)
    idx = torch.empty(k, dtype=torch.int64, device=DEV)
    val = torch.empty(k, dtype=torch.float32, device=DEV)
    cs.cs_heavy_hitters_topk(est, k, idx, val, ws)
    return idx, val


def _static_raw(lib, est, k, idx, val):
    """straight through the C ABI: pointers and sizes, the current stream"""
    stream = ctypes.c_void_p(torch.cuda.current_stream(est.device).cuda_stream)
    return lib.cs_heavy_hitters_topk_static(
        ctypes.c_void_p(est.data_ptr()), ctypes.c_int64(est.numel()), ctypes.c_int64(k),
        ctypes.c_void_p(idx.data_ptr()), ctypes.c_void_p(val.data_ptr() if val is not None else 0),
        stream)


def test_static_scratch_topk_matches_workspace_topk_on_calls_in_a_row():
    lib = cs.load_library()
    # first a large input (several tiles per block and a ragged tail), then a smaller one, then
    # k close to d: the array keeps the previous call's histograms and per-block counts
    for d, k, seed in [(3_000_017, 4_000, 1), (70_001, 250, 2), (4_099, 4_095, 3), (1, 1, 4)]:
        est = _estimates(d, seed)
        want_idx, want_val = _reference(est, k)
        idx = torch.full((k,), -1, dtype=torch.int64, device=DEV)
        val = torch.full((k,), float("nan"), dtype=torch.float32, device=DEV)
        assert _static_raw(lib, est, k, idx, val) == 0
        torch.cuda.synchronize()
        np.testing.assert_array_equal(idx.cpu().numpy(), want_idx.cpu().numpy())
        np.testing.assert_array_equal(val.cpu().numpy().view(np.uint32),
                                      want_val.cpu().numpy().view(np.uint32))
    # through the binding, without values
    est = _estimates(500_003, 5)
    want_idx, _ = _reference(est, 1_000)
    idx = torch.empty(1_000, dtype=torch.int64, device=DEV)
    cs.cs_heavy_hitters_topk_static(est, 1_000, idx, None)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(idx.cpu().numpy(), want_idx.cpu().numpy())


def test_static_scratch_topk_allocates_nothing_and_rejects_bad_sizes():
    lib = cs.load_library()
    est = _estimates(200_003, 6)
    idx = torch.empty(100, dtype=torch.int64, device=DEV)
    val = torch.empty(100, dtype=torch.float32, device=DEV)
    assert _static_raw(lib, est, 100, idx, val) == 0          # first call on this device: set-up
    torch.cuda.synchronize()
    free_before, _ = torch.cuda.mem_get_info()
    for _ in range(3):
        assert _static_raw(lib, est, 100, idx, val) == 0
    torch.cuda.synchronize()
    free_after, _ = torch.cuda.mem_get_info()
    assert free_after == free_before
    # limits and argument errors come back as status codes, nothing is launched
    stream = ctypes.c_void_p(0)
    too_big = ctypes.c_int64((1 << 32) + 1)
    assert lib.cs_heavy_hitters_topk_static(ctypes.c_void_p(est.data_ptr()), too_big, ctypes.c_int64(5),
                                            ctypes.c_void_p(idx.data_ptr()), None, stream) == -4
    assert "limit" in cs.cs_status_string(-4)
    assert _static_raw(lib, est, 0, idx, val) == -1
    assert _static_raw(lib, est, est.numel() + 1, idx, val) == -1
    assert lib.cs_heavy_hitters_topk_static(None, ctypes.c_int64(10), ctypes.c_int64(5),
                                            ctypes.c_void_p(idx.data_ptr()), None, stream) == -1
