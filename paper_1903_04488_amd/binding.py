"""ctypes binding of libcsketch.so: same names as include/csketch.h, argument marshalling only.

Tensors must live on a HIP device ("cuda" in torch), be contiguous and have the dtype the C
signature states; the binding checks that and the shapes, passes `tensor.data_ptr()` and the
current torch stream, and raises CsError on a non-zero status.  Nothing is computed here.
"""
from __future__ import annotations

import ctypes
import os

import torch

CS_MAX_R = 16
_PKG = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_PKG, "libcsketch.so")
_lib = None


class CsError(RuntimeError):
    pass


class CsRowPlan(ctypes.Structure):
    _fields_ = [("D", ctypes.c_uint64), ("AD", ctypes.c_uint64), ("ADs", ctypes.c_uint64),
                ("Dw", ctypes.c_uint64), ("ADw", ctypes.c_uint64), ("ADws", ctypes.c_uint64),
                ("lanes", ctypes.c_int32), ("scan_steps", ctypes.c_int32)]


CS_MAX_VISITS = 512
CS_FLAG_NO_VISIT_LIST = 1
CS_FLAG_NO_LDS_TABLE = 2


class CsVisitPlan(ctypes.Structure):
    _fields_ = [("K", ctypes.c_uint32), ("ncell", ctypes.c_uint32),
                ("cover", ctypes.c_uint64), ("gmax", ctypes.c_uint64),
                ("cost", ctypes.c_uint64), ("cost_walk", ctypes.c_uint64),
                ("gap", ctypes.c_uint64 * 4),
                ("A", ctypes.c_uint64 * 4), ("As", ctypes.c_uint64 * 4),
                ("code", ctypes.c_uint32 * (CS_MAX_VISITS // 16))]

    def gaps(self):
        """Gap of every visit, in order (decoded from the 2-bit codes)."""
        return [int(self.gap[(self.code[k // 16] >> (2 * (k % 16))) & 3]) for k in range(self.K)]


CS_ANYC_MAX_VISITS = 144


class CsAnycPlan(ctypes.Structure):
    _fields_ = [("K", ctypes.c_uint32), ("omega", ctypes.c_uint32),
                ("cover", ctypes.c_uint64), ("gmax", ctypes.c_uint64),
                ("cost", ctypes.c_uint64), ("cost_direct", ctypes.c_uint64),
                ("gap", ctypes.c_uint32 * CS_ANYC_MAX_VISITS)]

    def gaps(self):
        return [int(self.gap[k]) for k in range(self.K)]


class CsParams(ctypes.Structure):
    _fields_ = [("r", ctypes.c_uint32), ("c", ctypes.c_uint32),
                ("c_pow2", ctypes.c_uint32), ("flags", ctypes.c_uint32),
                ("seed", ctypes.c_uint64),
                ("a", ctypes.c_uint64 * CS_MAX_R), ("b", ctypes.c_uint64 * CS_MAX_R),
                ("as_", ctypes.c_uint64 * CS_MAX_R), ("bs", ctypes.c_uint64 * CS_MAX_R),
                ("plan", CsRowPlan * CS_MAX_R),
                ("visit", CsVisitPlan * CS_MAX_R),
                ("anyc", CsAnycPlan * CS_MAX_R)]


def library_path() -> str:
    return _LIB_PATH


_SIGNATURES = {
    "cs_params_init": [ctypes.POINTER(CsParams), ctypes.c_uint32, ctypes.c_uint32,
                       ctypes.c_uint64, ctypes.c_int64],
    "cs_hash_debug": [ctypes.POINTER(CsParams), ctypes.c_void_p, ctypes.c_int64,
                      ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p],
    "cs_hash_debug_range": [ctypes.POINTER(CsParams), ctypes.c_int64, ctypes.c_int64,
                            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p],
    "cs_sketch_zero": [ctypes.POINTER(CsParams), ctypes.c_void_p, ctypes.c_void_p],
    "cs_sketch_accumulate": [ctypes.POINTER(CsParams), ctypes.c_void_p, ctypes.c_void_p,
                             ctypes.c_int64, ctypes.c_int64, ctypes.c_float, ctypes.c_void_p],
    "cs_sketch_accumulate_batch": [ctypes.POINTER(CsParams), ctypes.POINTER(ctypes.c_void_p),
                                   ctypes.POINTER(ctypes.c_void_p), ctypes.c_int32,
                                   ctypes.c_int64, ctypes.c_int64, ctypes.c_float,
                                   ctypes.c_void_p],
    "cs_bundle_floats": [ctypes.POINTER(CsParams), ctypes.c_int32, ctypes.POINTER(ctypes.c_int64)],
    "cs_bundle_zero": [ctypes.POINTER(CsParams), ctypes.c_void_p, ctypes.c_int32, ctypes.c_void_p],
    "cs_sketch_accumulate_bundle": [ctypes.POINTER(CsParams), ctypes.c_void_p, ctypes.c_int32,
                                    ctypes.POINTER(ctypes.c_void_p), ctypes.c_int64,
                                    ctypes.c_int64, ctypes.c_float, ctypes.c_void_p],
    "cs_sketch_accumulate_sum": [ctypes.POINTER(CsParams), ctypes.c_void_p, ctypes.c_int32,
                                 ctypes.POINTER(ctypes.c_void_p), ctypes.c_int64,
                                 ctypes.c_int64, ctypes.c_float, ctypes.c_void_p],
    "cs_bundle_merge": [ctypes.POINTER(CsParams), ctypes.c_void_p, ctypes.c_float,
                        ctypes.c_void_p, ctypes.c_int32, ctypes.c_float, ctypes.c_void_p],
    "cs_sketch_accumulate_sparse": [ctypes.POINTER(CsParams), ctypes.c_void_p, ctypes.c_void_p,
                                    ctypes.c_void_p, ctypes.c_int64, ctypes.c_float,
                                    ctypes.c_void_p],
    "cs_sketch_merge": [ctypes.POINTER(CsParams), ctypes.c_void_p, ctypes.c_float,
                        ctypes.POINTER(ctypes.c_void_p), ctypes.c_int32, ctypes.c_float,
                        ctypes.c_void_p],
    "cs_sketch_count_nonfinite": [ctypes.POINTER(CsParams), ctypes.c_void_p, ctypes.c_void_p,
                                  ctypes.c_void_p],
    "cs_fixed_accumulate": [ctypes.POINTER(CsParams), ctypes.c_void_p, ctypes.c_void_p,
                            ctypes.c_int64, ctypes.c_int64, ctypes.c_float, ctypes.c_int32,
                            ctypes.c_void_p, ctypes.c_void_p],
    "cs_fixed_accumulate_sparse": [ctypes.POINTER(CsParams), ctypes.c_void_p, ctypes.c_void_p,
                                   ctypes.c_void_p, ctypes.c_int64, ctypes.c_float,
                                   ctypes.c_int32, ctypes.c_void_p, ctypes.c_void_p],
    "cs_fixed_to_float": [ctypes.POINTER(CsParams), ctypes.c_void_p, ctypes.c_int32,
                          ctypes.c_float, ctypes.c_void_p, ctypes.c_void_p],
    "cs_sketch_axpby": [ctypes.POINTER(CsParams), ctypes.c_void_p, ctypes.c_float,
                        ctypes.c_void_p, ctypes.c_float, ctypes.c_void_p],
    "cs_sketch_momentum": [ctypes.POINTER(CsParams), ctypes.c_void_p, ctypes.c_void_p,
                           ctypes.c_void_p, ctypes.c_float, ctypes.c_void_p],
    "cs_estimate_workspace_bytes": [ctypes.POINTER(CsParams), ctypes.c_int64,
                                    ctypes.POINTER(ctypes.c_size_t)],
    "cs_sketch_estimate": [ctypes.POINTER(CsParams), ctypes.c_void_p, ctypes.c_int64,
                           ctypes.c_int64, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                           ctypes.c_size_t, ctypes.c_void_p],
    "cs_sketch_estimate_sparse": [ctypes.POINTER(CsParams), ctypes.c_void_p, ctypes.c_void_p,
                                  ctypes.c_int64, ctypes.c_void_p, ctypes.c_void_p],
    "cs_topk_workspace_bytes": [ctypes.c_int64, ctypes.c_int64, ctypes.POINTER(ctypes.c_size_t)],
    "cs_heavy_hitters_topk": [ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64, ctypes.c_void_p,
                              ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t,
                              ctypes.c_void_p],
    "cs_heavy_hitters_topk_static": [ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64,
                                     ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p],
    "cs_select_exact_topk": [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64,
                             ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t,
                             ctypes.c_void_p],
    "cs_bundle_update_launches": [ctypes.POINTER(CsParams), ctypes.c_int32, ctypes.c_int64,
                                  ctypes.POINTER(ctypes.c_int32)],
    "cs_quantize16": [ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p, ctypes.c_int32, ctypes.c_void_p],
    "cs_dequantize16": [ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p, ctypes.c_int32, ctypes.c_void_p],
    "cs_bundle_merge16": [ctypes.POINTER(CsParams), ctypes.c_void_p, ctypes.c_float, ctypes.c_void_p,
                          ctypes.c_int32, ctypes.c_float, ctypes.c_int32, ctypes.c_void_p],
    "cs_sketch_l2sq": [ctypes.POINTER(CsParams), ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p],
    "cs_heavymix_select": [ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64, ctypes.c_void_p,
                           ctypes.c_uint64, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                           ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p],
    "cs_gather_exact": [ctypes.POINTER(ctypes.c_void_p), ctypes.c_int32, ctypes.c_void_p,
                        ctypes.c_int64, ctypes.c_float, ctypes.c_void_p, ctypes.c_void_p],
    "cs_dense_momentum": [ctypes.POINTER(ctypes.c_void_p), ctypes.POINTER(ctypes.c_void_p),
                          ctypes.POINTER(ctypes.c_void_p), ctypes.c_int32, ctypes.c_int64,
                          ctypes.c_float, ctypes.c_void_p],
    "cs_probe_stream_read": [ctypes.POINTER(ctypes.c_void_p), ctypes.c_int32, ctypes.c_int64,
                             ctypes.c_void_p, ctypes.c_void_p],
    "cs_dense_mask": [ctypes.POINTER(ctypes.c_void_p), ctypes.POINTER(ctypes.c_void_p),
                      ctypes.c_int32, ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p],
    "cs_sketch_feedback": [ctypes.POINTER(CsParams), ctypes.c_void_p, ctypes.c_void_p,
                           ctypes.c_int64, ctypes.c_void_p, ctypes.c_void_p],
}


def load_library():
    """Loads libcsketch.so built by paper_1903_04488_amd/build.py; fails loudly if absent."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise CsError(f"{_LIB_PATH} is not built: run `python -c 'import __graft_entry__ as g; "
                      "g.build()'` (there is no fallback path)")
    lib = ctypes.CDLL(_LIB_PATH)
    for name, argtypes in _SIGNATURES.items():
        fn = getattr(lib, name)
        fn.argtypes = argtypes
        fn.restype = ctypes.c_int
    lib.cs_status_string.argtypes = [ctypes.c_int]
    lib.cs_status_string.restype = ctypes.c_char_p
    _lib = lib
    return lib


def exported_symbols():
    return list(_SIGNATURES) + ["cs_status_string"]


def cs_status_string(status: int) -> str:
    return load_library().cs_status_string(int(status)).decode()


def _check(status: int, what: str):
    if status != 0:
        raise CsError(f"{what}: {cs_status_string(status)} ({status})")


def _dev(t: torch.Tensor, dtype, name: str, numel: int | None = None):
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise CsError(f"{name} must be a tensor on the GPU")
    if t.dtype != dtype:
        raise CsError(f"{name} must have dtype {dtype}, got {t.dtype}")
    if not t.is_contiguous():
        raise CsError(f"{name} must be contiguous")
    if numel is not None and t.numel() != numel:
        raise CsError(f"{name} must have {numel} elements, got {t.numel()}")
    return ctypes.c_void_p(t.data_ptr())


def _stream(t: torch.Tensor):
    return ctypes.c_void_p(torch.cuda.current_stream(t.device).cuda_stream)


def _ptr_array(tensors, dtype, name, numel=None):
    arr = (ctypes.c_void_p * len(tensors))()
    for w, t in enumerate(tensors):
        arr[w] = _dev(t, dtype, f"{name}[{w}]", numel).value
    return arr


def _cells(p: CsParams) -> int:
    return int(p.r) * int(p.c)


# ------------------------------------------------------------------------------------------
def cs_params_init(r: int, c: int, seed: int, d_hint: int = 0) -> CsParams:
    p = CsParams()
    _check(load_library().cs_params_init(ctypes.byref(p), r, c, seed, d_hint), "cs_params_init")
    return p


def cs_hash_debug(p, idx, bucket, sign):
    n = idx.numel()
    _check(load_library().cs_hash_debug(
        ctypes.byref(p), _dev(idx, torch.int64, "idx"), n,
        _dev(bucket, torch.int32, "bucket", p.r * n), _dev(sign, torch.int8, "sign", p.r * n),
        _stream(idx)), "cs_hash_debug")


def cs_hash_debug_range(p, i0, n, bucket, sign):
    _check(load_library().cs_hash_debug_range(
        ctypes.byref(p), i0, n,
        _dev(bucket, torch.int32, "bucket", p.r * n), _dev(sign, torch.int8, "sign", p.r * n),
        _stream(bucket)), "cs_hash_debug_range")


def cs_sketch_zero(p, S):
    _check(load_library().cs_sketch_zero(
        ctypes.byref(p), _dev(S, torch.float32, "S", _cells(p)), _stream(S)), "cs_sketch_zero")


def cs_sketch_accumulate(p, S, g, i0: int = 0, scale: float = 1.0):
    _check(load_library().cs_sketch_accumulate(
        ctypes.byref(p), _dev(S, torch.float32, "S", _cells(p)), _dev(g, torch.float32, "g"),
        g.numel(), i0, scale, _stream(S)), "cs_sketch_accumulate")


def cs_sketch_accumulate_batch(p, S_w, g_w, i0: int = 0, scale: float = 1.0):
    if len(S_w) != len(g_w) or len(S_w) == 0:
        raise CsError("S_w and g_w must be non-empty lists of equal length")
    d = g_w[0].numel()
    _check(load_library().cs_sketch_accumulate_batch(
        ctypes.byref(p), _ptr_array(S_w, torch.float32, "S_w", _cells(p)),
        _ptr_array(g_w, torch.float32, "g_w", d), len(S_w), d, i0, scale, _stream(S_w[0])),
        "cs_sketch_accumulate_batch")


CS_BUNDLE_GROUP = 8


def cs_bundle_floats(p, W: int) -> int:
    out = ctypes.c_int64(0)
    _check(load_library().cs_bundle_floats(ctypes.byref(p), W, ctypes.byref(out)),
           "cs_bundle_floats")
    return int(out.value)


def cs_bundle_zero(p, T, W: int):
    _check(load_library().cs_bundle_zero(
        ctypes.byref(p), _dev(T, torch.float32, "T", cs_bundle_floats(p, W)), W, _stream(T)),
        "cs_bundle_zero")


def cs_sketch_accumulate_bundle(p, T, g_w, i0: int = 0, scale: float = 1.0):
    W = len(g_w)
    if W == 0:
        raise CsError("g_w must be a non-empty list")
    d = g_w[0].numel()
    _check(load_library().cs_sketch_accumulate_bundle(
        ctypes.byref(p), _dev(T, torch.float32, "T", cs_bundle_floats(p, W)), W,
        _ptr_array(g_w, torch.float32, "g_w", d), d, i0, scale, _stream(T)),
        "cs_sketch_accumulate_bundle")


def cs_sketch_accumulate_sum(p, S, g_w, i0: int = 0, scale: float = 1.0):
    W = len(g_w)
    if W == 0:
        raise CsError("g_w must be a non-empty list")
    d = g_w[0].numel()
    _check(load_library().cs_sketch_accumulate_sum(
        ctypes.byref(p), _dev(S, torch.float32, "S", _cells(p)), W,
        _ptr_array(g_w, torch.float32, "g_w", d), d, i0, scale, _stream(S)),
        "cs_sketch_accumulate_sum")


def cs_bundle_update_launches(p, W: int, d: int) -> int:
    n = ctypes.c_int32(0)
    _check(load_library().cs_bundle_update_launches(ctypes.byref(p), W, d, ctypes.byref(n)),
           "cs_bundle_update_launches")
    return int(n.value)


def cs_bundle_merge(p, dst, T, W: int, alpha: float = 1.0, beta: float = 0.0):
    _check(load_library().cs_bundle_merge(
        ctypes.byref(p), _dev(dst, torch.float32, "dst", _cells(p)), beta,
        _dev(T, torch.float32, "T", cs_bundle_floats(p, W)), W, alpha, _stream(dst)),
        "cs_bundle_merge")


def cs_sketch_accumulate_sparse(p, S, idx, val, scale: float = 1.0):
    n = idx.numel()
    _check(load_library().cs_sketch_accumulate_sparse(
        ctypes.byref(p), _dev(S, torch.float32, "S", _cells(p)),
        _dev(idx, torch.int64, "idx"), _dev(val, torch.float32, "val", n), n, scale,
        _stream(S)), "cs_sketch_accumulate_sparse")


def cs_sketch_merge(p, dst, src, alpha: float = 1.0, beta: float = 0.0):
    _check(load_library().cs_sketch_merge(
        ctypes.byref(p), _dev(dst, torch.float32, "dst", _cells(p)), beta,
        _ptr_array(src, torch.float32, "src", _cells(p)), len(src), alpha, _stream(dst)),
        "cs_sketch_merge")


def cs_sketch_axpby(p, y, a: float, x, b: float):
    _check(load_library().cs_sketch_axpby(
        ctypes.byref(p), _dev(y, torch.float32, "y", _cells(p)), a,
        _dev(x, torch.float32, "x", _cells(p)), b, _stream(y)), "cs_sketch_axpby")


def cs_sketch_momentum(p, S_u, S_v, S_t, rho: float):
    _check(load_library().cs_sketch_momentum(
        ctypes.byref(p), _dev(S_u, torch.float32, "S_u", _cells(p)),
        _dev(S_v, torch.float32, "S_v", _cells(p)), _dev(S_t, torch.float32, "S_t", _cells(p)),
        rho, _stream(S_u)), "cs_sketch_momentum")


def cs_sketch_count_nonfinite(p, S, count):
    _check(load_library().cs_sketch_count_nonfinite(
        ctypes.byref(p), _dev(S, torch.float32, "S", _cells(p)), _dev(count, torch.int64, "count", 1),
        _stream(S)), "cs_sketch_count_nonfinite")


CS_FIXED_MAX_FRAC_BITS = 62


def _dropped(dropped):
    if dropped is None:
        return ctypes.c_void_p(0)
    return _dev(dropped, torch.int64, "dropped", 1)


def cs_fixed_accumulate(p, acc, g, frac_bits: int, i0: int = 0, scale: float = 1.0, dropped=None):
    _check(load_library().cs_fixed_accumulate(
        ctypes.byref(p), _dev(acc, torch.int64, "acc", _cells(p)), _dev(g, torch.float32, "g"),
        g.numel(), i0, scale, frac_bits, _dropped(dropped), _stream(acc)), "cs_fixed_accumulate")


def cs_fixed_accumulate_sparse(p, acc, idx, val, frac_bits: int, scale: float = 1.0, dropped=None):
    n = idx.numel()
    _check(load_library().cs_fixed_accumulate_sparse(
        ctypes.byref(p), _dev(acc, torch.int64, "acc", _cells(p)), _dev(idx, torch.int64, "idx"),
        _dev(val, torch.float32, "val", n), n, scale, frac_bits, _dropped(dropped),
        _stream(acc)), "cs_fixed_accumulate_sparse")


def cs_fixed_to_float(p, acc, frac_bits: int, S, alpha: float = 1.0):
    _check(load_library().cs_fixed_to_float(
        ctypes.byref(p), _dev(acc, torch.int64, "acc", _cells(p)), frac_bits, alpha,
        _dev(S, torch.float32, "S", _cells(p)), _stream(acc)), "cs_fixed_to_float")


def cs_estimate_workspace_bytes(p, d: int) -> int:
    out = ctypes.c_size_t(0)
    _check(load_library().cs_estimate_workspace_bytes(ctypes.byref(p), d, ctypes.byref(out)),
           "cs_estimate_workspace_bytes")
    return int(out.value)


CS_TOPK_HIST_BINS = 2048


def _hist(hist):
    if hist is None:
        return ctypes.c_void_p(0)
    return _dev(hist, torch.int64, "hist", CS_TOPK_HIST_BINS)


def cs_sketch_estimate(p, S, est, i0: int = 0, workspace=None, hist=None):
    d = est.numel()
    ws_ptr, ws_bytes = ctypes.c_void_p(0), 0
    if workspace is not None:
        ws_ptr = _dev(workspace, torch.uint8, "workspace")
        ws_bytes = workspace.numel()
    _check(load_library().cs_sketch_estimate(
        ctypes.byref(p), _dev(S, torch.float32, "S", _cells(p)), d, i0,
        _dev(est, torch.float32, "est"), _hist(hist), ws_ptr, ws_bytes, _stream(S)),
        "cs_sketch_estimate")


def cs_sketch_estimate_sparse(p, S, idx, out):
    n = idx.numel()
    _check(load_library().cs_sketch_estimate_sparse(
        ctypes.byref(p), _dev(S, torch.float32, "S", _cells(p)), _dev(idx, torch.int64, "idx"),
        n, _dev(out, torch.float32, "out", n), _stream(S)), "cs_sketch_estimate_sparse")


def cs_topk_workspace_bytes(d: int, k: int) -> int:
    out = ctypes.c_size_t(0)
    _check(load_library().cs_topk_workspace_bytes(d, k, ctypes.byref(out)),
           "cs_topk_workspace_bytes")
    return int(out.value)


def cs_heavy_hitters_topk(est, k: int, idx_out, val_out, workspace, hist=None):
    d = est.numel()
    _check(load_library().cs_heavy_hitters_topk(
        _dev(est, torch.float32, "est"), d, k, _hist(hist), _dev(idx_out, torch.int64, "idx_out", k),
        _dev(val_out, torch.float32, "val_out", k) if val_out is not None else ctypes.c_void_p(0),
        _dev(workspace, torch.uint8, "workspace"), workspace.numel(), _stream(est)),
        "cs_heavy_hitters_topk")


def cs_heavy_hitters_topk_static(est, k: int, idx_out, val_out):
    d = est.numel()
    _check(load_library().cs_heavy_hitters_topk_static(
        _dev(est, torch.float32, "est"), d, k, _dev(idx_out, torch.int64, "idx_out", k),
        _dev(val_out, torch.float32, "val_out", k) if val_out is not None else ctypes.c_void_p(0),
        _stream(est)), "cs_heavy_hitters_topk_static")


def cs_select_exact_topk(cand, x, k: int, idx_out, val_out, workspace):
    n = cand.numel()
    _check(load_library().cs_select_exact_topk(
        _dev(cand, torch.int64, "cand"), _dev(x, torch.float32, "x", n), n, k,
        _dev(idx_out, torch.int64, "idx_out", k),
        _dev(val_out, torch.float32, "val_out", k) if val_out is not None else ctypes.c_void_p(0),
        _dev(workspace, torch.uint8, "workspace"), workspace.numel(), _stream(x)),
        "cs_select_exact_topk")


CS_FMT_BF16, CS_FMT_F16 = 0, 1


def cs_quantize16(x, out, fmt: int):
    """out: int16 tensor (torch has no uint16 arithmetic; the bit patterns are what matters)"""
    n = x.numel()
    _check(load_library().cs_quantize16(_dev(x, torch.float32, "x"), n,
                                        _dev(out, torch.int16, "out", n), fmt, _stream(x)),
           "cs_quantize16")


def cs_dequantize16(q, out, fmt: int):
    n = q.numel()
    _check(load_library().cs_dequantize16(_dev(q, torch.int16, "q"), n,
                                          _dev(out, torch.float32, "out", n), fmt, _stream(q)),
           "cs_dequantize16")


def cs_bundle_merge16(p, dst, T16, W: int, fmt: int, alpha: float = 1.0, beta: float = 0.0):
    _check(load_library().cs_bundle_merge16(
        ctypes.byref(p), _dev(dst, torch.float32, "dst", _cells(p)), beta,
        _dev(T16, torch.int16, "T16", cs_bundle_floats(p, W)), W, alpha, fmt, _stream(dst)),
        "cs_bundle_merge16")


def cs_sketch_l2sq(p, S, out):
    _check(load_library().cs_sketch_l2sq(
        ctypes.byref(p), _dev(S, torch.float32, "S", _cells(p)),
        _dev(out, torch.float64, "out", 1 + p.r), _stream(S)), "cs_sketch_l2sq")


def cs_heavymix_select(est, k: int, l2sq, rng_seed: int, idx_out, val_out, n_heavy, workspace):
    d = est.numel()
    null = ctypes.c_void_p(0)
    _check(load_library().cs_heavymix_select(
        _dev(est, torch.float32, "est"), d, k, _dev(l2sq, torch.float64, "l2sq"),
        rng_seed & 0xFFFFFFFFFFFFFFFF, _dev(idx_out, torch.int64, "idx_out", k),
        _dev(val_out, torch.float32, "val_out", k) if val_out is not None else null,
        _dev(n_heavy, torch.int64, "n_heavy", 1) if n_heavy is not None else null,
        _dev(workspace, torch.uint8, "workspace"), workspace.numel(), _stream(est)),
        "cs_heavymix_select")


def cs_gather_exact(vec, idx, out, alpha: float = 1.0):
    k = idx.numel()
    d = vec[0].numel()
    _check(load_library().cs_gather_exact(
        _ptr_array(vec, torch.float32, "vec", d), len(vec), _dev(idx, torch.int64, "idx"), k,
        alpha, _dev(out, torch.float32, "out", k), _stream(out)), "cs_gather_exact")


def cs_dense_momentum(u_w, v_w, g_w, rho: float):
    W, d = len(g_w), g_w[0].numel()
    if len(u_w) != W or len(v_w) != W:
        raise CsError("u_w, v_w and g_w must have one tensor per worker")
    _check(load_library().cs_dense_momentum(
        _ptr_array(u_w, torch.float32, "u_w", d), _ptr_array(v_w, torch.float32, "v_w", d),
        _ptr_array(g_w, torch.float32, "g_w", d), W, d, rho, _stream(g_w[0])), "cs_dense_momentum")


def cs_dense_mask(u_w, v_w, idx):
    W = len(u_w)
    if len(v_w) != W:
        raise CsError("u_w and v_w must have one tensor per worker")
    d = u_w[0].numel()
    _check(load_library().cs_dense_mask(
        _ptr_array(u_w, torch.float32, "u_w", d), _ptr_array(v_w, torch.float32, "v_w", d), W,
        _dev(idx, torch.int64, "idx"), idx.numel(), _stream(idx)), "cs_dense_mask")


def cs_probe_stream_read(x_w, out):
    d = x_w[0].numel()
    _check(load_library().cs_probe_stream_read(
        _ptr_array(x_w, torch.float32, "x_w", d), len(x_w), d, _dev(out, torch.float32, "out", 1),
        _stream(out)), "cs_probe_stream_read")


def cs_sketch_feedback(p, S, idx, val):
    k = idx.numel()
    _check(load_library().cs_sketch_feedback(
        ctypes.byref(p), _dev(S, torch.float32, "S", _cells(p)), _dev(idx, torch.int64, "idx"),
        k, _dev(val, torch.float32, "val", k), _stream(S)), "cs_sketch_feedback")
