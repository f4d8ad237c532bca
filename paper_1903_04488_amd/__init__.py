"""Count Sketch hot path of Sketched-SGD for AMD MI355X.

A thin ctypes binding over libcsketch.so (include/csketch.h).  The functions below have the
names of the C entry points and only marshal arguments: torch tensors supply device memory
and the current HIP stream, every step of the computation runs in the library's kernels.
There is no CPU fallback: without the built library, or without a GPU, calls fail.
"""
from .binding import (  # noqa: F401
    CS_MAX_R,
    CsError,
    CsParams,
    CS_BUNDLE_GROUP,
    cs_bundle_floats,
    cs_bundle_merge,
    cs_bundle_zero,
    cs_sketch_accumulate_bundle,
    cs_estimate_workspace_bytes,
    cs_gather_exact,
    cs_hash_debug,
    cs_hash_debug_range,
    cs_heavy_hitters_topk,
    cs_params_init,
    cs_select_exact_topk,
    cs_sketch_l2sq,
    cs_bundle_update_launches,
    cs_quantize16,
    cs_dequantize16,
    cs_bundle_merge16,
    CS_FMT_BF16,
    CS_FMT_F16,
    cs_dense_momentum,
    cs_dense_mask,
    cs_probe_stream_read,
    cs_heavymix_select,
    cs_sketch_accumulate,
    cs_sketch_accumulate_batch,
    cs_sketch_accumulate_sparse,
    cs_sketch_axpby,
    cs_sketch_estimate,
    cs_sketch_estimate_sparse,
    cs_sketch_feedback,
    cs_sketch_merge,
    cs_sketch_momentum,
    cs_sketch_zero,
    cs_status_string,
    cs_topk_workspace_bytes,
    library_path,
    load_library,
)
