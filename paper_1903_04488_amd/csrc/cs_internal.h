// Declarations shared by the library's translation units (not part of the C ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "csketch.h"

namespace cs {

// What kernels receive by value: cs_params without the visit lists (kernel arguments are
// limited to 4 KB); a list travels separately to the one kernel that reads it.
struct KParams {
    uint32_t r, c, c_pow2, flags;
    uint64_t seed;
    uint64_t a[CS_MAX_R], b[CS_MAX_R];
    uint64_t as[CS_MAX_R], bs[CS_MAX_R];
    cs_row_plan plan[CS_MAX_R];
};
static_assert(offsetof(cs_params, visit) == sizeof(KParams), "KParams is the head of cs_params");
inline const KParams& kparams(const cs_params* p) { return *reinterpret_cast<const KParams*>(p); }

constexpr int kMaxBatch = 32;   // workers per launch of the batched update kernels

// kernel argument block: worker w's table and vector
struct LatticePtrs {
    float* S[kMaxBatch];
    const float* g[kMaxBatch];
};

// True when the stride-aligned traversal is used for vectors of length d with this sketch
// (power-of-two c, a stride found for every row, d large enough to fill tiles).
bool lattice_applies(const cs_params* p, int64_t d);

int launch_accumulate_lattice(const cs_params* p, const LatticePtrs& ptrs, int nw, int64_t d,
                              int64_t i0, float scale, hipStream_t stream);
// *hist_done = true when the kernels that wrote est also filled hist (see launch_estimate_walk)
int launch_estimate_lattice(const cs_params* p, const float* S, int64_t d, int64_t i0,
                            float* est, float* rows, uint64_t* hist, bool* hist_done,
                            hipStream_t stream);
// hist[b] = number of t < d with (bits(est[t]) & 0x7fffffff) >> 20 == b, b < 2048 (cs_topk.hip);
// the _zero form only clears the 2048 counters
int launch_magnitude_hist_zero(uint64_t* hist, hipStream_t stream);
int launch_magnitude_hist(const float* est, int64_t d, uint64_t* hist, hipStream_t stream);
int launch_hash_range_lattice(const cs_params* p, int64_t i0, int64_t n, uint32_t* bucket,
                              int8_t* sign, hipStream_t stream);

// Walk-order update of a worker bundle T = float[ceil(W/8)][r][c][8] (cs_walk.hip).
bool walk_applies(const cs_params* p, int64_t d);
// fold = true: T is one table float[r][c] and receives the sum over the W workers
// (all_rows_listed(p, d) must hold for launch_accumulate_walk, anyc_visits_apply for the other)
bool all_rows_listed(const cs_params* p, int64_t d);
int launch_accumulate_walk(const cs_params* p, float* T, int W, const float* const* g_w,
                           int64_t d, int64_t i0, float scale, bool fold, hipStream_t stream);
int count_accumulate_walk_launches(const cs_params* p, int W, int64_t d);
// the same along visit lists for column counts that are not a power of two
bool anyc_visits_apply(const cs_params* p, int64_t d);
bool anyc_visits_serve_query(const cs_params* p, int64_t d);
int launch_accumulate_anyc(const cs_params* p, float* T, int W, const float* const* g_w,
                           int64_t d, int64_t i0, float scale, bool fold, hipStream_t stream);
int count_accumulate_anyc_launches(const cs_params* p, int W);
int launch_estimate_anyc(const cs_params* p, const float* S, int64_t d, int64_t i0, float* est,
                         float* rows, hipStream_t stream);
int launch_estimate_walk(const cs_params* p, const float* S, int64_t d, int64_t i0,
                         float* est, float* rows, bool fuse_last, uint64_t* hist, hipStream_t stream);
int launch_bundle_zero(float* T, int64_t n, hipStream_t stream);
int launch_bundle_merge(float* dst, float beta, const float* T, int groups, float alpha,
                        int64_t cells, hipStream_t stream);
int launch_bundle_merge16(float* dst, float beta, const uint16_t* T16, int groups, float alpha,
                          int64_t cells, int fmt, hipStream_t stream);

}  // namespace cs
