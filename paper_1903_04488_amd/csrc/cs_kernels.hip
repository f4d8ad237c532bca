// Kernels and C ABI of the Count Sketch hot path (gfx950).  See include/csketch.h for what
// every entry point computes and which passage of the paper defines it.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "cs_device.h"
#include "cs_internal.h"
#include "csketch.h"
#include "csketch_probe.h"

namespace cs {

// ---------------------------------------------------------------------------------------
// launch helpers
// ---------------------------------------------------------------------------------------
inline hipStream_t as_stream(void* s) { return reinterpret_cast<hipStream_t>(s); }

inline int launch_status() { return hipGetLastError() == hipSuccess ? CS_OK : CS_EHIP; }

inline bool params_ok(const cs_params* p) {
    return p && p->r >= 1 && p->r <= CS_MAX_R && (p->r & 1u) && p->c >= 1 && p->c <= (1u << 31);
}

// number of workgroups for a grid-stride kernel over n items: enough to fill 256 CUs a few
// times over, never more than the items need.
inline unsigned grid_for(int64_t n, int per_block = kBlock, int max_blocks = 256 * 16) {
    int64_t b = (n + per_block - 1) / per_block;
    if (b < 1) b = 1;
    if (b > max_blocks) b = max_blocks;
    return static_cast<unsigned>(b);
}

// Dispatch on the (odd) row count and on "c is a power of two" so that the hash state of all
// rows lives in registers and loops over rows are unrolled.
#define CS_DISPATCH_R(p, CALL)                                                     \
    do {                                                                           \
        const bool pow2__ = (p)->c_pow2 != 0;                                      \
        switch ((p)->r) {                                                          \
            case 1: if (pow2__) { CALL(1, true); } else { CALL(1, false); } break;   \
            case 3: if (pow2__) { CALL(3, true); } else { CALL(3, false); } break;   \
            case 5: if (pow2__) { CALL(5, true); } else { CALL(5, false); } break;   \
            case 7: if (pow2__) { CALL(7, true); } else { CALL(7, false); } break;   \
            case 9: if (pow2__) { CALL(9, true); } else { CALL(9, false); } break;   \
            case 11: if (pow2__) { CALL(11, true); } else { CALL(11, false); } break; \
            case 13: if (pow2__) { CALL(13, true); } else { CALL(13, false); } break; \
            case 15: if (pow2__) { CALL(15, true); } else { CALL(15, false); } break; \
            default: return CS_EINVAL;                                             \
        }                                                                          \
    } while (0)

// ---------------------------------------------------------------------------------------
// hash parity hooks
// ---------------------------------------------------------------------------------------
template <bool POW2>
__global__ void __launch_bounds__(kBlock)
k_hash_list(KParams p, const int64_t* __restrict__ idx, int64_t n,
            uint32_t* __restrict__ bucket, int8_t* __restrict__ sign) {
    const int64_t stride = static_cast<int64_t>(gridDim.x) * kBlock;
    const Columns col = columns_of<POW2>(p.c);
    for (int64_t t = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x; t < n; t += stride) {
        const uint64_t i = static_cast<uint64_t>(idx[t]);
        for (uint32_t j = 0; j < p.r; ++j) {
            const uint64_t yb = hash_state(p.a[j], p.b[j], i);
            const uint64_t ys = hash_state(p.as[j], p.bs[j], i);
            bucket[static_cast<size_t>(j) * n + t] = bucket_of<POW2>(yb, col);
            sign[static_cast<size_t>(j) * n + t] = sign_flip_of(ys) ? -1 : 1;
        }
    }
}

// Streaming hash state of all R rows for one thread: start at coordinate `first`, then step
// by `stride` coordinates at a time.
template <int R>
struct RowStates {
    uint64_t yb[R], ys[R];    // y-form states of the bucket and sign hashes
    uint64_t Ab[R], As[R];    // (a_j * stride) mod p, (a'_j * stride) mod p

    __device__ __forceinline__ void init(const KParams& p, uint64_t first, uint64_t stride) {
#pragma unroll
        for (int j = 0; j < R; ++j) {
            yb[j] = hash_state(p.a[j], p.b[j], first);
            ys[j] = hash_state(p.as[j], p.bs[j], first);
            Ab[j] = mulmod_p(p.a[j], stride);
            As[j] = mulmod_p(p.as[j], stride);
        }
    }
    __device__ __forceinline__ void advance() {
#pragma unroll
        for (int j = 0; j < R; ++j) {
            yb[j] = hash_advance(yb[j], Ab[j]);
            ys[j] = hash_advance(ys[j], As[j]);
        }
    }
};

template <int R, bool POW2>
__global__ void __launch_bounds__(kBlock)
k_hash_range(KParams p, int64_t i0, int64_t n, uint32_t* __restrict__ bucket,
             int8_t* __restrict__ sign) {
    const int64_t stride = static_cast<int64_t>(gridDim.x) * kBlock;
    const Columns col = columns_of<POW2>(p.c);
    int64_t t = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x;
    if (t >= n) return;
    RowStates<R> st;
    st.init(p, static_cast<uint64_t>(i0 + t), static_cast<uint64_t>(stride));
    for (; t < n; t += stride) {
#pragma unroll
        for (int j = 0; j < R; ++j) {
            bucket[static_cast<size_t>(j) * n + t] = bucket_of<POW2>(st.yb[j], col);
            sign[static_cast<size_t>(j) * n + t] = sign_flip_of(st.ys[j]) ? -1 : 1;
        }
        st.advance();
    }
}

// ---------------------------------------------------------------------------------------
// sketch_accumulate: Alg. 4 update over a dense vector
// ---------------------------------------------------------------------------------------
using BatchPtrs = LatticePtrs;

// One thread per coordinate, grid-stride; the gradient is read coalesced, the r updates go
// out as fp32 atomics.  With NW > 1 the same hash values serve NW workers.
template <int R, bool POW2>
__global__ void __launch_bounds__(kBlock)
k_accumulate(KParams p, BatchPtrs ptrs, int nw, int64_t d, int64_t i0, float scale) {
    const int64_t stride = static_cast<int64_t>(gridDim.x) * kBlock;
    const Columns col = columns_of<POW2>(p.c);
    int64_t t = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x;
    if (t >= d) return;
    RowStates<R> st;
    st.init(p, static_cast<uint64_t>(i0 + t), static_cast<uint64_t>(stride));
    const uint32_t c = p.c;
    for (; t < d; t += stride) {
        uint32_t cell[R], flip[R];
#pragma unroll
        for (int j = 0; j < R; ++j) {
            cell[j] = static_cast<uint32_t>(j) * c + bucket_of<POW2>(st.yb[j], col);
            flip[j] = sign_flip_of(st.ys[j]);
        }
        for (int w = 0; w < nw; ++w) {
            const float v = scale * ptrs.g[w][t];
            float* S = ptrs.S[w];
#pragma unroll
            for (int j = 0; j < R; ++j)
                atomic_add_noret(S + cell[j], apply_sign(v, flip[j]));
        }
        st.advance();
    }
}

// Update of a worker bundle for any sketch shape.  Eight neighbouring lanes form a slot that
// takes one coordinate; lane q of the slot carries worker q of the group (blockIdx.y), so the
// slot's 8 updates of a cell T[group][j][b][0..8) are 32 contiguous bytes and leave the
// wavefront as ONE memory request per row instead of one per worker: the atomic unit, which
// bounds this kernel, sees W/8 times fewer requests than with one table per worker.  The 8
// lanes of a slot evaluate the same hashes; that work is hidden behind the atomics.
struct GroupedVectors {
    const float* g[kMaxBatch];   // worker w of the launch; group = w / 8
};

template <int R, bool POW2>
__global__ void __launch_bounds__(kBlock)
k_accumulate_cells(KParams p, GroupedVectors vec, int nw, float* __restrict__ T, int64_t d,
                   int64_t i0, float scale) {
    constexpr int kSlots = kBlock / CS_BUNDLE_GROUP;
    const int q = threadIdx.x % CS_BUNDLE_GROUP;
    const int w = blockIdx.y * CS_BUNDLE_GROUP + q;
    const int64_t stride = static_cast<int64_t>(gridDim.x) * kSlots;
    int64_t t = static_cast<int64_t>(blockIdx.x) * kSlots + threadIdx.x / CS_BUNDLE_GROUP;
    if (t >= d || w >= nw) return;
    const float* g = nullptr;
#pragma unroll
    for (int u = 0; u < CS_BUNDLE_GROUP; ++u)
        if (q == u) g = vec.g[blockIdx.y * CS_BUNDLE_GROUP + u];
    const uint32_t c = p.c;
    float* Tq = T + static_cast<size_t>(blockIdx.y) * R * c * CS_BUNDLE_GROUP + q;
    const Columns col = columns_of<POW2>(c);
    RowStates<R> st;
    st.init(p, static_cast<uint64_t>(i0 + t), static_cast<uint64_t>(stride));
    for (; t < d; t += stride) {
        const float v = scale * g[t];
#pragma unroll
        for (int j = 0; j < R; ++j) {
            const size_t cell = static_cast<size_t>(j) * c + bucket_of<POW2>(st.yb[j], col);
            atomic_add_noret(Tq + cell * CS_BUNDLE_GROUP, apply_sign(v, sign_flip_of(st.ys[j])));
        }
        st.advance();
    }
}

// The same update when one group's whole table fits in LDS (R * c * 8 floats <= 64 KB): a
// workgroup adds into a private copy with LDS atomics and sends every non-zero cell to memory
// once at the end.  Only narrow tables gain.  Measured per coordinate and row: through memory
// max(10 / c, 0.05) ns (few columns are a hot spot for the memory-side atomic unit), through
// LDS 0.045 ns plus ~10 us per launch for clearing and sending the copy; beyond ~200 columns
// the memory path is as fast as LDS float atomics.
constexpr uint32_t kLdsCells = 2048;      // R * c at most: 64 KB of LDS for 8 workers
constexpr uint32_t kLdsColumns = 128;     // c at most

inline bool lds_table_applies(const cs_params* p, int64_t d) {
    return !(p->flags & CS_FLAG_NO_LDS_TABLE) && p->c <= kLdsColumns &&
           static_cast<uint64_t>(p->r) * p->c <= kLdsCells &&
           d >= static_cast<int64_t>(2048) * p->c / p->r;
}

template <int R, bool POW2>
__global__ void __launch_bounds__(kBlock)
k_accumulate_cells_lds(KParams p, GroupedVectors vec, int nw, float* __restrict__ T, int64_t d,
                       int64_t i0, float scale) {
    extern __shared__ float part[];       // [R][c][8]
    constexpr int kSlots = kBlock / CS_BUNDLE_GROUP;
    const uint32_t c = p.c;
    const int floats = static_cast<int>(R * c * CS_BUNDLE_GROUP);
    for (int x = threadIdx.x; x < floats; x += kBlock) part[x] = 0.0f;
    __syncthreads();
    const int q = threadIdx.x % CS_BUNDLE_GROUP;
    const int w = blockIdx.y * CS_BUNDLE_GROUP + q;
    const int64_t stride = static_cast<int64_t>(gridDim.x) * kSlots;
    int64_t t = static_cast<int64_t>(blockIdx.x) * kSlots + threadIdx.x / CS_BUNDLE_GROUP;
    if (t < d && w < nw) {
        const float* g = nullptr;
#pragma unroll
        for (int u = 0; u < CS_BUNDLE_GROUP; ++u)
            if (q == u) g = vec.g[blockIdx.y * CS_BUNDLE_GROUP + u];
        const Columns col = columns_of<POW2>(c);
        RowStates<R> st;
        st.init(p, static_cast<uint64_t>(i0 + t), static_cast<uint64_t>(stride));
        for (; t < d; t += stride) {
            const float v = scale * g[t];
#pragma unroll
            for (int j = 0; j < R; ++j) {
                const uint32_t cell = static_cast<uint32_t>(j) * c + bucket_of<POW2>(st.yb[j], col);
                __hip_atomic_fetch_add(part + cell * CS_BUNDLE_GROUP + q,
                                       apply_sign(v, sign_flip_of(st.ys[j])), __ATOMIC_RELAXED,
                                       __HIP_MEMORY_SCOPE_WORKGROUP);
            }
            st.advance();
        }
    }
    __syncthreads();
    float* Tg = T + static_cast<size_t>(blockIdx.y) * floats;
    for (int x = threadIdx.x; x < floats; x += kBlock) {
        const float v = part[x];
        if (v != 0.0f) atomic_add_noret(Tg + x, v);     // NaN compares unequal: it is sent
    }
}

template <bool POW2>
__global__ void __launch_bounds__(kBlock)
k_accumulate_sparse(KParams p, float* __restrict__ S, const int64_t* __restrict__ idx,
                    const float* __restrict__ val, int64_t n, float scale) {
    const int64_t stride = static_cast<int64_t>(gridDim.x) * kBlock;
    const Columns col = columns_of<POW2>(p.c);
    for (int64_t t = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x; t < n; t += stride) {
        const uint64_t i = static_cast<uint64_t>(idx[t]);
        const float v = scale * val[t];
        for (uint32_t j = 0; j < p.r; ++j) {
            const uint64_t yb = hash_state(p.a[j], p.b[j], i);
            const uint64_t ys = hash_state(p.as[j], p.bs[j], i);
            atomic_add_noret(S + static_cast<size_t>(j) * p.c + bucket_of<POW2>(yb, col),
                             apply_sign(v, sign_flip_of(ys)));
        }
    }
}

// ---------------------------------------------------------------------------------------
// Alg. 4 update with order-independent sums: every contribution is rounded once to a multiple
// of 2^-F and added as a 64-bit integer, so a table does not depend on how the additions were
// scheduled (a debugging and checkpointing aid; the float kernels above are the product path)
// ---------------------------------------------------------------------------------------
// scale * g * 2^F as an integer, ties to even; the product of two binary32 numbers and a power
// of two is exact in binary64, so the one rounding is the one to an integer.  False (and no
// contribution) when the value is not finite or not below 2^62 in magnitude.
__device__ __forceinline__ bool fixed_of(float g, double scale_2F, long long* q) {
    const double x = static_cast<double>(g) * scale_2F;
    if (!(fabs(x) < 0x1p62)) return false;
    *q = __double2ll_rn(x);
    return true;
}

__device__ __forceinline__ void fixed_add(long long* acc, long long q, bool negative) {
    atomicAdd(reinterpret_cast<unsigned long long*>(acc),
              static_cast<unsigned long long>(negative ? -q : q));
}

// lanes that dropped a coordinate: one atomic per wavefront that saw any
__device__ __forceinline__ void count_dropped(unsigned long long* dropped, unsigned long long mine) {
    if (dropped == nullptr) return;
    for (int off = 32; off > 0; off >>= 1) mine += __shfl_xor(mine, off);
    if ((threadIdx.x & 63) == 0 && mine) atomicAdd(dropped, mine);
}

template <int R, bool POW2>
__global__ void __launch_bounds__(kBlock)
k_fixed_accumulate(KParams p, long long* __restrict__ acc, const float* __restrict__ g, int64_t d,
                   int64_t i0, double scale_2F, unsigned long long* __restrict__ dropped) {
    const int64_t stride = static_cast<int64_t>(gridDim.x) * kBlock;
    const Columns col = columns_of<POW2>(p.c);
    int64_t t = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x;
    unsigned long long bad = 0;
    if (t < d) {
        RowStates<R> st;
        st.init(p, static_cast<uint64_t>(i0 + t), static_cast<uint64_t>(stride));
        for (; t < d; t += stride) {
            long long q;
            if (fixed_of(g[t], scale_2F, &q)) {
#pragma unroll
                for (int j = 0; j < R; ++j)
                    fixed_add(acc + static_cast<size_t>(j) * p.c + bucket_of<POW2>(st.yb[j], col), q,
                              sign_flip_of(st.ys[j]) != 0u);
            } else {
                ++bad;
            }
            st.advance();
        }
    }
    count_dropped(dropped, bad);
}

template <bool POW2>
__global__ void __launch_bounds__(kBlock)
k_fixed_accumulate_sparse(KParams p, long long* __restrict__ acc, const int64_t* __restrict__ idx,
                          const float* __restrict__ val, int64_t n, double scale_2F,
                          unsigned long long* __restrict__ dropped) {
    const int64_t stride = static_cast<int64_t>(gridDim.x) * kBlock;
    const Columns col = columns_of<POW2>(p.c);
    unsigned long long bad = 0;
    for (int64_t t = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x; t < n; t += stride) {
        const uint64_t i = static_cast<uint64_t>(idx[t]);
        long long q;
        if (!fixed_of(val[t], scale_2F, &q)) {
            ++bad;
            continue;
        }
        for (uint32_t j = 0; j < p.r; ++j) {
            const uint64_t yb = hash_state(p.a[j], p.b[j], i);
            const uint64_t ys = hash_state(p.as[j], p.bs[j], i);
            fixed_add(acc + static_cast<size_t>(j) * p.c + bucket_of<POW2>(yb, col), q,
                      sign_flip_of(ys) != 0u);
        }
    }
    count_dropped(dropped, bad);
}

// S = binary32( binary64(acc) * 2^-F * alpha ): the integer to binary64 (exact below 2^53), an
// exact scaling, one multiplication rounded in binary64, one rounding to binary32.
__global__ void __launch_bounds__(kBlock)
k_fixed_to_float(const long long* __restrict__ acc, int64_t n, double inv_2F, double alpha,
                 float* __restrict__ S) {
    const int64_t stride = static_cast<int64_t>(gridDim.x) * kBlock;
    for (int64_t t = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x; t < n; t += stride) {
        const double cell = __ll2double_rn(acc[t]) * inv_2F;
        S[t] = __double2float_rn(cell * alpha);
    }
}

// ---------------------------------------------------------------------------------------
// table-wide elementwise kernels: zero, merge, axpby, momentum
// ---------------------------------------------------------------------------------------
__global__ void __launch_bounds__(kBlock) k_fill_zero(float* __restrict__ S, int64_t n) {
    const int64_t stride = static_cast<int64_t>(gridDim.x) * kBlock;
    for (int64_t t = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x; t < n; t += stride)
        S[t] = 0.0f;
}

constexpr int kMaxMerge = 128;   // source tables per launch of the merge kernel

struct MergePtrs {
    const float* src[kMaxMerge];
};

// dst = beta * dst + alpha * (src[0] + src[1] + ...), the sum taken in ascending order in
// binary64 and the result rounded to binary32 once (see k_bundle_merge for why).
__global__ void __launch_bounds__(kBlock)
k_merge(float* __restrict__ dst, float beta, MergePtrs ptrs, int nw, float alpha, int64_t n) {
    const int64_t stride = static_cast<int64_t>(gridDim.x) * kBlock;
    for (int64_t t = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x; t < n; t += stride) {
        double s = static_cast<double>(ptrs.src[0][t]);
        for (int w = 1; w < nw; ++w) s += static_cast<double>(ptrs.src[w][t]);
        const double base = (beta == 0.0f) ? 0.0 : static_cast<double>(beta) * static_cast<double>(dst[t]);
        dst[t] = static_cast<float>(base + static_cast<double>(alpha) * s);
    }
}

__global__ void __launch_bounds__(kBlock)
k_axpby(float* __restrict__ y, float a, const float* __restrict__ x, float b, int64_t n) {
    const int64_t stride = static_cast<int64_t>(gridDim.x) * kBlock;
    for (int64_t t = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x; t < n; t += stride) {
        const float by = (b == 0.0f) ? 0.0f : b * y[t];
        y[t] = a * x[t] + by;
    }
}

// cells that are NaN or infinite: exponent bits all ones
__global__ void __launch_bounds__(kBlock)
k_count_nonfinite(const float* __restrict__ S, int64_t n, unsigned long long* __restrict__ count) {
    const int64_t stride = static_cast<int64_t>(gridDim.x) * kBlock;
    unsigned long long mine = 0;
    for (int64_t t = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x; t < n; t += stride)
        mine += (__float_as_uint(S[t]) & 0x7f800000u) == 0x7f800000u ? 1u : 0u;
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) mine += __shfl_down(mine, off, 64);
    if ((threadIdx.x & 63) == 0 && mine) atomicAdd(count, mine);
}

__global__ void k_clear_count(unsigned long long* count) { *count = 0; }

__global__ void __launch_bounds__(kBlock)
k_momentum(float* __restrict__ Su, float* __restrict__ Sv, const float* __restrict__ St,
           float rho, int64_t n) {
    const int64_t stride = static_cast<int64_t>(gridDim.x) * kBlock;
    for (int64_t t = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x; t < n; t += stride) {
        const float u = rho * Su[t] + St[t];
        Su[t] = u;
        Sv[t] = Sv[t] + u;
    }
}

// ---------------------------------------------------------------------------------------
// sketch_estimate: Alg. 4 estimate
// ---------------------------------------------------------------------------------------
template <int R, bool POW2>
__global__ void __launch_bounds__(kBlock)
k_estimate(KParams p, const float* __restrict__ S, int64_t d, int64_t i0,
           float* __restrict__ est) {
    const int64_t stride = static_cast<int64_t>(gridDim.x) * kBlock;
    const Columns col = columns_of<POW2>(p.c);
    int64_t t = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x;
    if (t >= d) return;
    RowStates<R> st;
    st.init(p, static_cast<uint64_t>(i0 + t), static_cast<uint64_t>(stride));
    const uint32_t c = p.c;
    for (; t < d; t += stride) {
        float v[R];
#pragma unroll
        for (int j = 0; j < R; ++j) {
            const float cellv = S[static_cast<size_t>(j) * c + bucket_of<POW2>(st.yb[j], col)];
            v[j] = apply_sign(cellv, sign_flip_of(st.ys[j]));
        }
        est[t] = median_odd<R>(v);
        st.advance();
    }
}

template <int R, bool POW2>
__global__ void __launch_bounds__(kBlock)
k_estimate_sparse(KParams p, const float* __restrict__ S, const int64_t* __restrict__ idx,
                  int64_t n, float* __restrict__ out) {
    const int64_t stride = static_cast<int64_t>(gridDim.x) * kBlock;
    const Columns col = columns_of<POW2>(p.c);
    for (int64_t t = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x; t < n; t += stride) {
        const uint64_t i = static_cast<uint64_t>(idx[t]);
        float v[R];
#pragma unroll
        for (int j = 0; j < R; ++j) {
            const uint64_t yb = hash_state(p.a[j], p.b[j], i);
            const uint64_t ys = hash_state(p.as[j], p.bs[j], i);
            v[j] = apply_sign(S[static_cast<size_t>(j) * p.c + bucket_of<POW2>(yb, col)],
                              sign_flip_of(ys));
        }
        out[t] = median_odd<R>(v);
    }
}

// ---------------------------------------------------------------------------------------
// gather_exact: second round
// ---------------------------------------------------------------------------------------
struct GatherPtrs {
    const float* vec[kMaxBatch];
};

__global__ void __launch_bounds__(kBlock)
k_gather(GatherPtrs ptrs, int nw, const int64_t* __restrict__ idx, int64_t k, float alpha,
         float* __restrict__ out, int first_chunk, int last_chunk) {
    const int64_t stride = static_cast<int64_t>(gridDim.x) * kBlock;
    for (int64_t n = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x; n < k; n += stride) {
        const int64_t i = idx[n];
        float s = first_chunk ? 0.0f : out[n];
        for (int w = 0; w < nw; ++w) s += __builtin_nontemporal_load(ptrs.vec[w] + i);
        out[n] = last_chunk ? alpha * s : s;
    }
}

template <int FMT>
__global__ void __launch_bounds__(kBlock)
k_quantize16(const float* __restrict__ x, int64_t n, uint16_t* __restrict__ out) {
    const int64_t stride = static_cast<int64_t>(gridDim.x) * kBlock;
    for (int64_t t = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x; t < n; t += stride)
        out[t] = to_16<FMT>(x[t]);
}

template <int FMT>
__global__ void __launch_bounds__(kBlock)
k_dequantize16(const uint16_t* __restrict__ q, int64_t n, float* __restrict__ out) {
    const int64_t stride = static_cast<int64_t>(gridDim.x) * kBlock;
    for (int64_t t = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x; t < n; t += stride)
        out[t] = from_16<FMT>(q[t]);
}

// The momentum and error-accumulation steps of Alg. 3 with dense per-worker state:
// u = rho u + g (one fused multiply-add), v = v + u.  blockIdx.y = worker; 20 bytes of
// traffic per coordinate, 16-byte accesses when the three vectors are 16-byte aligned.
struct DensePtrs {
    float* u[kMaxBatch];
    float* v[kMaxBatch];
    const float* g[kMaxBatch];
};

template <bool VEC>
__global__ void __launch_bounds__(kBlock)
k_dense_momentum(DensePtrs ptrs, int64_t d, float rho) {
    float* __restrict__ u = ptrs.u[blockIdx.y];
    float* __restrict__ v = ptrs.v[blockIdx.y];
    const float* __restrict__ g = ptrs.g[blockIdx.y];
    const int64_t stride = static_cast<int64_t>(gridDim.x) * kBlock;
    const int64_t t0 = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x;
    int64_t done = 0;
    if (VEC) {
        const int64_t n4 = d / 4;
        for (int64_t t = t0; t < n4; t += stride) {
            float4 uu = reinterpret_cast<float4*>(u)[t], vv = reinterpret_cast<float4*>(v)[t];
            const float4 gg = reinterpret_cast<const float4*>(g)[t];
            uu.x = __fmaf_rn(rho, uu.x, gg.x); uu.y = __fmaf_rn(rho, uu.y, gg.y);
            uu.z = __fmaf_rn(rho, uu.z, gg.z); uu.w = __fmaf_rn(rho, uu.w, gg.w);
            vv.x += uu.x; vv.y += uu.y; vv.z += uu.z; vv.w += uu.w;
            reinterpret_cast<float4*>(u)[t] = uu;
            reinterpret_cast<float4*>(v)[t] = vv;
        }
        done = n4 * 4;
    }
    for (int64_t t = done + t0; t < d; t += stride) {
        const float un = __fmaf_rn(rho, u[t], g[t]);
        u[t] = un;
        v[t] += un;
    }
}

// Measurement aid: a plain streaming read of the workers' vectors, the access that every
// HBM-bound kernel here is compared with.  blockIdx.y = worker; 16-byte loads, two in flight
// per thread, when the vectors are 16-byte aligned; the sum of everything read is added to
// out[0] (one atomic per workgroup, a few thousand per launch) so that the loads cannot be
// dropped.
struct ProbePtrs {
    const float* x[kMaxBatch];
};

template <bool VEC>
__global__ void __launch_bounds__(kBlock)
k_probe_stream_read(ProbePtrs ptrs, int64_t d, float* __restrict__ out) {
    const float* __restrict__ x = ptrs.x[blockIdx.y];
    const int64_t stride = static_cast<int64_t>(gridDim.x) * kBlock;
    const int64_t t0 = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x;
    float acc = 0.0f;
    int64_t done = 0;
    if (VEC) {
        const float4* __restrict__ x4 = reinterpret_cast<const float4*>(x);
        const int64_t n4 = d / 4;
        int64_t t = t0;
        for (; t + stride < n4; t += 2 * stride) {
            const float4 p = x4[t], q = x4[t + stride];
            acc += ((p.x + p.y) + (p.z + p.w)) + ((q.x + q.y) + (q.z + q.w));
        }
        if (t < n4) {
            const float4 p = x4[t];
            acc += (p.x + p.y) + (p.z + p.w);
        }
        done = n4 * 4;
    }
    for (int64_t t = done + t0; t < d; t += stride) acc += x[t];
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) acc += __shfl_down(acc, off, 64);
    __shared__ float part[kBlock / 64];
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) {
        float s = 0.0f;
#pragma unroll
        for (int q = 0; q < kBlock / 64; ++q) s += part[q];
        atomic_add_noret(out, s);                       // one per workgroup
    }
}

// Alg. 3 last step: u, v <- 0 on the coordinates of the update, for every worker
__global__ void __launch_bounds__(kBlock)
k_dense_mask(DensePtrs ptrs, const int64_t* __restrict__ idx, int64_t k) {
    float* __restrict__ u = ptrs.u[blockIdx.y];
    float* __restrict__ v = ptrs.v[blockIdx.y];
    const int64_t stride = static_cast<int64_t>(gridDim.x) * kBlock;
    for (int64_t n = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x; n < k; n += stride) {
        const int64_t i = idx[n];
        u[i] = 0.0f;
        v[i] = 0.0f;
    }
}

}  // namespace cs

using namespace cs;

// =========================================================================================
// C ABI
// =========================================================================================
extern "C" int cs_hash_debug(const cs_params* p, const int64_t* idx, int64_t n,
                             uint32_t* bucket, int8_t* sign, void* stream) {
    if (!params_ok(p) || n < 0) return CS_EINVAL;
    if (n == 0) return CS_OK;
    if (!idx || !bucket || !sign) return CS_EINVAL;
    if (p->c_pow2)
        k_hash_list<true><<<grid_for(n), kBlock, 0, as_stream(stream)>>>(kparams(p), idx, n, bucket, sign);
    else
        k_hash_list<false><<<grid_for(n), kBlock, 0, as_stream(stream)>>>(kparams(p), idx, n, bucket, sign);
    return launch_status();
}

extern "C" int cs_hash_debug_range(const cs_params* p, int64_t i0, int64_t n,
                                   uint32_t* bucket, int8_t* sign, void* stream) {
    if (!params_ok(p) || n < 0 || i0 < 0 || i0 > (int64_t)kP61 - n) return CS_EINVAL;
    if (n == 0) return CS_OK;
    if (!bucket || !sign) return CS_EINVAL;
    if (lattice_applies(p, n)) return launch_hash_range_lattice(p, i0, n, bucket, sign, as_stream(stream));
    // a small grid on purpose: every thread takes several strided steps
    const unsigned grid = grid_for(n, kBlock * 8, 64);
#define CALL(R_, P2_) \
    k_hash_range<R_, P2_><<<grid, kBlock, 0, as_stream(stream)>>>(kparams(p), i0, n, bucket, sign)
    CS_DISPATCH_R(p, CALL);
#undef CALL
    return launch_status();
}

extern "C" int cs_sketch_zero(const cs_params* p, float* S, void* stream) {
    if (!params_ok(p) || !S) return CS_EINVAL;
    const int64_t n = static_cast<int64_t>(p->r) * p->c;
    k_fill_zero<<<grid_for(n), kBlock, 0, as_stream(stream)>>>(S, n);
    return launch_status();
}

static int accumulate_direct(const cs_params* p, const BatchPtrs& ptrs, int nw, int64_t d,
                             int64_t i0, float scale, void* stream) {
    // at least ~8 coordinates per thread so the per-thread hash set-up is amortised
    const unsigned grid = grid_for(d, kBlock * 8, 256 * 8);
#define CALL(R_, P2_)                                                                      \
    k_accumulate<R_, P2_><<<grid, kBlock, 0, as_stream(stream)>>>(kparams(p), ptrs, nw, d, i0, scale)
    CS_DISPATCH_R(p, CALL);
#undef CALL
    return launch_status();
}

static int accumulate_launch(const cs_params* p, const BatchPtrs& ptrs, int nw, int64_t d,
                             int64_t i0, float scale, void* stream) {
    if (lattice_applies(p, d))
        return launch_accumulate_lattice(p, ptrs, nw, d, i0, scale, as_stream(stream));
    return accumulate_direct(p, ptrs, nw, d, i0, scale, stream);
}

extern "C" int cs_sketch_accumulate(const cs_params* p, float* S, const float* g, int64_t d,
                                    int64_t i0, float scale, void* stream) {
    if (!params_ok(p) || d < 0 || i0 < 0 || i0 > (int64_t)kP61 - d) return CS_EINVAL;
    if (d == 0) return CS_OK;
    if (!S || !g) return CS_EINVAL;
    BatchPtrs ptrs{};
    ptrs.S[0] = S;
    ptrs.g[0] = g;
    return accumulate_launch(p, ptrs, 1, d, i0, scale, stream);
}

static int64_t bundle_groups(int32_t W) { return (static_cast<int64_t>(W) + CS_BUNDLE_GROUP - 1) / CS_BUNDLE_GROUP; }

static bool bundle_ok(const cs_params* p, int32_t W) {
    return params_ok(p) && W >= 1 &&
           static_cast<uint64_t>(p->r) * p->c * static_cast<uint64_t>(bundle_groups(W)) * CS_BUNDLE_GROUP < (1ull << 40);
}

extern "C" int cs_bundle_floats(const cs_params* p, int32_t W, int64_t* n) {
    if (!bundle_ok(p, W) || !n) return CS_EINVAL;
    *n = static_cast<int64_t>(p->r) * p->c * bundle_groups(W) * CS_BUNDLE_GROUP;
    return CS_OK;
}

extern "C" int cs_bundle_zero(const cs_params* p, float* T, int32_t W, void* stream) {
    if (!bundle_ok(p, W) || !T) return CS_EINVAL;
    return launch_bundle_zero(T, static_cast<int64_t>(p->r) * p->c * bundle_groups(W) * CS_BUNDLE_GROUP,
                              as_stream(stream));
}

extern "C" int cs_sketch_accumulate_bundle(const cs_params* p, float* T, int32_t W,
                                           const float* const* g_w, int64_t d, int64_t i0,
                                           float scale, void* stream) {
    if (!bundle_ok(p, W) || d < 0 || i0 < 0 || i0 > (int64_t)kP61 - d) return CS_EINVAL;
    if (!T || !g_w) return CS_EINVAL;
    for (int w = 0; w < W; ++w)
        if (!g_w[w] && d > 0) return CS_EINVAL;
    if (d == 0) return CS_OK;
    if (walk_applies(p, d)) return launch_accumulate_walk(p, T, W, g_w, d, i0, scale, false, as_stream(stream));
    if (anyc_visits_apply(p, d)) return launch_accumulate_anyc(p, T, W, g_w, d, i0, scale, false, as_stream(stream));
    // any other sketch: a slot of 8 lanes per coordinate, one lane per worker of a group
    const size_t group_floats = static_cast<size_t>(p->r) * p->c * CS_BUNDLE_GROUP;
    constexpr int kSlots = kBlock / CS_BUNDLE_GROUP;
    for (int w0 = 0; w0 < W; w0 += kMaxBatch) {
        const int nw = (W - w0 < kMaxBatch) ? (W - w0) : kMaxBatch;
        GroupedVectors vec{};
        for (int w = 0; w < nw; ++w) vec.g[w] = g_w[w0 + w];
        float* T0 = T + (w0 / CS_BUNDLE_GROUP) * group_floats;
        // at least ~8 coordinates per lane so the per-lane hash set-up is amortised
        const dim3 grid(grid_for(d, kSlots * 8, 256 * 8),
                        static_cast<unsigned>((nw + CS_BUNDLE_GROUP - 1) / CS_BUNDLE_GROUP));
        if (lds_table_applies(p, d)) {
            const dim3 lgrid(grid_for(d, kSlots * 8, 512), grid.y);
            const size_t lds = static_cast<size_t>(p->r) * p->c * CS_BUNDLE_GROUP * sizeof(float);
#define CALL(R_, P2_)                                                                      \
    k_accumulate_cells_lds<R_, P2_><<<lgrid, kBlock, lds, as_stream(stream)>>>(kparams(p), vec, nw, \
                                                                               T0, d, i0, scale)
            CS_DISPATCH_R(p, CALL);
#undef CALL
        } else {
#define CALL(R_, P2_)                                                                      \
    k_accumulate_cells<R_, P2_><<<grid, kBlock, 0, as_stream(stream)>>>(kparams(p), vec, nw, T0, d, \
                                                                        i0, scale)
            CS_DISPATCH_R(p, CALL);
#undef CALL
        }
        if (launch_status() != CS_OK) return CS_EHIP;
    }
    return CS_OK;
}

extern "C" int cs_sketch_accumulate_sum(const cs_params* p, float* S, int32_t W,
                                        const float* const* g_w, int64_t d, int64_t i0,
                                        float scale, void* stream) {
    if (!params_ok(p) || W < 1 || d < 0 || i0 < 0 || i0 > (int64_t)kP61 - d) return CS_EINVAL;
    if (!S || !g_w) return CS_EINVAL;
    for (int w = 0; w < W; ++w)
        if (!g_w[w] && d > 0) return CS_EINVAL;
    if (d == 0) return CS_OK;
    // along visit lists the 8 workers of a group are added up in registers and a cell receives
    // one request per group; everything else adds worker by worker into the same table
    if (all_rows_listed(p, d)) return launch_accumulate_walk(p, S, W, g_w, d, i0, scale, true, as_stream(stream));
    if (anyc_visits_apply(p, d)) return launch_accumulate_anyc(p, S, W, g_w, d, i0, scale, true, as_stream(stream));
    for (int w0 = 0; w0 < W; w0 += kMaxBatch) {
        const int nw = (W - w0 < kMaxBatch) ? (W - w0) : kMaxBatch;
        BatchPtrs ptrs{};
        for (int w = 0; w < nw; ++w) {
            ptrs.S[w] = S;
            ptrs.g[w] = g_w[w0 + w];
        }
        const int rc = accumulate_launch(p, ptrs, nw, d, i0, scale, stream);
        if (rc != CS_OK) return rc;
    }
    return CS_OK;
}

extern "C" int cs_bundle_update_launches(const cs_params* p, int32_t W, int64_t d, int32_t* n) {
    if (!bundle_ok(p, W) || d < 0 || !n) return CS_EINVAL;
    if (d == 0) { *n = 0; return CS_OK; }
    if (walk_applies(p, d)) { *n = count_accumulate_walk_launches(p, W, d); return CS_OK; }
    if (anyc_visits_apply(p, d)) { *n = count_accumulate_anyc_launches(p, W); return CS_OK; }
    *n = (W + kMaxBatch - 1) / kMaxBatch;
    return CS_OK;
}

extern "C" int cs_bundle_merge(const cs_params* p, float* dst, float beta, const float* T,
                               int32_t W, float alpha, void* stream) {
    if (!bundle_ok(p, W) || !dst || !T) return CS_EINVAL;
    if (reinterpret_cast<uintptr_t>(T) % 16 != 0) return CS_EINVAL;
    return launch_bundle_merge(dst, beta, T, static_cast<int>(bundle_groups(W)), alpha,
                               static_cast<int64_t>(p->r) * p->c, as_stream(stream));
}

extern "C" int cs_quantize16(const float* x, int64_t n, uint16_t* out, int32_t fmt, void* stream) {
    if (n < 0 || (fmt != CS_FMT_BF16 && fmt != CS_FMT_F16)) return CS_EINVAL;
    if (n == 0) return CS_OK;
    if (!x || !out) return CS_EINVAL;
    if (fmt == CS_FMT_BF16) k_quantize16<0><<<grid_for(n), kBlock, 0, as_stream(stream)>>>(x, n, out);
    else k_quantize16<1><<<grid_for(n), kBlock, 0, as_stream(stream)>>>(x, n, out);
    return launch_status();
}

extern "C" int cs_dequantize16(const uint16_t* q, int64_t n, float* out, int32_t fmt, void* stream) {
    if (n < 0 || (fmt != CS_FMT_BF16 && fmt != CS_FMT_F16)) return CS_EINVAL;
    if (n == 0) return CS_OK;
    if (!q || !out) return CS_EINVAL;
    if (fmt == CS_FMT_BF16) k_dequantize16<0><<<grid_for(n), kBlock, 0, as_stream(stream)>>>(q, n, out);
    else k_dequantize16<1><<<grid_for(n), kBlock, 0, as_stream(stream)>>>(q, n, out);
    return launch_status();
}

extern "C" int cs_bundle_merge16(const cs_params* p, float* dst, float beta, const uint16_t* T16,
                                 int32_t W, float alpha, int32_t fmt, void* stream) {
    if (!bundle_ok(p, W) || !dst || !T16) return CS_EINVAL;
    if (fmt != CS_FMT_BF16 && fmt != CS_FMT_F16) return CS_EINVAL;
    if (reinterpret_cast<uintptr_t>(T16) % 16 != 0) return CS_EINVAL;
    return launch_bundle_merge16(dst, beta, T16, static_cast<int>(bundle_groups(W)), alpha,
                                 static_cast<int64_t>(p->r) * p->c, fmt, as_stream(stream));
}

extern "C" int cs_sketch_accumulate_batch(const cs_params* p, float* const* S_w,
                                          const float* const* g_w, int32_t W, int64_t d,
                                          int64_t i0, float scale, void* stream) {
    if (!params_ok(p) || W < 1 || d < 0 || i0 < 0 || i0 > (int64_t)kP61 - d) return CS_EINVAL;
    if (!S_w || !g_w) return CS_EINVAL;
    for (int w = 0; w < W; ++w)
        if (!S_w[w] || (!g_w[w] && d > 0)) return CS_EINVAL;
    if (d == 0) return CS_OK;
    for (int w0 = 0; w0 < W; w0 += kMaxBatch) {
        const int nw = (W - w0 < kMaxBatch) ? (W - w0) : kMaxBatch;
        BatchPtrs ptrs{};
        for (int w = 0; w < nw; ++w) {
            ptrs.S[w] = S_w[w0 + w];
            ptrs.g[w] = g_w[w0 + w];
        }
        const int rc = accumulate_launch(p, ptrs, nw, d, i0, scale, stream);
        if (rc != CS_OK) return rc;
    }
    return CS_OK;
}

extern "C" int cs_sketch_accumulate_sparse(const cs_params* p, float* S, const int64_t* idx,
                                           const float* val, int64_t n, float scale,
                                           void* stream) {
    if (!params_ok(p) || n < 0) return CS_EINVAL;
    if (n == 0) return CS_OK;
    if (!S || !idx || !val) return CS_EINVAL;
    if (p->c_pow2)
        k_accumulate_sparse<true><<<grid_for(n), kBlock, 0, as_stream(stream)>>>(kparams(p), S, idx, val, n, scale);
    else
        k_accumulate_sparse<false><<<grid_for(n), kBlock, 0, as_stream(stream)>>>(kparams(p), S, idx, val, n, scale);
    return launch_status();
}

static bool fixed_args_ok(const cs_params* p, const void* acc, int32_t frac_bits) {
    return params_ok(p) && acc && frac_bits >= 0 && frac_bits <= CS_FIXED_MAX_FRAC_BITS;
}

extern "C" int cs_fixed_accumulate(const cs_params* p, int64_t* acc, const float* g, int64_t d,
                                   int64_t i0, float scale, int32_t frac_bits, int64_t* dropped,
                                   void* stream) {
    if (!fixed_args_ok(p, acc, frac_bits) || d < 0 || i0 < 0 || (d > 0 && !g)) return CS_EINVAL;
    if (d == 0) return CS_OK;
    const double scale_2F = ldexp(static_cast<double>(scale), frac_bits);
    auto* a = reinterpret_cast<long long*>(acc);
    auto* bad = reinterpret_cast<unsigned long long*>(dropped);
#define CS_CALL(R_, P2_) \
    k_fixed_accumulate<R_, P2_><<<grid_for(d), kBlock, 0, as_stream(stream)>>>(kparams(p), a, g, d, i0, scale_2F, bad)
    CS_DISPATCH_R(p, CS_CALL);
#undef CS_CALL
    return launch_status();
}

extern "C" int cs_fixed_accumulate_sparse(const cs_params* p, int64_t* acc, const int64_t* idx,
                                          const float* val, int64_t n, float scale,
                                          int32_t frac_bits, int64_t* dropped, void* stream) {
    if (!fixed_args_ok(p, acc, frac_bits) || n < 0 || (n > 0 && (!idx || !val))) return CS_EINVAL;
    if (n == 0) return CS_OK;
    const double scale_2F = ldexp(static_cast<double>(scale), frac_bits);
    auto* a = reinterpret_cast<long long*>(acc);
    auto* bad = reinterpret_cast<unsigned long long*>(dropped);
    if (p->c_pow2)
        k_fixed_accumulate_sparse<true><<<grid_for(n), kBlock, 0, as_stream(stream)>>>(kparams(p), a, idx, val, n, scale_2F, bad);
    else
        k_fixed_accumulate_sparse<false><<<grid_for(n), kBlock, 0, as_stream(stream)>>>(kparams(p), a, idx, val, n, scale_2F, bad);
    return launch_status();
}

extern "C" int cs_fixed_to_float(const cs_params* p, const int64_t* acc, int32_t frac_bits,
                                 float alpha, float* S, void* stream) {
    if (!fixed_args_ok(p, acc, frac_bits) || !S) return CS_EINVAL;
    const int64_t n = static_cast<int64_t>(p->r) * p->c;
    k_fixed_to_float<<<grid_for(n), kBlock, 0, as_stream(stream)>>>(
        reinterpret_cast<const long long*>(acc), n, ldexp(1.0, -frac_bits),
        static_cast<double>(alpha), S);
    return launch_status();
}

extern "C" int cs_sketch_merge(const cs_params* p, float* dst, float beta,
                               const float* const* src, int32_t W, float alpha, void* stream) {
    if (!params_ok(p) || !dst || !src || W < 1) return CS_EINVAL;
    for (int w = 0; w < W; ++w)
        if (!src[w] || (W > 1 && src[w] == dst)) return CS_EINVAL;
    const int64_t n = static_cast<int64_t>(p->r) * p->c;
    // More sources than one launch takes: later launches add their share on top (beta = 1).
    for (int w0 = 0; w0 < W; w0 += kMaxMerge) {
        const int nw = (W - w0 < kMaxMerge) ? (W - w0) : kMaxMerge;
        MergePtrs ptrs{};
        for (int w = 0; w < nw; ++w) ptrs.src[w] = src[w0 + w];
        k_merge<<<grid_for(n), kBlock, 0, as_stream(stream)>>>(dst, w0 == 0 ? beta : 1.0f, ptrs,
                                                               nw, alpha, n);
        if (launch_status() != CS_OK) return CS_EHIP;
    }
    return CS_OK;
}

extern "C" int cs_sketch_axpby(const cs_params* p, float* y, float a, const float* x, float b,
                               void* stream) {
    if (!params_ok(p) || !y || !x) return CS_EINVAL;
    const int64_t n = static_cast<int64_t>(p->r) * p->c;
    k_axpby<<<grid_for(n), kBlock, 0, as_stream(stream)>>>(y, a, x, b, n);
    return launch_status();
}

extern "C" int cs_sketch_count_nonfinite(const cs_params* p, const float* S, int64_t* count,
                                         void* stream) {
    if (!params_ok(p) || !S || !count || reinterpret_cast<uintptr_t>(count) % 8 != 0) return CS_EINVAL;
    const int64_t n = static_cast<int64_t>(p->r) * p->c;
    unsigned long long* out = reinterpret_cast<unsigned long long*>(count);
    k_clear_count<<<1, 1, 0, as_stream(stream)>>>(out);
    k_count_nonfinite<<<grid_for(n), kBlock, 0, as_stream(stream)>>>(S, n, out);
    return launch_status();
}

extern "C" int cs_sketch_momentum(const cs_params* p, float* S_u, float* S_v, const float* S_t,
                                  float rho, void* stream) {
    if (!params_ok(p) || !S_u || !S_v || !S_t) return CS_EINVAL;
    const int64_t n = static_cast<int64_t>(p->r) * p->c;
    k_momentum<<<grid_for(n), kBlock, 0, as_stream(stream)>>>(S_u, S_v, S_t, rho, n);
    return launch_status();
}

extern "C" int cs_estimate_workspace_bytes(const cs_params* p, int64_t d, size_t* bytes) {
    if (!params_ok(p) || d < 0 || !bytes) return CS_EINVAL;
    // the stride-aligned path stores the r signed cells of every coordinate before the median
    *bytes = (lattice_applies(p, d) || anyc_visits_serve_query(p, d))
                 ? sizeof(float) * static_cast<size_t>(p->r) * static_cast<size_t>(d) : 0;
    return CS_OK;
}

static int estimate_all(const cs_params* p, const float* S, int64_t d, int64_t i0, float* est,
                        uint64_t* hist, bool* hist_done, void* rows_ws, size_t ws_bytes,
                        void* stream) {
    *hist_done = false;
    if (lattice_applies(p, d)) {
        const size_t need = sizeof(float) * static_cast<size_t>(p->r) * static_cast<size_t>(d);
        if (!rows_ws || reinterpret_cast<uintptr_t>(rows_ws) % 4 != 0) return CS_EINVAL;
        if (ws_bytes < need) return CS_EWORKSPACE;
        return launch_estimate_lattice(p, S, d, i0, est, static_cast<float*>(rows_ws), hist, hist_done,
                                       as_stream(stream));
    }
    if (anyc_visits_serve_query(p, d)) {
        const size_t need = sizeof(float) * static_cast<size_t>(p->r) * static_cast<size_t>(d);
        if (!rows_ws || reinterpret_cast<uintptr_t>(rows_ws) % 4 != 0) return CS_EINVAL;
        if (ws_bytes < need) return CS_EWORKSPACE;
        return launch_estimate_anyc(p, S, d, i0, est, static_cast<float*>(rows_ws), as_stream(stream));
    }
    const unsigned grid = grid_for(d, kBlock * 8, 256 * 8);
#define CALL(R_, P2_) \
    k_estimate<R_, P2_><<<grid, kBlock, 0, as_stream(stream)>>>(kparams(p), S, d, i0, est)
    CS_DISPATCH_R(p, CALL);
#undef CALL
    return launch_status();
}

extern "C" int cs_sketch_estimate(const cs_params* p, const float* S, int64_t d, int64_t i0,
                                  float* est, uint64_t* hist_or_null, void* rows_ws,
                                  size_t ws_bytes, void* stream) {
    if (!params_ok(p) || d < 0 || i0 < 0 || i0 > (int64_t)kP61 - d) return CS_EINVAL;
    if (hist_or_null && reinterpret_cast<uintptr_t>(hist_or_null) % 8 != 0) return CS_EINVAL;
    if (d > 0 && (!S || !est)) return CS_EINVAL;
    if (hist_or_null) {
        const int rc = launch_magnitude_hist_zero(hist_or_null, as_stream(stream));
        if (rc != CS_OK) return rc;
    }
    if (d == 0) return CS_OK;
    bool hist_done = false;
    const int rc = estimate_all(p, S, d, i0, est, hist_or_null, &hist_done, rows_ws, ws_bytes, stream);
    if (rc != CS_OK || !hist_or_null || hist_done) return rc;
    // the kernels that wrote est did not count it: one more read of est
    return launch_magnitude_hist(est, d, hist_or_null, as_stream(stream));
}

extern "C" int cs_sketch_estimate_sparse(const cs_params* p, const float* S, const int64_t* idx,
                                         int64_t n, float* out, void* stream) {
    if (!params_ok(p) || n < 0) return CS_EINVAL;
    if (n == 0) return CS_OK;
    if (!S || !idx || !out) return CS_EINVAL;
#define CALL(R_, P2_) \
    k_estimate_sparse<R_, P2_><<<grid_for(n), kBlock, 0, as_stream(stream)>>>(kparams(p), S, idx, n, out)
    CS_DISPATCH_R(p, CALL);
#undef CALL
    return launch_status();
}

extern "C" int cs_gather_exact(const float* const* vec, int32_t W, const int64_t* idx, int64_t k,
                               float alpha, float* out, void* stream) {
    if (!vec || W < 1 || k < 0) return CS_EINVAL;
    for (int w = 0; w < W; ++w)
        if (!vec[w]) return CS_EINVAL;
    if (k == 0) return CS_OK;
    if (!idx || !out) return CS_EINVAL;
    for (int w0 = 0; w0 < W; w0 += kMaxBatch) {
        const int nw = (W - w0 < kMaxBatch) ? (W - w0) : kMaxBatch;
        GatherPtrs ptrs{};
        for (int w = 0; w < nw; ++w) ptrs.vec[w] = vec[w0 + w];
        k_gather<<<grid_for(k), kBlock, 0, as_stream(stream)>>>(ptrs, nw, idx, k, alpha, out,
                                                                w0 == 0, w0 + nw == W);
        if (launch_status() != CS_OK) return CS_EHIP;
    }
    return CS_OK;
}

extern "C" int cs_dense_momentum(float* const* u_w, float* const* v_w, const float* const* g_w,
                                 int32_t W, int64_t d, float rho, void* stream) {
    if (!u_w || !v_w || !g_w || W < 1 || d < 0) return CS_EINVAL;
    bool vec = true;
    for (int w = 0; w < W; ++w) {
        if (!u_w[w] || !v_w[w] || !g_w[w]) return CS_EINVAL;
        vec = vec && (reinterpret_cast<uintptr_t>(u_w[w]) | reinterpret_cast<uintptr_t>(v_w[w]) |
                      reinterpret_cast<uintptr_t>(g_w[w])) % 16 == 0;
    }
    if (d == 0) return CS_OK;
    for (int w0 = 0; w0 < W; w0 += kMaxBatch) {
        const int nw = (W - w0 < kMaxBatch) ? (W - w0) : kMaxBatch;
        DensePtrs ptrs{};
        for (int w = 0; w < nw; ++w) {
            ptrs.u[w] = u_w[w0 + w];
            ptrs.v[w] = v_w[w0 + w];
            ptrs.g[w] = g_w[w0 + w];
        }
        const dim3 grid(grid_for(vec ? (d + 3) / 4 : d, kBlock, 2048), static_cast<unsigned>(nw));
        if (vec) k_dense_momentum<true><<<grid, kBlock, 0, as_stream(stream)>>>(ptrs, d, rho);
        else k_dense_momentum<false><<<grid, kBlock, 0, as_stream(stream)>>>(ptrs, d, rho);
        if (launch_status() != CS_OK) return CS_EHIP;
    }
    return CS_OK;
}

extern "C" int cs_probe_stream_read(const float* const* x_w, int32_t W, int64_t d, float* out,
                                    void* stream) {
    if (!x_w || W < 1 || d < 0 || !out) return CS_EINVAL;
    bool vec = true;
    for (int w = 0; w < W; ++w) {
        if (!x_w[w]) return CS_EINVAL;
        vec = vec && reinterpret_cast<uintptr_t>(x_w[w]) % 16 == 0;
    }
    if (d == 0) return CS_OK;
    for (int w0 = 0; w0 < W; w0 += kMaxBatch) {
        const int nw = (W - w0 < kMaxBatch) ? (W - w0) : kMaxBatch;
        ProbePtrs ptrs{};
        for (int w = 0; w < nw; ++w) ptrs.x[w] = x_w[w0 + w];
        // about 4096 workgroups per launch, shared out among the workers
        const dim3 grid(grid_for(vec ? (d + 3) / 4 : d, kBlock * 2, (4096 + nw - 1) / nw),
                        static_cast<unsigned>(nw));
        if (vec) k_probe_stream_read<true><<<grid, kBlock, 0, as_stream(stream)>>>(ptrs, d, out);
        else k_probe_stream_read<false><<<grid, kBlock, 0, as_stream(stream)>>>(ptrs, d, out);
        if (launch_status() != CS_OK) return CS_EHIP;
    }
    return CS_OK;
}

extern "C" int cs_dense_mask(float* const* u_w, float* const* v_w, int32_t W, const int64_t* idx,
                             int64_t k, void* stream) {
    if (!u_w || !v_w || W < 1 || k < 0) return CS_EINVAL;
    for (int w = 0; w < W; ++w)
        if (!u_w[w] || !v_w[w]) return CS_EINVAL;
    if (k == 0) return CS_OK;
    if (!idx) return CS_EINVAL;
    for (int w0 = 0; w0 < W; w0 += kMaxBatch) {
        const int nw = (W - w0 < kMaxBatch) ? (W - w0) : kMaxBatch;
        DensePtrs ptrs{};
        for (int w = 0; w < nw; ++w) {
            ptrs.u[w] = u_w[w0 + w];
            ptrs.v[w] = v_w[w0 + w];
        }
        const dim3 grid(grid_for(k), static_cast<unsigned>(nw));
        k_dense_mask<<<grid, kBlock, 0, as_stream(stream)>>>(ptrs, idx, k);
        if (launch_status() != CS_OK) return CS_EHIP;
    }
    return CS_OK;
}

extern "C" int cs_sketch_feedback(const cs_params* p, float* S, const int64_t* idx, int64_t k,
                                  float* val, void* stream) {
    if (!params_ok(p) || k < 0) return CS_EINVAL;
    if (k == 0) return CS_OK;
    if (!S || !idx || !val) return CS_EINVAL;
    // all k estimates are taken from the table as it is on entry (first kernel), and only
    // then is the sketch of (idx, val) subtracted (second kernel, same stream).
    int rc = cs_sketch_estimate_sparse(p, S, idx, k, val, stream);
    if (rc != CS_OK) return rc;
    return cs_sketch_accumulate_sparse(p, S, idx, val, k, -1.0f, stream);
}
