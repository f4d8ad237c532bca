// Stride-aligned ("lattice") traversal for power-of-two column counts.
//
// Fact used.  The bucket hash h(i) = ((a i + b) mod p) mod c is affine modulo p, and with c a
// power of two p = 2^61 - 1 = -1 (mod c).  Hence for any stride D
//     h(i + D) = h(i) + (a D mod p) mod c  (+1 if the sum wrapped past p)      (mod c),
// i.e. coordinates D apart advance through the row by a constant number of buckets.  The
// host picks, per row, a stride D whose advance is a fraction of a bucket (cs_row_plan).  A
// group of L lanes then takes L coordinates D apart, one per lane: its atomic adds (Alg. 4
// update) or gathers (Alg. 4 estimate) fall into one short contiguous stretch of the row and
// travel as one or two 64-byte requests instead of L.  The memory system processes atomic
// requests at a fixed rate per request, not per lane (measured: ~21 G requests/s whatever
// the table size), so this is worth more than an order of magnitude.  Lanes that fall into
// the same cell are added up in registers first (segment_sum16).  No result changes: every
// lane still evaluates the hash of its own coordinate exactly; only the order in which
// coordinates are visited differs.
//
// Traversal.  For a row with stride D and group width L the vector [0, d) is cut into
// super-tiles of L D coordinates; lane l' of a group owns the block [l' D, (l'+1) D) of its
// super-tile and walks it in chunks of kRun consecutive coordinates.  A wavefront holds
// G = 64 / L groups working on G neighbouring chunks, so a wavefront tile is 64 runs of kRun
// coordinates.  Global memory is always touched in whole runs: a run is loaded (stored) as
// 16-byte pieces by neighbouring lanes and the 64 x kRun tile is transposed through LDS, so
// that afterwards each lane reads (writes) its own run.  A workgroup is one wavefront;
// nothing is shared between wavefronts, so LDS needs no barrier.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "cs_device.h"
#include "cs_internal.h"
#include "csketch.h"

namespace cs {

constexpr int kRun = 16;                            // consecutive coordinates per lane and tile
constexpr int kLdsStride = kRun + 1;                // padded: transposed access, no bank conflicts
constexpr int kLanesPerRun = kRun / 4;              // lanes that move one run as 16-byte pieces
constexpr int kRunsPerPass = 64 / kLanesPerRun;     // runs covered by one wavefront-wide access
constexpr int kPasses = 64 / kRunsPerPass;          // accesses per lane and tile

// four floats that are only 4-byte aligned: global memory takes a 16-byte access at any dword
// address, and a lane's run starts wherever its stride puts it
struct __attribute__((packed, aligned(4))) float4u {
    float x, y, z, w;
};

struct TileGeom {
    int64_t D;         // lane stride
    int L;             // lanes per group
    int G;             // groups per wavefront = 64 / L
    int64_t chunks;    // chunks per lane block = ceil(D / kRun)
    int64_t wtiles;    // wavefront tiles per super-tile = ceil(chunks / G)
    int64_t ntiles;    // super-tiles * wtiles
};

__host__ __device__ __forceinline__ TileGeom tile_geom(const KParams& p, int j, int64_t d) {
    TileGeom g;
    g.D = static_cast<int64_t>(p.plan[j].D);
    g.L = p.plan[j].lanes;
    g.G = 64 / g.L;
    g.chunks = (g.D + kRun - 1) / kRun;
    g.wtiles = (g.chunks + g.G - 1) / g.G;
    const int64_t span = g.D * g.L;
    g.ntiles = ((d + span - 1) / span) * g.wtiles;
    return g;
}

// Run `rho` (0..63) of wavefront tile `tile`: index of its first coordinate relative to the
// vector, and how many of its kRun coordinates exist (inside the lane's block and below d).
__device__ __forceinline__ int run_span(const TileGeom& g, int64_t tile, int rho, int64_t d,
                                        int64_t* first) {
    const int64_t s = tile / g.wtiles, tq = tile - s * g.wtiles;
    const int h = rho / g.L, l = rho - h * g.L;
    const int64_t t = tq * g.G + h;                        // chunk of this group
    const int64_t rel = (s * g.L + l) * g.D + t * kRun;
    *first = rel;
    int64_t len = g.D - t * kRun;                          // left in the lane's block
    if (d - rel < len) len = d - rel;                      // left in the vector
    if (len > kRun) len = kRun;
    return len > 0 ? static_cast<int>(len) : 0;
}

// packed (bucket | sign bit 31) of the kRun coordinates starting at global index `first`
__device__ __forceinline__ void run_hashes(const KParams& p, int j, uint64_t first,
                                           uint32_t (&packed)[kRun]) {
    uint64_t yb = hash_state(p.a[j], p.b[j], first);
    uint64_t ys = hash_state(p.as[j], p.bs[j], first);
    const uint64_t Ab = p.a[j], As = p.as[j];              // step of one coordinate
    const uint32_t mask = p.c - 1u;
#pragma unroll
    for (int m = 0; m < kRun; ++m) {
        packed[m] = ((static_cast<uint32_t>(yb) - 1u) & mask) | sign_flip_of(ys);
        yb = hash_advance(yb, Ab);
        ys = hash_advance(ys, As);
    }
}

// Brings the 64 x kRun tile of one vector into registers: lane T takes floats
// 4 (T % kLanesPerRun) .. +3 of runs T / kLanesPerRun, + kRunsPerPass, ...; positions that do
// not exist read as 0.
__device__ __forceinline__ void load_tile(const float* __restrict__ gw, const TileGeom& g,
                                          int64_t tile, int64_t d, float4 (&pre)[kPasses]) {
    const int lane = threadIdx.x;
    const int m4 = (lane % kLanesPerRun) * 4, r0 = lane / kLanesPerRun;
#pragma unroll
    for (int q = 0; q < kPasses; ++q) {
        int64_t first;
        const int len = run_span(g, tile, q * kRunsPerPass + r0, d, &first);
        const float* src = gw + first + m4;
        float4 v = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
        if (m4 + 4 <= len) {
            const float4u u = *reinterpret_cast<const float4u*>(src);
            v = make_float4(u.x, u.y, u.z, u.w);
        } else if (m4 < len) {
            v.x = src[0];
            if (m4 + 1 < len) v.y = src[1];
            if (m4 + 2 < len) v.z = src[2];
        }
        pre[q] = v;
    }
}

// ---------------------------------------------------------------------------------------
// Alg. 4 update, lattice order.  grid = (tiles, rows).
// ---------------------------------------------------------------------------------------
template <int NSTEPS>
__device__ __forceinline__ void accumulate_row(const KParams& p, const LatticePtrs& ptrs, int nw,
                                               int64_t d, int64_t i0, float scale, int j,
                                               float* tile_lds) {
    const int lane = threadIdx.x;
    const TileGeom g = tile_geom(p, j, d);
    const size_t row_off = static_cast<size_t>(j) * p.c;
    const int m4 = (lane % kLanesPerRun) * 4, r0 = lane / kLanesPerRun;
    for (int64_t tile = blockIdx.x; tile < g.ntiles; tile += gridDim.x) {
        int64_t my_first;
        run_span(g, tile, lane, d, &my_first);
        uint32_t packed[kRun];
        run_hashes(p, j, static_cast<uint64_t>(i0 + my_first), packed);
        float4 pre[kPasses];
        load_tile(ptrs.g[0], g, tile, d, pre);
        for (int w = 0; w < nw; ++w) {
            float* __restrict__ Sw = ptrs.S[w] + row_off;
#pragma unroll
            for (int q = 0; q < kPasses; ++q) {
                float* dst = tile_lds + (q * kRunsPerPass + r0) * kLdsStride + m4;
                dst[0] = pre[q].x;
                dst[1] = pre[q].y;
                dst[2] = pre[q].z;
                dst[3] = pre[q].w;
            }
            __builtin_amdgcn_wave_barrier();
            float mine[kRun];
#pragma unroll
            for (int m = 0; m < kRun; ++m) mine[m] = tile_lds[lane * kLdsStride + m];
            __builtin_amdgcn_wave_barrier();
            // the next worker's tile is fetched while this one is applied
            if (w + 1 < nw) load_tile(ptrs.g[w + 1], g, tile, d, pre);
#pragma unroll
            for (int m = 0; m < kRun; ++m) {
                // Neighbouring lanes often fall into the same cell (the bucket advances by a
                // fraction of a cell per lane): add them up in registers, so that one lane per
                // distinct cell issues the atomic.  Positions that do not exist hold 0 and are
                // harmless wherever they land; totals of exactly 0 are not sent.
                const uint32_t cell = packed[m] & 0x7fffffffu;
                float v = apply_sign(scale * mine[m], packed[m] & 0x80000000u);
                const bool last = segment_sum16(cell, v, NSTEPS);
                if (last && v != 0.0f) atomic_add_noret(Sw + cell, v);
            }
        }
    }
}

__global__ void __launch_bounds__(64)
k_accumulate_lattice(KParams p, LatticePtrs ptrs, int nw, int64_t d, int64_t i0, float scale) {
    __shared__ float tile_lds[64 * kLdsStride];
    const int j = blockIdx.y;
    switch (p.plan[j].scan_steps) {       // uniform: compile-time scan depth inside
        case 0: accumulate_row<0>(p, ptrs, nw, d, i0, scale, j, tile_lds); break;
        case 1: accumulate_row<1>(p, ptrs, nw, d, i0, scale, j, tile_lds); break;
        case 2: accumulate_row<2>(p, ptrs, nw, d, i0, scale, j, tile_lds); break;
        case 3: accumulate_row<3>(p, ptrs, nw, d, i0, scale, j, tile_lds); break;
        default: accumulate_row<4>(p, ptrs, nw, d, i0, scale, j, tile_lds); break;
    }
}

// ---------------------------------------------------------------------------------------
// Alg. 4 estimate, lattice order: per row, the signed cell s_j(i) S[j][h_j(i)] of every
// coordinate goes to rows[j][i]; a second kernel takes the median over rows.
// ---------------------------------------------------------------------------------------
__global__ void __launch_bounds__(64)
k_row_values_lattice(KParams p, const float* __restrict__ S, int64_t d, int64_t i0,
                     float* __restrict__ rows) {
    __shared__ float tile_lds[64 * kLdsStride];
    const int j = blockIdx.y;
    const int lane = threadIdx.x;
    const TileGeom g = tile_geom(p, j, d);
    const float* __restrict__ Sj = S + static_cast<size_t>(j) * p.c;
    float* __restrict__ out = rows + static_cast<size_t>(j) * d;
    const int m4 = (lane % kLanesPerRun) * 4, r0 = lane / kLanesPerRun;
    for (int64_t tile = blockIdx.x; tile < g.ntiles; tile += gridDim.x) {
        int64_t my_first;
        const int my_len = run_span(g, tile, lane, d, &my_first);
        uint32_t packed[kRun];
        run_hashes(p, j, static_cast<uint64_t>(i0 + my_first), packed);
#pragma unroll
        for (int m = 0; m < kRun; ++m) {
            float v = 0.0f;
            if (m < my_len) v = apply_sign(Sj[packed[m] & 0x7fffffffu], packed[m] & 0x80000000u);
            tile_lds[lane * kLdsStride + m] = v;
        }
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int q = 0; q < kPasses; ++q) {
            int64_t first;
            const int len = run_span(g, tile, q * kRunsPerPass + r0, d, &first);
            const float* src = tile_lds + (q * kRunsPerPass + r0) * kLdsStride + m4;
            float* dst = out + first + m4;
            if (m4 + 4 <= len) {
                float4u u;
                u.x = src[0]; u.y = src[1]; u.z = src[2]; u.w = src[3];
                *reinterpret_cast<float4u*>(dst) = u;
            } else if (m4 < len) {
                dst[0] = src[0];
                if (m4 + 1 < len) dst[1] = src[1];
                if (m4 + 2 < len) dst[2] = src[2];
            }
        }
        __builtin_amdgcn_wave_barrier();
    }
}

// est[t] = median over rows of rows[j][t]; VEC: four coordinates per thread with 16-byte
// accesses (d a multiple of 4, both arrays 16-byte aligned, so every row is aligned too)
template <int R, bool VEC>
__global__ void __launch_bounds__(kBlock)
k_median_rows(const float* __restrict__ rows, int64_t d, float* __restrict__ est) {
    const int64_t stride = static_cast<int64_t>(gridDim.x) * kBlock;
    const int64_t t0 = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x;
    if (VEC) {
        const int64_t n4 = d / 4;
        for (int64_t t = t0; t < n4; t += stride) {
            typedef float f4 __attribute__((ext_vector_type(4)));
            float vx[R], vy[R], vz[R], vw[R];
#pragma unroll
            for (int j = 0; j < R; ++j) {
                const f4 q = __builtin_nontemporal_load(
                    reinterpret_cast<const f4*>(rows + static_cast<size_t>(j) * d) + t);
                vx[j] = q.x; vy[j] = q.y; vz[j] = q.z; vw[j] = q.w;
            }
            reinterpret_cast<float4*>(est)[t] =
                make_float4(median_odd<R>(vx), median_odd<R>(vy), median_odd<R>(vz), median_odd<R>(vw));
        }
        return;
    }
    for (int64_t t = t0; t < d; t += stride) {
        float v[R];
#pragma unroll
        for (int j = 0; j < R; ++j) v[j] = rows[static_cast<size_t>(j) * d + t];
        est[t] = median_odd<R>(v);
    }
}

// parity hook: buckets and signs of a contiguous range, visited in lattice order
__global__ void __launch_bounds__(64)
k_hash_range_lattice(KParams p, int64_t i0, int64_t n, uint32_t* __restrict__ bucket,
                     int8_t* __restrict__ sign) {
    const int j = blockIdx.y;
    const int lane = threadIdx.x;
    const TileGeom g = tile_geom(p, j, n);
    for (int64_t tile = blockIdx.x; tile < g.ntiles; tile += gridDim.x) {
        int64_t my_first;
        const int my_len = run_span(g, tile, lane, n, &my_first);
        uint32_t packed[kRun];
        run_hashes(p, j, static_cast<uint64_t>(i0 + my_first), packed);
#pragma unroll
        for (int m = 0; m < kRun; ++m) {
            if (m < my_len) {
                bucket[static_cast<size_t>(j) * n + my_first + m] = packed[m] & 0x7fffffffu;
                sign[static_cast<size_t>(j) * n + my_first + m] = (packed[m] >> 31) ? -1 : 1;
            }
        }
    }
}

// ---------------------------------------------------------------------------------------
// host launchers
// ---------------------------------------------------------------------------------------
static unsigned lattice_grid_x(const cs_params* p, int64_t d) {
    int64_t most = 1;
    for (uint32_t j = 0; j < p->r; ++j) {
        const TileGeom g = tile_geom(kparams(p), static_cast<int>(j), d);
        if (g.ntiles > most) most = g.ntiles;
    }
    const int64_t cap = 256 * 64;      // workgroups of one wavefront: plenty per CU
    return static_cast<unsigned>(most < cap ? most : cap);
}

bool lattice_applies(const cs_params* p, int64_t d) {
    if (!p->c_pow2 || p->c < 64 || d < 4096) return false;
    for (uint32_t j = 0; j < p->r; ++j) {
        const int L = p->plan[j].lanes;
        if (p->plan[j].D <= 1 || (L != 16 && L != 32 && L != 64)) return false;
        if (p->plan[j].scan_steps < 0 || p->plan[j].scan_steps > 4) return false;
    }
    return true;
}

int launch_accumulate_lattice(const cs_params* p, const LatticePtrs& ptrs, int nw, int64_t d,
                              int64_t i0, float scale, hipStream_t stream) {
    const dim3 grid(lattice_grid_x(p, d), p->r);
    k_accumulate_lattice<<<grid, 64, 0, stream>>>(kparams(p), ptrs, nw, d, i0, scale);
    return hipGetLastError() == hipSuccess ? CS_OK : CS_EHIP;
}

int launch_estimate_lattice(const cs_params* p, const float* S, int64_t d, int64_t i0,
                            float* est, float* rows, uint64_t* hist, bool* hist_done,
                            hipStream_t stream) {
    *hist_done = false;
    if (walk_applies(p, d)) {
        const bool fuse_last = d >= (static_cast<int64_t>(1) << 24);
        const int rc = launch_estimate_walk(p, S, d, i0, est, rows, fuse_last, fuse_last ? hist : nullptr, stream);
        *hist_done = fuse_last && hist != nullptr;
        if (rc != CS_OK || fuse_last) return rc;
    } else {
        const dim3 grid(lattice_grid_x(p, d), p->r);
        k_row_values_lattice<<<grid, 64, 0, stream>>>(kparams(p), S, d, i0, rows);
    }
    int64_t b = (d + kBlock - 1) / kBlock;
    if (b > 256 * 16) b = 256 * 16;
    const unsigned mg = static_cast<unsigned>(b);
    const bool vec = d % 4 == 0 && (reinterpret_cast<uintptr_t>(rows) | reinterpret_cast<uintptr_t>(est)) % 16 == 0;
#define CS_MEDIAN(R_)                                                                   \
    case R_:                                                                            \
        if (vec) k_median_rows<R_, true><<<mg, kBlock, 0, stream>>>(rows, d, est);       \
        else k_median_rows<R_, false><<<mg, kBlock, 0, stream>>>(rows, d, est);          \
        break;
    switch (p->r) {
        CS_MEDIAN(1) CS_MEDIAN(3) CS_MEDIAN(5) CS_MEDIAN(7) CS_MEDIAN(9) CS_MEDIAN(11) CS_MEDIAN(13) CS_MEDIAN(15)
        default: return CS_EINVAL;
    }
#undef CS_MEDIAN
    return hipGetLastError() == hipSuccess ? CS_OK : CS_EHIP;
}

int launch_hash_range_lattice(const cs_params* p, int64_t i0, int64_t n, uint32_t* bucket,
                              int8_t* sign, hipStream_t stream) {
    const dim3 grid(lattice_grid_x(p, n), p->r);
    k_hash_range_lattice<<<grid, 64, 0, stream>>>(kparams(p), i0, n, bucket, sign);
    return hipGetLastError() == hipSuccess ? CS_OK : CS_EHIP;
}

}  // namespace cs
