// Stride-aligned ("lattice") traversal for power-of-two column counts.
//
// Fact used.  The bucket hash h(i) = ((a i + b) mod p) mod c is affine modulo p, and with c a
// power of two p = 2^61 - 1 = -1 (mod c).  Hence for any stride D
//     h(i + D) = h(i) + (a D mod p) mod c  (+1 if the sum wrapped past p)      (mod c),
// i.e. coordinates D apart advance through the row by a constant number of buckets.  The
// host picks, per row, a stride D whose advance is a fraction of a bucket to a few buckets
// (cs_row_plan).  One wavefront then takes 64 coordinates D apart, one per lane: its 64
// atomic adds (Alg. 4 update) or 64 gathers (Alg. 4 estimate) fall into one short contiguous
// stretch of the row and travel as a handful of 64-byte requests instead of 64.  The hardware
// processes atomic requests at a fixed rate per request, not per lane, so this is worth an
// order of magnitude.  No result changes: every lane still evaluates the hash of its own
// coordinate exactly; only the order in which coordinates are visited differs.
//
// Traversal.  For a row with stride D the vector [0, d) is cut into super-tiles of 64 D
// coordinates; lane l owns the block [l D, (l+1) D) of its super-tile and walks it in
// chunks of kRun consecutive coordinates.  A tile = (super-tile, chunk) = 64 runs of kRun
// coordinates.  Global memory is always touched coalesced: a run is loaded (stored) by
// consecutive lanes and the 64 x kRun tile is transposed through LDS, so that afterwards each
// lane reads (writes) its own run.  A workgroup is one wavefront; nothing is shared between
// wavefronts.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "cs_device.h"
#include "cs_internal.h"
#include "csketch.h"

namespace cs {

constexpr int kRun = 16;              // consecutive coordinates per lane and tile
constexpr int kLdsStride = kRun + 1;  // padded: transposed access without bank conflicts

struct TileGeom {
    int64_t D;         // lane stride
    int64_t chunks;    // ceil(D / kRun)
    int64_t ntiles;    // super-tiles * chunks
};

__device__ __forceinline__ TileGeom tile_geom(const cs_params& p, int j, int64_t d) {
    TileGeom g;
    g.D = static_cast<int64_t>(p.plan[j].D);
    g.chunks = (g.D + kRun - 1) / kRun;
    const int64_t span = g.D * 64;
    g.ntiles = ((d + span - 1) / span) * g.chunks;
    return g;
}

// Walks the 64 x kRun tile `tile` of row j: computes, for this lane's run, the packed
// (bucket | sign bit 31) of each of its coordinates.  Returns the index (relative to the
// vector) of the lane's first coordinate and the run length of this chunk.
__device__ __forceinline__ void tile_hashes(const cs_params& p, int j, const TileGeom& g,
                                            int64_t tile, int64_t i0, uint32_t (&packed)[kRun],
                                            int64_t* base, int* mlen) {
    const int lane = threadIdx.x;
    const int64_t s = tile / g.chunks, t = tile - s * g.chunks;
    *base = s * g.D * 64 + t * kRun;                       // lane 0's first coordinate
    const int64_t left = g.D - t * kRun;
    *mlen = left < kRun ? static_cast<int>(left) : kRun;
    const uint64_t first = static_cast<uint64_t>(i0 + *base + static_cast<int64_t>(lane) * g.D);
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

// ---------------------------------------------------------------------------------------
// Alg. 4 update, lattice order.  grid = (tiles, rows); one wavefront per workgroup, so LDS
// traffic of a wavefront is ordered by itself and no barrier is needed.
// ---------------------------------------------------------------------------------------
constexpr int kLanesPerRun = kRun / 4;              // lanes that fetch one run as float4 pieces
constexpr int kRunsPerLoad = 64 / kLanesPerRun;     // runs covered by one wavefront-wide load
constexpr int kLoads = 64 / kRunsPerLoad;           // float4 loads per lane and tile

// four floats that are only 4-byte aligned: global memory takes a 16-byte load at any dword
// address, and a lane's run starts wherever its stride puts it
struct __attribute__((packed, aligned(4))) float4u {
    float x, y, z, w;
};

// Brings the 64 x kRun tile of one worker's vector into registers: lane L takes floats
// 4 (L % kLanesPerRun) .. +3 of runs L / kLanesPerRun, + kRunsPerLoad, ..., each piece as one
// 16-byte load.
__device__ __forceinline__ void load_tile(const float* __restrict__ gw, int64_t base, int64_t D,
                                          int mlen, int64_t d, float4 (&pre)[kLoads]) {
    const int lane = threadIdx.x;
    const int m4 = (lane % kLanesPerRun) * 4, r0 = lane / kLanesPerRun;
#pragma unroll
    for (int q = 0; q < kLoads; ++q) {
        const int64_t rel = base + static_cast<int64_t>(q * kRunsPerLoad + r0) * D + m4;
        float4 v = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
        if (m4 < mlen) {
            if (rel + 4 <= d && m4 + 4 <= mlen) {
                const float4u u = *reinterpret_cast<const float4u*>(gw + rel);
                v = make_float4(u.x, u.y, u.z, u.w);
            } else {
                if (rel + 0 < d && m4 + 0 < mlen) v.x = gw[rel + 0];
                if (rel + 1 < d && m4 + 1 < mlen) v.y = gw[rel + 1];
                if (rel + 2 < d && m4 + 2 < mlen) v.z = gw[rel + 2];
                if (rel + 3 < d && m4 + 3 < mlen) v.w = gw[rel + 3];
            }
        }
        pre[q] = v;
    }
}

__global__ void __launch_bounds__(64)
k_accumulate_lattice(cs_params p, LatticePtrs ptrs, int nw, int64_t d, int64_t i0, float scale) {
    __shared__ float tile_lds[64 * kLdsStride];
    const int j = blockIdx.y;
    const int lane = threadIdx.x;
    const TileGeom g = tile_geom(p, j, d);
    const size_t row_off = static_cast<size_t>(j) * p.c;
    const int nsteps = p.plan[j].scan_steps;
    const int m4 = (lane % kLanesPerRun) * 4, r0 = lane / kLanesPerRun;
    for (int64_t tile = blockIdx.x; tile < g.ntiles; tile += gridDim.x) {
        uint32_t packed[kRun];
        int64_t base;
        int mlen;
        tile_hashes(p, j, g, tile, i0, packed, &base, &mlen);
        const int64_t my_first = base + static_cast<int64_t>(lane) * g.D;
        float4 pre[kLoads];
        load_tile(ptrs.g[0], base, g.D, mlen, d, pre);
        for (int w = 0; w < nw; ++w) {
            float* __restrict__ Sw = ptrs.S[w] + row_off;
#pragma unroll
            for (int q = 0; q < kLoads; ++q) {
                float* dst = tile_lds + (q * kRunsPerLoad + r0) * kLdsStride + m4;
                dst[0] = pre[q].x;
                dst[1] = pre[q].y;
                dst[2] = pre[q].z;
                dst[3] = pre[q].w;
            }
            __builtin_amdgcn_wave_barrier();
            // next worker's tile is fetched while this one is applied
            if (w + 1 < nw) load_tile(ptrs.g[w + 1], base, g.D, mlen, d, pre);
#pragma unroll
            for (int m = 0; m < kRun; ++m) {
                // neighbouring lanes often fall into the same cell (the bucket advances by a
                // fraction of a cell per lane): add them up in registers first, so that one
                // lane per distinct cell issues the atomic
                const bool valid = m < mlen && my_first + m < d;
                const uint32_t cell = packed[m] & 0x7fffffffu;
                const uint32_t key = valid ? cell : (0xfffffff0u - static_cast<uint32_t>(lane));
                float v = valid ? apply_sign(scale * tile_lds[lane * kLdsStride + m],
                                             packed[m] & 0x80000000u)
                                : 0.0f;
                const bool issue = segment_sum16(key, v, nsteps);
                if (issue && valid) atomic_add_noret(Sw + cell, v);
            }
            __builtin_amdgcn_wave_barrier();
        }
    }
}

// ---------------------------------------------------------------------------------------
// Alg. 4 estimate, lattice order: per row, the signed cell s_j(i) S[j][h_j(i)] of every
// coordinate goes to rows[j][i]; a second kernel takes the median over rows.
// ---------------------------------------------------------------------------------------
__global__ void __launch_bounds__(64)
k_row_values_lattice(cs_params p, const float* __restrict__ S, int64_t d, int64_t i0,
                     float* __restrict__ rows) {
    __shared__ float tile_lds[64 * kLdsStride];
    const int j = blockIdx.y;
    const int lane = threadIdx.x;
    const TileGeom g = tile_geom(p, j, d);
    const float* __restrict__ Sj = S + static_cast<size_t>(j) * p.c;
    float* __restrict__ out = rows + static_cast<size_t>(j) * d;
    for (int64_t tile = blockIdx.x; tile < g.ntiles; tile += gridDim.x) {
        uint32_t packed[kRun];
        int64_t base;
        int mlen;
        tile_hashes(p, j, g, tile, i0, packed, &base, &mlen);
        const int64_t my_first = base + static_cast<int64_t>(lane) * g.D;
#pragma unroll
        for (int m = 0; m < kRun; ++m) {
            float v = 0.0f;
            if (m < mlen && my_first + m < d)
                v = apply_sign(Sj[packed[m] & 0x7fffffffu], packed[m] & 0x80000000u);
            tile_lds[lane * kLdsStride + m] = v;
        }
        __syncthreads();
        const int m_st = lane % kRun, r_st = lane / kRun;
#pragma unroll 8
        for (int rr = 0; rr < 64; rr += 64 / kRun) {
            const int run = rr + r_st;
            const int64_t rel = base + static_cast<int64_t>(run) * g.D + m_st;
            if (m_st < mlen && rel < d) out[rel] = tile_lds[run * kLdsStride + m_st];
        }
        __syncthreads();
    }
}

template <int R>
__global__ void __launch_bounds__(kBlock)
k_median_rows(const float* __restrict__ rows, int64_t d, float* __restrict__ est) {
    const int64_t stride = static_cast<int64_t>(gridDim.x) * kBlock;
    for (int64_t t = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x; t < d; t += stride) {
        float v[R];
#pragma unroll
        for (int j = 0; j < R; ++j) v[j] = rows[static_cast<size_t>(j) * d + t];
        est[t] = median_odd<R>(v);
    }
}

// parity hook: buckets and signs of a contiguous range, visited in lattice order
__global__ void __launch_bounds__(64)
k_hash_range_lattice(cs_params p, int64_t i0, int64_t n, uint32_t* __restrict__ bucket,
                     int8_t* __restrict__ sign) {
    const int j = blockIdx.y;
    const int lane = threadIdx.x;
    const TileGeom g = tile_geom(p, j, n);
    for (int64_t tile = blockIdx.x; tile < g.ntiles; tile += gridDim.x) {
        uint32_t packed[kRun];
        int64_t base;
        int mlen;
        tile_hashes(p, j, g, tile, i0, packed, &base, &mlen);
        const int64_t my_first = base + static_cast<int64_t>(lane) * g.D;
#pragma unroll
        for (int m = 0; m < kRun; ++m) {
            if (m < mlen && my_first + m < n) {
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
        const int64_t D = static_cast<int64_t>(p->plan[j].D);
        const int64_t chunks = (D + kRun - 1) / kRun;
        const int64_t nt = ((d + D * 64 - 1) / (D * 64)) * chunks;
        if (nt > most) most = nt;
    }
    const int64_t cap = 256 * 64;      // workgroups of one wavefront: plenty per CU
    return static_cast<unsigned>(most < cap ? most : cap);
}

bool lattice_applies(const cs_params* p, int64_t d) {
    if (!p->c_pow2 || p->c < 64 || d < 4096) return false;
    for (uint32_t j = 0; j < p->r; ++j)
        if (p->plan[j].D <= 1) return false;
    return true;
}

int launch_accumulate_lattice(const cs_params* p, const LatticePtrs& ptrs, int nw, int64_t d,
                              int64_t i0, float scale, hipStream_t stream) {
    const dim3 grid(lattice_grid_x(p, d), p->r);
    k_accumulate_lattice<<<grid, 64, 0, stream>>>(*p, ptrs, nw, d, i0, scale);
    return hipGetLastError() == hipSuccess ? CS_OK : CS_EHIP;
}

int launch_estimate_lattice(const cs_params* p, const float* S, int64_t d, int64_t i0,
                            float* est, float* rows, hipStream_t stream) {
    const dim3 grid(lattice_grid_x(p, d), p->r);
    k_row_values_lattice<<<grid, 64, 0, stream>>>(*p, S, d, i0, rows);
    int64_t b = (d + kBlock - 1) / kBlock;
    if (b > 256 * 16) b = 256 * 16;
    const unsigned mg = static_cast<unsigned>(b);
    switch (p->r) {
        case 1: k_median_rows<1><<<mg, kBlock, 0, stream>>>(rows, d, est); break;
        case 3: k_median_rows<3><<<mg, kBlock, 0, stream>>>(rows, d, est); break;
        case 5: k_median_rows<5><<<mg, kBlock, 0, stream>>>(rows, d, est); break;
        case 7: k_median_rows<7><<<mg, kBlock, 0, stream>>>(rows, d, est); break;
        case 9: k_median_rows<9><<<mg, kBlock, 0, stream>>>(rows, d, est); break;
        case 11: k_median_rows<11><<<mg, kBlock, 0, stream>>>(rows, d, est); break;
        case 13: k_median_rows<13><<<mg, kBlock, 0, stream>>>(rows, d, est); break;
        case 15: k_median_rows<15><<<mg, kBlock, 0, stream>>>(rows, d, est); break;
        default: return CS_EINVAL;
    }
    return hipGetLastError() == hipSuccess ? CS_OK : CS_EHIP;
}

int launch_hash_range_lattice(const cs_params* p, int64_t i0, int64_t n, uint32_t* bucket,
                              int8_t* sign, hipStream_t stream) {
    const dim3 grid(lattice_grid_x(p, n), p->r);
    k_hash_range_lattice<<<grid, 64, 0, stream>>>(*p, i0, n, bucket, sign);
    return hipGetLastError() == hipSuccess ? CS_OK : CS_EHIP;
}

}  // namespace cs
