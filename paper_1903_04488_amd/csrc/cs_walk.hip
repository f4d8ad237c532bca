// Alg. 4 update for a bundle of workers (power-of-two column counts), and the bundle-wide
// elementwise kernels.
//
// Done naively the update is one atomic add per coordinate, row and worker, and this machine
// executes fp32 atomics at the memory side at a fixed ~21-24 G requests per second (measured,
// whatever the table size; a request is one aligned 64-byte block touched by one instruction).  Three facts cut the requests by a factor of ~300, after
// which the kernel is bound by reading the vectors:
//
//  1. The bucket hash is affine modulo p = 2^61 - 1, so moving s coordinates on moves a
//     coordinate through a row by an amount that depends on s only.  The host lists offsets for
//     which that amount is a fraction of a cell (cs_row_plan: one stride and its multiples;
//     cs_visit_plan: every such offset below the vector length), and a lane visits its
//     coordinates in that order, keeping running sums in registers: one per coordinate,
//     flushed when the cell changes, in the stride walk (k_accumulate_walk); two to four per
//     coordinate, flushed once at the very end, with a visit list (k_accumulate_visits, the
//     kernel that normally runs).
//  2. All workers use the same hash functions, so in the bundle layout T[w/8][j][b][w%8] the
//     sums of 8 workers for one cell are 32 contiguous bytes: 8 lanes (one per worker) flush
//     them as one request.
//  3. Every row needs its own visiting order, so a group's vectors are read once per row; the
//     rows of a group run in one launch.
//
// Work decomposition for row j: the residues below the stride (or below the largest gap of the
// list) are cut into chunks of RUN consecutive coordinates; a "walker" owns one chunk and
// visits it at every listed offset.  A wavefront holds 64 / WL walkers of WL lanes each, lane
// wl of a walker serving worker wl of the group.  Every hash value is evaluated exactly
// (incremental form of the definition), so results are the same sums as in any other order,
// up to fp32 rounding order.
//
// Data movement per visit: the 64 x RUN tile (64 runs = walkers x workers, RUN floats each) is
// requested as contiguous pieces by neighbouring lanes, transposed through LDS so that every
// lane gets its own run, and the (bucket, sign) of a walker's RUN coordinates are computed once
// per walker by its lanes and shared through LDS.  Nothing is shared between the wavefronts of
// a workgroup, so LDS needs no barrier.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "cs_device.h"
#include "cs_internal.h"
#include "csketch.h"

namespace cs {

namespace {

constexpr int kGroup = CS_BUNDLE_GROUP;  // workers per bundle group
constexpr int kWavesPerGroupOf8 = 2;      // wavefronts per workgroup of the 8-worker kernels

// Vectors are addressed as global memory explicitly: the pointers pass through an LDS table,
// and a generic ("flat") load would count against the LDS counter as well and force the
// hardware to drain both before any data can be used.
typedef const __attribute__((address_space(1))) float* gfloat_ptr;
typedef float vec4f __attribute__((ext_vector_type(4)));
typedef vec4f __attribute__((aligned(4))) vec4f_u;           // 16 bytes at any dword address
typedef const __attribute__((address_space(1))) vec4f_u* gvec4_ptr;

struct WalkArgs {
    const float* g[kGroup];      // vectors of the workers of this group
    float* T;                    // the group's table, float[r][c][kGroup]
    int32_t js[CS_MAX_R];        // sketch rows of this launch; blockIdx.y picks one
    int32_t nw;                  // workers in this group (<= kGroup)
    int64_t d, i0;
    float scale;
};

// WL  = lanes per walker = workers served together (1, 2, 4 or 8);
// RUN = consecutive coordinates per walker and visit (16 or 32).
// A wavefront holds WPW = 64 / WL walkers on neighbouring chunks of RUN residues, so one visit
// reads WPW * RUN * 4 contiguous bytes of every worker's vector (512 bytes for WL = 8,
// RUN = 16: measured to stream at 5.7 TB/s, against 4.5 TB/s with 256-byte and
// 3.5 TB/s with 128-byte pieces).
// NWAVE = wavefronts per workgroup; they work on neighbouring sets of walkers at about the same
// time (nothing is shared and nothing is synchronised between them), which widens the
// contiguous stretch of every vector that is being read at one moment.
template <int WL, int RUN, int NWAVE>
__global__ void __launch_bounds__(64 * NWAVE) k_accumulate_walk(KParams p, WalkArgs a) {
    constexpr int WPW = 64 / WL;                       // walkers per wavefront
    constexpr int PPL = RUN / WL > 0 ? RUN / WL : 1;   // hash values each lane computes
    constexpr int kStride = RUN + 1;                   // padded LDS row of the value tile
    constexpr int kPieces = RUN / 4;                   // 16-byte pieces per run
    constexpr int kRunsPerPass = 64 / kPieces;
    constexpr int kPasses = kPieces;                   // 64 runs / kRunsPerPass
    static_assert(WL * PPL == RUN || WL > RUN, "every coordinate of a walker gets a hash lane");
    __shared__ float tile_lds_all[NWAVE][64 * kStride];
    __shared__ uint32_t hash_lds_all[NWAVE][2][WPW * RUN];   // (bucket | sign), this and previous visit
    __shared__ gfloat_ptr gptr_lds_all[NWAVE][kGroup];

    const int lane = threadIdx.x & 63;
    const int wq = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // wavefront-uniform
    float* tile_lds = tile_lds_all[wq];
    uint32_t (*hash_lds)[WPW * RUN] = hash_lds_all[wq];
    gfloat_ptr* gptr_lds = gptr_lds_all[wq];
    const int j = a.js[blockIdx.y];
    const int h = lane / WL, wl = lane % WL;           // my walker, my worker slot
    if (lane < kGroup) gptr_lds[lane] = (gfloat_ptr)a.g[lane < a.nw ? lane : 0];
    __builtin_amdgcn_wave_barrier();

    const int64_t D = static_cast<int64_t>(p.plan[j].Dw);
    const uint64_t ADb = p.plan[j].ADw, ADs = p.plan[j].ADws;
    const int64_t chunks = (D + RUN - 1) / RUN;
    const int64_t nwaves = (chunks + WPW - 1) / WPW;
    const uint32_t mask = p.c - 1u;
    const int64_t d = a.d;
    float* __restrict__ Tcol = a.T + static_cast<size_t>(j) * p.c * kGroup + wl;

    // loader role: piece m4 of runs r0, r0 + kRunsPerPass, ...; run rho = worker * WPW + walker,
    // so that one load instruction covers neighbouring walkers (contiguous bytes) of few workers
    const int m4 = (lane % kPieces) * 4, r0 = lane / kPieces;
    // hash role: values m0 .. m0 + PPL - 1 of my walker
    const int m0 = (wl * PPL) % RUN;
    const bool hash_duty = wl * PPL < RUN;

    // Workgroups are dealt to the 8 XCDs round-robin; giving XCD x the x-th eighth of the
    // walkers makes each XCD (and its L2) stream through its own contiguous part of every
    // vector.  gridDim.x is a multiple of 8.
    const int64_t ngroups = (nwaves + NWAVE - 1) / NWAVE;      // workgroup-sized sets of walkers
    const int64_t per_xcd = (ngroups + 7) / 8;
    const int64_t xcd_first = static_cast<int64_t>(blockIdx.x & 7) * per_xcd;
    for (int64_t k = blockIdx.x >> 3; k < per_xcd; k += gridDim.x >> 3) {
        const int64_t wv = (xcd_first + k) * NWAVE + wq;
        if (xcd_first + k >= ngroups || wv >= nwaves) break;
        const int64_t chunk0 = wv * WPW;               // first walker's chunk
        const int64_t my_off = (chunk0 + h) * RUN;     // my walker's residue offset in [0, Dw)
        // hash state of coordinate i0 + my_off + m0 (visit n = 0)
        uint64_t yb = hash_state(p.a[j], p.b[j], static_cast<uint64_t>(a.i0 + my_off + m0));
        uint64_t ys = hash_state(p.as[j], p.bs[j], static_cast<uint64_t>(a.i0 + my_off + m0));

        float acc[RUN];                                // running sum of the cell each coordinate is in
#pragma unroll
        for (int m = 0; m < RUN; ++m) acc[m] = 0.0f;

        // All pieces are requested back to back without a branch in between (a piece that is
        // not wholly inside its run reads a safe address and is discarded); runs cut short by
        // the end of the vector or of the residue range are patched up afterwards, which only
        // the last visit or the last chunk ever needs.
        float4 pre[kPasses];
        auto load_visit = [&](int64_t nD) {
            bool any_partial = false;
#pragma unroll
            for (int q = 0; q < kPasses; ++q) {
                const int rho = q * kRunsPerPass + r0;
                const int rw = rho / WPW, rh = rho % WPW;     // worker-major: neighbouring lanes, neighbouring walkers
                const int64_t off = (chunk0 + rh) * RUN;           // residue offset of that run
                const int64_t rel = nD + off;
                int64_t len = D - off;
                if (d - rel < len) len = d - rel;
                if (rw >= a.nw) len = 0;
                const bool full = m4 + 4 <= len;
                const bool part = !full && m4 < len;
                const gfloat_ptr base = gptr_lds[rw < kGroup ? rw : 0];
                const gfloat_ptr src = full ? base + rel + m4 : base;
                const vec4f u = *(gvec4_ptr)src;
                pre[q] = full ? make_float4(u.x, u.y, u.z, u.w) : make_float4(0.0f, 0.0f, 0.0f, 0.0f);
                any_partial |= part;
            }
            if (__builtin_amdgcn_ballot_w64(any_partial) != 0) {
#pragma unroll
                for (int q = 0; q < kPasses; ++q) {
                    const int rho = q * kRunsPerPass + r0;
                    const int rw = rho / WPW, rh = rho % WPW;     // worker-major: neighbouring lanes, neighbouring walkers
                    const int64_t off = (chunk0 + rh) * RUN;
                    const int64_t rel = nD + off;
                    int64_t len = D - off;
                    if (d - rel < len) len = d - rel;
                    if (rw >= a.nw) len = 0;
                    if (m4 + 4 > len && m4 < len) {
                        const gfloat_ptr src = gptr_lds[rw < kGroup ? rw : 0] + rel + m4;
                        pre[q].x = src[0];
                        if (m4 + 1 < len) pre[q].y = src[1];
                        if (m4 + 2 < len) pre[q].z = src[2];
                    }
                }
            }
        };

        int64_t nD = 0;
        int par = 0;                                   // which hash buffer holds this visit
        load_visit(nD);
        while (nD + chunk0 * RUN < d) {
            // values: registers -> LDS (run-major); each lane then reads its own run
#pragma unroll
            for (int q = 0; q < kPasses; ++q) {
                const int rho = q * kRunsPerPass + r0;
                float* dst = tile_lds + ((rho % WPW) * WL + rho / WPW) * kStride + m4;
                dst[0] = pre[q].x;
                dst[1] = pre[q].y;
                dst[2] = pre[q].z;
                dst[3] = pre[q].w;
            }
            // hashes of this visit: PPL consecutive coordinates from my state; the first visit
            // also fills the "previous" buffer, so that nothing looks like a left cell
            if (hash_duty) {
                uint64_t tb = yb, ts = ys;
#pragma unroll
                for (int q = 0; q < PPL; ++q) {
                    const uint32_t pk = ((static_cast<uint32_t>(tb) - 1u) & mask) | sign_flip_of(ts);
                    hash_lds[par][h * RUN + m0 + q] = pk;
                    if (nD == 0) hash_lds[par ^ 1][h * RUN + m0 + q] = pk;
                    if (q + 1 < PPL) {
                        tb = hash_advance(tb, p.a[j]);
                        ts = hash_advance(ts, p.as[j]);
                    }
                }
            }
            yb = hash_advance(yb, ADb);
            ys = hash_advance(ys, ADs);
            __builtin_amdgcn_wave_barrier();
            const float* my_run = tile_lds + lane * kStride;
            const uint32_t* now = hash_lds[par] + h * RUN;
            const uint32_t* before = hash_lds[par ^ 1] + h * RUN;
#pragma unroll
            for (int m = 0; m < RUN; ++m) {
                const uint32_t pk = now[m];
                const uint32_t cell = pk & 0x7fffffffu;
                const uint32_t was = before[m] & 0x7fffffffu;
                if (cell != was) {                         // left the cell: send its sum
                    if (acc[m] != 0.0f)
                        atomic_add_noret(Tcol + static_cast<size_t>(was) * kGroup, acc[m]);
                    acc[m] = 0.0f;
                }
                acc[m] += apply_sign(a.scale * my_run[m], pk & 0x80000000u);
            }
            __builtin_amdgcn_wave_barrier();
            // The next visit's loads are issued after this visit's atomics: the memory counter
            // retires in order, so the wait for those loads at the top of the loop also covers
            // the (older) atomics.
            nD += D;
            par ^= 1;
            if (nD + chunk0 * RUN < d) load_visit(nD);
        }
        // the cells the walkers ended in (buffer of the last visit)
        const uint32_t* last = hash_lds[par ^ 1] + h * RUN;
#pragma unroll
        for (int m = 0; m < RUN; ++m)
            if (acc[m] != 0.0f)
                atomic_add_noret(Tcol + static_cast<size_t>(last[m] & 0x7fffffffu) * kGroup, acc[m]);
        __builtin_amdgcn_wave_barrier();
    }
}

// one launch: the rows a.js[0 .. nrows-1] of one group of workers (blockIdx.y = row of the set)
template <int WL, int RUN, int NWAVE>
int launch_walk(const cs_params* p, const WalkArgs& a, int nrows, hipStream_t stream) {
    constexpr int WPW = 64 / WL;
    int64_t most = 1;
    for (int q = 0; q < nrows; ++q) {
        const int64_t chunks = (static_cast<int64_t>(p->plan[a.js[q]].Dw) + RUN - 1) / RUN;
        const int64_t nwaves = (chunks + WPW - 1) / WPW;
        const int64_t ngroups = (nwaves + NWAVE - 1) / NWAVE;
        if (ngroups > most) most = ngroups;
    }
    const int64_t cap = 256 * 64 / NWAVE;
    int64_t gx = most < cap ? most : cap;
    gx = (gx + 7) / 8 * 8;                   // the kernel deals workgroups to XCDs in eights
    const dim3 grid(static_cast<unsigned>(gx), static_cast<unsigned>(nrows));
    k_accumulate_walk<WL, RUN, NWAVE><<<grid, 64 * NWAVE, 0, stream>>>(kparams(p), a);
    return hipGetLastError() == hipSuccess ? CS_OK : CS_EHIP;
}

// ---------------------------------------------------------------------------------------
// The same update along a visit list (cs_visit_plan) instead of a single stride.
//
// The list s_0 = 0 < s_1 < ... holds every offset whose bucket advance is below a bound of
// ncell - 1 cells, so whatever a lane meets at i + s_k lies in one of the NC = ncell cells
// that start at the cell of i.  A lane therefore keeps NC running sums per coordinate of its
// run for the whole kernel and sends each to memory exactly once at the end: NC atomic
// requests per RUN-residue and worker group for the entire vector, and none inside the loop.
// Visit k covers [s_k, s_k + gap_k); the walker that owns residues [off, off + RUN) takes part
// in it when off < gap_k, so lanes own the residues below the largest gap.  Loads, the LDS
// transpose and the roles of lanes are those of the stride walk above.
// ---------------------------------------------------------------------------------------
struct VisitArgs {
    uint32_t K;                  // visits
    int32_t j;                   // sketch row
    uint64_t gmax;
    uint64_t a, b, as, bs;       // hash constants of row j
    uint64_t gap[4], A[4], As[4];
    uint32_t code[CS_MAX_VISITS / 16];
};
// The rows of a sketch are updated by one launch (blockIdx.y = row of the set): their serial
// chains of visits overlap, and there are fewer launch tails.
constexpr int kRowsPerLaunch = 8;
// Neighbouring sets of walkers that go to the same XCD (the kernel deals sets to XCDs in blocks
// of this many, so that an XCD reads a few KB of contiguous addresses per visit).  Five, not a
// power of two: with 4 sets of 2 wavefronts an XCD's block is exactly 4 KB of every vector, each
// XCD then keeps meeting the same addresses modulo 32 KB, and the update measured 1 % slower
// (1, 2, 4, 16: slower; 3, 5, 6, 8: within 0.5 % of each other).
constexpr int kVisitSetBlock = 5;
struct VisitRows {
    VisitArgs row[kRowsPerLaunch];
    __device__ __forceinline__ const VisitArgs& at(unsigned y) const { return row[y]; }
};
// The list of one row when the column count is not a power of two (cs_anyc_plan): the gaps visit
// by visit.  The hash advances (a_j gap_k) mod p and (a'_j gap_k) mod p do not travel with it:
// every workgroup computes them once into LDS, so that several rows' lists fit into the 4 KB of
// kernel arguments and share a launch.
struct VisitGaps {
    uint32_t K;
    int32_t j;
    uint64_t gmax;
    uint64_t a, b, as, bs;
    uint32_t omega;              // running sums: omega cells from the first one, omega more after a wrap
    uint32_t pc;                 // p mod c: how far back a wrap past p sets the bucket
    uint32_t gap[CS_ANYC_MAX_VISITS];
};
constexpr int kAnycRowsPerLaunch = 6;
struct VisitGapsRows {
    VisitGaps row[kAnycRowsPerLaunch];
    __device__ __forceinline__ const VisitGaps& at(unsigned y) const { return row[y]; }
};
static_assert(sizeof(VisitGapsRows) + 128 <= 4096, "the lists of a launch and its other arguments are kernel arguments");
struct VisitWorkers {
    const float* g[kGroup];      // vectors of the workers of this group
    float* T;                    // the group's table, float[r][c][kGroup]; with `fold` one table float[r][c]
    int64_t d, i0;
    uint32_t c;
    int32_t nw;                  // workers in this group (<= kGroup)
    float scale;
    int32_t fold;                // != 0: the workers' sums of a cell are added up across the lanes
                                 // of a walker and leave as one 4-byte request into a single table
};


typedef float vec2f __attribute__((ext_vector_type(2)));
typedef vec2f __attribute__((aligned(4))) vec2f_u;            // 8 bytes at any dword address
typedef const __attribute__((address_space(1))) vec2f_u* gvec2_ptr;

// N consecutive floats from global memory at any dword address, as the widest requests
template <int N>
__device__ __forceinline__ void load_floats(gfloat_ptr src, float (&out)[N]) {
    static_assert(N == 2 || N % 4 == 0, "pieces of 2, 4, 8 or 16 floats");
    if constexpr (N == 2) {
        const vec2f u = *(gvec2_ptr)src;
        out[0] = u.x;
        out[1] = u.y;
    } else {
#pragma unroll
        for (int t = 0; t < N; t += 4) {
            const vec4f u = *(gvec4_ptr)(src + t);
            out[t] = u.x;
            out[t + 1] = u.y;
            out[t + 2] = u.z;
            out[t + 3] = u.w;
        }
    }
}

// LIST = VisitRows (power-of-two column counts: three gaps and 2-bit codes, the NC cells are
// neighbours) or VisitGapsRows (any column count: gaps one by one, NC = 2 omega cells of which
// the second half lies p mod c cells back).
template <int WL, int RUN, int NWAVE, int NC, typename LIST>
__global__ void __launch_bounds__(64 * NWAVE)
k_accumulate_visits(LIST rows, VisitWorkers a) {
    constexpr bool POW2 = std::is_same<LIST, VisitRows>::value;
    const auto& v = rows.at(blockIdx.y);
    constexpr int WPW = 64 / WL;                       // walkers per wavefront
    constexpr int PPL = RUN / WL;                      // hash values each lane computes
    constexpr int FPL = RUN / WL;                      // floats each lane requests per worker
    constexpr int SPAN = WPW * RUN;                    // residues a wavefront owns
    constexpr int kStride = RUN + 1;
    constexpr int kSetBlock = kVisitSetBlock;          // neighbouring walker sets per XCD turn
    constexpr int kRec = NC == 2 ? 2 : 4;              // words of a coordinate's record
    // records of one walker, padded by one record: the 8 lanes of a walker read the same record
    // (a broadcast), the walkers of a wavefront different ones, which without the pad would
    // all start in the same LDS bank
    constexpr int kRecWalker = (RUN + 1) * kRec;
    static_assert(WL <= 8 && WL * PPL == RUN, "every coordinate of a walker gets a hash lane");
    static_assert(NC >= 2 && NC <= 4, "two to four running sums");
    // Per wavefront: the value tile (one padded row per lane), one record per coordinate of
    // every walker (sign word, then one all-ones / all-zeros word per cell but the last,
    // telling which running sum the coordinate belongs to in this visit), the walkers' first
    // cells, and the (bucket | sign) words of the stride walk, for the fallback.
    __shared__ float tile_lds_all[NWAVE][64 * kStride];
    __shared__ __attribute__((aligned(16))) uint32_t rec_lds_all[NWAVE][WPW * kRecWalker];
    __shared__ uint32_t first_lds_all[NWAVE][SPAN];
    __shared__ uint32_t raw_lds_all[NWAVE][SPAN];

    const int lane = threadIdx.x & 63;
    const int wq = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // wavefront-uniform
    float* tile_lds = tile_lds_all[wq];
    uint32_t* rec_lds = rec_lds_all[wq];
    uint32_t* first_lds = first_lds_all[wq];
    uint32_t* raw_lds = raw_lds_all[wq];
    const int h = lane / WL, wl = lane % WL;
    const int nw = a.nw;
    const bool live = wl < nw;                          // my worker exists

    const int64_t chunks = (static_cast<int64_t>(v.gmax) + RUN - 1) / RUN;
    const int64_t nwaves = (chunks + WPW - 1) / WPW;
    const uint32_t mask = a.c - 1u;
    const Columns col = columns_of<POW2>(a.c);
    const int64_t d = a.d;
    const bool fold = a.fold != 0;
    const size_t cell_floats = fold ? 1 : kGroup;      // floats from one cell to the next
    float* __restrict__ Tcol = fold ? a.T + static_cast<size_t>(v.j) * a.c
                                    : a.T + static_cast<size_t>(v.j) * a.c * kGroup + wl;
    // which running sum a coordinate now in `cell` belongs to, given the cell it started in;
    // >= NC: none of them (never with a list of cs_params_init)
    auto sum_of = [&](uint32_t cell, uint32_t first) -> uint32_t {
        if constexpr (POW2) {
            return (cell - first) & mask;
        } else {
            const uint32_t c = a.c, omega = v.omega;
            const uint32_t t = cell >= first ? cell - first : cell + c - first;    // (cell - first) mod c
            if (t < omega) return t;
            const uint32_t t2 = t + v.pc >= c ? t + v.pc - c : t + v.pc;            // after a wrap past p
            return t2 < omega ? omega + t2 : static_cast<uint32_t>(NC);
        }
    };
    // the cell of running sum q of a coordinate that started in cell `first`
    auto cell_of_sum = [&](uint32_t first, int q) -> uint32_t {
        if constexpr (POW2) {
            return (first + static_cast<uint32_t>(q)) & mask;
        } else {
            const uint32_t c = a.c, omega = v.omega;
            uint32_t x = static_cast<uint32_t>(q) < omega ? first + q : first + (q - omega) + (c - v.pc);
            return x >= c ? x - c : x;
        }
    };
    const int m0 = wl * PPL;                           // hash role: coordinates m0 .. m0 + PPL - 1
    float* my_row = tile_lds + lane * kStride;         // consumer role: my walker's run of my worker
    const uint32_t* my_rec = rec_lds + h * kRecWalker;
    uint32_t* rec_dst = rec_lds + h * kRecWalker + m0 * kRec;
    const uint64_t Aj = v.a, Asj = v.as;
    // loader role: floats lspan .. lspan + FPL - 1 of the wavefront's span, of every worker;
    // they belong to walker lspan / RUN and go to that walker's row of each worker
    // With 8 workers and 8-byte pieces, two workers share a request instead: the lower 32 lanes
    // take 16 bytes each of one worker's 512-byte span, the upper 32 lanes of the next worker's.
    // Same bytes and the same time, but half the load instructions and half the address
    // registers (16 VGPRs fewer).
    constexpr bool PAIR = WL == 8 && FPL == 2;
    constexpr int kLoads = PAIR ? WL / 2 : WL;         // load instructions per visit
    constexpr int kPer = PAIR ? 2 * FPL : FPL;         // floats per lane and instruction
    const int half = PAIR ? lane >> 5 : 0;
    const int lspan = PAIR ? (lane & 31) * kPer : lane * FPL;
    float* tile_dst = tile_lds + ((lspan / RUN) * WL + half) * kStride + lspan % RUN;
    constexpr int kRowStep = PAIR ? 2 * kStride : kStride;   // tile rows between my loads
    // gap and hash advances of visit k.  Power-of-two lists: three gaps and the cut last one
    // live in scalar registers and a 2-bit code per visit picks among them; other lists are
    // read visit by visit from the kernel arguments.
    auto pick = [](uint32_t code, uint64_t x0, uint64_t x1, uint64_t x2, uint64_t x3) {
        return code == 0u ? x0 : code == 1u ? x1 : code == 2u ? x2 : x3;
    };
    auto code_of = [&](uint32_t k) -> uint32_t {
        if constexpr (POW2) return (v.code[k >> 4] >> ((k & 15u) * 2u)) & 3u;
        else return k;
    };
    auto gap_of = [&](uint32_t code) -> int64_t {
        if constexpr (POW2) return static_cast<int64_t>(pick(code, v.gap[0], v.gap[1], v.gap[2], v.gap[3]));
        else return static_cast<int64_t>(v.gap[code]);
    };
    // hash advances of the visits of an any-c list: once per workgroup into LDS
    __shared__ uint64_t adv_b[POW2 ? 1 : CS_ANYC_MAX_VISITS], adv_s[POW2 ? 1 : CS_ANYC_MAX_VISITS];
    if constexpr (!POW2) {
        for (uint32_t k = threadIdx.x; k < v.K; k += 64 * NWAVE) {
            adv_b[k] = mulmod_p(v.a, v.gap[k]);
            adv_s[k] = mulmod_p(v.as, v.gap[k]);
        }
        __syncthreads();
    }
    auto A_of = [&](uint32_t code) -> uint64_t {
        if constexpr (POW2) return pick(code, v.A[0], v.A[1], v.A[2], v.A[3]);
        else return adv_b[code];
    };
    auto As_of = [&](uint32_t code) -> uint64_t {
        if constexpr (POW2) return pick(code, v.As[0], v.As[1], v.As[2], v.As[3]);
        else return adv_s[code];
    };

    // Walkers with small residues take part in every visit, those with large ones only in
    // the visits with the largest gap, so the sets of walkers are dealt to the XCDs in short
    // blocks rather than as eight long ranges: every XCD gets the same mix.
    const int64_t ngroups = (nwaves + NWAVE - 1) / NWAVE;
    for (int64_t vi = blockIdx.x; ; vi += gridDim.x) {
        const int64_t slot = vi >> 3;
        const int64_t set = ((slot / kSetBlock) * 8 + (vi & 7)) * kSetBlock + slot % kSetBlock;
        if ((slot / kSetBlock) * 8 * kSetBlock >= ngroups) break;
        const int64_t wv = set * NWAVE + wq;
        if (set >= ngroups || wv >= nwaves) continue;
        const int64_t first_res = wv * SPAN;           // first residue of this wavefront's walkers
        uint64_t yb = hash_state(v.a, v.b, static_cast<uint64_t>(a.i0 + first_res + h * RUN + m0));
        uint64_t ys = hash_state(v.as, v.bs, static_cast<uint64_t>(a.i0 + first_res + h * RUN + m0));

        // the cells my coordinates start in (visit 0, whether or not I take part in it)
        uint32_t first_cell[PPL];
        {
            uint64_t tb = yb;
#pragma unroll
            for (int q = 0; q < PPL; ++q) {
                first_cell[q] = bucket_of<POW2>(tb, col);
                first_lds[h * RUN + m0 + q] = first_cell[q];
                if (q + 1 < PPL) tb = hash_advance(tb, Aj);
            }
        }

        float acc[NC][RUN];
#pragma unroll
        for (int q = 0; q < NC; ++q)
#pragma unroll
            for (int m = 0; m < RUN; ++m) acc[q][m] = 0.0f;

        // Requests of the visit at offset s.  `room` = residues from first_res on that belong
        // to the visit and exist; when the whole span does, every piece is whole and needs no
        // check (one wavefront-uniform base per worker plus a fixed lane offset).  Otherwise
        // pieces are cut where the visit or the vector ends, and missing values count as 0.
        float pre[kLoads][kPer];
        // the vector that load instruction `w` of this lane reads
        auto vector_of = [&](int w) -> gfloat_ptr {
            if constexpr (PAIR) {
                const float* lo = a.g[2 * w < nw ? 2 * w : 0];
                const float* hi = a.g[2 * w + 1 < nw ? 2 * w + 1 : 0];
                return (gfloat_ptr)(half ? hi : lo);
            } else {
                return (gfloat_ptr)a.g[w < nw ? w : 0];
            }
        };
        auto load_visit = [&](int64_t s, int64_t room) {
            if (room >= SPAN) {
#pragma unroll
                for (int w = 0; w < kLoads; ++w)
                    load_floats<kPer>(vector_of(w) + (first_res + s) + lspan, pre[w]);
            } else {
                const int len = static_cast<int>(room) - lspan;    // of my piece: >= kPer whole, <= 0 none
#pragma unroll
                for (int w = 0; w < kLoads; ++w) {
                    const gfloat_ptr src = vector_of(w) + (first_res + s) + lspan;
#pragma unroll
                    for (int t = 0; t < kPer; ++t) pre[w][t] = 0.0f;
                    if (len >= kPer) {
                        load_floats<kPer>(src, pre[w]);
                    } else {
#pragma unroll
                        for (int t = 0; t < kPer; ++t)
                            if (t < len) pre[w][t] = src[t];
                    }
                }
            }
        };
        // room of the visit with gap `gap` at offset s; > 0 means this wavefront takes part
        auto room_of = [&](int64_t s, int64_t gap) {
            const int64_t in_gap = gap - first_res, in_vec = d - s - first_res;
            return in_gap < in_vec ? in_gap : in_vec;
        };

        int64_t s = 0;                                 // offset of visit k
        uint32_t code = code_of(0);
        bool active = room_of(0, gap_of(code)) > 0;
        if (active) load_visit(0, room_of(0, gap_of(code)));
        for (uint32_t k = 0; k < v.K; ++k) {
            // visit k: its values are on their way (requested one turn earlier)
            const bool was_active = active;
            if (was_active) {
#pragma unroll
                for (int w = 0; w < kLoads; ++w)
#pragma unroll
                    for (int t = 0; t < kPer; ++t) tile_dst[w * kRowStep + t] = pre[w][t];
            }
            // request visit k + 1 as soon as the registers of visit k are free, to fly while
            // visit k is hashed and added up
            const uint32_t code_k = code;
            s += gap_of(code_k);
            active = false;
            if (k + 1 < v.K) {
                code = code_of(k + 1);
                const int64_t room = room_of(s, gap_of(code));
                active = room > 0;
                if (active) load_visit(s, room);
            }
            bool bad = false;
            if (was_active) {
                uint64_t tb = yb, ts = ys;
#pragma unroll
                for (int q = 0; q < PPL; ++q) {
                    const uint32_t cell = bucket_of<POW2>(tb, col);
                    const uint32_t rel = sum_of(cell, first_cell[q]);
                    const uint32_t flip = sign_flip_of(ts);
                    bad |= rel >= static_cast<uint32_t>(NC);
                    if (NC == 2) {
                        *reinterpret_cast<uint2*>(rec_dst + q * kRec) =
                            make_uint2(flip, rel == 0u ? ~0u : 0u);
                    } else {
                        *reinterpret_cast<uint4*>(rec_dst + q * kRec) = make_uint4(
                            flip, rel == 0u ? ~0u : 0u, rel == 1u ? ~0u : 0u, rel == 2u ? ~0u : 0u);
                    }
                    if (q + 1 < PPL) {
                        tb = hash_advance(tb, Aj);
                        ts = hash_advance(ts, Asj);
                    }
                }
            }
            // A coordinate outside the NC cells cannot happen with a list built by
            // cs_params_init; the check is kept so that a wrong list costs time, never
            // correctness: such a visit's values go to memory one by one, and the tile is
            // cleared so that the sums below take nothing from it.
            const bool stray = was_active && __builtin_amdgcn_ballot_w64(bad) != 0;
            if (stray) {
                uint64_t tb = yb, ts = ys;
#pragma unroll
                for (int q = 0; q < PPL; ++q) {
                    raw_lds[h * RUN + m0 + q] = bucket_of<POW2>(tb, col) | sign_flip_of(ts);
                    if (q + 1 < PPL) {
                        tb = hash_advance(tb, Aj);
                        ts = hash_advance(ts, Asj);
                    }
                }
            }
            yb = hash_advance(yb, A_of(code_k));
            ys = hash_advance(ys, As_of(code_k));
            __builtin_amdgcn_wave_barrier();
            if (stray) {
                const uint32_t* raw = raw_lds + h * RUN;
#pragma unroll
                for (int m = 0; m < RUN; ++m) {
                    const uint32_t pk = raw[m];
                    const float val = apply_sign(a.scale * my_row[m], pk & 0x80000000u);
                    if (live && val != 0.0f)
                        atomic_add_noret(Tcol + static_cast<size_t>(pk & 0x7fffffffu) * cell_floats, val);
                    my_row[m] = 0.0f;
                }
            }
            if (was_active) {
#pragma unroll
                for (int m = 0; m < RUN; ++m) {
                    if (NC == 2) {
                        const uint2 rec = *reinterpret_cast<const uint2*>(my_rec + m * kRec);
                        const uint32_t bits = __float_as_uint(my_row[m]) ^ rec.x;
                        const uint32_t t0 = bits & rec.y;
                        acc[0][m] += __uint_as_float(t0);
                        acc[1][m] += __uint_as_float(bits ^ t0);
                    } else {
                        const uint4 rec = *reinterpret_cast<const uint4*>(my_rec + m * kRec);
                        const uint32_t bits = __float_as_uint(my_row[m]) ^ rec.x;
                        const uint32_t t0 = bits & rec.y, t1 = bits & rec.z;
                        acc[0][m] += __uint_as_float(t0);
                        acc[1][m] += __uint_as_float(t1);
                        if (NC == 3) {
                            acc[2][m] += __uint_as_float(bits ^ t0 ^ t1);
                        } else {
                            const uint32_t t2 = bits & rec.w;
                            acc[2][m] += __uint_as_float(t2);
                            acc[NC - 1][m] += __uint_as_float(bits ^ t0 ^ t1 ^ t2);
                        }
                    }
                    // keeps the LDS reads of later coordinates from being hoisted over the sums
                    // of earlier ones, which would cost a register per read in flight
                    if (m % 4 == 3) __builtin_amdgcn_sched_barrier(0);
                }
            }
            __builtin_amdgcn_wave_barrier();
        }
        // every running sum goes to memory once
        const uint32_t* first = first_lds + h * RUN;
#pragma unroll
        for (int m = 0; m < RUN; ++m) {
            const uint32_t c0 = first[m];
#pragma unroll
            for (int q = 0; q < NC; ++q) {
                if (!fold) {
                    if (live && acc[q][m] != 0.0f)
                        atomic_add_noret(Tcol + static_cast<size_t>(cell_of_sum(c0, q)) * kGroup,
                                         a.scale * acc[q][m]);
                } else {
                    // the WL lanes of my walker hold the same cell's sums of the WL workers
                    float sum = live ? acc[q][m] : 0.0f;
#pragma unroll
                    for (int off = 1; off < WL; off <<= 1) sum += __shfl_xor(sum, off);
                    if (wl == 0 && sum != 0.0f)
                        atomic_add_noret(Tcol + cell_of_sum(c0, q), a.scale * sum);
                }
            }
        }
        __builtin_amdgcn_wave_barrier();
    }
}

// one launch: the rows `js` (all with ncell running sums) of one group of workers
template <int WL, int RUN, int NWAVE>
int launch_visits(const cs_params* p, const VisitWorkers& a, const uint32_t* js, int nrows,
                  uint32_t ncell, hipStream_t stream) {
    constexpr int WPW = 64 / WL;
    VisitRows rows{};
    int64_t most = 1;
    for (int q = 0; q < nrows; ++q) {
        const uint32_t j = js[q];
        const cs_visit_plan& vp = p->visit[j];
        VisitArgs& v = rows.row[q];
        v.K = vp.K;
        v.j = static_cast<int32_t>(j);
        v.gmax = vp.gmax;
        v.a = p->a[j]; v.b = p->b[j]; v.as = p->as[j]; v.bs = p->bs[j];
        for (int t = 0; t < 4; ++t) { v.gap[t] = vp.gap[t]; v.A[t] = vp.A[t]; v.As[t] = vp.As[t]; }
        for (int t = 0; t < CS_MAX_VISITS / 16; ++t) v.code[t] = vp.code[t];
        const int64_t chunks = (static_cast<int64_t>(vp.gmax) + RUN - 1) / RUN;
        const int64_t nwaves = (chunks + WPW - 1) / WPW;
        const int64_t ngroups = (nwaves + NWAVE - 1) / NWAVE;
        if (ngroups > most) most = ngroups;
    }
    const int64_t cap = 256 * 64 / NWAVE;
    int64_t gx = most < cap ? most : cap;
    // the kernel deals sets to the 8 XCDs in blocks of kVisitSetBlock: whole blocks, so that
    // no workgroup takes a second set
    gx = (gx + 8 * kVisitSetBlock - 1) / (8 * kVisitSetBlock) * (8 * kVisitSetBlock);
    const dim3 grid(static_cast<unsigned>(gx), static_cast<unsigned>(nrows)), block(64 * NWAVE);
    switch (ncell) {
        case 2: k_accumulate_visits<WL, RUN, NWAVE, 2, VisitRows><<<grid, block, 0, stream>>>(rows, a); break;
        case 3: k_accumulate_visits<WL, RUN, NWAVE, 3, VisitRows><<<grid, block, 0, stream>>>(rows, a); break;
        case 4: k_accumulate_visits<WL, RUN, NWAVE, 4, VisitRows><<<grid, block, 0, stream>>>(rows, a); break;
        default: return CS_EINVAL;
    }
    return hipGetLastError() == hipSuccess ? CS_OK : CS_EHIP;
}

// the visit list of row j serves vectors of length d, and (unless any_cost) is expected to take
// less time than the stride walk
bool visits_apply(const cs_params* p, uint32_t j, int64_t d, bool any_cost = false) {
    const cs_visit_plan& vp = p->visit[j];
    if ((p->flags & CS_FLAG_NO_VISIT_LIST) != 0 || vp.K == 0) return false;
    if (vp.ncell < 2 || vp.ncell > 4 || vp.K > CS_MAX_VISITS) return false;
    if (static_cast<uint64_t>(d) > vp.cover) return false;
    return any_cost || vp.cost < vp.cost_walk;
}

void fill_visit_gaps(const cs_params* p, uint32_t j, VisitGaps& v) {
    const cs_anyc_plan& vp = p->anyc[j];
    v.K = vp.K;
    v.j = static_cast<int32_t>(j);
    v.gmax = vp.gmax;
    v.a = p->a[j]; v.b = p->b[j]; v.as = p->as[j]; v.bs = p->bs[j];
    v.omega = vp.omega;
    v.pc = static_cast<uint32_t>(kP61 % p->c);
    for (uint32_t k = 0; k < vp.K; ++k) v.gap[k] = vp.gap[k];
}

// The rows of an any-c sketch in the launches that take them: rows with the same number of
// running sums (omega = 1 or 2) together, up to kAnycRowsPerLaunch per launch, the longest lists
// first.  fn(rows, n, omega) is called per launch.
template <typename FN>
int for_each_anyc_launch(const cs_params* p, uint32_t nrows_of_sketch, FN fn) {
    for (uint32_t omega = 1; omega <= 2; ++omega) {
        uint32_t order[CS_MAX_R];
        int n = 0;
        for (uint32_t j = 0; j < nrows_of_sketch; ++j) {
            if (p->anyc[j].omega != omega) continue;
            int at = n++;
            for (; at > 0 && p->anyc[order[at - 1]].K < p->anyc[j].K; --at) order[at] = order[at - 1];
            order[at] = j;
        }
        for (int q0 = 0; q0 < n; q0 += kAnycRowsPerLaunch) {
            const int m = n - q0 < kAnycRowsPerLaunch ? n - q0 : kAnycRowsPerLaunch;
            const int rc = fn(order + q0, m, omega);
            if (rc != CS_OK) return rc;
        }
    }
    return CS_OK;
}

// one launch: rows js[0 .. n) (all with the same omega) of one group of workers, each along
// its list for any column count
template <int WL, int RUN, int NWAVE>
int launch_visits_anyc(const cs_params* p, const VisitWorkers& a, const uint32_t* js, int n,
                       uint32_t omega, hipStream_t stream) {
    constexpr int WPW = 64 / WL;
    VisitGapsRows rows{};
    int64_t most = 1;
    for (int q = 0; q < n; ++q) {
        fill_visit_gaps(p, js[q], rows.row[q]);
        const int64_t chunks = (static_cast<int64_t>(p->anyc[js[q]].gmax) + RUN - 1) / RUN;
        const int64_t nwaves = (chunks + WPW - 1) / WPW;
        const int64_t ngroups = (nwaves + NWAVE - 1) / NWAVE;
        if (ngroups > most) most = ngroups;
    }
    const int64_t cap = 256 * 64 / NWAVE;
    int64_t gx = most < cap ? most : cap;
    gx = (gx + 8 * kVisitSetBlock - 1) / (8 * kVisitSetBlock) * (8 * kVisitSetBlock);
    const dim3 grid(static_cast<unsigned>(gx), static_cast<unsigned>(n)), block(64 * NWAVE);
    if (omega == 1) k_accumulate_visits<WL, RUN, NWAVE, 2, VisitGapsRows><<<grid, block, 0, stream>>>(rows, a);
    else if (omega == 2) k_accumulate_visits<WL, RUN, NWAVE, 4, VisitGapsRows><<<grid, block, 0, stream>>>(rows, a);
    else return CS_EINVAL;
    return hipGetLastError() == hipSuccess ? CS_OK : CS_EHIP;
}

}  // namespace

// Every row has a list for this column count and vector length, and by its own estimate the
// list beats one request per coordinate.
bool anyc_visits_apply(const cs_params* p, int64_t d) {
    if (p->c_pow2 || (p->flags & CS_FLAG_NO_VISIT_LIST) != 0) return false;
    for (uint32_t j = 0; j < p->r; ++j) {
        const cs_anyc_plan& vp = p->anyc[j];
        if (vp.K == 0 || vp.K > CS_ANYC_MAX_VISITS || (vp.omega != 1 && vp.omega != 2)) return false;
        if (static_cast<uint64_t>(d) > vp.cover || vp.cost >= vp.cost_direct) return false;
    }
    return true;
}

// The query follows the lists when there is enough of it: one launch per row with short chains
// of visits loses to r gathers per coordinate on small inputs (measured: 5 rows over 6.5 M
// coordinates 0.19 against 0.15 ms, 15 rows over 6.5 M 0.59 against 0.90 ms).
bool anyc_visits_serve_query(const cs_params* p, int64_t d) {
    return anyc_visits_apply(p, d) && d * static_cast<int64_t>(p->r - 1) >= (static_cast<int64_t>(1) << 26);
}

int count_accumulate_anyc_launches(const cs_params* p, int W) {
    int per_group = 0;
    for_each_anyc_launch(p, p->r, [&](const uint32_t*, int, uint32_t) { ++per_group; return CS_OK; });
    return per_group * ((W + kGroup - 1) / kGroup);
}

// Per group of 8 workers one launch for up to kAnycRowsPerLaunch rows: every row has its own
// visiting order, so the group's vectors are read once per row (where the direct form reads them
// once in all but sends d requests per row to the atomic unit, which is what bounds it); rows
// that share a launch overlap their serial chains of visits and have one tail.
int launch_accumulate_anyc(const cs_params* p, float* T, int W, const float* const* g_w,
                           int64_t d, int64_t i0, float scale, bool fold, hipStream_t stream) {
    const size_t row_floats = static_cast<size_t>(p->c) * kGroup;
    for (int w0 = 0; w0 < W; w0 += kGroup) {
        const int nw = (W - w0 < kGroup) ? (W - w0) : kGroup;
        VisitWorkers vw{};
        for (int w = 0; w < nw; ++w) vw.g[w] = g_w[w0 + w];
        vw.T = fold ? T : T + static_cast<size_t>(w0 / kGroup) * p->r * row_floats;
        vw.d = d;
        vw.i0 = i0;
        vw.c = p->c;
        vw.nw = nw;
        vw.scale = scale;
        vw.fold = fold ? 1 : 0;
        const int rc = for_each_anyc_launch(p, p->r, [&](const uint32_t* js, int n, uint32_t omega) {
            if (nw > 4) return launch_visits_anyc<8, 16, kWavesPerGroupOf8>(p, vw, js, n, omega, stream);
            if (nw > 2) return launch_visits_anyc<4, 16, 1>(p, vw, js, n, omega, stream);
            if (nw > 1) return launch_visits_anyc<2, 16, 1>(p, vw, js, n, omega, stream);
            return launch_visits_anyc<1, 16, 1>(p, vw, js, n, omega, stream);
        });
        if (rc != CS_OK) return rc;
    }
    return CS_OK;
}

bool walk_applies(const cs_params* p, int64_t d) {
    if (!p->c_pow2 || p->c < 64 || d < 4096) return false;
    for (uint32_t j = 0; j < p->r; ++j)
        if (p->plan[j].Dw <= 1) return false;
    return true;
}

// kernel launches one call of launch_accumulate_walk makes (same grouping as below)
int count_accumulate_walk_launches(const cs_params* p, int W, int64_t d) {
    int listed = 0, per_group = 0;
    for (uint32_t j = 0; j < p->r; ++j) {
        if (visits_apply(p, j, d)) ++listed;
        else ++per_group;
    }
    const int launches = (listed + kRowsPerLaunch - 1) / kRowsPerLaunch + (per_group > 0 ? 1 : 0);
    return launches * ((W + kGroup - 1) / kGroup);
}

// every row of the sketch has a visit list for vectors of length d (what the folded form of
// the update needs: only the list kernel adds the workers up before it writes; a list that the
// time model likes less than the stride walk is used all the same)
bool all_rows_listed(const cs_params* p, int64_t d) {
    if (!walk_applies(p, d)) return false;
    for (uint32_t j = 0; j < p->r; ++j)
        if (!visits_apply(p, j, d, true)) return false;
    return true;
}

// fold: T is one table float[r][c] that receives the sum over all W workers (all_rows_listed
// must hold); otherwise T is the bundle and every worker has its own slot.
int launch_accumulate_walk(const cs_params* p, float* T, int W, const float* const* g_w,
                           int64_t d, int64_t i0, float scale, bool fold, hipStream_t stream) {
    if (fold && !all_rows_listed(p, d)) return CS_EINVAL;
    const size_t row_floats = static_cast<size_t>(p->c) * kGroup;
    for (int w0 = 0; w0 < W; w0 += kGroup) {
        const int nw = (W - w0 < kGroup) ? (W - w0) : kGroup;
        float* Tg = fold ? T : T + static_cast<size_t>(w0 / kGroup) * p->r * row_floats;
        VisitWorkers vw{};
        for (int w = 0; w < nw; ++w) vw.g[w] = g_w[w0 + w];
        vw.T = Tg;
        vw.d = d;
        vw.i0 = i0;
        vw.c = p->c;
        vw.nw = nw;
        vw.scale = scale;
        vw.fold = fold ? 1 : 0;
        // All rows with a visit list go into one launch (per 8 rows), compiled for the largest
        // number of running sums among them: a row that needs fewer simply never touches the
        // extra ones.  One launch overlaps the rows' serial chains of visits and has one tail.
        // Rows with the longest lists go first: workgroups are started in order, so the launch
        // then ends on the wavefronts that live shortest and the chip drains quickly (measured
        // against the rows in index order: 1.5 % at d = 100 M with 5 rows, 4 % at d = 25 M
        // with 7; the opposite order costs as much again).
        uint32_t ncell = 2;
        uint32_t listed[CS_MAX_R];
        int nlisted = 0;
        for (uint32_t j = 0; j < p->r; ++j) {
            if (!visits_apply(p, j, d, fold)) continue;
            if (p->visit[j].ncell > ncell) ncell = p->visit[j].ncell;
            int at = nlisted++;
            for (; at > 0 && p->visit[listed[at - 1]].K < p->visit[j].K; --at) listed[at] = listed[at - 1];
            listed[at] = j;
        }
        for (int q0 = 0; q0 < nlisted; q0 += kRowsPerLaunch) {
            const int nrows = nlisted - q0 < kRowsPerLaunch ? nlisted - q0 : kRowsPerLaunch;
            const uint32_t* js = listed + q0;
            int rc;
            if (nw > 4) rc = launch_visits<8, 16, kWavesPerGroupOf8>(p, vw, js, nrows, ncell, stream);
            else if (nw > 2) rc = launch_visits<4, 16, 1>(p, vw, js, nrows, ncell, stream);
            else if (nw > 1) rc = launch_visits<2, 16, 1>(p, vw, js, nrows, ncell, stream);
            else rc = launch_visits<1, 16, 1>(p, vw, js, nrows, ncell, stream);
            if (rc != CS_OK) return rc;
        }
        // the other rows: stride walk, all in one launch, the longest chains of visits
        // (smallest strides) first
        WalkArgs a{};
        a.nw = nw;
        for (int w = 0; w < nw; ++w) a.g[w] = g_w[w0 + w];
        a.T = Tg;
        a.d = d;
        a.i0 = i0;
        a.scale = scale;
        int nwalked = 0;
        for (uint32_t j = 0; j < p->r; ++j) {
            if (visits_apply(p, j, d, fold)) continue;
            int at = nwalked++;
            for (; at > 0 && p->plan[a.js[at - 1]].Dw > p->plan[j].Dw; --at) a.js[at] = a.js[at - 1];
            a.js[at] = static_cast<int32_t>(j);
        }
        if (nwalked > 0) {
            int rc;
            if (nw > 4) rc = launch_walk<8, 16, kWavesPerGroupOf8>(p, a, nwalked, stream);
            else if (nw > 2) rc = launch_walk<4, 16, 1>(p, a, nwalked, stream);
            else if (nw > 1) rc = launch_walk<2, 16, 1>(p, a, nwalked, stream);
            else rc = launch_walk<1, 16, 1>(p, a, nwalked, stream);
            if (rc != CS_OK) return rc;
        }
    }
    return CS_OK;
}

// ---------------------------------------------------------------------------------------
// Alg. 4 estimate, walk order: rows[j][i] = s_j(i) S[j][h_j(i)] for every coordinate.
//
// The same stride serves the query: a lane that walks i, i + Dw, i + 2 Dw, ... stays in one
// cell for ~1/sigma visits, so it keeps that cell's value in a register and gathers again
// only when it leaves the cell (one gather per ~10 coordinates instead of one per
// coordinate).  The 64 lanes of a wavefront own 64 neighbouring chunks of 4 residues, so
// every visit writes 1 KB of contiguous output, 16 bytes per lane.  A second kernel takes the
// median over rows.
// ---------------------------------------------------------------------------------------
namespace {

// Coordinates per lane and visit.  Four: a lane's values are one 16-byte piece of output, so no
// transpose is needed, and the registers that 16 coordinates took (cell and value of each) are
// better spent on twice as many resident wavefronts -- the kernel waits on its gathers.
constexpr int kQRun = 4;

// A short vector leaves a row with few chunks (Dw / 256 wavefronts) and a long serial chain
// of visits each; the chain is then cut into segments that separate wavefronts walk
// (blockIdx.z), at the price of one more gather per lane and segment.
struct RowSegments {
    int n[CS_MAX_R];
};

// RF = 0: rows[j][i] for the rows j = blockIdx.y.  RF = R (the row count): the walk of the last
// row, which instead of storing its values reads those of rows 0 .. R-2 at the same coordinates
// and writes their median, est[i] -- the last row never goes through memory.
// HIST (with RF > 0): the kernel also counts the estimates it writes by the top 11 bits of their
// magnitude (bits 30..20 of the binary32 pattern) into hist[2048], which is the first
// histogram of the selection that follows (Sec. 5.2: query every coordinate, keep the
// largest): one read of est less.  Counts are kept per workgroup in LDS and added to hist at
// the end; a workgroup of kHistWaves wavefronts shares one set of counters (8 KB), so that LDS
// does not limit how many wavefronts a CU holds.
constexpr int kHistWaves = 4;
template <int RF, bool HIST>
__global__ void __launch_bounds__(HIST ? 64 * kHistWaves : 64)
k_row_values_walk(KParams p, RowSegments segs, const float* __restrict__ S, int64_t d, int64_t i0,
                  float* __restrict__ rows, float* __restrict__ est,
                  unsigned long long* __restrict__ hist) {
    static_assert(kQRun == 4, "one 16-byte piece per lane");
    static_assert(!HIST || RF > 0, "only the kernel that writes est can count it");
    constexpr int NW = HIST ? kHistWaves : 1;          // wavefronts per workgroup
    const int lane = threadIdx.x & 63;
    const int wq = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int j = RF ? RF - 1 : blockIdx.y;
    const int nseg = segs.n[j];
    if (static_cast<int>(blockIdx.z) >= nseg) return;
    __shared__ uint32_t lh[HIST ? 2048 : 1];
    if (HIST) {
        for (int t = threadIdx.x; t < 2048; t += 64 * NW) lh[t] = 0;
        __syncthreads();
    }
    auto tally = [&](float v) {
        if (HIST) atomicAdd(&lh[(__float_as_uint(v) & 0x7fffffffu) >> 20], 1u);
    };
    const int64_t D = static_cast<int64_t>(p.plan[j].Dw);
    const int64_t visits = (d + D - 1) / D;
    const int64_t nD0 = visits * blockIdx.z / nseg * D;          // my segment of the chain
    const int64_t nD1 = visits * (blockIdx.z + 1) / nseg * D;
    const uint64_t ADb = p.plan[j].ADw, ADs = p.plan[j].ADws;
    const uint64_t Ab = p.a[j], As = p.as[j];
    const int64_t chunks = (D + kQRun - 1) / kQRun;
    const int64_t nwaves = (chunks + 63) / 64;
    const uint32_t mask = p.c - 1u;
    const float* __restrict__ Sj = S + static_cast<size_t>(j) * p.c;
    float* __restrict__ out = rows + static_cast<size_t>(j) * d;

    const int64_t per_xcd = (nwaves + 7) / 8;
    const int64_t xcd_first = static_cast<int64_t>(blockIdx.x & 7) * per_xcd;
    for (int64_t k = static_cast<int64_t>(blockIdx.x >> 3) * NW + wq; k < per_xcd;
         k += static_cast<int64_t>(gridDim.x >> 3) * NW) {
        const int64_t wv = xcd_first + k;
        if (wv >= nwaves) break;
        const int64_t chunk0 = wv * 64;
        const int64_t my_off = (chunk0 + lane) * kQRun;          // my residue offset in [0, Dw)
        uint64_t yb = hash_state(p.a[j], p.b[j], static_cast<uint64_t>(i0 + nD0 + my_off));
        uint64_t ys = hash_state(p.as[j], p.bs[j], static_cast<uint64_t>(i0 + nD0 + my_off));
        uint32_t cur[kQRun];
        float val[kQRun];
#pragma unroll
        for (int m = 0; m < kQRun; ++m) { cur[m] = 0xffffffffu; val[m] = 0.0f; }

        for (int64_t nD = nD0; nD < nD1 && nD + chunk0 * kQRun < d; nD += D) {
            int64_t my_len = D - my_off;                         // coordinates of mine that exist
            if (d - (nD + my_off) < my_len) my_len = d - (nD + my_off);
            [[maybe_unused]] vec4f other[RF > 1 ? RF - 1 : 1];       // the other rows' values, requested early
            if constexpr (RF > 1) {
                if (my_len >= kQRun) {
#pragma unroll
                    for (int q = 0; q < RF - 1; ++q)
                        other[q] = __builtin_nontemporal_load(reinterpret_cast<const vec4f_u*>(
                            rows + static_cast<size_t>(q) * d + nD + my_off));
                }
            }
            uint64_t tb = yb, ts = ys;
            float o[kQRun];
#pragma unroll
            for (int m = 0; m < kQRun; ++m) {
                const uint32_t cell = (static_cast<uint32_t>(tb) - 1u) & mask;
                if (cell != cur[m] && m < my_len) {              // entered a new cell: fetch it
                    cur[m] = cell;
                    val[m] = Sj[cell];
                }
                o[m] = apply_sign(val[m], sign_flip_of(ts));
                tb = hash_advance(tb, Ab);
                ts = hash_advance(ts, As);
            }
            yb = hash_advance(yb, ADb);
            ys = hash_advance(ys, ADs);
            if constexpr (RF > 0) {
                float* dst = est + nD + my_off;
                if (my_len >= kQRun) {
                    float vx[RF], vy[RF], vz[RF], vw[RF];
#pragma unroll
                    for (int q = 0; q < RF - 1; ++q) {
                        vx[q] = other[q].x; vy[q] = other[q].y; vz[q] = other[q].z; vw[q] = other[q].w;
                    }
                    vx[RF - 1] = o[0]; vy[RF - 1] = o[1]; vz[RF - 1] = o[2]; vw[RF - 1] = o[3];
                    vec4f u;
                    u.x = median_odd<RF>(vx); u.y = median_odd<RF>(vy);
                    u.z = median_odd<RF>(vz); u.w = median_odd<RF>(vw);
                    __builtin_nontemporal_store(u, reinterpret_cast<vec4f_u*>(dst));
                    tally(u.x); tally(u.y); tally(u.z); tally(u.w);
                } else {
                    for (int m = 0; m < kQRun; ++m) {
                        if (m >= my_len) break;
                        float v[RF];
#pragma unroll
                        for (int q = 0; q < RF - 1; ++q) v[q] = rows[static_cast<size_t>(q) * d + nD + my_off + m];
                        v[RF - 1] = o[m];
                        const float med = median_odd<RF>(v);
                        dst[m] = med;
                        tally(med);
                    }
                }
                continue;
            }
            // the wavefront's 64 pieces are 1 KB of contiguous rows[j][i]
            float* dst = out + nD + my_off;
            if (my_len >= kQRun) {
                vec4f u;
                u.x = o[0]; u.y = o[1]; u.z = o[2]; u.w = o[3];
                // streamed out, read once by the median kernel: kept out of the way of the
                // table row that the gathers want to find in L2
                __builtin_nontemporal_store(u, reinterpret_cast<vec4f_u*>(dst));
            } else if (my_len > 0) {
                dst[0] = o[0];
                if (my_len > 1) dst[1] = o[1];
                if (my_len > 2) dst[2] = o[2];
            }
        }
    }
    if (HIST) {
        __syncthreads();
        for (int t = threadIdx.x; t < 2048; t += 64 * NW) {
            const uint32_t n = lh[t];
            if (n) atomicAdd(&hist[t], static_cast<unsigned long long>(n));
        }
    }
}


// ---------------------------------------------------------------------------------------
// Alg. 4 estimate along a visit list, for column counts that are not a power of two.
//
// The list that serves the update serves the query: whatever a lane meets at i + s_k lies in
// one of the NC = 2 omega cells that the cell of i fixes, so the lane fetches those NC cell
// values once, keeps them in registers, and for the rest of the vector picks one of them per
// visit -- no gather inside the loop.  (Without a list the query is r random gathers per
// coordinate from a table that L2 does not hold: ~80 G gathers/s.  For power-of-two column
// counts the stride walk above does the same job faster than this kernel's form with three
// gaps: both are then bound by their hashing and the walk balances its load better.)
// A lane owns 4 neighbouring residues below the largest gap, a wavefront 256, and every visit
// writes 1 KB of contiguous rows[j][i] (RF = 0) or, for the last row (RF = R), reads the other
// rows' values there, takes the median and writes est.  A coordinate outside the NC cells
// cannot occur with a list from cs_params_init; it is checked all the same and such a value
// is gathered from the table directly.
// ---------------------------------------------------------------------------------------
template <int RF, int NC>
__global__ void __launch_bounds__(64)
k_row_values_visits(VisitGapsRows vr, const float* __restrict__ S, uint32_t c, int64_t d, int64_t i0,
                    float* __restrict__ rows, float* __restrict__ est, int nseg) {
    static_assert(kQRun == 4, "one 16-byte piece per lane");
    static_assert(NC == 2 || NC == 4, "omega = 1 or 2");
    const int lane = threadIdx.x;
    const VisitGaps& v = vr.row[blockIdx.y];           // the rows of a launch run side by side
    const int j = v.j;
    // hash advances of the visits, (a_j gap_k) mod p and (a'_j gap_k) mod p: computed here once
    // per wavefront instead of travelling with the list
    __shared__ uint64_t A_of[CS_ANYC_MAX_VISITS], As_of[CS_ANYC_MAX_VISITS];
    __shared__ uint32_t Ac_of[CS_ANYC_MAX_VISITS];     // A_of[k] mod c
    const Columns colc = columns_of<false>(c);
    for (uint32_t k = lane; k < v.K; k += 64) {
        const uint64_t A = mulmod_p(v.a, v.gap[k]);
        A_of[k] = A;
        As_of[k] = mulmod_p(v.as, v.gap[k]);
        Ac_of[k] = bucket_of<false>(A + 1, colc);     // bucket_of takes the y form, x + 1
    }
    __syncthreads();
    const Columns col = columns_of<false>(c);
    const float* __restrict__ Sj = S + static_cast<size_t>(j) * c;
    float* __restrict__ out = rows + static_cast<size_t>(j) * d;
    const uint64_t Aj = v.a, Asj = v.as;
    const uint32_t omega = v.omega, pc = v.pc;
    auto sum_of = [&](uint32_t cell, uint32_t first) -> uint32_t {
        const uint32_t t = cell >= first ? cell - first : cell + c - first;
        if (t < omega) return t;
        const uint32_t t2 = t + pc >= c ? t + pc - c : t + pc;
        return t2 < omega ? omega + t2 : static_cast<uint32_t>(NC);
    };
    auto cell_of_sum = [&](uint32_t first, int q) -> uint32_t {
        const uint32_t x = static_cast<uint32_t>(q) < omega ? first + q : first + (q - omega) + (c - pc);
        return x >= c ? x - c : x;
    };
    // The bucket x mod c is carried along with the hash value instead of being taken again by a
    // 64-bit remainder at every coordinate: when x moves on by A (mod p), x mod c moves on by
    // A mod c, less p mod c if x wrapped past p.  All terms are below c <= 2^31, so the sums
    // stay below 2^32.  Exact, like the hash state itself.
    const uint32_t Ajc = bucket_of<false>(Aj + 1, colc);          // a_j mod c
    auto advance = [&](uint64_t& y, uint32_t& rem, uint64_t A, uint32_t Ac) {
        const uint64_t t = y + A;
        const bool wrapped = (t >> 61) != 0;
        y = (t & kP61) + (t >> 61);
        uint32_t u = rem + Ac;
        u = u >= c ? u - c : u;
        const uint32_t u2 = u + (c - pc);
        rem = !wrapped ? u : (u2 >= c ? u2 - c : u2);
    };
    const int64_t nwaves = (static_cast<int64_t>(v.gmax) + 64 * kQRun - 1) / (64 * kQRun);
    const int64_t per_xcd = (nwaves + 7) / 8;
    const int64_t xcd_first = static_cast<int64_t>(blockIdx.x & 7) * per_xcd;
    for (int64_t kk = blockIdx.x >> 3; kk < per_xcd; kk += gridDim.x >> 3) {
        const int64_t wv = xcd_first + kk;
        if (wv >= nwaves) break;
        const int64_t wave_res = wv * 64 * kQRun;                   // first residue of the wavefront
        const int64_t my_res = wave_res + static_cast<int64_t>(lane) * kQRun;
        uint64_t yb = hash_state(v.a, v.b, static_cast<uint64_t>(i0 + my_res));
        uint64_t ys = hash_state(v.as, v.bs, static_cast<uint64_t>(i0 + my_res));
        uint32_t rb = bucket_of<false>(yb, col);                    // bucket of my first coordinate
        uint32_t first_cell[kQRun];
        float cellv[kQRun][NC];
        {
            uint64_t tb = yb;
            uint32_t tr = rb;
#pragma unroll
            for (int m = 0; m < kQRun; ++m) {
                first_cell[m] = tr;
#pragma unroll
                for (int n = 0; n < NC; ++n) cellv[m][n] = Sj[cell_of_sum(first_cell[m], n)];
                advance(tb, tr, Aj, Ajc);
            }
        }
        // A launch with few rows leaves the chip half empty and waits on its longest chain of
        // visits, so the chains are cut into nseg pieces walked by separate wavefronts
        // (blockIdx.z); a piece that does not start at visit 0 takes its hash state from the
        // definition at its first coordinate (the cells it can meet are still those of visit 0).
        const uint32_t k0 = v.K * blockIdx.z / nseg, k1 = v.K * (blockIdx.z + 1) / nseg;
        int64_t s = 0;
        if (k0 > 0) {
            for (uint32_t k = 0; k < k0; ++k) s += static_cast<int64_t>(v.gap[k]);
            yb = hash_state(v.a, v.b, static_cast<uint64_t>(i0 + my_res + s));
            ys = hash_state(v.as, v.bs, static_cast<uint64_t>(i0 + my_res + s));
            rb = bucket_of<false>(yb, col);
        }
        for (uint32_t k = k0; k < k1; ++k) {
            const int64_t gap = static_cast<int64_t>(v.gap[k]);
            // residues from wave_res on that take part in this visit and exist in the vector
            const int64_t in_gap = gap - wave_res, in_vec = d - s - wave_res;
            const int64_t room = in_gap < in_vec ? in_gap : in_vec;
            if (room > 0) {
                const int64_t my_len = room - static_cast<int64_t>(lane) * kQRun;   // of my 4: >= 4 all, <= 0 none
                [[maybe_unused]] vec4f other[RF > 1 ? RF - 1 : 1];
                if constexpr (RF > 1) {
                    if (my_len >= kQRun) {
#pragma unroll
                        for (int q = 0; q < RF - 1; ++q)
                            other[q] = __builtin_nontemporal_load(reinterpret_cast<const vec4f_u*>(
                                rows + static_cast<size_t>(q) * d + s + my_res));
                    }
                }
                uint64_t tb = yb, ts = ys;
                uint32_t tr = rb;
                float o[kQRun];
#pragma unroll
                for (int m = 0; m < kQRun; ++m) {
                    const uint32_t cell = tr;
                    const uint32_t rel = sum_of(cell, first_cell[m]);
                    float x = cellv[m][NC - 1];
#pragma unroll
                    for (int n = NC - 2; n >= 0; --n) x = rel == static_cast<uint32_t>(n) ? cellv[m][n] : x;
                    if (rel >= static_cast<uint32_t>(NC) && m < my_len) x = Sj[cell];
                    o[m] = apply_sign(x, sign_flip_of(ts));
                    advance(tb, tr, Aj, Ajc);
                    ts = hash_advance(ts, Asj);
                }
                if constexpr (RF > 0) {
                    float* dst = est + s + my_res;
                    if (my_len >= kQRun) {
                        float vx[RF], vy[RF], vz[RF], vw[RF];
#pragma unroll
                        for (int q = 0; q < RF - 1; ++q) {
                            vx[q] = other[q].x; vy[q] = other[q].y; vz[q] = other[q].z; vw[q] = other[q].w;
                        }
                        vx[RF - 1] = o[0]; vy[RF - 1] = o[1]; vz[RF - 1] = o[2]; vw[RF - 1] = o[3];
                        vec4f u;
                        u.x = median_odd<RF>(vx); u.y = median_odd<RF>(vy);
                        u.z = median_odd<RF>(vz); u.w = median_odd<RF>(vw);
                        __builtin_nontemporal_store(u, reinterpret_cast<vec4f_u*>(dst));
                    } else {
                        for (int m = 0; m < kQRun; ++m) {
                            if (m >= my_len) break;
                            float t[RF];
#pragma unroll
                            for (int q = 0; q < RF - 1; ++q) t[q] = rows[static_cast<size_t>(q) * d + s + my_res + m];
                            t[RF - 1] = o[m];
                            dst[m] = median_odd<RF>(t);
                        }
                    }
                } else {
                    float* dst = out + s + my_res;
                    if (my_len >= kQRun) {
                        vec4f u;
                        u.x = o[0]; u.y = o[1]; u.z = o[2]; u.w = o[3];
                        __builtin_nontemporal_store(u, reinterpret_cast<vec4f_u*>(dst));
                    } else if (my_len > 0) {
                        dst[0] = o[0];
                        if (my_len > 1) dst[1] = o[1];
                        if (my_len > 2) dst[2] = o[2];
                    }
                }
            }
            s += gap;
            advance(yb, rb, A_of[k], Ac_of[k]);
            ys = hash_advance(ys, As_of[k]);
        }
    }
}

}  // namespace

// The query along the rows' visit lists for any column count: rows 0 .. r-2 into the scratch,
// up to kAnycRowsPerLaunch rows per launch (one row's wavefronts alone fill a third to two
// thirds of the chip, and every launch has the tail of its longest chain of visits), then the
// last row together with the median.  The rows of a launch use the same number of cells.
int launch_estimate_anyc(const cs_params* p, const float* S, int64_t d, int64_t i0, float* est,
                         float* rows, hipStream_t stream) {
    auto grid_x = [](uint64_t gmax) {
        const int64_t nwaves = (static_cast<int64_t>(gmax) + 64 * kQRun - 1) / (64 * kQRun);
        const int64_t cap = 256 * 64;
        const int64_t gx = nwaves < cap ? nwaves : cap;
        return static_cast<unsigned>((gx + 7) / 8 * 8);
    };
    // pieces per chain of a launch: enough wavefronts for about two per SIMD slot of the chip,
    // at least 8 visits per piece
    auto pieces = [](uint64_t waves, uint32_t shortest_list) {
        int64_t n = static_cast<int64_t>((16384 + waves - 1) / (waves > 0 ? waves : 1));
        if (n > shortest_list / 8) n = shortest_list / 8;
        if (n > 16) n = 16;
        return static_cast<unsigned>(n < 1 ? 1 : n);
    };
    const uint32_t last = p->r - 1;
    VisitGapsRows vr{};
    const int rc = for_each_anyc_launch(p, last, [&](const uint32_t* js, int n, uint32_t omega) {
        uint64_t most = 0, waves = 0;
        uint32_t shortest = CS_ANYC_MAX_VISITS;
        for (int q = 0; q < n; ++q) {
            fill_visit_gaps(p, js[q], vr.row[q]);
            const cs_anyc_plan& vp = p->anyc[js[q]];
            if (vp.gmax > most) most = vp.gmax;
            waves += (vp.gmax + 64 * kQRun - 1) / (64 * kQRun);
            if (vp.K < shortest) shortest = vp.K;
        }
        const unsigned nseg = pieces(waves, shortest);
        const dim3 grid(grid_x(most), static_cast<unsigned>(n), nseg);
        if (omega == 1) k_row_values_visits<0, 2><<<grid, 64, 0, stream>>>(vr, S, p->c, d, i0, rows, est, static_cast<int>(nseg));
        else k_row_values_visits<0, 4><<<grid, 64, 0, stream>>>(vr, S, p->c, d, i0, rows, est, static_cast<int>(nseg));
        return hipGetLastError() == hipSuccess ? CS_OK : CS_EHIP;
    });
    if (rc != CS_OK) return rc;
    fill_visit_gaps(p, last, vr.row[0]);
    const uint32_t omega_last = p->anyc[last].omega;
    const unsigned nseg_last = pieces((p->anyc[last].gmax + 64 * kQRun - 1) / (64 * kQRun), p->anyc[last].K);
    const dim3 gx(grid_x(p->anyc[last].gmax), 1, nseg_last);
#define CS_LASTR(R_)                                                                                 \
    case R_:                                                                                         \
        if (omega_last == 1) k_row_values_visits<R_, 2><<<gx, 64, 0, stream>>>(vr, S, p->c, d, i0, rows, est, static_cast<int>(nseg_last)); \
        else k_row_values_visits<R_, 4><<<gx, 64, 0, stream>>>(vr, S, p->c, d, i0, rows, est, static_cast<int>(nseg_last));             \
        break;
    switch (p->r) {
        CS_LASTR(1) CS_LASTR(3) CS_LASTR(5) CS_LASTR(7) CS_LASTR(9) CS_LASTR(11) CS_LASTR(13) CS_LASTR(15)
        default: return CS_EINVAL;
    }
#undef CS_LASTR
    return hipGetLastError() == hipSuccess ? CS_OK : CS_EHIP;
}

// fuse_last = false: all rows into the scratch (the caller takes the median).  fuse_last = true:
// the last row's walk takes the median itself; worth it for long vectors, where the scratch
// traffic it saves (write and read of one row) outweighs a second, narrower launch.
// hist (with fuse_last): zeroed by the caller; receives the counts of est by magnitude bin.
int launch_estimate_walk(const cs_params* p, const float* S, int64_t d, int64_t i0,
                         float* est, float* rows, bool fuse_last, uint64_t* hist, hipStream_t stream) {
    int64_t most = 1;
    for (uint32_t j = 0; j < p->r; ++j) {
        const int64_t chunks = (static_cast<int64_t>(p->plan[j].Dw) + kQRun - 1) / kQRun;
        const int64_t nwaves = (chunks + 63) / 64;
        if (nwaves > most) most = nwaves;
    }
    const int64_t cap = 256 * 64;
    int64_t gx = most < cap ? most : cap;
    gx = (gx + 7) / 8 * 8;
    // about 2048 wavefronts per row, at least 4 visits per segment
    RowSegments segs{};
    int most_segs = 1;
    for (uint32_t j = 0; j < p->r; ++j) {
        const int64_t Dw = static_cast<int64_t>(p->plan[j].Dw);
        const int64_t nwaves = ((Dw + kQRun - 1) / kQRun + 63) / 64;
        const int64_t visits = (d + Dw - 1) / Dw;
        int64_t n = 2048 / nwaves;
        if (n > visits / 4) n = visits / 4;
        if (n < 1) n = 1;
        if (n > 1024) n = 1024;
        segs.n[j] = static_cast<int>(n);
        if (segs.n[j] > most_segs) most_segs = segs.n[j];
    }
    if (!fuse_last) {
        const dim3 grid(static_cast<unsigned>(gx), p->r, static_cast<unsigned>(most_segs));
        k_row_values_walk<0, false><<<grid, 64, 0, stream>>>(kparams(p), segs, S, d, i0, rows, est, nullptr);
        return hipGetLastError() == hipSuccess ? CS_OK : CS_EHIP;
    }
    // rows 0 .. r-2 into the scratch, then the last row together with the median
    if (p->r > 1) {
        const dim3 grid(static_cast<unsigned>(gx), p->r - 1, static_cast<unsigned>(most_segs));
        k_row_values_walk<0, false><<<grid, 64, 0, stream>>>(kparams(p), segs, S, d, i0, rows, est, nullptr);
    }
    const dim3 grid(static_cast<unsigned>(gx), 1, static_cast<unsigned>(segs.n[p->r - 1]));
    unsigned long long* h = reinterpret_cast<unsigned long long*>(hist);
    const dim3 hgrid(static_cast<unsigned>(((gx + kHistWaves - 1) / kHistWaves + 7) / 8 * 8), 1, grid.z);
#define CS_LAST(R_)                                                                                    \
    case R_:                                                                                           \
        if (h) k_row_values_walk<R_, true><<<hgrid, 64 * kHistWaves, 0, stream>>>(kparams(p), segs, S, d, i0, rows, est, h); \
        else k_row_values_walk<R_, false><<<grid, 64, 0, stream>>>(kparams(p), segs, S, d, i0, rows, est, h);  \
        break;
    switch (p->r) {
        CS_LAST(1) CS_LAST(3) CS_LAST(5) CS_LAST(7) CS_LAST(9) CS_LAST(11) CS_LAST(13) CS_LAST(15)
        default: return CS_EINVAL;
    }
#undef CS_LAST
    return hipGetLastError() == hipSuccess ? CS_OK : CS_EHIP;
}

// ---------------------------------------------------------------------------------------
// bundle-wide elementwise kernels
// ---------------------------------------------------------------------------------------
namespace {

__global__ void __launch_bounds__(kBlock) k_bundle_zero(float4* __restrict__ T4, int64_t n4,
                                                        float* __restrict__ T, int64_t n) {
    const int64_t stride = static_cast<int64_t>(gridDim.x) * kBlock;
    const int64_t t0 = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x;
    for (int64_t t = t0; t < n4; t += stride) T4[t] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
    for (int64_t t = n4 * 4 + t0; t < n; t += stride) T[t] = 0.0f;
}

// one thread per cell: adds the 8 slots of every group (32 contiguous bytes per group, and
// neighbouring lanes read neighbouring cells, so every load instruction is coalesced).
// The sum over workers is accumulated in binary64 and rounded to binary32 once, together with
// alpha and beta.  A binary32 running sum of W values of similar size loses up to log2(W) bits
// on cells that hold a heavy coordinate; with momentum and error feedback kept as sketches
// that loss is fed back every step and grows (measured at W = 256: the state cells drift
// past 1e-5 of their operands within 8 steps).  The kernel waits on its reads either way.
__global__ void __launch_bounds__(kBlock)
k_bundle_merge(float* __restrict__ dst, float beta, const float4* __restrict__ T4, int groups,
               float alpha, int64_t cells) {
    const int64_t stride = static_cast<int64_t>(gridDim.x) * kBlock;
    for (int64_t t = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x; t < cells; t += stride) {
        double s = 0.0;
        for (int g = 0; g < groups; ++g) {
            const float4* src = T4 + (static_cast<size_t>(g) * cells + t) * (kGroup / 4);
#pragma unroll
            for (int q = 0; q < kGroup / 4; ++q) {
                const float4 u = src[q];
                s += (static_cast<double>(u.x) + static_cast<double>(u.y)) +
                     (static_cast<double>(u.z) + static_cast<double>(u.w));
            }
        }
        const double base = (beta == 0.0f) ? 0.0 : static_cast<double>(beta) * static_cast<double>(dst[t]);
        dst[t] = static_cast<float>(base + static_cast<double>(alpha) * s);
    }
}

// the same merge from a bundle stored in 16 bits per cell: one 16-byte load per group and cell
template <int FMT>
__global__ void __launch_bounds__(kBlock)
k_bundle_merge16(float* __restrict__ dst, float beta, const uint4* __restrict__ T16, int groups,
                 float alpha, int64_t cells) {
    static_assert(kGroup == 8, "8 cells of 16 bits are one 16-byte load");
    const int64_t stride = static_cast<int64_t>(gridDim.x) * kBlock;
    for (int64_t t = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x; t < cells; t += stride) {
        double s = 0.0;
        for (int g = 0; g < groups; ++g) {
            const uint4 q = T16[static_cast<size_t>(g) * cells + t];
            const uint32_t w[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
            for (int h = 0; h < 4; h += 2)
                s += (static_cast<double>(from_16<FMT>(static_cast<uint16_t>(w[h]))) +
                      static_cast<double>(from_16<FMT>(static_cast<uint16_t>(w[h] >> 16)))) +
                     (static_cast<double>(from_16<FMT>(static_cast<uint16_t>(w[h + 1]))) +
                      static_cast<double>(from_16<FMT>(static_cast<uint16_t>(w[h + 1] >> 16))));
        }
        const double base = (beta == 0.0f) ? 0.0 : static_cast<double>(beta) * static_cast<double>(dst[t]);
        dst[t] = static_cast<float>(base + static_cast<double>(alpha) * s);
    }
}

}  // namespace

int launch_bundle_merge16(float* dst, float beta, const uint16_t* T16, int groups, float alpha,
                          int64_t cells, int fmt, hipStream_t stream) {
    int64_t b = (cells + kBlock - 1) / kBlock;
    if (b > 256 * 16) b = 256 * 16;
    const uint4* src = reinterpret_cast<const uint4*>(T16);
    if (fmt == CS_FMT_BF16)
        k_bundle_merge16<0><<<static_cast<unsigned>(b), kBlock, 0, stream>>>(dst, beta, src, groups, alpha, cells);
    else
        k_bundle_merge16<1><<<static_cast<unsigned>(b), kBlock, 0, stream>>>(dst, beta, src, groups, alpha, cells);
    return hipGetLastError() == hipSuccess ? CS_OK : CS_EHIP;
}

int launch_bundle_zero(float* T, int64_t n, hipStream_t stream) {
    const bool aligned = reinterpret_cast<uintptr_t>(T) % 16 == 0;
    const int64_t n4 = aligned ? n / 4 : 0;
    int64_t b = (n / 4 + kBlock - 1) / kBlock;
    if (b < 1) b = 1;
    if (b > 256 * 16) b = 256 * 16;
    k_bundle_zero<<<static_cast<unsigned>(b), kBlock, 0, stream>>>(reinterpret_cast<float4*>(T),
                                                                   n4, T, n);
    return hipGetLastError() == hipSuccess ? CS_OK : CS_EHIP;
}

int launch_bundle_merge(float* dst, float beta, const float* T, int groups, float alpha,
                        int64_t cells, hipStream_t stream) {
    int64_t b = (cells + kBlock - 1) / kBlock;
    if (b > 256 * 32) b = 256 * 32;
    k_bundle_merge<<<static_cast<unsigned>(b), kBlock, 0, stream>>>(
        dst, beta, reinterpret_cast<const float4*>(T), groups, alpha, cells);
    return hipGetLastError() == hipSuccess ? CS_OK : CS_EHIP;
}

}  // namespace cs
