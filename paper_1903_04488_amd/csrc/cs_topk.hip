// heavy_hitters_topk: the selection half of Sec. 5.2 of the paper, where every coordinate is
// queried and the k estimates of largest magnitude are kept.
//
// Exact radix select on the 31-bit magnitude key  bits(est) & 0x7fffffff  (monotone in |est|
// for IEEE binary32): three histograms (11 + 10 + 10 bits) find the key theta of the
// k-th largest magnitude and how many entries equal to theta are still needed; an ordered
// compaction (per-block counts, scan over blocks, write) then emits, in ascending index
// order, every index with key > theta plus the lowest-index entries with key == theta.
// Everything is integer work, so the result is a deterministic function of est.
//
// Passes over est.  Done plainly that is five reads of est (three histograms, count, write).
// After the first histogram the bin of the k-th largest key is known, and only entries in that
// bin or above can be selected: with k << d they are a small multiple of k.  One pass copies
// them, block by block in index order, into a candidate list (k_topk_compact), and the two
// remaining histograms, the count and the write run over that list only: two reads of est
// (one when the caller brings the first histogram, which the estimate kernel can fill as it
// writes est).  The list has a fixed capacity; if the input does not fit it (many equal
// magnitudes, k close to d) a flag is raised on the device and the five-pass form, whose
// kernels are enqueued behind and return at once otherwise, does the work instead.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <mutex>

#include "cs_device.h"
#include "cs_internal.h"
#include "csketch.h"

namespace cs {

constexpr int kBins = 2048;           // bins of the widest pass
constexpr int kItems = 4;             // consecutive elements per thread in a tile
constexpr int kTile = kBlock * kItems;
constexpr int kMaxSelBlocks = 4096;   // blocks of the count / write passes

struct TopkSel {
    uint32_t prefix;      // key bits fixed so far (after pass n: the top 11, 21, 31 bits)
    uint32_t pad;
    uint64_t k_rem;       // how many of the entries sharing `prefix` are still wanted
};

constexpr int kStage = 4096;          // candidates one block can hold in LDS for its chunk

// workspace layout (all 8-byte aligned); the candidate list follows the struct
struct TopkWs {
    uint64_t hist[3][kBins];
    TopkSel sel;
    uint32_t failed;                // != 0: the candidate list could not be built, est is read instead
    uint32_t ncand;                 // candidates appended so far
    uint64_t gt[kMaxSelBlocks];     // per block: entries with key > theta  -> exclusive scan
    uint64_t eq[kMaxSelBlocks];     // per block: entries with key == theta -> exclusive scan
    uint32_t seg_base[kMaxSelBlocks];    // block b's candidates are cand[seg_base[b] .. + seg_count[b])
    uint32_t seg_count[kMaxSelBlocks];
};
constexpr size_t kCandBytes = sizeof(int64_t) + sizeof(float);   // index and value of a candidate

// candidates worth providing for: a few times k, never a large part of d.  When k itself is a
// few per cent of d (the P k candidates of Alg. 3 with P in the tens) the list is sized more
// tightly: the entries of the k-th largest key's bin and above are k plus that bin's own
// population, at most a few tenths of k for magnitudes that fall off smoothly (a bin is an
// eighth of a binade wide); should they not fit, the five-pass form takes over on the device.
__host__ inline int64_t candidate_capacity_for(int64_t d, int64_t k) {
    const int64_t roomy = 8 * k + 65536;
    if (roomy <= d / 4) return roomy;
    const int64_t tight = 3 * k + 65536;
    return tight <= d / 5 ? tight : 0;
}

// Selection keys (31 bits, larger = selected first; equal keys: lower index first).
// KeyMagnitude: the magnitude bits of the estimate (top-k by |est|).
struct KeyMagnitude {
    __device__ __forceinline__ void init() {}
    __device__ __forceinline__ uint32_t operator()(float v, int64_t) const {
        return __float_as_uint(v) & 0x7fffffffu;
    }
};
// KeyHeavymix (Alg. 1 steps 3-4): a coordinate is heavy when est^2 >= l2sq / k (binary32
// estimate, squared and compared in binary64: the product of two binary32 values is exact
// there).  Heavy coordinates get bit 30 plus the top 30 magnitude bits, so they come before
// every other coordinate and, should more than k be heavy, in order of magnitude; the others
// get the top 30 bits of a counter-based random word -- the (i+1)-th output of SplitMix64
// started at `seed` -- so the k - |H| of them with the largest words are a uniform draw
// without replacement.
struct KeyHeavymix {
    const double* l2sq;       // device: the norm estimate of cs_sketch_l2sq
    double k;
    uint64_t seed;
    double theta;
    __device__ __forceinline__ void init() { theta = *l2sq / k; }
    __device__ __forceinline__ bool heavy(float v) const {
        return static_cast<double>(v) * static_cast<double>(v) >= theta;
    }
    __device__ __forceinline__ uint32_t operator()(float v, int64_t i) const {
        if (heavy(v)) return 0x40000000u | ((__float_as_uint(v) & 0x7fffffffu) >> 1);
        uint64_t z = seed + (static_cast<uint64_t>(i) + 1u) * 0x9E3779B97F4A7C15ull;
        z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
        z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
        z ^= z >> 31;
        return static_cast<uint32_t>(z >> 34);
    }
};

__global__ void __launch_bounds__(kBlock) k_topk_clear(TopkWs* ws, uint64_t k) {
    for (int t = threadIdx.x; t < 3 * kBins; t += kBlock) (&ws->hist[0][0])[t] = 0;
    if (threadIdx.x == 0) {
        ws->sel.prefix = 0;
        ws->sel.pad = 0;
        ws->sel.k_rem = k;
        ws->failed = 0;
        ws->ncand = 0;
    }
}

// The histogram, count and write kernels below exist once and work either on the candidate
// list or on est itself: `listed` says that a list was asked for, and ws->failed, which the
// compaction sets on the device, that it could not be built -- then the same launches fall
// back to reading est (the five-pass form), without the host having to know.
__device__ __forceinline__ bool use_list(const TopkWs* ws, bool listed) {
    return listed && ws->failed == 0;
}

// PASS 0: bin = key >> 20 (2048 bins); PASS 1: entries with key >> 20 == prefix, bin = bits
// 19..10; PASS 2: entries with key >> 10 == prefix, bin = bits 9..0.
template <int PASS, bool VEC, typename KEY>
__global__ void __launch_bounds__(kBlock)
k_topk_hist(const float* __restrict__ est, int64_t d, TopkWs* ws, uint64_t* __restrict__ hist_out,
            bool listed, const int64_t* __restrict__ cand_idx, const float* __restrict__ cand_val,
            KEY kf) {
    kf.init();
    // Magnitudes crowd into a few of the pass-0 bins (same exponent), and lanes that hit the same
    // LDS word are served one after the other: pass 0 keeps kCopies histograms and lane l adds
    // into copy l mod kCopies.
    constexpr int kCopies = (PASS == 0) ? 4 : 1;
    constexpr int nb = (PASS == 0) ? 2048 : 1024;
    __shared__ uint32_t lh_all[kCopies][nb];
    const bool from_list = PASS > 0 && use_list(ws, listed);
    constexpr unsigned kListBlocks = 128;           // the list is short: a few blocks are plenty
    if (from_list && blockIdx.x >= kListBlocks) return;
    for (int t = threadIdx.x; t < kCopies * nb; t += kBlock) (&lh_all[0][0])[t] = 0;
    __syncthreads();
    uint32_t* lh = lh_all[threadIdx.x % kCopies];
    const uint32_t prefix = PASS > 0 ? ws->sel.prefix : 0u;
    auto tally = [&](uint32_t key) {
        if (PASS == 0) {
            atomicAdd(&lh[key >> 20], 1u);
        } else if (PASS == 1) {
            if ((key >> 20) == prefix) atomicAdd(&lh[(key >> 10) & 1023u], 1u);
        } else {
            if ((key >> 10) == prefix) atomicAdd(&lh[key & 1023u], 1u);
        }
    };
    if (from_list) {
        const uint32_t n = ws->ncand;
        const unsigned blocks = gridDim.x < kListBlocks ? gridDim.x : kListBlocks;
        for (uint32_t t = blockIdx.x * kBlock + threadIdx.x; t < n; t += blocks * kBlock)
            tally(kf(cand_val[t], cand_idx[t]));
    } else {
        const int64_t stride = static_cast<int64_t>(gridDim.x) * kBlock;
        const int64_t t0 = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x;
        int64_t done = 0;
        if (VEC) {                                   // est is 16-byte aligned: four elements per load
            const int64_t n4 = d / 4;
            const float4* est4 = reinterpret_cast<const float4*>(est);
            int64_t t = t0;
            for (; t + stride < n4; t += 2 * stride) {   // two loads in flight
                const float4 u = est4[t], w = est4[t + stride];
                tally(kf(u.x, 4 * t)); tally(kf(u.y, 4 * t + 1)); tally(kf(u.z, 4 * t + 2)); tally(kf(u.w, 4 * t + 3));
                const int64_t t2 = t + stride;
                tally(kf(w.x, 4 * t2)); tally(kf(w.y, 4 * t2 + 1)); tally(kf(w.z, 4 * t2 + 2)); tally(kf(w.w, 4 * t2 + 3));
            }
            if (t < n4) {
                const float4 u = est4[t];
                tally(kf(u.x, 4 * t)); tally(kf(u.y, 4 * t + 1)); tally(kf(u.z, 4 * t + 2)); tally(kf(u.w, 4 * t + 3));
            }
            done = n4 * 4;
        }
        for (int64_t t = done + t0; t < d; t += stride) tally(kf(est[t], t));
    }
    __syncthreads();
    for (int t = threadIdx.x; t < nb; t += kBlock) {
        uint32_t v = 0;
#pragma unroll
        for (int q = 0; q < kCopies; ++q) v += lh_all[q][t];
        if (v) atomicAdd(reinterpret_cast<unsigned long long*>(&hist_out[t]),
                         static_cast<unsigned long long>(v));
    }
}

// One workgroup: walk the histogram of this pass from the top bin down to the bin that holds
// the k_rem-th largest entry; append that bin to the prefix, and drop from k_rem the entries
// in higher bins (they are all selected).
// Sum of v over the threads before this one in the workgroup (shuffles within a wavefront, one
// LDS word per wavefront); *total receives the sum over all threads.
__device__ __forceinline__ uint64_t block_exclusive_sum64(uint64_t v, uint64_t* lds, uint64_t* total) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    uint64_t inc = v;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const uint64_t up = __shfl_up(inc, off, 64);
        if (lane >= off) inc += up;
    }
    if (lane == 63) lds[wave] = inc;
    __syncthreads();
    uint64_t before = 0, all = 0;
#pragma unroll
    for (int wv = 0; wv < kBlock / 64; ++wv) {
        const uint64_t s = lds[wv];
        if (wv < wave) before += s;
        all += s;
    }
    *total = all;
    return before + inc - v;
}

// h: the histogram of this pass (for PASS 0 possibly one the caller brought)
template <int PASS>
__global__ void __launch_bounds__(kBlock) k_topk_find(TopkWs* ws, const uint64_t* __restrict__ h) {
    constexpr int nb = (PASS == 0) ? 2048 : 1024;
    constexpr int per = nb / kBlock;              // bins per thread: 8 or 4
    __shared__ uint64_t wave_sum[kBlock / 64];
    const uint64_t k_rem = ws->sel.k_rem;
    const uint32_t prefix = ws->sel.prefix;
    uint64_t mine = 0;
    for (int q = 0; q < per; ++q) mine += h[threadIdx.x * per + q];
    uint64_t all;
    const uint64_t below = block_exclusive_sum64(mine, wave_sum, &all);
    const uint64_t above = all - below - mine;     // entries in bins above my segment
    if (above < k_rem && k_rem <= above + mine) {  // true for exactly one thread
        uint64_t acc = above;
        for (int q = per - 1; q >= 0; --q) {
            const int bin = threadIdx.x * per + q;
            const uint64_t cnt = h[bin];
            if (k_rem <= acc + cnt) {
                constexpr int bits = (PASS == 0) ? 11 : 10;
                ws->sel.prefix = (PASS == 0) ? static_cast<uint32_t>(bin)
                                             : ((prefix << bits) | static_cast<uint32_t>(bin));
                ws->sel.k_rem = k_rem - acc;
                break;
            }
            acc += cnt;
        }
    }
}

// flags of one element against theta, packed: low 16 bits count "greater", high 16 "equal"
__device__ __forceinline__ uint32_t classify(uint32_t key, uint32_t theta) {
    return (key > theta ? 1u : 0u) | (key == theta ? 0x10000u : 0u);
}

// inclusive scan of a packed counter over the workgroup; returns the inclusive value and
// writes the workgroup total to *total.  `lds` holds one word per wavefront.
__device__ __forceinline__ uint32_t block_inclusive_scan(uint32_t v, uint32_t* lds, uint32_t* total) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const uint32_t up = __shfl_up(v, off, 64);
        if (lane >= off) v += up;
    }
    if (lane == 63) lds[wave] = v;
    __syncthreads();
    uint32_t before = 0, all = 0;
#pragma unroll
    for (int wv = 0; wv < kBlock / 64; ++wv) {
        const uint32_t s = lds[wv];
        if (wv < wave) before += s;
        all += s;
    }
    __syncthreads();
    *total = all;
    return v + before;
}

template <bool VEC>
__device__ __forceinline__ void load_items(const float* __restrict__ est, int64_t base, int64_t d,
                                           float (&v)[kItems], int& nvalid) {
    // base = index of this thread's first element
    if (VEC && base + kItems <= d) {
        const float4 q = *reinterpret_cast<const float4*>(est + base);
        v[0] = q.x; v[1] = q.y; v[2] = q.z; v[3] = q.w;
        nvalid = kItems;
        return;
    }
    nvalid = 0;
#pragma unroll
    for (int q = 0; q < kItems; ++q) {
        if (base + q < d) { v[q] = est[base + q]; nvalid = q + 1; } else { v[q] = 0.0f; }
    }
}

// The candidate list.  Block b scans its chunk of est (the chunks of the count / write passes)
// and keeps, in index order, every entry whose key lies in the bin of the k-th largest key or
// above (sel.prefix after the first histogram).  Each wavefront takes a consecutive quarter of
// the chunk, 256 entries at a time, and stages its candidates in its own part of LDS (their
// places come from wavefront ballots, no barrier inside the loop); the block then appends
// them to the list as one segment, whose place comes from a single atomic add.  Segments lie
// in the list in the order the blocks finished; (seg_base[b], seg_count[b]) lets the later
// kernels visit them in block order, i.e. in index order.  A wavefront with more than
// kStage / 4 candidates, or a list that would exceed `cap`, raises ws->failed.
template <bool VEC, typename KEY>
__global__ void __launch_bounds__(kBlock)
k_topk_compact(const float* __restrict__ est, int64_t d, int64_t chunk, TopkWs* ws, uint32_t cap,
               int64_t* __restrict__ cand_idx, float* __restrict__ cand_val, KEY kf) {
    kf.init();
    constexpr int kWaves = kBlock / 64;
    constexpr int kWaveStage = kStage / kWaves;
    constexpr int kWaveTile = 64 * kItems;
    __shared__ uint32_t st_off[kStage];
    __shared__ float st_val[kStage];
    __shared__ uint32_t wave_n[kWaves];
    __shared__ uint32_t seg[2];                     // base, ok
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint32_t bin0 = ws->sel.prefix;
    const int64_t lo = static_cast<int64_t>(blockIdx.x) * chunk;
    const int64_t hi = (lo + chunk < d) ? lo + chunk : d;
    const int64_t part = (chunk / kWaves + kWaveTile - 1) / kWaveTile * kWaveTile;
    const int64_t wlo = lo + wave * part;
    const int64_t whi = (wlo + part < hi) ? wlo + part : hi;
    uint32_t* my_off = st_off + wave * kWaveStage;
    float* my_val = st_val + wave * kWaveStage;
    const uint64_t below = (lane == 0) ? 0ull : (~0ull >> (64 - lane));   // lanes before mine
    uint32_t staged = 0;                            // the same in every lane of the wavefront
    bool overflow = false;
    auto take = [&](const float (&v)[kItems], int nvalid, int64_t base) {
        bool f[kItems];
        uint32_t before = 0, total = 0;
#pragma unroll
        for (int q = 0; q < kItems; ++q) {
            f[q] = q < nvalid && (kf(v[q], base + q) >> 20) >= bin0;
            const uint64_t m = __builtin_amdgcn_ballot_w64(f[q]);
            before += __builtin_popcountll(m & below);
            total += __builtin_popcountll(m);
        }
        if (total == 0) return;
        if (staged + total > static_cast<uint32_t>(kWaveStage)) { overflow = true; return; }
        uint32_t pos = staged + before;
#pragma unroll
        for (int q = 0; q < kItems; ++q)
            if (f[q]) {
                my_off[pos] = static_cast<uint32_t>(base + q - lo);
                my_val[pos] = v[q];
                ++pos;
            }
        staged += total;
    };
    for (int64_t tile = wlo; tile < whi && !overflow; tile += 2 * kWaveTile) {   // two loads in flight
        float v0[kItems], v1[kItems];
        int n0, n1 = 0;
        const int64_t b0 = tile + static_cast<int64_t>(lane) * kItems, b1 = b0 + kWaveTile;
        load_items<VEC>(est, b0, whi, v0, n0);
        if (tile + kWaveTile < whi) load_items<VEC>(est, b1, whi, v1, n1);
        take(v0, n0, b0);
        if (tile + kWaveTile < whi && !overflow) take(v1, n1, b1);
    }
    if (lane == 0) wave_n[wave] = overflow ? 0xffffffffu : staged;
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t total = 0;
        bool ok = true;
        for (int w = 0; w < kWaves; ++w) {
            if (wave_n[w] == 0xffffffffu) ok = false;
            else total += wave_n[w];
        }
        uint32_t base = 0;
        if (ok && total) {
            base = atomicAdd(&ws->ncand, total);
            ok = static_cast<uint64_t>(base) + total <= cap;
        }
        if (!ok) atomicOr(&ws->failed, 1u);
        ws->seg_base[blockIdx.x] = base;
        ws->seg_count[blockIdx.x] = ok ? total : 0u;
        seg[0] = base;
        seg[1] = ok ? 1u : 0u;
    }
    __syncthreads();
    if (seg[1] == 0u) return;
    uint32_t at = seg[0];
    for (int w = 0; w < wave; ++w) at += wave_n[w];
    for (uint32_t t = lane; t < staged; t += 64) {
        cand_idx[at + t] = lo + my_off[t];
        cand_val[at + t] = my_val[t];
    }
}

// per block: how many entries of its chunk (or of its segment of the list) are above / equal
// to theta
template <bool VEC, typename KEY>
__global__ void __launch_bounds__(kBlock)
k_topk_count(const float* __restrict__ est, int64_t d, int64_t chunk, TopkWs* ws, int nblocks,
             bool listed, const int64_t* __restrict__ cand_idx, const float* __restrict__ cand_val,
             KEY kf) {
    kf.init();
    const uint32_t theta = ws->sel.prefix;
    if (use_list(ws, listed)) {                     // one wavefront per segment
        const int b = blockIdx.x * (kBlock / 64) + (threadIdx.x >> 6);
        if (b >= nblocks) return;
        const int lane = threadIdx.x & 63;
        const uint32_t base = ws->seg_base[b], n = ws->seg_count[b];
        uint32_t n_gt = 0, n_eq = 0;
        for (uint32_t t = lane; t < n; t += 64) {
            const uint32_t key = kf(cand_val[base + t], cand_idx[base + t]);
            n_gt += key > theta ? 1u : 0u;
            n_eq += key == theta ? 1u : 0u;
        }
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) {
            n_gt += __shfl_down(n_gt, off, 64);
            n_eq += __shfl_down(n_eq, off, 64);
        }
        if (lane == 0) {
            ws->gt[b] = n_gt;
            ws->eq[b] = n_eq;
        }
        return;
    }
    __shared__ uint32_t lds[kBlock / 64];
    const int64_t lo = static_cast<int64_t>(blockIdx.x) * chunk;
    const int64_t hi = (lo + chunk < d) ? lo + chunk : d;
    uint64_t n_gt = 0, n_eq = 0;
    for (int64_t tile = lo; tile < hi; tile += kTile) {
        float v[kItems];
        int nvalid;
        const int64_t base = tile + static_cast<int64_t>(threadIdx.x) * kItems;
        load_items<VEC>(est, base, hi, v, nvalid);
        uint32_t c = 0;
#pragma unroll
        for (int q = 0; q < kItems; ++q)
            if (q < nvalid) c += classify(kf(v[q], base + q), theta);
        uint32_t total;
        block_inclusive_scan(c, lds, &total);
        n_gt += total & 0xffffu;
        n_eq += total >> 16;
    }
    if (threadIdx.x == 0) {
        ws->gt[blockIdx.x] = n_gt;
        ws->eq[blockIdx.x] = n_eq;
    }
}

// one workgroup: exclusive scan of the per-block counts, in place
__global__ void __launch_bounds__(kBlock) k_topk_scan(TopkWs* ws, int nblocks) {
    __shared__ uint64_t wave_gt[kBlock / 64], wave_eq[kBlock / 64];
    constexpr int per = kMaxSelBlocks / kBlock;     // 16 consecutive blocks per thread
    uint64_t g[per], e[per], sg = 0, se = 0;
    for (int q = 0; q < per; ++q) {
        const int b = threadIdx.x * per + q;
        g[q] = (b < nblocks) ? ws->gt[b] : 0;
        e[q] = (b < nblocks) ? ws->eq[b] : 0;
        sg += g[q];
        se += e[q];
    }
    uint64_t all;
    uint64_t bg = block_exclusive_sum64(sg, wave_gt, &all);
    uint64_t be = block_exclusive_sum64(se, wave_eq, &all);
    for (int q = 0; q < per; ++q) {
        const int b = threadIdx.x * per + q;
        if (b < nblocks) { ws->gt[b] = bg; ws->eq[b] = be; }
        bg += g[q];
        be += e[q];
    }
}

// ordered compaction: index t is selected when key > theta, or key == theta and fewer than
// need_eq equal entries precede it; its output slot is (#greater before t) + min(#equal
// before t, need_eq), which is its rank among the selected in ascending index order.
template <bool VEC, typename KEY>
__global__ void __launch_bounds__(kBlock)
k_topk_write(const float* __restrict__ est, int64_t d, int64_t chunk, const TopkWs* ws, int nblocks,
             int64_t k, int64_t* __restrict__ idx_out, float* __restrict__ val_out, bool listed,
             const int64_t* __restrict__ cand_idx, const float* __restrict__ cand_val, KEY kf) {
    kf.init();
    const uint32_t theta = ws->sel.prefix;
    const uint64_t need_eq = ws->sel.k_rem;
    if (use_list(ws, listed)) {                     // one wavefront per segment, 64 candidates at a time
        const int b = blockIdx.x * (kBlock / 64) + (threadIdx.x >> 6);
        if (b >= nblocks) return;
        const int lane = threadIdx.x & 63;
        uint64_t g = ws->gt[b], e = ws->eq[b];      // greater / equal entries before this batch
        const uint32_t base = ws->seg_base[b], n = ws->seg_count[b];
        const uint64_t below = (lane == 0) ? 0ull : (~0ull >> (64 - lane));   // lanes before mine
        for (uint32_t t0 = 0; t0 < n; t0 += 64) {
            const uint32_t t = t0 + lane;
            bool is_gt = false, is_eq = false;
            int64_t i = 0;
            float v = 0.0f;
            if (t < n) {
                i = cand_idx[base + t];
                v = cand_val[base + t];
                const uint32_t key = kf(v, i);
                is_gt = key > theta;
                is_eq = key == theta;
            }
            const uint64_t m_gt = __builtin_amdgcn_ballot_w64(is_gt);
            const uint64_t m_eq = __builtin_amdgcn_ballot_w64(is_eq);
            const uint64_t my_g = g + __builtin_popcountll(m_gt & below);
            const uint64_t my_e = e + __builtin_popcountll(m_eq & below);
            if (is_gt || (is_eq && my_e < need_eq)) {
                const uint64_t slot = my_g + (my_e < need_eq ? my_e : need_eq);
                if (slot < static_cast<uint64_t>(k)) {
                    idx_out[slot] = i;
                    if (val_out) val_out[slot] = v;
                }
            }
            g += __builtin_popcountll(m_gt);
            e += __builtin_popcountll(m_eq);
        }
        return;
    }
    __shared__ uint32_t lds[kBlock / 64];
    uint64_t gt_before = ws->gt[blockIdx.x];
    uint64_t eq_before = ws->eq[blockIdx.x];
    const int64_t lo = static_cast<int64_t>(blockIdx.x) * chunk;
    const int64_t hi = (lo + chunk < d) ? lo + chunk : d;
    for (int64_t tile = lo; tile < hi; tile += kTile) {
        float v[kItems];
        int nvalid;
        const int64_t base = tile + static_cast<int64_t>(threadIdx.x) * kItems;
        load_items<VEC>(est, base, hi, v, nvalid);
        uint32_t c = 0;
#pragma unroll
        for (int q = 0; q < kItems; ++q)
            if (q < nvalid) c += classify(kf(v[q], base + q), theta);
        uint32_t total;
        const uint32_t incl = block_inclusive_scan(c, lds, &total);
        if (c) {
            uint64_t g = gt_before + ((incl - c) & 0xffffu);
            uint64_t e = eq_before + ((incl - c) >> 16);
#pragma unroll
            for (int q = 0; q < kItems; ++q) {
                if (q >= nvalid) break;
                const uint32_t key = kf(v[q], base + q);
                const bool is_gt = key > theta, is_eq = key == theta;
                if (is_gt || (is_eq && e < need_eq)) {
                    const uint64_t slot = g + (e < need_eq ? e : need_eq);
                    if (slot < static_cast<uint64_t>(k)) {
                        idx_out[slot] = base + q;
                        if (val_out) val_out[slot] = v[q];
                    }
                }
                g += is_gt;
                e += is_eq;
            }
        }
        gt_before += total & 0xffffu;
        eq_before += total >> 16;
    }
}

// idx[t] = cand[idx[t]]: positions within the candidate list -> coordinates
__global__ void __launch_bounds__(kBlock)
k_remap_positions(int64_t* __restrict__ idx, const int64_t* __restrict__ cand, int64_t k) {
    const int64_t stride = static_cast<int64_t>(gridDim.x) * kBlock;
    for (int64_t t = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x; t < k; t += stride)
        idx[t] = cand[idx[t]];
}

// Alg. 1 step 1: out[1 + j] = sum_b S[j][b]^2, one workgroup of 1024 threads per row, binary64
// sums in a fixed order (each thread a strided share in four independent chains, then a tree
// over the workgroup), 16-byte loads when the row allows.
constexpr int kSumBlock = 1024;
__global__ void __launch_bounds__(kSumBlock)
k_row_sumsq(const float* __restrict__ S, uint32_t c, double* __restrict__ out) {
    __shared__ double part[kSumBlock];
    const float* row = S + static_cast<size_t>(blockIdx.x) * c;
    double a0 = 0.0, a1 = 0.0, a2 = 0.0, a3 = 0.0;
    uint32_t done = 0;
    if (reinterpret_cast<uintptr_t>(row) % 16 == 0) {
        const uint32_t n4 = c / 4;
        const float4* row4 = reinterpret_cast<const float4*>(row);
        for (uint32_t q = threadIdx.x; q < n4; q += kSumBlock) {
            const float4 u = row4[q];
            a0 += static_cast<double>(u.x) * static_cast<double>(u.x);
            a1 += static_cast<double>(u.y) * static_cast<double>(u.y);
            a2 += static_cast<double>(u.z) * static_cast<double>(u.z);
            a3 += static_cast<double>(u.w) * static_cast<double>(u.w);
        }
        done = n4 * 4;
    }
    for (uint32_t b = done + threadIdx.x; b < c; b += kSumBlock) {
        const double v = static_cast<double>(row[b]);
        a0 += v * v;
    }
    part[threadIdx.x] = (a0 + a1) + (a2 + a3);
    __syncthreads();
    for (int off = kSumBlock / 2; off > 0; off >>= 1) {
        if (static_cast<int>(threadIdx.x) < off) part[threadIdx.x] += part[threadIdx.x + off];
        __syncthreads();
    }
    if (threadIdx.x == 0) out[1 + blockIdx.x] = part[0];
}

// out[0] = median of out[1 .. r] (r odd, <= CS_MAX_R): insertion sort by one thread
__global__ void k_median_of_rows(double* out, int r) {
    double v[CS_MAX_R];
    for (int j = 0; j < r; ++j) {
        double x = out[1 + j];
        int q = j;
        while (q > 0 && v[q - 1] > x) { v[q] = v[q - 1]; --q; }
        v[q] = x;
    }
    out[0] = v[r / 2];
}

// how many of the selected coordinates passed the threshold
__global__ void __launch_bounds__(kBlock)
k_count_heavy(const float* __restrict__ est, const int64_t* __restrict__ idx, int64_t k,
              KeyHeavymix kf, unsigned long long* __restrict__ n_heavy) {
    kf.init();
    const int64_t stride = static_cast<int64_t>(gridDim.x) * kBlock;
    unsigned long long mine = 0;
    for (int64_t t = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x; t < k; t += stride)
        mine += kf.heavy(est[idx[t]]) ? 1u : 0u;
    for (int off = 32; off > 0; off >>= 1) mine += __shfl_down(mine, off, 64);
    if ((threadIdx.x & 63) == 0 && mine) atomicAdd(n_heavy, mine);
}

__global__ void k_clear_u64(unsigned long long* x) { *x = 0; }

__global__ void __launch_bounds__(kBlock) k_hist_zero(uint64_t* hist) {
    for (int t = threadIdx.x; t < kBins; t += kBlock) hist[t] = 0;
}

int launch_magnitude_hist_zero(uint64_t* hist, hipStream_t stream) {
    k_hist_zero<<<1, kBlock, 0, stream>>>(hist);
    return hipGetLastError() == hipSuccess ? CS_OK : CS_EHIP;
}

int launch_magnitude_hist(const float* est, int64_t d, uint64_t* hist, hipStream_t stream) {
    const unsigned hgrid = static_cast<unsigned>(
        (d + kBlock * 16 - 1) / (kBlock * 16) < 2048 ? (d + kBlock * 16 - 1) / (kBlock * 16) : 2048);
    if (reinterpret_cast<uintptr_t>(est) % 16 == 0)
        k_topk_hist<0, true, KeyMagnitude><<<hgrid, kBlock, 0, stream>>>(est, d, nullptr, hist, false, nullptr,
                                                                        nullptr, KeyMagnitude{});
    else
        k_topk_hist<0, false, KeyMagnitude><<<hgrid, kBlock, 0, stream>>>(est, d, nullptr, hist, false, nullptr,
                                                                         nullptr, KeyMagnitude{});
    return hipGetLastError() == hipSuccess ? CS_OK : CS_EHIP;
}

}  // namespace cs

using namespace cs;

static void topk_geometry(int64_t d, int* nblocks, int64_t* chunk) {
    int64_t tiles = (d + kTile - 1) / kTile;
    int64_t nb = tiles < kMaxSelBlocks ? tiles : kMaxSelBlocks;
    if (nb < 1) nb = 1;
    int64_t tiles_per_block = (tiles + nb - 1) / nb;
    *chunk = tiles_per_block * kTile;
    *nblocks = static_cast<int>((d + *chunk - 1) / *chunk);
    if (*nblocks < 1) *nblocks = 1;
}

extern "C" int cs_topk_workspace_bytes(int64_t d, int64_t k, size_t* bytes) {
    if (!bytes || d < 1 || k < 1 || k > d) return CS_EINVAL;
    *bytes = sizeof(TopkWs) + static_cast<size_t>(candidate_capacity_for(d, k)) * kCandBytes;
    return CS_OK;
}

// the k entries with the largest keys, ascending by index (see the header of this file).
// hist0: device uint64[2048], the histogram of key >> 20 over est, when the caller has it.
template <typename KEY, bool VEC>
static void enqueue_selection(const float* est, int64_t d, int64_t k, const uint64_t* hist0,
                              int64_t* idx_out, float* val_out, TopkWs* ws, int64_t cap, bool listed,
                              hipStream_t s, KEY kf) {
    int64_t* cand_idx = reinterpret_cast<int64_t*>(ws + 1);
    float* cand_val = reinterpret_cast<float*>(cand_idx + cap);
    const unsigned hgrid = static_cast<unsigned>(
        (d + kBlock * 16 - 1) / (kBlock * 16) < 2048 ? (d + kBlock * 16 - 1) / (kBlock * 16) : 2048);
    int nblocks;
    int64_t chunk;
    topk_geometry(d, &nblocks, &chunk);
    k_topk_clear<<<1, kBlock, 0, s>>>(ws, static_cast<uint64_t>(k));
    if (!hist0)
        k_topk_hist<0, VEC, KEY><<<hgrid, kBlock, 0, s>>>(est, d, ws, ws->hist[0], false, cand_idx, cand_val, kf);
    k_topk_find<0><<<1, kBlock, 0, s>>>(ws, hist0 ? hist0 : ws->hist[0]);
    if (listed)
        k_topk_compact<VEC, KEY><<<nblocks, kBlock, 0, s>>>(est, d, chunk, ws, static_cast<uint32_t>(cap),
                                                            cand_idx, cand_val, kf);
    k_topk_hist<1, VEC, KEY><<<hgrid, kBlock, 0, s>>>(est, d, ws, ws->hist[1], listed, cand_idx, cand_val, kf);
    k_topk_find<1><<<1, kBlock, 0, s>>>(ws, ws->hist[1]);
    k_topk_hist<2, VEC, KEY><<<hgrid, kBlock, 0, s>>>(est, d, ws, ws->hist[2], listed, cand_idx, cand_val, kf);
    k_topk_find<2><<<1, kBlock, 0, s>>>(ws, ws->hist[2]);
    k_topk_count<VEC, KEY><<<nblocks, kBlock, 0, s>>>(est, d, chunk, ws, nblocks, listed, cand_idx, cand_val, kf);
    k_topk_scan<<<1, kBlock, 0, s>>>(ws, nblocks);
    k_topk_write<VEC, KEY><<<nblocks, kBlock, 0, s>>>(est, d, chunk, ws, nblocks, k, idx_out, val_out, listed,
                                                      cand_idx, cand_val, kf);
}

template <typename KEY>
static int select_largest(const float* est, int64_t d, int64_t k, const uint64_t* hist0,
                          int64_t* idx_out, float* val_out, void* workspace, size_t ws_bytes,
                          hipStream_t s, KEY kf) {
    if (d < 1 || k < 1 || k > d || !est || !idx_out || !workspace) return CS_EINVAL;
    if (reinterpret_cast<uintptr_t>(workspace) % 8 != 0) return CS_EINVAL;
    if (hist0 && reinterpret_cast<uintptr_t>(hist0) % 8 != 0) return CS_EINVAL;
    if (ws_bytes < sizeof(TopkWs)) return CS_EWORKSPACE;
    TopkWs* ws = static_cast<TopkWs*>(workspace);
    // The candidate list takes what the workspace holds beyond the struct, up to what is worth
    // having; it is used when that is at least 2 k + kStage entries (the k-th largest key's own
    // bin has to fit beside the k entries above it) and clearly less than d.
    int64_t cap = static_cast<int64_t>((ws_bytes - sizeof(TopkWs)) / kCandBytes);
    if (cap > candidate_capacity_for(d, k)) cap = candidate_capacity_for(d, k);
    if (cap > 0xffffffffll) cap = 0xffffffffll;
    const bool listed = cap >= 2 * k + kStage;
    if (reinterpret_cast<uintptr_t>(est) % 16 == 0)
        enqueue_selection<KEY, true>(est, d, k, hist0, idx_out, val_out, ws, cap, listed, s, kf);
    else
        enqueue_selection<KEY, false>(est, d, k, hist0, idx_out, val_out, ws, cap, listed, s, kf);
    return hipGetLastError() == hipSuccess ? CS_OK : CS_EHIP;
}

extern "C" int cs_heavy_hitters_topk(const float* est, int64_t d, int64_t k,
                                     const uint64_t* hist_or_null, int64_t* idx_out,
                                     float* val_out, void* workspace, size_t ws_bytes,
                                     void* stream) {
    return select_largest(est, d, k, hist_or_null, idx_out, val_out, workspace, ws_bytes,
                          reinterpret_cast<hipStream_t>(stream), KeyMagnitude{});
}

// ---------------------------------------------------------------------------------------
// The selection for callers that cannot allocate: its workspace is an array in the library's
// own device image.  Every GPU holds its own copy at its own address, so the address is asked
// for once per device (with that device current) and kept; host code never passes the array's
// name to a kernel.
// ---------------------------------------------------------------------------------------
constexpr size_t kStaticCandidates = 131072;     // room for a candidate list: selections up to k ~ 60 000 read est twice
static __device__ __align__(256) unsigned char
    scratch[(sizeof(cs::TopkWs) + kStaticCandidates * cs::kCandBytes + 255) / 256 * 256];

static int static_scratch(void** out) {
    constexpr int kMaxDevices = 64;
    static std::mutex mu;
    static void* ptr_of_device[kMaxDevices] = {};
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) return CS_EHIP;
    if (dev < 0 || dev >= kMaxDevices) return CS_EINVAL;
    std::lock_guard<std::mutex> lock(mu);
    if (!ptr_of_device[dev]) {
        void* ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return CS_EHIP;
        ptr_of_device[dev] = ptr;
    }
    *out = ptr_of_device[dev];
    return CS_OK;
}

extern "C" int cs_heavy_hitters_topk_static(const float* est, int64_t d, int64_t k,
                                            int64_t* idx_out, float* val_out, void* stream) {
    if (d > CS_TOPK_STATIC_MAX_D) return CS_ELIMIT;
    void* ws = nullptr;
    const int rc = static_scratch(&ws);
    if (rc != CS_OK) return rc;
    return select_largest(est, d, k, nullptr, idx_out, val_out, ws, sizeof(scratch),
                          reinterpret_cast<hipStream_t>(stream), KeyMagnitude{});
}

extern "C" int cs_sketch_l2sq(const cs_params* p, const float* S, double* out, void* stream) {
    if (!p || !S || !out) return CS_EINVAL;
    if (p->r == 0 || p->r > CS_MAX_R || (p->r & 1u) == 0 || p->c == 0) return CS_EINVAL;
    if (reinterpret_cast<uintptr_t>(out) % 8 != 0) return CS_EINVAL;
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    k_row_sumsq<<<p->r, kSumBlock, 0, s>>>(S, p->c, out);
    k_median_of_rows<<<1, 1, 0, s>>>(out, static_cast<int>(p->r));
    return hipGetLastError() == hipSuccess ? CS_OK : CS_EHIP;
}

extern "C" int cs_heavymix_select(const float* est, int64_t d, int64_t k, const double* l2sq,
                                  uint64_t rng_seed, int64_t* idx_out, float* val_out,
                                  int64_t* n_heavy, void* workspace, size_t ws_bytes,
                                  void* stream) {
    if (!l2sq || reinterpret_cast<uintptr_t>(l2sq) % 8 != 0) return CS_EINVAL;
    if (n_heavy && reinterpret_cast<uintptr_t>(n_heavy) % 8 != 0) return CS_EINVAL;
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    KeyHeavymix kf{l2sq, static_cast<double>(k), rng_seed, 0.0};
    const int rc = select_largest(est, d, k, nullptr, idx_out, val_out, workspace, ws_bytes, s, kf);
    if (rc != CS_OK || !n_heavy) return rc;
    unsigned long long* cnt = reinterpret_cast<unsigned long long*>(n_heavy);
    k_clear_u64<<<1, 1, 0, s>>>(cnt);
    int64_t b = (k + kBlock - 1) / kBlock;
    if (b > 1024) b = 1024;
    k_count_heavy<<<static_cast<unsigned>(b), kBlock, 0, s>>>(est, idx_out, k, kf, cnt);
    return hipGetLastError() == hipSuccess ? CS_OK : CS_EHIP;
}

extern "C" int cs_select_exact_topk(const int64_t* cand, const float* x, int64_t n, int64_t k,
                                    int64_t* idx_out, float* val_out, void* workspace,
                                    size_t ws_bytes, void* stream) {
    if (!cand) return CS_EINVAL;
    // positions of the k largest |x| (ascending), then positions -> coordinates; cand is
    // ascending, so the result is ascending too
    const int rc = cs_heavy_hitters_topk(x, n, k, nullptr, idx_out, val_out, workspace, ws_bytes, stream);
    if (rc != CS_OK) return rc;
    int64_t b = (k + kBlock - 1) / kBlock;
    if (b > 4096) b = 4096;
    k_remap_positions<<<static_cast<unsigned>(b), kBlock, 0, reinterpret_cast<hipStream_t>(stream)>>>(
        idx_out, cand, k);
    return hipGetLastError() == hipSuccess ? CS_OK : CS_EHIP;
}
