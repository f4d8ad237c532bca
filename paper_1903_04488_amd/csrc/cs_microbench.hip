// Microbenchmarks of the MI355X memory system that the kernel design rests on (standalone
// program, not part of libcsketch.so): rate of fp32 / integer global atomics by access pattern,
// table size and number of active XCDs; random and contiguous gathers; streaming read bandwidth
// by buffer size; the reads of the bundle update without its processing; lane-strided
// streaming; LDS atomics.  Every access is in bounds by
// construction (indices are masked with the table size).
//
//   hipcc -O3 --offload-arch=gfx950 -munsafe-fp-atomics -o cs_microbench cs_microbench.hip
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

#define CK(x) do { hipError_t e = (x); if (e != hipSuccess) { printf("HIP error %s at %s:%d\n", hipGetErrorString(e), __FILE__, __LINE__); exit(1); } } while (0)

__device__ __forceinline__ uint32_t mix(uint32_t x) {
    x ^= x >> 16; x *= 0x7feb352du; x ^= x >> 15; x *= 0x846ca68bu; x ^= x >> 16; return x;
}

// mode 0: every lane its own random cell. mode 1: wave picks a random base, lanes base+lane.
// mode 2: lanes base + floor(lane*1.3). mode 3: base aligned to 64 floats, + lane.
// mode 4: groups of 16 lanes contiguous (4 random bases per wave)
// modes 5-7: groups of 8 / 16 / 32 lanes at random addresses aligned to 32 / 64 / 128 bytes
template <int MODE, bool ATOMIC>
__global__ void __launch_bounds__(256) k_scatter(float* table, uint32_t mask, int iters, float* sink) {
    const uint32_t gtid = blockIdx.x * 256 + threadIdx.x;
    const uint32_t wave = gtid >> 6, lane = threadIdx.x & 63;
    float acc = 0.f;
    for (int it = 0; it < iters; ++it) {
        uint32_t cell;
        if (MODE == 0) cell = mix(gtid * 9781u + it * 0x9e3779b9u) & mask;
        else {
            uint32_t base = mix(wave * 9781u + it * 0x9e3779b9u);
            if (MODE == 1) cell = (base + lane) & mask;
            else if (MODE == 2) cell = (base + (lane * 13u) / 10u) & mask;
            else if (MODE == 3) cell = ((base & ~63u) + lane) & mask;
            else if (MODE == 4) { base = mix((wave * 4 + (lane >> 4)) * 9781u + it * 0x9e3779b9u); cell = (base + (lane & 15)) & mask; }
            else {
                // modes 5, 6, 7: groups of 8, 16, 32 lanes, each group at a random address
                // aligned to its own size (32, 64, 128 bytes)
                const uint32_t gl = MODE == 5 ? 8u : MODE == 6 ? 16u : 32u;
                base = mix((wave * (64u / gl) + lane / gl) * 9781u + it * 0x9e3779b9u);
                cell = ((base & ~(gl - 1u)) + (lane & (gl - 1u))) & mask;
            }
        }
        if (ATOMIC) __hip_atomic_fetch_add(table + cell, 1.0f, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        else acc += table[cell];
    }
    if (!ATOMIC && acc == 12345.678f) sink[0] = acc;
}

__global__ void __launch_bounds__(256) k_read(const float4* __restrict__ buf, size_t n4, float* sink) {
    size_t stride = (size_t)gridDim.x * 256;
    float acc = 0.f;
    for (size_t t = (size_t)blockIdx.x * 256 + threadIdx.x; t < n4; t += stride) {
        float4 v = buf[t]; acc += v.x + v.y + v.z + v.w;
    }
    if (acc == 12345.678f) sink[0] = acc;
}

// each lane streams its own contiguous run of `run` floats; runs of a wave are D floats apart.
template <int VEC>
__global__ void __launch_bounds__(256) k_lane_runs(const float* __restrict__ buf, size_t D, int run, size_t nwaves_total, float* sink) {
    const size_t wave = ((size_t)blockIdx.x * 256 + threadIdx.x) >> 6;
    const uint32_t lane = threadIdx.x & 63;
    // wave q handles offset q*run within each of the 64 lane-blocks of size D (needs nwaves*run <= D)
    const float* p = buf + (size_t)lane * D + wave * run;
    float acc = 0.f;
    if (VEC == 4) { for (int m = 0; m < run; m += 4) { float4 v = *reinterpret_cast<const float4*>(p + m); acc += v.x + v.y + v.z + v.w; } }
    else if (VEC == 1) { for (int m = 0; m < run; ++m) acc += p[m]; }
    if (acc == 12345.678f) sink[0] = acc;
}

__device__ __forceinline__ uint32_t xcc_id() {
    uint32_t x; asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID)" : "=s"(x)); return x & 15u;
}

__global__ void k_xcc_map(uint32_t* out) { if (threadIdx.x == 0) out[blockIdx.x] = xcc_id(); }

// TYPE 0: f32, 1: u32, 2: u64, 3: plain store f32, 4: f32 atomic with return
// MODE 0 random lanes, 1 wave-contiguous
template <int TYPE, int MODE>
__global__ void __launch_bounds__(256) k_atomic(void* table, uint32_t mask, int iters, uint32_t xcd_limit, float* sink) {
    if (xcc_id() >= xcd_limit) return;
    const uint32_t gtid = blockIdx.x * 256 + threadIdx.x;
    const uint32_t wave = gtid >> 6, lane = threadIdx.x & 63;
    float acc = 0.f;
    for (int it = 0; it < iters; ++it) {
        uint32_t cell = MODE == 0 ? (mix(gtid * 9781u + it * 0x9e3779b9u) & mask)
                                  : ((mix(wave * 9781u + it * 0x9e3779b9u) + lane) & mask);
        if (TYPE == 0) __hip_atomic_fetch_add((float*)table + cell, 1.0f, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        else if (TYPE == 1) __hip_atomic_fetch_add((uint32_t*)table + cell, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        else if (TYPE == 2) __hip_atomic_fetch_add((unsigned long long*)table + cell, 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        else if (TYPE == 3) ((float*)table)[cell] = (float)it;
        else acc += __hip_atomic_fetch_add((float*)table + cell, 1.0f, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    if (TYPE == 4 && acc == 12345.678f) sink[0] = acc;
}

// LDS atomics: LDSW words of LDS per block
template <int LDSW, int TYPE, int MODE>
__global__ void __launch_bounds__(256) k_lds(int iters, float* sink) {
    __shared__ uint32_t lds[LDSW];
    for (int t = threadIdx.x; t < LDSW; t += 256) lds[t] = 0;
    __syncthreads();
    const uint32_t gtid = blockIdx.x * 256 + threadIdx.x;
    for (int it = 0; it < iters; ++it) {
        uint32_t cell = MODE == 0 ? (mix(gtid * 9781u + it * 0x9e3779b9u) & (LDSW - 1))
                                  : ((mix((gtid >> 6) * 9781u + it * 0x9e3779b9u) + (threadIdx.x & 63)) & (LDSW - 1));
        if (TYPE == 0) atomicAdd(reinterpret_cast<float*>(&lds[cell]), 1.0f);
        else atomicAdd(&lds[cell], 1u);
    }
    __syncthreads();
    if (lds[threadIdx.x] == 0x12345678u) sink[0] = 1.f;
}

// ---- reads in the order and piece size of the bundle update, without its processing ----------
// Eight vectors; a wavefront owns 128 residues and visits base + k G for k = 0 .. K-1 (G = the
// gap of a visit list), reading 512 bytes of every vector per visit, the next visit requested
// before the current one is consumed.  MODE 0: 8 bytes per lane and vector (8 loads); MODE 1:
// 16 bytes per lane, two vectors per load (4 loads).  k_plain8 is the plain read of the same
// vectors (blockIdx.y = vector).  All addresses are below d by the `ok` test.
typedef float vec2f __attribute__((ext_vector_type(2)));
typedef float vec4f __attribute__((ext_vector_type(4)));
typedef vec2f __attribute__((aligned(4))) vec2f_u;
typedef vec4f __attribute__((aligned(4))) vec4f_u;
struct Vectors8 { const float* g[8]; };

__global__ void __launch_bounds__(256) k_plain8(Vectors8 p, int64_t d, float* sink) {
    const float4* x4 = (const float4*)p.g[blockIdx.y];
    const int64_t n4 = d / 4, stride = (int64_t)gridDim.x * 256;
    float acc = 0.f;
    int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
    for (; t + stride < n4; t += 2 * stride) {
        float4 a = x4[t], b = x4[t + stride];
        acc += a.x + a.y + a.z + a.w + b.x + b.y + b.z + b.w;
    }
    if (t < n4) { float4 a = x4[t]; acc += a.x + a.y + a.z + a.w; }
    if (acc == 12345.678f) sink[0] = acc;
}

// DEAL 1: workgroups are dealt to the XCDs (blockIdx.x mod 8) in blocks of 4 neighbours, as the
// update does, so that most of the lines that two neighbouring pieces share are fetched by one L2.
template <int MODE, int NWAVE, int DEAL>
__global__ void __launch_bounds__(64 * NWAVE) k_visit_reads(Vectors8 p, int64_t d, int64_t G, int K, float* sink) {
    const int lane = threadIdx.x & 63;
    int64_t set = blockIdx.x;
    if (DEAL) {
        const int64_t slot = set >> 3;
        set = ((slot / 4) * 8 + (set & 7)) * 4 + slot % 4;
    }
    const int64_t base = (set * NWAVE + (threadIdx.x >> 6)) * 128;
    if (base >= G) return;
    float acc = 0.f, pre[16];
    auto load = [&](int64_t pos) {
        if (MODE == 0) {
#pragma unroll
            for (int w = 0; w < 8; ++w) {
                vec2f u = *(const vec2f_u*)(p.g[w] + pos + lane * 2);
                pre[2 * w] = u.x; pre[2 * w + 1] = u.y;
            }
        } else {
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                const float* src = (lane >> 5) ? p.g[2 * w + 1] : p.g[2 * w];
                vec4f u = *(const vec4f_u*)(src + pos + (lane & 31) * 4);
                pre[4 * w] = u.x; pre[4 * w + 1] = u.y; pre[4 * w + 2] = u.z; pre[4 * w + 3] = u.w;
            }
        }
    };
    int64_t pos = base;
    bool ok = pos + 128 <= d;
    if (ok) load(pos);
    for (int k = 0; k < K; ++k) {
        float cur[16];
#pragma unroll
        for (int t = 0; t < 16; ++t) cur[t] = ok ? pre[t] : 0.f;
        pos += G;
        ok = (k + 1 < K) && pos + 128 <= d;
        if (ok) load(pos);
#pragma unroll
        for (int t = 0; t < 16; ++t) acc += cur[t];
    }
    if (acc == 12345.678f) sink[0] = acc;
}

template <typename F>
float time_ms(F f, int reps = 3) {
    hipEvent_t a, b; CK(hipEventCreate(&a)); CK(hipEventCreate(&b));
    f(); CK(hipDeviceSynchronize());
    float best = 1e30f;
    for (int r = 0; r < reps; ++r) {
        CK(hipEventRecord(a)); f(); CK(hipEventRecord(b)); CK(hipEventSynchronize(b));
        float ms; CK(hipEventElapsedTime(&ms, a, b)); if (ms < best) best = ms;
    }
    CK(hipGetLastError());
    return best;
}

int main() {
    hipDeviceProp_t prop; CK(hipGetDeviceProperties(&prop, 0));
    printf("device %s CUs=%d clock=%d kHz l2=%d B lds/block=%zu\n", prop.name, prop.multiProcessorCount, prop.clockRate, prop.l2CacheSize, prop.sharedMemPerBlock);
    float* sink; CK(hipMalloc(&sink, 16));
    const int blocks = 256 * 8, iters = 256;
    const double nops = (double)blocks * 256 * iters;
    for (uint32_t cells : {163840u / 1u, 1u << 20, 5u << 20, 32u << 20, 168u << 20}) {
        uint32_t pow2 = 1; while (pow2 * 2 <= cells) pow2 *= 2;
        float* table; CK(hipMalloc(&table, (size_t)pow2 * 4)); CK(hipMemset(table, 0, (size_t)pow2 * 4));
        uint32_t mask = pow2 - 1;
        printf("table %u cells (%.2f MB):\n", pow2, pow2 * 4.0 / 1e6);
        float ms;
        ms = time_ms([&] { k_scatter<0, true><<<blocks, 256>>>(table, mask, iters, sink); });  printf("  atomic random lanes      : %8.3f ms  %7.1f Gop/s\n", ms, nops / ms / 1e6);
        ms = time_ms([&] { k_scatter<1, true><<<blocks, 256>>>(table, mask, iters, sink); });  printf("  atomic wave-contiguous   : %8.3f ms  %7.1f Gop/s\n", ms, nops / ms / 1e6);
        ms = time_ms([&] { k_scatter<3, true><<<blocks, 256>>>(table, mask, iters, sink); });  printf("  atomic wave-contig align : %8.3f ms  %7.1f Gop/s\n", ms, nops / ms / 1e6);
        ms = time_ms([&] { k_scatter<2, true><<<blocks, 256>>>(table, mask, iters, sink); });  printf("  atomic stride 1.3        : %8.3f ms  %7.1f Gop/s\n", ms, nops / ms / 1e6);
        ms = time_ms([&] { k_scatter<4, true><<<blocks, 256>>>(table, mask, iters, sink); });  printf("  atomic 16-lane groups    : %8.3f ms  %7.1f Gop/s\n", ms, nops / ms / 1e6);
        ms = time_ms([&] { k_scatter<5, true><<<blocks, 256>>>(table, mask, iters, sink); });  printf("  atomic 8 x 32 B aligned  : %8.3f ms  %7.1f Gop/s  %6.1f G groups/s\n", ms, nops / ms / 1e6, nops / 8 / ms / 1e6);
        ms = time_ms([&] { k_scatter<6, true><<<blocks, 256>>>(table, mask, iters, sink); });  printf("  atomic 4 x 64 B aligned  : %8.3f ms  %7.1f Gop/s  %6.1f G groups/s\n", ms, nops / ms / 1e6, nops / 16 / ms / 1e6);
        ms = time_ms([&] { k_scatter<7, true><<<blocks, 256>>>(table, mask, iters, sink); });  printf("  atomic 2 x 128 B aligned : %8.3f ms  %7.1f Gop/s  %6.1f G groups/s\n", ms, nops / ms / 1e6, nops / 32 / ms / 1e6);
        ms = time_ms([&] { k_scatter<0, false><<<blocks, 256>>>(table, mask, iters, sink); }); printf("  gather random lanes      : %8.3f ms  %7.1f Gop/s\n", ms, nops / ms / 1e6);
        ms = time_ms([&] { k_scatter<1, false><<<blocks, 256>>>(table, mask, iters, sink); }); printf("  gather wave-contiguous   : %8.3f ms  %7.1f Gop/s\n", ms, nops / ms / 1e6);
        ms = time_ms([&] { k_scatter<2, false><<<blocks, 256>>>(table, mask, iters, sink); }); printf("  gather stride 1.3        : %8.3f ms  %7.1f Gop/s\n", ms, nops / ms / 1e6);
        CK(hipFree(table));
        fflush(stdout);
    }
    // streaming read bandwidth vs buffer size, buffer re-read `passes` times back to back
    for (size_t mb : {32, 64, 128, 192, 256, 512, 1024, 4096, 12800}) {
        size_t bytes = mb * 1000000ull / 16 * 16;
        float4* buf; CK(hipMalloc(&buf, bytes)); CK(hipMemset(buf, 0, bytes));
        size_t n4 = bytes / 16;
        int passes = mb <= 1024 ? 8 : 2;
        float ms = time_ms([&] { for (int p = 0; p < passes; ++p) k_read<<<256 * 16, 256>>>(buf, n4, sink); });
        printf("read %6zu MB x%d : %8.3f ms  %7.2f TB/s\n", mb, passes, ms, (double)bytes * passes / ms / 1e9);
        CK(hipFree(buf));
        fflush(stdout);
    }
    // reads of the bundle update without its processing: 8 vectors of 10^8 floats
    {
        const int64_t d = 100000000;
        Vectors8 v8;
        for (int w = 0; w < 8; ++w) { float* x; CK(hipMalloc(&x, d * 4)); CK(hipMemset(x, 0, d * 4)); v8.g[w] = x; }
        const double bytes = 8.0 * d * 4;
        float t = time_ms([&] { k_plain8<<<dim3(512, 8), 256>>>(v8, d, sink); }, 5);
        printf("8 vectors plain read               : %8.3f ms  %7.2f TB/s\n", t, bytes / t / 1e9);
        for (int64_t G : {456789ll, 456788ll, 456792ll, 456800ll, 456704ll, 594161ll, 594160ll, 594176ll, 877855ll, 1324789ll}) {
            const int K = (int)((d + G - 1) / G);
            const unsigned nwaves = (unsigned)((G + 127) / 128);
            const unsigned wg2 = ((nwaves + 1) / 2 + 31) / 32 * 32, wg4 = ((nwaves + 3) / 4 + 31) / 32 * 32;
            t = time_ms([&] { k_visit_reads<0, 2, 0><<<wg2, 128>>>(v8, d, G, K, sink); }, 5);
            printf("visits G=%7lld K=%3d 8 B/lane                 : %8.3f ms  %7.2f TB/s\n", (long long)G, K, t, bytes / t / 1e9);
            t = time_ms([&] { k_visit_reads<1, 2, 0><<<wg2, 128>>>(v8, d, G, K, sink); }, 5);
            printf("visits G=%7lld K=%3d 16 B/lane                : %8.3f ms  %7.2f TB/s\n", (long long)G, K, t, bytes / t / 1e9);
            t = time_ms([&] { k_visit_reads<1, 2, 1><<<wg2, 128>>>(v8, d, G, K, sink); }, 5);
            printf("visits G=%7lld K=%3d 16 B/lane, dealt in fours: %8.3f ms  %7.2f TB/s\n", (long long)G, K, t, bytes / t / 1e9);
            t = time_ms([&] { k_visit_reads<1, 4, 0><<<wg4, 256>>>(v8, d, G, K, sink); }, 5);
            printf("visits G=%7lld K=%3d 16 B/lane, 4 wavefronts  : %8.3f ms  %7.2f TB/s\n", (long long)G, K, t, bytes / t / 1e9);
            fflush(stdout);
        }
        for (int w = 0; w < 8; ++w) CK(hipFree((void*)v8.g[w]));
    }
    // lane-strided streaming: 64 lane-blocks of D floats each; all waves together cover them once
    {
        size_t D = 1u << 19;                       // floats between lanes
        size_t total = 64 * D;                     // 33.5M floats = 134 MB
        float* buf; CK(hipMalloc(&buf, total * 4)); CK(hipMemset(buf, 0, total * 4));
        for (int run : {16, 64, 256}) {
            size_t nwaves = D / run;               // waves needed
            int nblocks = (int)(nwaves / 4);
            float ms = time_ms([&] { k_lane_runs<4><<<nblocks, 256>>>(buf, D, run, nwaves, sink); });
            printf("lane-runs float4 run=%3d: %8.3f ms  %7.2f TB/s\n", run, ms, (double)total * 4 / ms / 1e9);
            ms = time_ms([&] { k_lane_runs<1><<<nblocks, 256>>>(buf, D, run, nwaves, sink); });
            printf("lane-runs dword  run=%3d: %8.3f ms  %7.2f TB/s\n", run, ms, (double)total * 4 / ms / 1e9);
        }
        float ms = time_ms([&] { k_read<<<256 * 16, 256>>>((const float4*)buf, total / 4, sink); });
        printf("same buffer coalesced   : %8.3f ms  %7.2f TB/s\n", ms, (double)total * 4 / ms / 1e9);
        CK(hipFree(buf));
    }
    uint32_t* map; CK(hipMalloc(&map, 64 * 4));
    k_xcc_map<<<64, 64>>>(map); CK(hipDeviceSynchronize());
    uint32_t h[64]; CK(hipMemcpy(h, map, sizeof(h), hipMemcpyDeviceToHost));
    printf("blockIdx -> XCC_ID:"); for (int i = 0; i < 64; ++i) printf(" %u", h[i]); printf("\n");

    const int iters2 = 128;
    const double nops2 = (double)blocks * 256 * iters2;
    const uint32_t cells2 = 4u << 20;     // 4M cells
    void* table; CK(hipMalloc(&table, (size_t)cells2 * 8)); CK(hipMemset(table, 0, (size_t)cells2 * 8));
    const uint32_t mask = cells2 - 1;
    float ms;
#define RUN(T, M, X, label) ms = time_ms([&] { k_atomic<T, M><<<blocks, 256>>>(table, mask, iters2, X, sink); }); \
    printf("  %-34s xcds<%u: %8.3f ms  %8.1f Gop/s\n", label, X, ms, nops2 * (X > 8 ? 8 : X) / 8 / ms / 1e6);
    RUN(0, 0, 8, "f32 atomic random");
    RUN(0, 1, 8, "f32 atomic wave-contiguous");
    RUN(4, 0, 8, "f32 atomic+return random");
    RUN(1, 0, 8, "u32 atomic random");
    RUN(1, 1, 8, "u32 atomic wave-contiguous");
    RUN(2, 0, 8, "u64 atomic random");
    RUN(2, 1, 8, "u64 atomic wave-contiguous");
    RUN(3, 0, 8, "plain store random");
    RUN(3, 1, 8, "plain store wave-contiguous");
    RUN(0, 0, 1, "f32 atomic random");
    RUN(0, 0, 2, "f32 atomic random");
    RUN(0, 0, 4, "f32 atomic random");
    RUN(0, 1, 1, "f32 atomic wave-contiguous");
    RUN(1, 0, 1, "u32 atomic random");
    fflush(stdout);
    // small table (fits one L2): does the rate change when one XCD works alone?
    const uint32_t small_mask = (1u << 17) - 1;
    ms = time_ms([&] { k_atomic<0, 0><<<blocks, 256>>>(table, small_mask, iters2, 1, sink); });
    printf("  f32 atomic random 0.5MB table, 1 XCD: %8.3f ms %8.1f Gop/s\n", ms, nops2 / 8 / ms / 1e6);
    ms = time_ms([&] { k_atomic<0, 0><<<blocks, 256>>>(table, small_mask, iters2, 8, sink); });
    printf("  f32 atomic random 0.5MB table, 8 XCD: %8.3f ms %8.1f Gop/s\n", ms, nops2 / ms / 1e6);

    const int lb = 256 * 16, li = 512;
    const double ln = (double)lb * 256 * li;
    ms = time_ms([&] { k_lds<4096, 0, 0><<<lb, 256>>>(li, sink); }); printf("LDS 16KB f32 random     : %8.3f ms %8.1f Gop/s\n", ms, ln / ms / 1e6);
    ms = time_ms([&] { k_lds<4096, 0, 1><<<lb, 256>>>(li, sink); }); printf("LDS 16KB f32 contiguous : %8.3f ms %8.1f Gop/s\n", ms, ln / ms / 1e6);
    ms = time_ms([&] { k_lds<4096, 1, 0><<<lb, 256>>>(li, sink); }); printf("LDS 16KB u32 random     : %8.3f ms %8.1f Gop/s\n", ms, ln / ms / 1e6);
    ms = time_ms([&] { k_lds<4096, 1, 1><<<lb, 256>>>(li, sink); }); printf("LDS 16KB u32 contiguous : %8.3f ms %8.1f Gop/s\n", ms, ln / ms / 1e6);
    ms = time_ms([&] { k_lds<16384, 0, 0><<<lb, 256>>>(li, sink); }); printf("LDS 64KB f32 random     : %8.3f ms %8.1f Gop/s\n", ms, ln / ms / 1e6);
    ms = time_ms([&] { k_lds<16384, 1, 0><<<lb, 256>>>(li, sink); }); printf("LDS 64KB u32 random     : %8.3f ms %8.1f Gop/s\n", ms, ln / ms / 1e6);
    return 0;
}
