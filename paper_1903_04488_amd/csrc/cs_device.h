// Device-side arithmetic shared by the kernels: hashing modulo the Mersenne prime
// p = 2^61 - 1 kept in registers, and a few wavefront helpers.  gfx950 only.
//
// Hash family (the sign and bucket hashes that Alg. 4 of the paper's App. C initialises):
//     h_j(i) = ((a_j * i + b_j) mod p) mod c,     s_j(i) = +1 / -1 by the parity of
//     ((a'_j * i + b'_j) mod p).
// A hash value x in [0, p) is carried as y = x + 1 in [1, p].  In that form "add a constant
// A in [0, p) modulo p" needs no comparison: t = y + A < 2^62, and x + A >= p exactly when
// bit 61 of t is set, in which case subtracting p = 2^61 - 1 is "clear bit 61, add 1":
//     y' = (t & p) + (t >> 61).
// The streaming kernels use this to step a thread's hash state from coordinate i to i + D
// with two 64-bit adds, a shift and a mask instead of a 61 x 61 bit multiplication; the
// results are bit-identical to the definition because the identity holds over the integers.
#pragma once

#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "csketch.h"

namespace cs {

constexpr uint64_t kP61 = (1ull << 61) - 1;
constexpr int kBlock = 256;                 // threads per workgroup (4 wavefronts)

// s < 2^63  ->  s mod p in [0, p)
__host__ __device__ __forceinline__ uint64_t reduce_p(uint64_t s) {
    s = (s & kP61) + (s >> 61);             // <= p + 3
    s = (s & kP61) + (s >> 61);             // <= p
    return s == kP61 ? 0 : s;
}

__device__ __forceinline__ uint64_t mulhi64(uint64_t a, uint64_t b) { return __umul64hi(a, b); }

// (a * i) mod p for a, i < 2^61.  a*i = hi * 2^64 + lo with 2^64 = 8 (mod p), 2^61 = 1 (mod p).
__device__ __forceinline__ uint64_t mulmod_p(uint64_t a, uint64_t i) {
    const uint64_t lo = a * i;
    const uint64_t hi = mulhi64(a, i);                    // < 2^58
    return reduce_p((hi << 3) + (lo >> 61) + (lo & kP61)); // < 2^61 + 8 + 2^61
}

// y-form state of  (a * i + b) mod p
__device__ __forceinline__ uint64_t hash_state(uint64_t a, uint64_t b, uint64_t i) {
    return reduce_p(mulmod_p(a, i) + b) + 1;
}

// state of coordinate i  ->  state of coordinate i + D, where A = (a * D) mod p
__device__ __forceinline__ uint64_t hash_advance(uint64_t y, uint64_t A) {
    const uint64_t t = y + A;
    return (t & kP61) + (t >> 61);
}

// Column count with what the reduction of a hash value modulo c needs.  For a power of two
// that is a mask.  Otherwise (the paper's 180 000-column sketches, Table 1) the remainder
// of a 61-bit value by a 32-bit one is taken with one high multiplication: with
// M = floor((2^64 - 1) / c), q = floor(x M / 2^64) is floor(x / c) or one less for every
// x < 2^61 (the error x (2^64 - M c) / (c 2^64) is below x / 2^64 < 1/8), so x - q c lies in
// [0, 2c) and one conditional subtraction finishes it.  M costs one division per thread.
struct Columns {
    uint32_t c;
    uint64_t M;
};
template <bool POW2>
__device__ __forceinline__ Columns columns_of(uint32_t c) {
    return Columns{c, POW2 ? 0ull : ~0ull / c};
}
template <bool POW2>
__device__ __forceinline__ uint32_t bucket_of(uint64_t y, const Columns& col) {
    if (POW2) return (static_cast<uint32_t>(y) - 1u) & (col.c - 1u);
    const uint64_t x = y - 1;
    const uint64_t rem = x - mulhi64(x, col.M) * col.c;      // < 2c
    return static_cast<uint32_t>(rem >= col.c ? rem - col.c : rem);
}

// 0x80000000 when s = -1 (x odd, i.e. y even), 0 when s = +1: XOR it into a float's bits.
__device__ __forceinline__ uint32_t sign_flip_of(uint64_t y) {
    return (~static_cast<uint32_t>(y)) << 31;
}

__device__ __forceinline__ float apply_sign(float v, uint32_t flip) {
    return __uint_as_float(__float_as_uint(v) ^ flip);
}

// 16-bit storage of sketch cells (Sec. 6 of the paper remarks that 16 bits per cell suffice):
// round to nearest, ties to even.  FMT 0 = bfloat16 (upper half of the binary32 pattern),
// FMT 1 = IEEE binary16 (the hardware conversion, whose default rounding is the same).
template <int FMT>
__device__ __forceinline__ uint16_t to_16(float v) {
    if (FMT == 1) return __half_as_ushort(__float2half_rn(v));
    const uint32_t bits = __float_as_uint(v);
    if ((bits & 0x7fffffffu) > 0x7f800000u) return static_cast<uint16_t>((bits >> 16) | 0x0040u);  // NaN
    return static_cast<uint16_t>((bits + 0x7fffu + ((bits >> 16) & 1u)) >> 16);
}
template <int FMT>
__device__ __forceinline__ float from_16(uint16_t q) {
    if (FMT == 1) return __half2float(__ushort_as_half(q));
    return __uint_as_float(static_cast<uint32_t>(q) << 16);
}

// fp32 add into global memory, result not needed: one hardware global_atomic_add_f32.
__device__ __forceinline__ void atomic_add_noret(float* addr, float v) {
    __hip_atomic_fetch_add(addr, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Lane l receives the value of lane l - N of its row of 16 lanes (DPP row_shr); lanes whose
// source would lie outside the row receive `fill`.
template <int N>
__device__ __forceinline__ uint32_t row_shr(uint32_t v, uint32_t fill) {
    return static_cast<uint32_t>(__builtin_amdgcn_update_dpp(
        static_cast<int>(fill), static_cast<int>(v), 0x110 + N, 0xf, 0xf, false));
}
// Lane l receives the value of lane l + 1 of its row of 16 lanes (DPP row_shl:1), else `fill`.
__device__ __forceinline__ uint32_t row_shl1(uint32_t v, uint32_t fill) {
    return static_cast<uint32_t>(__builtin_amdgcn_update_dpp(
        static_cast<int>(fill), static_cast<int>(v), 0x101, 0xf, 0xf, false));
}

// Wavefront-level pre-aggregation of an atomic add.  Within each row of 16 lanes, every
// maximal run of consecutive lanes holding the same key is summed (segmented inclusive scan
// with head flags, offsets 1, 2, 4, 8); returns true in the last lane of each run, whose `v`
// then holds the run's total.  Only adjacent lanes are ever merged, so the result is right
// for any key pattern provided no run is longer than 2^nsteps lanes (nsteps = 4 covers a
// whole row and is always safe; the caller passes the bound that holds for its stride).
__device__ __forceinline__ bool segment_sum16(uint32_t key, float& v, int nsteps) {
    const uint32_t kNone = 0xffffffffu;                      // never a valid key
    const uint32_t head = row_shr<1>(key, kNone) != key ? 1u : 0u;   // first lane of its run
    uint32_t f = head;
#define CS_SEG_STEP(N)                                                          \
    {                                                                           \
        const float v2 = __uint_as_float(row_shr<N>(__float_as_uint(v), 0u));   \
        const uint32_t f2 = row_shr<N>(f, 1u);                                  \
        v += f ? 0.0f : v2;                                                     \
        f |= f2;                                                                \
    }
    if (nsteps > 0) CS_SEG_STEP(1)
    if (nsteps > 1) CS_SEG_STEP(2)
    if (nsteps > 2) CS_SEG_STEP(4)
    if (nsteps > 3) CS_SEG_STEP(8)
#undef CS_SEG_STEP
    return row_shl1(head, 1u) != 0u;                         // next lane starts a new run
}

// Median of an odd number R of floats held in registers (compile-time R), as Alg. 4's estimate
// takes it: sort, then the middle element.  The sort is an insertion sort written as a fixed
// sequence of compare-exchanges on "left > right": element x is exchanged downwards through
// the sorted prefix; once a comparison fails the remaining ones of that pass compare
// neighbours of the prefix, which are in order, and change nothing.  With ordinary numbers
// any sorting network gives the same middle element; with a NaN among the values (every
// comparison with it is false) the result depends on the sequence of comparisons, and this
// sequence is the one a plain insertion sort with ">" makes: a NaN stays where it was put and
// blocks what lies above it from moving down.  Infinities order as usual; -0 and +0 compare
// equal and keep their order.
template <int R>
__device__ __forceinline__ float median_odd(float (&v)[R]) {
#pragma unroll
    for (int x = 1; x < R; ++x) {
#pragma unroll
        for (int y = x - 1; y >= 0; --y) {
            const bool exchange = v[y] > v[y + 1];
            const float lo = exchange ? v[y + 1] : v[y];
            const float hi = exchange ? v[y] : v[y + 1];
            v[y] = lo;
            v[y + 1] = hi;
        }
    }
    return v[R / 2];
}

}  // namespace cs
