/*
 * Count Sketch reference ("oracle") -- TEST INFRASTRUCTURE, NOT THE PRODUCT.
 *
 * A plain, slow, single-threaded CPU implementation of the Count Sketch data
 * structure (paper App. C, Alg. 4: init / update / estimate) with fp64
 * counters and exact integer hashing through unsigned __int128.  Only tests,
 * the smoke check and the benchmark's cpu_baseline leg may call it.  It shares
 * no source with the HIP library and is written to be checked against the
 * paper by eye: one loop nest per operation, in the order the algorithm states,
 * no blocking, no incremental tricks.
 *
 * Hash family (fixed by the benchmark definition, since the init of Alg. 4 names
 * no family for its sign and bucket hashes):
 *     p      = 2^61 - 1
 *     h_j(i) = ((a_j  * i + b_j ) mod p) mod c          bucket, 0-based
 *     s_j(i) = +1 if ((a'_j * i + b'_j) mod p) is even, else -1
 * with (a_j, b_j, a'_j, b'_j), j = 0..r-1, drawn in that order from the
 * SplitMix64 generator started at `seed`:  a = 1 + z mod (p-1),  b = z mod p.
 * Coordinates are 0-based (i in [0, d)); `i0` is the global index of g[0].
 */
#include <stdint.h>
#include <stddef.h>

typedef unsigned __int128 u128;

#define CSO_P ((((uint64_t)1) << 61) - 1)

/* SplitMix64 (Steele, Lea, Flood 2014; public-domain generator). */
static uint64_t splitmix64_next(uint64_t *state)
{
    uint64_t z;
    *state += 0x9E3779B97F4A7C15ULL;
    z = *state;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ULL;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBULL;
    return z ^ (z >> 31);
}

/* Expose the raw generator so a test can compare it with published vectors. */
void cso_splitmix64(uint64_t seed, int n, uint64_t *out)
{
    uint64_t st = seed;
    for (int t = 0; t < n; ++t) out[t] = splitmix64_next(&st);
}

/* Alg. 4 "init": draw the r bucket hashes and r sign hashes. */
void cso_derive_params(uint64_t seed, int r,
                       uint64_t *a, uint64_t *b, uint64_t *as, uint64_t *bs)
{
    uint64_t st = seed;
    for (int j = 0; j < r; ++j) {
        a[j]  = 1 + splitmix64_next(&st) % (CSO_P - 1);
        b[j]  =     splitmix64_next(&st) % CSO_P;
        as[j] = 1 + splitmix64_next(&st) % (CSO_P - 1);
        bs[j] =     splitmix64_next(&st) % CSO_P;
    }
}

static uint64_t affine_mod_p(uint64_t a, uint64_t b, uint64_t i)
{
    return (uint64_t)(((u128)a * (u128)i + (u128)b) % (u128)CSO_P);
}

static uint32_t bucket_of(uint64_t a, uint64_t b, uint32_t c, uint64_t i)
{
    return (uint32_t)(affine_mod_p(a, b, i) % (uint64_t)c);
}

static double sign_of(uint64_t as, uint64_t bs, uint64_t i)
{
    return (affine_mod_p(as, bs, i) & 1u) ? -1.0 : 1.0;
}

/* bucket[j*n + t] = h_j(idx[t]),  sign[j*n + t] = s_j(idx[t]) */
void cso_hash(int r, uint32_t c,
              const uint64_t *a, const uint64_t *b,
              const uint64_t *as, const uint64_t *bs,
              const int64_t *idx, int64_t n, uint32_t *bucket, int8_t *sign)
{
    for (int j = 0; j < r; ++j)
        for (int64_t t = 0; t < n; ++t) {
            uint64_t i = (uint64_t)idx[t];
            bucket[(size_t)j * n + t] = bucket_of(a[j], b[j], c, i);
            sign[(size_t)j * n + t] = (int8_t)sign_of(as[j], bs[j], i);
        }
}

/* Alg. 4 "update" applied to every coordinate of a dense fp32 vector:
 * T[j, h_j(i)] += scale * s_j(i) * g_i. */
void cso_accumulate_f32(int r, uint32_t c,
                        const uint64_t *a, const uint64_t *b,
                        const uint64_t *as, const uint64_t *bs,
                        double *T, const float *g, int64_t d, int64_t i0, double scale)
{
    for (int64_t t = 0; t < d; ++t) {
        uint64_t i = (uint64_t)(i0 + t);
        for (int j = 0; j < r; ++j)
            T[(size_t)j * c + bucket_of(a[j], b[j], c, i)] +=
                scale * sign_of(as[j], bs[j], i) * (double)g[t];
    }
}

/* Same update for an fp64 vector (used when a sum of workers' gradients is
 * sketched once, which by linearity equals the sum of their sketches). */
void cso_accumulate_f64(int r, uint32_t c,
                        const uint64_t *a, const uint64_t *b,
                        const uint64_t *as, const uint64_t *bs,
                        double *T, const double *g, int64_t d, int64_t i0, double scale)
{
    for (int64_t t = 0; t < d; ++t) {
        uint64_t i = (uint64_t)(i0 + t);
        for (int j = 0; j < r; ++j)
            T[(size_t)j * c + bucket_of(a[j], b[j], c, i)] +=
                scale * sign_of(as[j], bs[j], i) * g[t];
    }
}

/* Alg. 4 "update" for a list of (index, value) pairs. */
void cso_accumulate_sparse(int r, uint32_t c,
                           const uint64_t *a, const uint64_t *b,
                           const uint64_t *as, const uint64_t *bs,
                           double *T, const int64_t *idx, const double *val,
                           int64_t n, double scale)
{
    for (int64_t t = 0; t < n; ++t) {
        uint64_t i = (uint64_t)idx[t];
        for (int j = 0; j < r; ++j)
            T[(size_t)j * c + bucket_of(a[j], b[j], c, i)] +=
                scale * sign_of(as[j], bs[j], i) * val[t];
    }
}

/* median of an odd number of values: sort them, take the middle one */
static double median_odd(double *v, int r)
{
    for (int x = 1; x < r; ++x) {
        double key = v[x];
        int y = x - 1;
        while (y >= 0 && v[y] > key) { v[y + 1] = v[y]; --y; }
        v[y + 1] = key;
    }
    return v[r / 2];
}

/* Alg. 4 "estimate" of coordinate i: median_j s_j(i) * T[j, h_j(i)]. */
static double estimate_one(int r, uint32_t c,
                           const uint64_t *a, const uint64_t *b,
                           const uint64_t *as, const uint64_t *bs,
                           const double *T, uint64_t i)
{
    double v[64];
    for (int j = 0; j < r; ++j)
        v[j] = sign_of(as[j], bs[j], i) * T[(size_t)j * c + bucket_of(a[j], b[j], c, i)];
    return median_odd(v, r);
}

/* The query of every coordinate (Sec. 5.2): est[t] for i = i0 + t. */
void cso_estimate(int r, uint32_t c,
                  const uint64_t *a, const uint64_t *b,
                  const uint64_t *as, const uint64_t *bs,
                  const double *T, int64_t d, int64_t i0, double *est)
{
    for (int64_t t = 0; t < d; ++t)
        est[t] = estimate_one(r, c, a, b, as, bs, T, (uint64_t)(i0 + t));
}

void cso_estimate_sparse(int r, uint32_t c,
                         const uint64_t *a, const uint64_t *b,
                         const uint64_t *as, const uint64_t *bs,
                         const double *T, const int64_t *idx, int64_t n, double *out)
{
    for (int64_t t = 0; t < n; ++t)
        out[t] = estimate_one(r, c, a, b, as, bs, T, (uint64_t)idx[t]);
}

/* single-row estimates s_j(i) * T[j, h_j(i)] (before the median), rows[j*d + t];
 * lets tests look at the per-row error the l2 guarantee is stated for. */
void cso_row_estimates(int r, uint32_t c,
                       const uint64_t *a, const uint64_t *b,
                       const uint64_t *as, const uint64_t *bs,
                       const double *T, int64_t d, int64_t i0, double *rows)
{
    for (int j = 0; j < r; ++j)
        for (int64_t t = 0; t < d; ++t) {
            uint64_t i = (uint64_t)(i0 + t);
            rows[(size_t)j * d + t] =
                sign_of(as[j], bs[j], i) * T[(size_t)j * c + bucket_of(a[j], b[j], c, i)];
        }
}
