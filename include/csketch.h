/*
 * csketch.h -- C ABI of the Count Sketch hot path of Sketched-SGD for AMD MI355X (gfx950).
 *
 * What the library computes (paper = "Communication-efficient Distributed SGD with
 * Sketching", arXiv 1903.04488):
 *   - Count Sketch update / estimate                      App. C, Alg. 4
 *   - merge of workers' sketches, S = (1/W) sum_i S^i     Sec. 3; aggregation step of Alg. 2
 *                                                         and Alg. 3
 *   - recovery of the largest coordinates by querying     Sec. 5.2; recovery step of Alg. 3
 *     every coordinate and keeping the k largest
 *   - second round: exact values of the chosen            Sec. 4; Alg. 1 step 5; worker-query
 *     coordinates, summed over workers                    step of Alg. 3
 *   - momentum and error accumulation (Alg. 3's momentum and error-accumulation steps and its
 *     zeroing of u, v on updated coordinates) held as sketches, which is possible because
 *     the sketch is linear (Sec. 3).
 *
 * Conventions
 *   - Every function returns CS_OK (0) or a negative cs_status; none throws, exits or prints.
 *   - "device" pointers are HIP device memory owned by the caller; "host" pointers are
 *     ordinary host memory.  The library allocates no device memory and keeps no state:
 *     cs_params is a plain struct, immutable after cs_params_init, so calls are re-entrant.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Kernels are
 *     enqueued on it and the call returns without synchronising.  Launch failures are
 *     reported as CS_EHIP; faults inside a kernel surface at the caller's next synchronise.
 *   - A sketch table is float[r][c], row-major, contiguous.  Coordinates are 0-based int64.
 *   - Device data are not validated: NaN / Inf propagate.  In cs_heavy_hitters_topk a NaN
 *     magnitude orders above every finite value (comparison is on the bit pattern).
 *   - fp32 atomic adds make sketch cells depend on summation order in the last bits; every
 *     other output is a deterministic function of its inputs.  cs_fixed_accumulate is the
 *     update with order-independent (64-bit fixed-point) sums, for debugging and checkpoints.
 *   - The one entry point with memory of its own is cs_heavy_hitters_topk_static (a fixed
 *     array in the library's device image, for callers that cannot allocate).
 *
 * Hash family (Alg. 4 init draws r sign and r bucket hashes; the family itself is fixed by
 * the benchmark definition): with p = 2^61 - 1,
 *     h_j(i) = ((a_j  * i + b_j ) mod p) mod c                       bucket of row j
 *     s_j(i) = +1 if ((a'_j * i + b'_j) mod p) is even, -1 if odd     sign of row j
 * The 4r constants are drawn, in the order a_0, b_0, a'_0, b'_0, a_1, ..., from the
 * SplitMix64 generator started at `seed`:  a = 1 + z mod (p - 1),  b = z mod p.
 */
#ifndef CSKETCH_H
#define CSKETCH_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define CS_MAX_R 16          /* covers the paper's largest sketch (15 rows, Table 1) */

typedef enum cs_status {
    CS_OK = 0,
    CS_EINVAL = -1,       /* bad argument (null pointer, size out of range, even r, ...) */
    CS_EWORKSPACE = -2,   /* workspace smaller than cs_topk_workspace_bytes() says */
    CS_EHIP = -3,         /* a HIP runtime call or kernel launch failed */
    CS_ELIMIT = -4        /* input larger than an entry point with built-in scratch accepts */
} cs_status;

/* Traversal of one row (derived from a_j and c; does not change any result).  Because the
 * bucket hash is affine mod p, coordinates i, i + D, i + 2D, ... fall into buckets that
 * advance by a constant (a*D mod p) mod c, plus one for every wrap around p.  Two strides
 * with a small advance are kept per row:
 *   D  for the estimate: a group of `lanes` lanes takes coordinates D apart and so gathers
 *      from neighbouring cells of the row (shared cache lines);
 *   Dw for the update: one lane walks i, i + Dw, i + 2 Dw, ... and keeps the running sum of
 *      the cell it is in, issuing one atomic add per cell it leaves instead of one per
 *      coordinate. */
typedef struct cs_row_plan {
    uint64_t D;           /* lane stride of the estimate, >= 1 */
    uint64_t AD;          /* (a_j  * D) mod p */
    uint64_t ADs;         /* (a'_j * D) mod p */
    uint64_t Dw;          /* walk stride of the update, >= 1 */
    uint64_t ADw;         /* (a_j  * Dw) mod p */
    uint64_t ADws;        /* (a'_j * Dw) mod p */
    int32_t  lanes;       /* lanes per group: 16, 32 or 64 (a wavefront holds 64 / lanes groups) */
    int32_t  scan_steps;  /* 0..4: doubling steps of the in-register pre-aggregation that are
                             enough to add up the longest run of neighbouring lanes that can
                             fall into one bucket with stride D */
} cs_row_plan;

/* Visit list of one row for the update of a worker bundle (derived from a_j, c and d_hint;
 * does not change any result).  With c a power of two, h_j(i) is the top log2(c) bits of
 * u(i) = (2^(61 - log2 c) * (a_j i + b_j)) mod p, and u(i + s) = (u(i) + U(s)) mod p with
 * U(s) = (2^(61 - log2 c) * a_j * s) mod p.  The list holds, in increasing order, s_0 = 0 and
 * every offset s < d_hint with U(s) below a chosen bound of at most (ncell - 1) cells, so
 * that  h_j(i + s_k) - h_j(i)  (mod c)  lies in  [0, ncell)  for every i and k.  A lane that
 * visits i + s_0, i + s_1, ... therefore needs only ncell running sums and sends each to
 * memory once, after its last visit.  Visit k covers the coordinates [s_k, s_k + gap_k),
 * gap_k = s_{k+1} - s_k (s_K = d_hint); return times of a rotation to an interval take at most
 * three values, so gaps are stored as 2-bit codes into gap[] (code 3 = the last, cut gap). */
#define CS_MAX_VISITS 512
typedef struct cs_visit_plan {
    uint32_t K;                 /* number of visits; 0 = no list (the stride walk is used) */
    uint32_t ncell;             /* running sums per lane and coordinate: 2, 3 or 4 */
    uint64_t cover;             /* the list covers vectors of length <= cover (= d_hint) */
    uint64_t gmax;              /* largest gap = number of residues that lanes own */
    uint64_t cost;              /* estimated time of one launch with this list, nanoseconds */
    uint64_t cost_walk;         /* the same for the stride walk with cs_row_plan.Dw */
    uint64_t gap[4];            /* gap value per code */
    uint64_t A[4], As[4];       /* (a_j * gap) mod p, (a'_j * gap) mod p per code */
    uint32_t code[CS_MAX_VISITS / 16];   /* 2 bits per visit, visit k in word k / 16 */
} cs_visit_plan;

/* Visit list of one row for column counts that are not a power of two (the paper's sketches of
 * 180 000 columns, Table 1).  Here h_j(i + s) = (x(i) + X(s) - [wrap] p) mod c with
 * X(s) = (a_j s) mod p and [wrap] = 1 when x(i) + X(s) >= p, so for an offset s with
 * X(s) mod c = delta < omega the bucket of i + s is h_j(i) + delta, or, after a wrap,
 * h_j(i) + delta - (p mod c)  (mod c): one of 2 omega cells that depend on i only.  Such offsets
 * occur about every c / omega coordinates; the list is a subset of them, picked so that the
 * gaps are as even as they come (gaps are stored one by one: they take no three values here).
 * A lane that visits i + s_0, i + s_1, ... keeps 2 omega running sums per coordinate and sends
 * each to memory once.  K = 0: no list, the update sends one request per coordinate and row. */
#define CS_ANYC_MAX_VISITS 144
typedef struct cs_anyc_plan {
    uint32_t K;                 /* number of visits; 0 = no list */
    uint32_t omega;             /* 1 or 2 */
    uint64_t cover;             /* the list covers vectors of length <= cover (= d_hint) */
    uint64_t gmax;              /* largest gap = number of residues that lanes own */
    uint64_t cost;              /* estimated time of one launch with this list, nanoseconds */
    uint64_t cost_direct;       /* the same for one request per coordinate */
    uint32_t gap[CS_ANYC_MAX_VISITS];   /* gap_k = s_{k+1} - s_k, s_0 = 0, s_K = d_hint */
} cs_anyc_plan;

#define CS_FLAG_NO_VISIT_LIST 1u   /* cs_params.flags: always use the stride walk (testing) */
#define CS_FLAG_NO_LDS_TABLE 2u    /* cs_params.flags: tiny tables are updated in memory, not in a
                                      workgroup-private LDS copy (testing) */

typedef struct cs_params {
    uint32_t r;                 /* rows, odd, 1..CS_MAX_R */
    uint32_t c;                 /* columns, 1..2^31 */
    uint32_t c_pow2;            /* 1 if c is a power of two (fast bucket extraction) */
    uint32_t flags;             /* 0, or CS_FLAG_* set by the caller after cs_params_init */
    uint64_t seed;
    uint64_t a[CS_MAX_R], b[CS_MAX_R];     /* bucket hashes */
    uint64_t as[CS_MAX_R], bs[CS_MAX_R];   /* sign hashes */
    cs_row_plan plan[CS_MAX_R];
    cs_visit_plan visit[CS_MAX_R];
    cs_anyc_plan anyc[CS_MAX_R];
} cs_params;

/* Alg. 4 init: fills *p for an r x c sketch from `seed` (host, no GPU needed).
 * `d_hint` is the vector length the sketch will mostly be used with (0 = unknown); it only
 * steers the traversal plan.  Cost: the plan is found by scanning, per row, every candidate
 * stride up to d_hint / 2 and every offset below d_hint (capped at 2^28 each), about 3.5 ns per
 * coordinate of d_hint and row on one host core: 1.7 s for r = 5, d_hint = 10^8; a few
 * milliseconds for d_hint = 0 or vectors below 10^6.  Call it once per sketch shape and keep
 * the struct.  Vectors longer than 2^28 get no visit list (the stride walk serves them).
 * CS_EINVAL: p null, r even or outside 1..CS_MAX_R, c == 0,
 * c > 2^31 or r * c >= 2^32 (a 16 GiB table). */
int cs_params_init(cs_params* p, uint32_t r, uint32_t c, uint64_t seed, int64_t d_hint);

/* Parity hook: bucket[j*n + t] = h_j(idx[t]) and sign[j*n + t] = s_j(idx[t]) (+1 / -1),
 * computed on the device with the same code path the kernels use.
 * idx, bucket, sign: device.  0 <= idx[t] < 2^61.  n >= 0. */
int cs_hash_debug(const cs_params* p, const int64_t* idx, int64_t n,
                  uint32_t* bucket, int8_t* sign, void* stream);

/* Same for the contiguous range i0 .. i0+n-1, computed through the incremental hash state
 * of the streaming kernels (the traversal plan's order), so that path is bit-checked too. */
int cs_hash_debug_range(const cs_params* p, int64_t i0, int64_t n,
                        uint32_t* bucket, int8_t* sign, void* stream);

/* S = 0.  S: device float[r][c]. */
int cs_sketch_zero(const cs_params* p, float* S, void* stream);

/* Alg. 4 update applied to a dense vector (the sketching step of Alg. 3):
 *     S[j][h_j(i0 + t)] += scale * s_j(i0 + t) * g[t]      for t in [0, d), j in [0, r)
 * S: device float[r][c], accumulated into (not cleared).  g: device float[d].
 * i0 = global index of g[0] (>= 0, i0 + d <= 2^61).  d >= 0 (0 is a no-op). */
int cs_sketch_accumulate(const cs_params* p, float* S, const float* g, int64_t d,
                         int64_t i0, float scale, void* stream);

/* The same update for W workers at once, worker w's vector into worker w's table; hashes
 * are evaluated once per coordinate and shared by all workers (they use the same seed).
 * S_w, g_w: HOST arrays of W device pointers (float[r][c] and float[d] each). W >= 1. */
int cs_sketch_accumulate_batch(const cs_params* p, float* const* S_w, const float* const* g_w,
                               int32_t W, int64_t d, int64_t i0, float scale, void* stream);

/* Worker bundle: the sketches of W workers stored cell-major in groups of CS_BUNDLE_GROUP = 8
 * workers,  T[w / 8][j][b][w % 8] = S^w[j][b],  i.e. float[ceil(W / 8)][r][c][8] contiguous
 * (cs_bundle_floats() elements; slots of a last, partial group are padding and stay 0).
 * Workers hash identically (same seed), so their updates to one cell land in 8 neighbouring
 * floats: one 32-byte memory request carries the updates of 8 workers.  One group's table is
 * small enough to stay in the memory-side cache while that group is being updated.
 *
 * cs_bundle_floats:      number of floats in a bundle of W workers.
 * cs_bundle_zero:        T = 0.
 * cs_sketch_accumulate_bundle:  S^w[j][h_j(i0+t)] += scale * s_j(i0+t) * g_w[w][t] for all
 *                        w < W, t < d, j < r (the sketching step of Alg. 3, every worker).
 *                        g_w: HOST array of W device pointers to float[d].  W >= 1.
 *                        (Placement matters on MI355X: the call measured 9 % faster with the
 *                        vectors in another ~100 GB part of device memory than T; a caller
 *                        that owns both can time the call on candidate buffers and choose.)
 * cs_bundle_merge:       dst[j][b] = beta * dst[j][b] + alpha * sum_{w<W} S^w[j][b]
 *                        (the aggregation step of Alg. 3 with alpha = 1/W); dst: device
 *                        float[r][c], not read when beta == 0; the sum over workers is
 *                        accumulated in binary64 in a fixed order and the result rounded to
 *                        binary32 once (a binary32 running sum over hundreds of workers loses
 *                        bits that momentum and error feedback in sketch space feed back
 *                        every step).
 * The bundle must be below 2^40 floats and 16-byte aligned. */
#define CS_BUNDLE_GROUP 8
int cs_bundle_floats(const cs_params* p, int32_t W, int64_t* n);
/* *n = number of kernel launches one cs_sketch_accumulate_bundle(p, T, W, g_w, d, ...) call
 * makes (rows that share a traversal share a launch); for reading profiles and for dividing
 * a timed call into per-launch figures.  Host only. */
int cs_bundle_update_launches(const cs_params* p, int32_t W, int64_t d, int32_t* n);
int cs_bundle_zero(const cs_params* p, float* T, int32_t W, void* stream);
int cs_sketch_accumulate_bundle(const cs_params* p, float* T, int32_t W,
                                const float* const* g_w, int64_t d, int64_t i0, float scale,
                                void* stream);

/* The workers that share a GPU summed as they are sketched (Sec. 3: the sketch of a sum is
 * the sum of the sketches, so the workers of one device need no tables of their own before
 * the aggregation step of Alg. 3):
 *     S[j][h_j(i0+t)] += scale * s_j(i0+t) * sum_{w<W} g_w[w][t]      for all t < d, j < r,
 * the sum over the workers of a group of 8 taken in registers, in binary32, before the cell
 * is touched.  Equal to cs_bundle_zero + cs_sketch_accumulate_bundle + cs_bundle_merge
 * (alpha = scale, beta = 1) up to the order of the binary32 additions, without the
 * W r c floats of worker tables written and read back, and with one table of r c floats as
 * the only target of the atomic adds.  S: device float[r][c], updated; g_w: HOST array of W
 * device pointers to float[d].  W >= 1, d >= 0, i0 as for cs_sketch_accumulate. */
int cs_sketch_accumulate_sum(const cs_params* p, float* S, int32_t W, const float* const* g_w,
                             int64_t d, int64_t i0, float scale, void* stream);
int cs_bundle_merge(const cs_params* p, float* dst, float beta, const float* T, int32_t W,
                    float alpha, void* stream);

/* Alg. 4 update for a list of (index, value) pairs:
 *     S[j][h_j(idx[t])] += scale * s_j(idx[t]) * val[t]
 * idx: device int64[n] (0 <= idx[t] < 2^61, repeats allowed and summed), val: device float[n]. */
int cs_sketch_accumulate_sparse(const cs_params* p, float* S, const int64_t* idx,
                                const float* val, int64_t n, float scale, void* stream);

/* Failure detector for a diverged run (no passage of the paper; a sketch is linear, so one
 * NaN or infinite gradient element poisons r cells and, through them, every estimate that
 * reads those cells): *count = number of cells of S that are NaN or infinite.
 * S: device float[r][c]; count: device int64, 8-byte aligned, overwritten. */
int cs_sketch_count_nonfinite(const cs_params* p, const float* S, int64_t* count, void* stream);

/* Alg. 4 update with sums that do not depend on the order of the additions.  The float
 * updates above add with atomic operations in whatever order the hardware takes them, so two
 * runs agree only to rounding.  Here every contribution is rounded once to a multiple of
 * 2^-frac_bits and summed as a 64-bit integer, which is associative: equal inputs give equal
 * bits whatever the launch shape, and a reference can be matched bit for bit (a debugging and
 * checkpointing aid that separates "wrong" from "reordered"; about one atomic request per
 * coordinate and row, so far slower than the float path).
 *     q        = (double)scale * (double)g[t] * 2^frac_bits   rounded to an integer, ties to even
 *                (the product is exact in binary64, so this is the only rounding)
 *     acc[j][h_j(i0+t)] += s_j(i0+t) * q                      in int64 (wraps on overflow)
 * A coordinate whose q is not finite or not below 2^62 in magnitude contributes nothing and
 * is counted: *dropped += number of such coordinates (dropped may be NULL).  The caller picks
 * frac_bits (0 .. CS_FIXED_MAX_FRAC_BITS) so that the sums fit: magnitudes below 2^m and at
 * most n coordinates per cell need frac_bits + m + log2(n) <= 62.  Sums over workers are the
 * same integer sums: accumulate every worker into one acc.
 * acc: device int64[r][c], updated (the caller clears it); g: device float[d]; idx, val as
 * for cs_sketch_accumulate_sparse; dropped: device int64, 8-byte aligned, or NULL.
 * cs_fixed_to_float:  S[j][b] = (float)( (double)acc[j][b] * 2^-frac_bits * (double)alpha ),
 * the integer converted to binary64 (exact below 2^53), scaled exactly, multiplied once and
 * rounded once to binary32.  S: device float[r][c], overwritten. */
#define CS_FIXED_MAX_FRAC_BITS 62
int cs_fixed_accumulate(const cs_params* p, int64_t* acc, const float* g, int64_t d, int64_t i0,
                        float scale, int32_t frac_bits, int64_t* dropped, void* stream);
int cs_fixed_accumulate_sparse(const cs_params* p, int64_t* acc, const int64_t* idx,
                               const float* val, int64_t n, float scale, int32_t frac_bits,
                               int64_t* dropped, void* stream);
int cs_fixed_to_float(const cs_params* p, const int64_t* acc, int32_t frac_bits, float alpha,
                      float* S, void* stream);

/* Mergeability (Sec. 3; the aggregation step of Alg. 3, S_t = (1/W) sum_i S_t^i):
 *     dst = beta * dst + alpha * sum_{w<W} src[w]
 * dst: device float[r][c]; with beta == 0 it is not read.  src: HOST array of W device
 * pointers; dst may not alias any src[w] unless W == 1.  The sum over w is taken in
 * ascending w in binary64 and the result is rounded to binary32 once. */
int cs_sketch_merge(const cs_params* p, float* dst, float beta, const float* const* src,
                    int32_t W, float alpha, void* stream);

/* y = a * x + b * y over a whole table (device float[r][c] each; x may equal y). */
int cs_sketch_axpby(const cs_params* p, float* y, float a, const float* x, float b,
                    void* stream);

/* Momentum and error accumulation of Alg. 3 in sketch space, one pass:
 *     S_u = rho * S_u + S_t ;   S_v = S_v + S_u
 * (the images under the sketch of  u <- m u + g  and  v <- v + u). All device float[r][c]. */
int cs_sketch_momentum(const cs_params* p, float* S_u, float* S_v, const float* S_t,
                       float rho, void* stream);

/* Alg. 4 estimate of every coordinate of a range (Sec. 5.2: the implementation queries all d
 * coordinates rather than running a heavy-hitter search):
 *     est[t] = median_{j<r} s_j(i0 + t) * S[j][h_j(i0 + t)]       t in [0, d)
 * S: device float[r][c]; est: device float[d].
 * The median is the middle of the r signed cells after an insertion sort on ">" (what a plain
 * reading of Alg. 4 does).  Infinite cells order as usual.  A NaN cell compares false with
 * everything, so it stays where the sort put it and the estimate is NaN exactly when that
 * position is the middle one; this is a deterministic function of the r values in row order.
 * hist_or_null: NULL, or device uint64[CS_TOPK_HIST_BINS], 8-byte aligned, which receives the
 * number of estimates per magnitude bin, hist[b] = #{ t : (bits(est[t]) & 0x7fffffff) >> 20 == b }
 * (cleared by the call).  It is the first histogram of the selection that follows (Sec. 5.2
 * queries every coordinate and keeps the largest); handing it to cs_heavy_hitters_topk saves
 * that call one read of est.  For long vectors the kernel that writes est counts as it goes;
 * otherwise est is read once more here.
 * rows_ws: device scratch of cs_estimate_workspace_bytes(p, d) bytes (may be NULL when that
 * size is 0).  */
#define CS_TOPK_HIST_BINS 2048
int cs_estimate_workspace_bytes(const cs_params* p, int64_t d, size_t* bytes);
int cs_sketch_estimate(const cs_params* p, const float* S, int64_t d, int64_t i0,
                       float* est, uint64_t* hist_or_null, void* rows_ws, size_t ws_bytes,
                       void* stream);

/* Alg. 4 estimate of listed coordinates: out[t] = median_j s_j(idx[t]) * S[j][h_j(idx[t])].
 * idx: device int64[n]; out: device float[n]. */
int cs_sketch_estimate_sparse(const cs_params* p, const float* S, const int64_t* idx,
                              int64_t n, float* out, void* stream);

/* Selection of the largest estimates (Sec. 5.2): the k indices t in [0, d) with the
 * largest |est[t]|; equal magnitudes are resolved towards the lower index; the result is in
 * ascending index order.  idx_out: device int64[k] (index t, NOT offset by any i0);
 * val_out: device float[k], val_out[n] = est[idx_out[n]] (may be NULL).
 * hist_or_null: NULL, or the histogram cs_sketch_estimate filled for exactly this est[0..d)
 * (device uint64[CS_TOPK_HIST_BINS], read only); a histogram of other data gives a wrong
 * selection.
 * workspace: device, 8-byte aligned, contents irrelevant on entry.  cs_topk_workspace_bytes(d, k)
 * is what makes the call fastest: about 114 KiB of histograms and counters plus, when k is
 * small against d, room for a list of 8 k + 65 536 candidates (12 bytes each; 3 k + 65 536
 * when k is a few per cent of d), with which est is read twice (once with hist_or_null)
 * instead of five times.  Any size from cs_topk_workspace_bytes(1, 1) (the fixed
 * part alone) upwards is accepted and gives the same result; below that CS_EWORKSPACE.
 * 1 <= k <= d. */
int cs_topk_workspace_bytes(int64_t d, int64_t k, size_t* bytes);
int cs_heavy_hitters_topk(const float* est, int64_t d, int64_t k, const uint64_t* hist_or_null,
                          int64_t* idx_out, float* val_out,
                          void* workspace, size_t ws_bytes, void* stream);

/* cs_heavy_hitters_topk for callers that cannot allocate device memory or hand over a
 * workspace: code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same result as cs_heavy_hitters_topk (same kernels); the workspace is a fixed
 * array of 1.7 MB inside the library's device image (histograms, counters and room for
 * 131 072 candidates), which every GPU the library runs on holds until the process ends.  The call allocates and frees nothing, clears what it
 * needs with a kernel (no memset node under capture), and looks up the array's address once
 * per device, on the first call with that device current (`stream` must belong to the current
 * device).  All calls on one GPU share the array: calls that overlap on one GPU (different
 * streams, different threads) race and give wrong selections -- serialise them.
 * CS_ELIMIT when d > CS_TOPK_STATIC_MAX_D (2^32: the supported range of this entry point;
 * the array's size does not grow with d); other arguments and errors as cs_heavy_hitters_topk. */
#define CS_TOPK_STATIC_MAX_D (((int64_t)1) << 32)
int cs_heavy_hitters_topk_static(const float* est, int64_t d, int64_t k,
                                 int64_t* idx_out, float* val_out, void* stream);

/* Second round (Sec. 4; the worker-query step of Alg. 3, which keeps the sum over workers):
 *     out[n] = alpha * sum_{w<W} vec[w][idx[n]]          (sum in ascending w, fp32)
 * vec: HOST array of W device pointers to float vectors; idx: device int64[k] with every
 * idx[n] inside the vectors; out: device float[k]. */
int cs_gather_exact(const float* const* vec, int32_t W, const int64_t* idx, int64_t k,
                    float alpha, float* out, void* stream);

/* Alg. 3 as the paper trains with it (Sec. 5.1: sketch and workers are asked for P k
 * coordinates, P > 1, and the k largest exact sums are applied): of n = Pk candidate coordinates cand[0..n)
 * (ascending, as cs_heavy_hitters_topk returns them) with exact second-round values x[0..n)
 * (cs_gather_exact), keep the k of largest |x| (equal magnitudes -> lower index), in ascending
 * index order:  idx_out[t] = cand[pos_t],  val_out[t] = x[pos_t].
 * cand: device int64[n]; x: device float[n]; idx_out: device int64[k]; val_out: device
 * float[k] (may be NULL); workspace as for cs_heavy_hitters_topk(n, k).  1 <= k <= n. */
int cs_select_exact_topk(const int64_t* cand, const float* x, int64_t n, int64_t k,
                         int64_t* idx_out, float* val_out, void* workspace, size_t ws_bytes,
                         void* stream);

/* Sketches in 16 bits per cell (Sec. 6 reports that 16-bit sketch cells cost no accuracy in
 * preliminary runs): what a worker would put on the wire.  Round to nearest, ties to even; NaN stays
 * NaN, overflow gives infinity.  fmt: CS_FMT_BF16 (upper half of the binary32 pattern: 8
 * exponent, 7 fraction bits -- keeps the range of sums of gradient elements) or CS_FMT_F16
 * (IEEE binary16).
 * cs_quantize16 / cs_dequantize16: elementwise over n values (a table float[r][c] or a whole
 *   worker bundle -- the layout is kept).  x, out, q: device.
 * cs_bundle_merge16: cs_bundle_merge reading a quantised bundle (uint16[ceil(W/8)][r][c][8],
 *   16-byte aligned): dst = beta * dst + alpha * sum_w value(S16^w); binary64 sum in a
 *   fixed order, rounded once. */
#define CS_FMT_BF16 0
#define CS_FMT_F16 1
int cs_quantize16(const float* x, int64_t n, uint16_t* out, int32_t fmt, void* stream);
int cs_dequantize16(const uint16_t* q, int64_t n, float* out, int32_t fmt, void* stream);
int cs_bundle_merge16(const cs_params* p, float* dst, float beta, const uint16_t* T16, int32_t W,
                      float alpha, int32_t fmt, void* stream);

/* HEAVYMIX (Sec. 4, Alg. 1), the recovery the convergence proof is stated for.
 *
 * cs_sketch_l2sq -- Alg. 1 step 1, the squared l2 norm read off the sketch: by the AMS argument of
 * App. C a row's sum of squared counters estimates ||g||^2; the median over the r rows is
 * taken.  out: device double[1 + r], 8-byte aligned: out[0] = the median, out[1 + j] =
 * sum_b S[j][b]^2 (binary64 sums in a fixed order).  S: device float[r][c].
 *
 * cs_heavymix_select -- Alg. 1 steps 3-4.  H = { i : est[i]^2 >= l2sq[0] / k } (the listing's
 * comparison is read in the squared form that Sec. 4's proof and App. C's definition of an
 * l2^2-heavy hitter use; est in binary32, square and threshold in binary64), and the selection
 * is H plus  l = k - |H|  of the remaining coordinates drawn uniformly at random without
 * replacement: coordinate i is given the top 30 bits of the (i+1)-th output of SplitMix64
 * started at rng_seed, and the l largest of these win (equal ones: lower index first).  If
 * k or more estimates pass the threshold, the k largest of them by the top 30 bits of their
 * binary32 magnitude are returned (equal ones: lower index first).
 * est: device float[d]; l2sq: device double (the out[0] above, read on the device, no host
 * synchronisation); idx_out: device int64[k], ascending; val_out: device float[k] or NULL,
 * val_out[t] = est[idx_out[t]]; n_heavy: device int64 or NULL, receives min(|H|, k);
 * workspace as for cs_heavy_hitters_topk.  1 <= k <= d.  The exact values of the selection
 * (Alg. 1 step 5) are what cs_gather_exact returns. */
int cs_sketch_l2sq(const cs_params* p, const float* S, double* out, void* stream);
int cs_heavymix_select(const float* est, int64_t d, int64_t k, const double* l2sq,
                       uint64_t rng_seed, int64_t* idx_out, float* val_out, int64_t* n_heavy,
                       void* workspace, size_t ws_bytes, void* stream);

/* Alg. 3 as printed, with dense state on every worker (the sketch-space form above keeps only
 * r x c numbers per state vector; this form keeps 2 d floats per worker and is exact).
 * cs_dense_momentum -- the momentum and error-accumulation steps for W workers:
 *     u_w[t] = rho * u_w[t] + g_w[t]  (one fused multiply-add),   v_w[t] = v_w[t] + u_w[t].
 *   The sketch of v_w is then taken with cs_sketch_accumulate_bundle(v_w), and the second
 *   round reads v_w through cs_gather_exact.
 * cs_dense_mask -- the last step of the loop body, zeroing on the coordinates of the update:
 *     u_w[idx[n]] = v_w[idx[n]] = 0   for every worker w and n < k.
 * u_w, v_w, g_w: HOST arrays of W device pointers to float[d]; u_w, v_w updated in place.
 * idx: device int64[k], each in [0, d).  W >= 1, d >= 0, k >= 0. */
int cs_dense_momentum(float* const* u_w, float* const* v_w, const float* const* g_w,
                      int32_t W, int64_t d, float rho, void* stream);
int cs_dense_mask(float* const* u_w, float* const* v_w, int32_t W, const int64_t* idx,
                  int64_t k, void* stream);

/* Error feedback / momentum masking in sketch space (the error-accumulation step
 * of Alg. 2 and the zeroing of u, v in Alg. 3, as far as a sketch can express them):
 *     val[n] = estimate(S, idx[n])   for all n, from the table as it is on entry, then
 *     S     -= sketch of the k-sparse vector (idx, val)
 * S: device float[r][c]; idx: device int64[k], distinct; val: device float[k] (output). */
int cs_sketch_feedback(const cs_params* p, float* S, const int64_t* idx, int64_t k,
                       float* val, void* stream);

const char* cs_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* CSKETCH_H */
