"""Pins for the CPU reference: every function of oracle/ is checked against something the
paper or the mathematics fixes, not against itself.

  hashing        published SplitMix64 vector; Python big-int arithmetic on edge cases;
                 universality statistics (collision rate 1/c, balanced signs)
  update         S(f) = A f with the dense sign/bucket matrix A (App. C), MNIST-sized sketch
                 7 x 40 over d = 784 (App. E)
  fixed point    the order-independent update: exact rational arithmetic, big-integer sums,
                 and the fp64 update on inputs that are multiples of 2^-F
  merge          S(g1) + S(g2) = S(g1 + g2) (Sec. 3, App. C)
  estimate       numpy's median over rows; r = 1; c = 1 (AMS sum, App. C); 1-sparse input
  error bound    row variance (||g||^2 - g_i^2)/c and the +-eps ||g||_2 guarantee (Sec. 3, 5.2)
  recovery       planted k-sparse vector recovered exactly (Lemma 1's regime)
  top-k, gather  numpy lexsort / fancy indexing
  state          sketch-space momentum / error feedback equals the sketch of its dense twin
  accounting     compression factors printed in Table 1 and App. E
  16-bit cells   hand-computed bit patterns (ties to even, overflow, subnormals) and PyTorch's
                 CPU conversions
  HEAVYMIX       l2 estimate exact on sparse vectors and inside the (1 +- 0.5) band of Alg. 1;
                 threshold split against a plain loop; fill keys against the published
                 generator; uniformity of the fill; the k/d contraction of Lemma 1
"""
import os

import numpy as np
import pytest

from oracle import cs_oracle as orc

P = (1 << 61) - 1


def bigint_hash(a, b, c, i):
    return ((int(a) * int(i) + int(b)) % P) % int(c)


def bigint_sign(a, b, i):
    return -1 if ((int(a) * int(i) + int(b)) % P) & 1 else 1


# ----------------------------------------------------------------------------- hashing
def test_splitmix64_matches_published_vector(golden_dir):
    want = [int(l) for l in open(os.path.join(golden_dir, "splitmix64_seed1234567.txt"))
            if l.strip() and not l.startswith("#")]
    got = [int(x) for x in orc.splitmix64(1234567, len(want))]
    assert got == want


def test_parameter_derivation_order_and_ranges():
    seed, r = 424242, 7
    z = [int(x) for x in orc.splitmix64(seed, 4 * r)]
    sk = orc.SketchOracle(r, 1 << 10, seed)
    for j in range(r):
        assert int(sk.a[j]) == 1 + z[4 * j] % (P - 1)
        assert int(sk.b[j]) == z[4 * j + 1] % P
        assert int(sk.as_[j]) == 1 + z[4 * j + 2] % (P - 1)
        assert int(sk.bs[j]) == z[4 * j + 3] % P
        assert 1 <= int(sk.a[j]) < P and 0 <= int(sk.b[j]) < P
        assert 1 <= int(sk.as_[j]) < P and 0 <= int(sk.bs[j]) < P
    # more rows extend the same stream
    sk2 = orc.SketchOracle(3, 1 << 10, seed)
    assert list(sk2.a) == list(sk.a[:3]) and list(sk2.bs) == list(sk.bs[:3])


@pytest.mark.parametrize("c", [1, 2, 40, 1000, 180000, 1 << 15, 1 << 20, (1 << 32) - 1])
def test_hash_against_bigint_random_and_edges(c):
    sk = orc.SketchOracle(5, c, 99)
    rng = np.random.default_rng(1)
    idx = np.concatenate([
        np.array([0, 1, 2, 63, 64, 65, (1 << 20) - 1, 10**8 - 1, (1 << 32) - 1, 1 << 32,
                  (1 << 40) + 12345, (1 << 60) + 7], dtype=np.int64),
        rng.integers(0, 1 << 40, size=200),
    ])
    bucket, sign = sk.hash(idx)
    for j in range(sk.r):
        for t, i in enumerate(idx):
            assert int(bucket[j, t]) == bigint_hash(sk.a[j], sk.b[j], c, i)
            assert int(sign[j, t]) == bigint_sign(sk.as_[j], sk.bs[j], i)


def test_hash_edge_parameters():
    c = 1 << 15
    sk = orc.SketchOracle(5, c, 5)
    i_star = 123456789
    a3 = 987654321987654321 % P
    edge = [(1, 0), (P - 1, P - 1), (1, P - 1), (P - 1, 0), (a3, (-a3 * i_star) % P)]
    for j, (a, b) in enumerate(edge):
        sk.a[j], sk.b[j] = a, b
        sk.as_[j], sk.bs[j] = a, b
    idx = np.array([0, 1, 2, i_star - 1, i_star, i_star + 1, (1 << 32) - 1], dtype=np.int64)
    bucket, sign = sk.hash(idx)
    for j, (a, b) in enumerate(edge):
        for t, i in enumerate(idx):
            assert int(bucket[j, t]) == bigint_hash(a, b, c, i)
            assert int(sign[j, t]) == bigint_sign(a, b, i)
    # a*i + b = 0 (mod p) lands in bucket 0 with sign +1
    t_star = list(idx).index(i_star)
    assert bucket[4, t_star] == 0 and sign[4, t_star] == 1


def test_hash_universality_statistics():
    c, n = 1 << 10, 1 << 16
    sk = orc.SketchOracle(5, c, 2024)
    # random keys: buckets look uniform, signs balanced, pair collision rate 1/c
    keys = np.random.default_rng(2).choice(1 << 40, size=n, replace=False)
    bucket, sign = sk.hash(keys)
    for j in range(sk.r):
        counts = np.bincount(bucket[j], minlength=c)
        chi2 = ((counts - n / c) ** 2 / (n / c)).sum()
        # chi-square with c-1 dof: mean c-1, std sqrt(2(c-1)) ~ 45
        assert abs(chi2 - (c - 1)) < 6 * np.sqrt(2 * (c - 1))
        assert abs(sign[j].astype(np.int64).sum()) < 5 * np.sqrt(n)
        assert set(np.unique(sign[j])) == {-1, 1}
        pairs = (counts.astype(np.int64) * (counts - 1) // 2).sum()
        expect = n * (n - 1) / 2 / c
        assert abs(pairs - expect) < 0.05 * expect
    # consecutive keys (a gradient's coordinates): an affine map mod p spreads them at
    # least as evenly as a random function would
    bucket, sign = sk.hash(np.arange(n))
    for j in range(sk.r):
        counts = np.bincount(bucket[j], minlength=c)
        chi2 = ((counts - n / c) ** 2 / (n / c)).sum()
        assert chi2 < (c - 1) + 6 * np.sqrt(2 * (c - 1))
        assert abs(sign[j].astype(np.int64).sum()) < 5 * np.sqrt(n)
    # rows are different functions, and signs are not tied to buckets
    assert (bucket[0] != bucket[1]).mean() > 0.99
    assert abs(np.corrcoef(sign[0], bucket[0] & 1)[0, 1]) < 0.02


# ----------------------------------------------------------------------------- update
def dense_sketch_matrix(sk, d, i0=0):
    """A in S(f) = A f: one +-1 per column in each row block (App. C)."""
    bucket, sign = sk.hash(np.arange(i0, i0 + d))
    A = np.zeros((sk.r * sk.c, d))
    for j in range(sk.r):
        A[j * sk.c + bucket[j].astype(np.int64), np.arange(d)] = sign[j]
    return A


@pytest.mark.parametrize("dtype", [np.float32, np.float64])
def test_accumulate_is_dense_matrix_product_mnist_shape(dtype):
    d, r, c = 784, 7, 40
    sk = orc.SketchOracle(r, c, 7)
    g = np.random.default_rng(0).standard_normal(d).astype(dtype)
    A = dense_sketch_matrix(sk, d)
    assert (np.abs(A).sum(axis=0) == r).all()
    want = (A @ g.astype(np.float64)).reshape(r, c)
    got = sk.sketch(g)
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-12)


def test_accumulate_offset_scale_and_accumulation():
    d, r, c, i0 = 300, 5, 64, 1000
    sk = orc.SketchOracle(r, c, 11)
    rng = np.random.default_rng(3)
    g = rng.standard_normal(d).astype(np.float32)
    A = dense_sketch_matrix(sk, d, i0)
    T = np.ones((r, c))
    sk.accumulate(T, g, i0=i0, scale=-0.25)
    want = 1.0 - 0.25 * (A @ g.astype(np.float64)).reshape(r, c)
    np.testing.assert_allclose(T, want, rtol=0, atol=1e-12)
    # chunked accumulation with i0 equals one pass
    T2 = sk.zeros()
    sk.accumulate(T2, g[:100], i0=i0)
    sk.accumulate(T2, g[100:], i0=i0 + 100)
    np.testing.assert_allclose(T2, (A @ g.astype(np.float64)).reshape(r, c), atol=1e-12)


def test_accumulate_sparse_equals_dense_of_scattered_vector():
    d, r, c = 5000, 5, 128
    sk = orc.SketchOracle(r, c, 13)
    rng = np.random.default_rng(5)
    idx = np.sort(rng.choice(d, 100, replace=False))
    val = rng.standard_normal(100)
    dense = np.zeros(d)
    dense[idx] = val
    np.testing.assert_allclose(sk.accumulate_sparse(sk.zeros(), idx, val, scale=2.0),
                               sk.sketch(dense, scale=2.0), atol=1e-13)
    # repeated indices add up (streaming model of Sec. 3)
    T = sk.accumulate_sparse(sk.zeros(), np.array([7, 7, 7]), np.array([1.0, 2.0, 4.0]))
    one = np.zeros(d)
    one[7] = 7.0
    np.testing.assert_allclose(T, sk.sketch(one), atol=1e-13)


def test_fixed_point_update_against_exact_rationals_and_the_fp64_update():
    """The order-independent form of the update: (i) every contribution equals the exact
    rational scale * g * 2^F rounded half to even (Python Fractions, big integers), including
    halves, the 2^62 limit and non-finite inputs; (ii) the table is the big-integer sum of the
    signed contributions over the dense sign/bucket matrix; (iii) on inputs that are multiples
    of 2^-F nothing is rounded, so the table equals 2^F times the fp64 update of Alg. 4."""
    from fractions import Fraction
    r, c, d, i0, F = 5, 16, 400, 77, 20
    sk = orc.SketchOracle(r, c, 23)
    rng = np.random.default_rng(9)
    g = rng.standard_normal(d).astype(np.float32)
    g[:8] = np.float32([0.5 * 2.0 ** -F, 1.5 * 2.0 ** -F, -0.5 * 2.0 ** -F, -2.5 * 2.0 ** -F,
                        np.nan, np.inf, -np.inf, 2.0 ** 43])        # halves; dropped; 2^63 >= 2^62
    scale = np.float32(0.75)
    q, ok = sk.fixed_contributions(g, scale, F)
    for t in range(d):
        if not np.isfinite(g[t]):
            assert not ok[t] and q[t] == 0
            continue
        exact = Fraction(float(g[t])) * Fraction(float(scale)) * 2 ** F
        if abs(exact) >= 2 ** 62:
            assert not ok[t] and q[t] == 0
        else:
            assert ok[t] and int(q[t]) == round(exact)       # round(Fraction): ties to even
    assert [int(v) for v in sk.fixed_contributions(g[:4], 1.0, F)[0]] == [0, 2, 0, -2]
    assert int((~ok).sum()) == 4
    acc = np.zeros((r, c), dtype=np.int64)
    dropped = sk.accumulate_fixed(acc, g, F, i0=i0, scale=float(scale))
    assert dropped == 4
    A = dense_sketch_matrix(sk, d, i0)                       # entries -1, 0, +1
    want = [sum(int(A[row, t]) * int(q[t]) for t in range(d) if A[row, t]) for row in range(r * c)]
    assert [int(v) for v in acc.ravel()] == want
    # (iii) dyadic inputs: no rounding anywhere, fixed point = 2^F * fp64 update
    gd = (rng.integers(-2 ** 12, 2 ** 12, d) * 2.0 ** -10).astype(np.float32)
    acc2 = np.zeros((r, c), dtype=np.int64)
    assert sk.accumulate_fixed(acc2, gd, F, i0=i0, scale=-0.5) == 0
    T = sk.sketch(gd, i0=i0, scale=-0.5)
    assert (acc2.astype(np.float64) == T * 2.0 ** F).all()
    np.testing.assert_array_equal(sk.fixed_to_float(acc2, F, alpha=0.25), (0.25 * T).astype(np.float32))
    # sparse form, repeated indices, and sums over "workers" are the same integer sums
    acc3 = np.zeros((r, c), dtype=np.int64)
    sk.accumulate_fixed_sparse(acc3, np.arange(i0, i0 + d)[::-1], gd[::-1], F, scale=-0.5)
    np.testing.assert_array_equal(acc3, acc2)
    acc4 = np.zeros((r, c), dtype=np.int64)
    sk.accumulate_fixed(acc4, gd[:150], F, i0=i0, scale=-0.5)
    sk.accumulate_fixed(acc4, gd[150:], F, i0=i0 + 150, scale=-0.5)
    np.testing.assert_array_equal(acc4, acc2)


def test_fixed_point_conversion_rounds_once_per_step():
    sk = orc.SketchOracle(1, 4, 1)
    acc = np.array([[(1 << 53) + 1, -(1 << 24) - 1, 3, 0]], dtype=np.int64)
    out = sk.fixed_to_float(acc, 0, alpha=1.0)
    # 2^53 + 1 -> binary64 ties to even 2^53; -(2^24 + 1) -> binary32 ties to even -2^24
    assert out.dtype == np.float32 and out.tolist() == [[2.0 ** 53, -(2.0 ** 24), 3.0, 0.0]]
    np.testing.assert_array_equal(sk.fixed_to_float(acc, 2, alpha=0.5)[0, 2:], np.float32([0.375, 0.0]))


# ----------------------------------------------------------------------------- linearity / merge
def test_linearity_and_merge():
    d, r, c, W = 20000, 5, 512, 6
    sk = orc.SketchOracle(r, c, 17)
    rng = np.random.default_rng(7)
    gs = [rng.standard_normal(d).astype(np.float32) for _ in range(W)]
    tables = [sk.sketch(g) for g in gs]
    total = np.sum([g.astype(np.float64) for g in gs], axis=0)
    np.testing.assert_allclose(tables[0] + tables[1],
                               sk.sketch(gs[0].astype(np.float64) + gs[1]), atol=1e-12)
    merged = orc.merge(tables, alpha=1.0 / W)
    np.testing.assert_allclose(merged, sk.sketch(total, scale=1.0 / W), atol=1e-12)
    np.testing.assert_allclose(merged, np.sum(tables, axis=0) / W, atol=1e-13)
    # beta * dst + alpha * sum
    dst = rng.standard_normal((r, c))
    np.testing.assert_allclose(orc.merge(tables[:2], alpha=0.5, beta=-2.0, dst=dst),
                               -2.0 * dst + 0.5 * (tables[0] + tables[1]), atol=1e-13)
    # dropping a worker and rescaling = sketch of the remaining workers' mean
    np.testing.assert_allclose(orc.merge(tables[:-1], alpha=1.0 / (W - 1)),
                               sk.sketch(total - gs[-1], scale=1.0 / (W - 1)), atol=1e-12)


# ----------------------------------------------------------------------------- estimate
def test_estimate_is_median_of_signed_cells():
    d, r, c = 3000, 7, 97
    sk = orc.SketchOracle(r, c, 19)
    g = np.random.default_rng(9).standard_normal(d)
    T = sk.sketch(g)
    bucket, sign = sk.hash(np.arange(d))
    rows = np.stack([sign[j] * T[j, bucket[j].astype(np.int64)] for j in range(r)])
    np.testing.assert_array_equal(sk.row_estimates(T, d), rows)
    np.testing.assert_array_equal(sk.estimate(T, d), np.median(rows, axis=0))
    sub = np.array([5, 17, 2999, 0])
    np.testing.assert_array_equal(sk.estimate_sparse(T, sub), np.median(rows, axis=0)[sub])
    np.testing.assert_array_equal(sk.estimate(T, 100, i0=50), np.median(rows, axis=0)[50:150])


def test_estimate_single_row_and_ams_column():
    d = 2000
    g = np.random.default_rng(10).standard_normal(d)
    sk1 = orc.SketchOracle(1, 64, 23)
    T = sk1.sketch(g)
    bucket, sign = sk1.hash(np.arange(d))
    np.testing.assert_array_equal(sk1.estimate(T, d), sign[0] * T[0, bucket[0].astype(np.int64)])
    # c = 1: every row is the AMS sum  sum_i s(i) g_i, and E[S^2] = ||g||^2 (App. C)
    ams = orc.SketchOracle(63, 1, 29)
    Ta = ams.sketch(g)
    _, s = ams.hash(np.arange(d))
    np.testing.assert_allclose(Ta[:, 0], (s * g).sum(axis=1), atol=1e-10)
    ratio = (Ta[:, 0] ** 2).mean() / (g ** 2).sum()
    assert 0.5 < ratio < 1.6


def test_estimate_one_sparse_input():
    d, r, c = 50000, 5, 256
    sk = orc.SketchOracle(r, c, 31)
    g = np.zeros(d)
    g[31337] = -2.5
    est = sk.estimate(sk.sketch(g), d)
    assert est[31337] == -2.5
    assert set(np.unique(est)) <= {0.0, 2.5, -2.5}
    # a coordinate is wrong only if it collides with 31337 in a majority of rows
    bucket, _ = sk.hash(np.arange(d))
    coll = (bucket == bucket[:, [31337]]).sum(axis=0)
    assert ((est != 0) == (coll >= 3)).all()


# ----------------------------------------------------------------------------- error bound
@pytest.mark.parametrize("kind", ["gauss", "heavy"])
def test_row_variance_and_l2_error_bound(kind):
    d, r, c = 1 << 18, 5, 1 << 14
    rng = np.random.default_rng(12)
    g = rng.standard_normal(d) * 0.01
    if kind == "heavy":
        g[rng.choice(d, 200, replace=False)] += rng.uniform(0.5, 1.0, 200) * rng.choice([-1, 1], 200)
    sk = orc.SketchOracle(r, c, 37)
    T = sk.sketch(g)
    rows = sk.row_estimates(T, d)
    norm2 = (g ** 2).sum()
    # single-row estimate s(i) T[h(i)] = g_i + sum of the other coordinates of the bucket with
    # random signs: unbiased, variance (||g||^2 - g_i^2)/c over the draw of the hash (pairwise
    # independence).  For the one function drawn here, averaging over the signs only, the mean
    # squared error over all i is (1/d) sum_b (n_b - 1) sum_{i in b} g_i^2  (n_b = bucket size),
    # which for the evenly spread buckets of consecutive keys is ~ (1 - c/d) of the bound.
    universal = ((norm2 - g ** 2) / c).mean()
    bucket, _ = sk.hash(np.arange(d))
    tol = 0.03 if kind == "gauss" else 0.35   # planted mass sits in few buckets: few sign draws
    for j in range(r):
        bj = bucket[j].astype(np.int64)
        n_b = np.bincount(bj, minlength=c)
        mass_b = np.bincount(bj, weights=g ** 2, minlength=c)
        predicted = ((n_b - 1) * mass_b).sum() / d
        assert predicted <= 1.02 * universal
        err2 = ((rows[j] - g) ** 2).mean()
        assert abs(err2 - predicted) < tol * predicted, (j, err2, predicted)
    assert abs((rows - g).mean()) < 0.05 * np.sqrt(universal)
    # Chebyshev per row (fail prob <= 1/8 at sqrt(8/c)||g||), majority of 5 rows
    est = sk.estimate(T, d)
    bad = np.abs(est - g) > np.sqrt(8.0 / c) * np.sqrt(norm2)
    assert bad.mean() <= 0.02
    # squared form of Sec. 3 with eps = 8/c on the coordinates within the value bound
    eps = 8.0 / c
    ok = ~bad
    assert (est[ok] ** 2 <= g[ok] ** 2 + 2 * np.abs(g[ok]) * np.sqrt(eps * norm2) + eps * norm2 + 1e-18).all()


# ----------------------------------------------------------------------------- recovery
def test_planted_sparse_recovery_exact():
    d, r, c, k = 1 << 20, 5, 1 << 15, 16
    rng = np.random.default_rng(14)
    idx = np.sort(rng.choice(d, k, replace=False))
    val = rng.uniform(0.5, 1.0, k) * rng.choice([-1.0, 1.0], k)
    g = np.zeros(d)
    g[idx] = val
    sk = orc.SketchOracle(r, c, 41)
    T = sk.sketch(g)
    est = sk.estimate(T, d)
    np.testing.assert_array_equal(est, g)
    np.testing.assert_array_equal(orc.topk(est, k), idx)
    np.testing.assert_array_equal(orc.gather_exact([g, g], orc.topk(est, k), 0.5), val)


def test_planted_recovery_follows_collision_pattern():
    d, r, c, k = 1 << 16, 5, 1 << 10, 400
    rng = np.random.default_rng(15)
    idx = np.sort(rng.choice(d, k, replace=False))
    g = np.zeros(d)
    g[idx] = rng.uniform(0.5, 1.0, k) * rng.choice([-1.0, 1.0], k)
    sk = orc.SketchOracle(r, c, 43)
    est = sk.estimate(sk.sketch(g), d)
    bucket, _ = sk.hash(np.arange(d))
    occupied = np.zeros((r, c), dtype=np.int64)
    for j in range(r):
        np.add.at(occupied[j], bucket[j, idx].astype(np.int64), 1)
    own = np.zeros(d, dtype=np.int64)
    own[idx] = 1
    # rows in which coordinate i shares its bucket with no *other* non-zero
    clean = np.stack([occupied[j, bucket[j].astype(np.int64)] - own == 0 for j in range(r)]).sum(axis=0)
    sure = clean >= 3
    assert sure.mean() > 0.5 and (~sure).sum() > 0
    np.testing.assert_array_equal(est[sure], g[sure])


# ----------------------------------------------------------------------------- top-k / gather
def test_topk_against_lexsort_with_ties():
    rng = np.random.default_rng(16)
    for d, k in [(1, 1), (10, 10), (1000, 1), (1000, 37), (5000, 4999), (4096, 256)]:
        est = np.round(rng.standard_normal(d) * 4) / 4      # many exact ties, both signs
        order = np.lexsort((np.arange(d), -np.abs(est)))      # |est| desc, index asc
        want = np.sort(order[:k])
        np.testing.assert_array_equal(orc.topk(est, k), want)
        np.testing.assert_array_equal(orc.topk_threshold(est, k), want)
    est = np.array([0.0, -3.0, 3.0, 1.0, -3.0, 2.0])
    np.testing.assert_array_equal(orc.topk(est, 2), [1, 2])
    np.testing.assert_array_equal(orc.topk(est, 3), [1, 2, 4])
    np.testing.assert_array_equal(orc.topk(est, 4), [1, 2, 4, 5])
    np.testing.assert_array_equal(orc.topk(np.zeros(7), 3), [0, 1, 2])
    np.testing.assert_array_equal(orc.topk_threshold(np.zeros(7), 3), [0, 1, 2])


def test_select_exact_topk_against_lexsort():
    rng = np.random.default_rng(21)
    n, k = 600, 50
    cand = np.sort(rng.choice(10**6, n, replace=False))
    x = np.round(rng.standard_normal(n) * 3) / 3            # ties
    order = np.lexsort((cand, -np.abs(x)))[:k]                # |x| desc, coordinate asc
    want = np.sort(cand[order])
    got_idx, got_val = orc.select_exact_topk(cand, x, k)
    np.testing.assert_array_equal(got_idx, want)
    np.testing.assert_array_equal(got_val, x[np.searchsorted(cand, want)])
    # P = 1: the selection is the whole candidate list
    i1, v1 = orc.select_exact_topk(cand, x, n)
    np.testing.assert_array_equal(i1, cand)
    np.testing.assert_array_equal(v1, x)


def test_gather_exact_is_fancy_indexing():
    rng = np.random.default_rng(17)
    vecs = [rng.standard_normal(1000).astype(np.float32) for _ in range(5)]
    idx = np.array([3, 999, 0, 500])
    want = 0.2 * np.stack(vecs).astype(np.float64).sum(axis=0)[idx]
    np.testing.assert_allclose(orc.gather_exact(vecs, idx, 0.2), want, atol=1e-15)


def test_topk_scale_invariance_and_merged_topk():
    d, r, c, W, k = 1 << 15, 5, 1 << 13, 4, 20
    rng = np.random.default_rng(18)
    sk = orc.SketchOracle(r, c, 47)
    heavy = np.sort(rng.choice(d, k, replace=False))
    gs = []
    for _ in range(W):
        g = rng.standard_normal(d) * 0.01
        g[heavy] += 1.0
        gs.append(g)
    S = orc.merge([sk.sketch(g) for g in gs], alpha=1.0)
    sel = orc.topk(sk.estimate(S, d), k)
    # dividing the summed sketch by W does not change the selected set (proof of Thm 1)
    np.testing.assert_array_equal(orc.topk(sk.estimate(S / W, d), k), sel)
    np.testing.assert_array_equal(orc.topk(sk.estimate(S * 0.125, d), k), sel)
    # the merged sketch finds the heavy coordinates of the summed vector
    np.testing.assert_array_equal(sel, heavy)
    np.testing.assert_array_equal(sel, orc.topk(np.sum(gs, axis=0), k))


# ----------------------------------------------------------------------------- state
def test_sketch_space_state_equals_sketch_of_dense_state():
    d, r, c, W, k, steps = 1 << 14, 5, 1 << 10, 4, 64, 6
    rng = np.random.default_rng(19)
    sk = orc.SketchOracle(r, c, 53)
    st = orc.SketchSpaceState(sk, 0.9)
    dense = orc.DenseState(d, st.rho)
    heavy = rng.choice(d, 40, replace=False)
    for t in range(steps):
        gs = []
        for _ in range(W):
            g = (rng.standard_normal(d) * 0.01).astype(np.float32)
            g[heavy] += 0.5
            gs.append(g)
        S_t = orc.merge([sk.sketch(g) for g in gs], alpha=1.0 / W)
        gbar = np.mean([g.astype(np.float64) for g in gs], axis=0)
        st.momentum(S_t)
        dense.momentum(gbar)
        np.testing.assert_allclose(st.S_u, sk.sketch(dense.u), atol=1e-10)
        np.testing.assert_allclose(st.S_v, sk.sketch(dense.v), atol=1e-10)
        est, idx = st.select(d, k)
        assert idx.size == k and (np.diff(idx) > 0).all()
        delta, uhat = st.feedback(idx)
        np.testing.assert_array_equal(delta, est[idx])
        dense.feedback(idx, delta, uhat)
        np.testing.assert_allclose(st.S_u, sk.sketch(dense.u), atol=1e-10)
        np.testing.assert_allclose(st.S_v, sk.sketch(dense.v), atol=1e-10)
        if t == 0:
            # first step: u = v = mean gradient, so the heavy coordinates are selected and
            # the fed-back value is close to the exact second-round value
            assert set(heavy) <= set(idx)
            x = orc.gather_exact(gs, idx, 1.0 / W)
            on_heavy = np.isin(idx, heavy)
            assert np.median(np.abs(x - delta)[on_heavy]) < 0.05
    # error feedback keeps the accumulated vector bounded on the planted coordinates
    assert np.abs(dense.v[heavy]).max() < 2.0


def test_dense_worker_state_worked_example_and_mean_recursion():
    """Alg. 3 with per-worker u, v: a two-step example computed by hand, and the fact that the
    workers' mean follows the single-vector recursion (DenseState) when the fed-back values
    are the exact means -- zeroing u^i, v^i at idx subtracts exactly their means there."""
    st = orc.DenseWorkerState(2, 3, 0.5)
    st.momentum([np.array([1.0, 2.0, 0.0]), np.array([3.0, 0.0, -1.0])])
    assert st.u[0].tolist() == [1.0, 2.0, 0.0] and st.v[1].tolist() == [3.0, 0.0, -1.0]
    assert st.exact(np.array([0])).tolist() == [2.0]                    # (1 + 3) / 2
    st.mask(np.array([0]))
    assert st.u[0].tolist() == [0.0, 2.0, 0.0] and st.v[1].tolist() == [0.0, 0.0, -1.0]
    st.momentum([np.array([1.0, 1.0, 1.0]), np.array([0.0, 0.0, 2.0])])
    # worker 0: u = 0.5 * [0, 2, 0] + [1, 1, 1] = [1, 2, 1];  v = [0, 2, 0] + u = [1, 4, 1]
    # worker 1: u = 0.5 * [0, 0, -1] + [0, 0, 2] = [0, 0, 1.5];  v = [0, 0, -1] + u = [0, 0, 0.5]
    assert st.u[0].tolist() == [1.0, 2.0, 1.0] and st.v[0].tolist() == [1.0, 4.0, 1.0]
    assert st.u[1].tolist() == [0.0, 0.0, 1.5] and st.v[1].tolist() == [0.0, 0.0, 0.5]
    assert st.mean_v().tolist() == [0.5, 2.0, 0.75]

    rng = np.random.default_rng(2)
    W, d, rho = 3, 500, 0.9
    workers = orc.DenseWorkerState(W, d, rho)
    mean = orc.DenseState(d, workers.rho)
    for t in range(5):
        g_w = [rng.standard_normal(d) for _ in range(W)]
        workers.momentum(g_w)
        mean.momentum(sum(g_w) / W)
        np.testing.assert_allclose(workers.mean_v(), mean.v, rtol=0, atol=1e-12)
        idx = np.sort(rng.choice(d, 40, replace=False))
        x = workers.exact(idx)
        np.testing.assert_allclose(x, mean.v[idx], rtol=0, atol=1e-12)
        mean_u = sum(workers.u) / W
        mean.feedback(idx, mean.v[idx].copy(), mean_u[idx].copy())
        workers.mask(idx)
        assert all((u[idx] == 0).all() and (v[idx] == 0).all() for u, v in zip(workers.u, workers.v))
        np.testing.assert_allclose(workers.mean_v(), mean.v, rtol=0, atol=1e-12)


def test_momentum_recursion_closed_form():
    # constant sketch input: S_u after n steps = (1 - rho^n)/(1 - rho) S, S_v = sum of those
    sk = orc.SketchOracle(3, 16, 59)
    st = orc.SketchSpaceState(sk, 0.9)
    S = np.random.default_rng(20).standard_normal((3, 16))
    rho = float(np.float32(0.9))
    sv = 0.0
    for n in range(1, 6):
        st.momentum(S)
        su = (1 - rho ** n) / (1 - rho)
        sv += su
        np.testing.assert_allclose(st.S_u, su * S, rtol=1e-13)
        np.testing.assert_allclose(st.S_v, sv * S, rtol=1e-13)


# ----------------------------------------------------------------------------- accounting
# ----------------------------------------------------------------------------- HEAVYMIX
def test_l2sq_exact_on_sparse_and_in_band_on_dense():
    sk = orc.SketchOracle(5, 1 << 12, 21)
    d = 1 << 16
    g = np.zeros(d)
    g[777] = -3.0
    l2, rows = orc.l2sq_estimate(sk.sketch(g))
    assert l2 == 9.0 and (rows == 9.0).all()                 # 1-sparse: every row holds g_i once
    g = np.zeros(d)
    idx = np.array([5, 1000, 40000, 65535])
    g[idx] = [1.0, -2.0, 0.5, 4.0]
    b, _ = sk.hash(idx)
    assert all(len(set(row)) == idx.size for row in b)       # no two share a bucket in any row
    l2, rows = orc.l2sq_estimate(sk.sketch(g))
    assert l2 == pytest.approx(21.25, rel=1e-15) and np.allclose(rows, 21.25, rtol=1e-15)
    rng = np.random.default_rng(3)
    g = rng.standard_normal(d)
    true = float(g @ g)
    l2, rows = orc.l2sq_estimate(sk.sketch(g))
    assert 0.5 * true <= l2 <= 1.5 * true                    # Alg. 1 step 1
    # AMS: a row's estimate has relative standard deviation about sqrt(2 / c) = 2.2 %
    assert np.abs(rows / true - 1).max() < 0.12 and abs(l2 / true - 1) < 0.06
    assert l2 == np.median(rows)


def test_heavymix_fill_keys_are_the_published_generator():
    for seed in (0, 1234567, (1 << 64) - 3):
        want = orc.splitmix64(seed, 1000) >> np.uint64(34)     # C version, pinned to the published vector
        np.testing.assert_array_equal(orc.heavymix_fill_keys(seed, 1000), want.astype(np.uint32))


def test_heavymix_split_and_fill_against_plain_loops():
    rng = np.random.default_rng(8)
    d, k = 60, 12
    est = rng.standard_normal(d).astype(np.float32)
    est[[3, 17, 41]] = [5.0, -6.0, 4.5]
    est[20] = np.nan                                          # never heavy, may be drawn
    l2sq = 100.0                                              # threshold 100 / 12: |est| >= 2.887
    got, n_heavy = orc.heavymix_select(est, k, l2sq, rng_seed=99)
    H = [i for i in range(d) if float(est[i]) * float(est[i]) >= l2sq / k]
    assert H == [3, 17, 41] and n_heavy == 3
    keys = [int(x) >> 34 for x in orc.splitmix64(99, d)]
    NH = sorted((i for i in range(d) if i not in H), key=lambda i: (-keys[i], i))
    assert got.tolist() == sorted(H + NH[: k - len(H)])
    assert len(set(got.tolist())) == k
    # a different seed draws a different fill but the same heavy part
    other, _ = orc.heavymix_select(est, k, l2sq, rng_seed=100)
    assert set(H) <= set(other.tolist()) and other.tolist() != got.tolist()
    # more than k pass a tiny threshold: the k largest magnitudes, ties to the lower index
    est2 = est.copy()
    est2[20] = 0.0
    est2[50] = est2[3]
    sel, n_heavy = orc.heavymix_select(est2, 4, 1e-6, rng_seed=1)
    assert n_heavy == 4 and sel.tolist() == [3, 17, 41, 50]
    sel, _ = orc.heavymix_select(est2, 3, 1e-6, rng_seed=1)
    assert sel.tolist() == [3, 17, 50]                        # 5.0 twice (3, 50) and -6.0; 4.5 is out


def test_heavymix_fill_is_uniform_without_replacement():
    d, k, trials = 120, 12, 4000
    est = np.zeros(d, dtype=np.float32)
    counts = np.zeros(d)
    for seed in range(trials):
        sel, n_heavy = orc.heavymix_select(est, k, 1.0, rng_seed=seed * 7919 + 1)
        assert n_heavy == 0 and sel.size == k and np.unique(sel).size == k
        counts[sel] += 1
    expect = trials * k / d
    chi2 = float(((counts - expect) ** 2 / (expect * (1 - k / d))).sum())
    assert 70 < chi2 < 175, chi2                              # d - 1 = 119 degrees of freedom


def test_heavymix_is_a_k_over_d_contraction():
    """Lemma 1: E ||g - HEAVYMIX(g)||^2 <= (1 - k/d) ||g||^2, with equality when nothing is
    heavy (a uniform draw of k of d coordinates keeps k/d of the energy in expectation)."""
    rng = np.random.default_rng(12)
    d, k, trials = 3000, 60, 400
    sk = orc.SketchOracle(5, 1 << 10, 4)
    for n_planted in (0, 6):
        g = rng.standard_normal(d)
        planted = rng.choice(d, n_planted, replace=False)
        g[planted] = 40.0 * np.sign(g[planted])
        T = sk.sketch(g)
        est = sk.estimate(T, d)
        l2sq, _ = orc.l2sq_estimate(T)
        total = float(g @ g)
        err = []
        for seed in range(trials):
            sel, n_heavy = orc.heavymix_select(est, k, l2sq, rng_seed=seed)
            assert n_heavy == n_planted and set(planted.tolist()) <= set(sel.tolist())
            rest = g.copy()
            rest[sel] = 0.0                                    # second round: exact values
            err.append(float(rest @ rest))
        ratio = np.mean(err) / total
        if n_planted == 0:
            assert ratio == pytest.approx(1 - k / d, rel=0.01)
        else:
            assert ratio < (1 - k / d) * (1 - 0.5)             # the planted part alone is > half


# ----------------------------------------------------------------------------- 16-bit sketches
def test_quantize16_known_patterns_and_library_conversions():
    import torch
    f = np.float32
    cases = [                                   # value, bf16 pattern, f16 pattern
        (0.0, 0x0000, 0x0000), (-0.0, 0x8000, 0x8000), (1.0, 0x3F80, 0x3C00),
        (-2.5, 0xC020, 0xC100), (np.inf, 0x7F80, 0x7C00), (-np.inf, 0xFF80, 0xFC00),
        (1.0 + 2.0 ** -8, 0x3F80, 0x3C04),      # bf16: exactly half way, even neighbour below
        (1.0 + 3 * 2.0 ** -8, 0x3F82, 0x3C0C),  # bf16: half way, even neighbour above
        (1.0 + 2.0 ** -8 + 2.0 ** -20, 0x3F81, 0x3C04),   # just above half way
        (1.0 + 2.0 ** -11, 0x3F80, 0x3C00),     # f16: half way between 1 and 1 + 2^-10, even below
        (1.0 + 3 * 2.0 ** -11, 0x3F80, 0x3C02),
        (65504.0, 0x4780, 0x7BFF), (65520.0, 0x4780, 0x7C00),   # f16: largest finite; overflow
        (3.4e38, 0x7F80, None),                 # bf16: rounds up past the largest finite value
        (2.0 ** -24, 0x3380, 0x0001), (2.0 ** -25, 0x3300, 0x0000),   # f16 subnormals
    ]
    for x, bf, hf in cases:
        assert int(orc.quantize16([f(x)], "bf16")[0]) == bf, (x, hex(bf))
        if hf is not None:
            assert int(orc.quantize16([f(x)], "f16")[0]) == hf, (x, hex(hf))
    assert np.isnan(orc.dequantize16(orc.quantize16([np.nan], "bf16"), "bf16")[0])
    rng = np.random.default_rng(5)
    x = np.concatenate([(rng.standard_normal(200_000) * 10.0 ** rng.uniform(-12, 12, 200_000)).astype(np.float32),
                        rng.integers(0, 1 << 32, 200_000, dtype=np.uint64).astype(np.uint32).view(np.float32)])
    ok = ~np.isnan(x)
    t = torch.from_numpy(x)
    np.testing.assert_array_equal(orc.quantize16(x, "bf16")[ok],
                                  t.to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)[ok])
    np.testing.assert_array_equal(orc.quantize16(x, "f16")[ok],
                                  t.to(torch.float16).view(torch.int16).numpy().view(np.uint16)[ok])
    for fmt, ulp in (("bf16", 2.0 ** -8), ("f16", 2.0 ** -11)):
        back = orc.dequantize16(orc.quantize16(x, fmt), fmt)
        fin = ok & np.isfinite(back) & (np.abs(x) > 1e-4) & (np.abs(x) < 6e4)
        assert (np.abs(back[fin] - x[fin].astype(np.float64)) <= ulp * np.abs(x[fin])).all()


def test_compression_numbers_printed_in_paper(golden_dir):
    rows = [l.split() for l in open(os.path.join(golden_dir, "compression_table.txt"))
            if l.strip() and not l.startswith("#")]
    assert len(rows) == 4
    for d, r, c, Pk, k, printed, tol, _ in rows:
        got = orc.compression_factor(int(d), int(r) * int(c), int(Pk), int(k))
        assert abs(got - float(printed)) <= float(tol), (got, printed)


def test_constructor_rejects_even_rows():
    with pytest.raises(ValueError):
        orc.SketchOracle(4, 16, 1)
    with pytest.raises(ValueError):
        orc.SketchOracle(5, 0, 1)
