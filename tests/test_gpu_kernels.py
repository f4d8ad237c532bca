"""Kernel-by-kernel parity of the HIP library (through its C ABI) against the CPU reference.
Integer results (hash buckets, signs, selected indices) must be bit-exact; a median picks one
of its inputs, so estimates computed from the same fp32 table must be bit-exact too; sums
(sketch cells, merges, gathers) must be within the stated fp32 tolerance."""
import numpy as np
import pytest
import torch

import paper_1903_04488_amd as cs
from paper_1903_04488_amd import binding
from oracle import cs_oracle as orc
from parity_util import assert_cells_close, assert_values_close

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def dev(a, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(a))
    if dtype is not None:
        t = t.to(dtype)
    return t.to(DEV)


def ref_table_from_device(S):
    return S.detach().cpu().numpy().astype(np.float64)


SHAPES = [  # (r, c, seed)
    (5, 1 << 15, 190304489),
    (7, 1 << 19, 190304493),
    (5, 1 << 20, 190304492),
    (15, 180000, 77),        # the paper's non-power-of-two column count, 15 rows
    (7, 40, 5),              # MNIST-sized sketch of App. E
    (1, 1 << 10, 3),
    (3, 1, 4),               # c = 1: AMS rows
]


# ------------------------------------------------------------------------------ hashing
@pytest.mark.parametrize("r,c,seed", SHAPES)
def test_hash_list_bit_exact(r, c, seed):
    p = cs.cs_params_init(r, c, seed)
    sk = orc.SketchOracle(r, c, seed)
    rng = np.random.default_rng(seed)
    idx = np.concatenate([
        np.array([0, 1, 2, 63, 64, 65, 255, 256, (1 << 20) - 1, 10**8 - 1, (1 << 32) - 1,
                  1 << 32, (1 << 40) + 12345, (1 << 61) - 1], dtype=np.int64),
        rng.integers(0, 1 << 61, size=5000), rng.integers(0, 1 << 27, size=5000)])
    n = idx.size
    bucket = torch.empty(r * n, dtype=torch.int32, device=DEV)
    sign = torch.empty(r * n, dtype=torch.int8, device=DEV)
    cs.cs_hash_debug(p, dev(idx), bucket, sign)
    rb, rs = sk.hash(idx)
    np.testing.assert_array_equal(bucket.cpu().numpy().view(np.uint32).reshape(r, n), rb)
    np.testing.assert_array_equal(sign.cpu().numpy().reshape(r, n), rs)


def test_hash_edge_constants_bit_exact():
    P = (1 << 61) - 1
    c = 1 << 15
    p = cs.cs_params_init(5, c, 5)
    sk = orc.SketchOracle(5, c, 5)
    i_star = 123456789
    a3 = 987654321987654321 % P
    edge = [(1, 0), (P - 1, P - 1), (1, P - 1), (P - 1, 0), (a3, (-a3 * i_star) % P)]
    for j, (a, b) in enumerate(edge):
        p.a[j] = p.as_[j] = a
        p.b[j] = p.bs[j] = b
        sk.a[j] = sk.as_[j] = a
        sk.b[j] = sk.bs[j] = b
    idx = np.array([0, 1, 2, i_star - 1, i_star, i_star + 1, (1 << 32) - 1, P - 1, P], dtype=np.int64)
    n = idx.size
    bucket = torch.empty(5 * n, dtype=torch.int32, device=DEV)
    sign = torch.empty(5 * n, dtype=torch.int8, device=DEV)
    cs.cs_hash_debug(p, dev(idx), bucket, sign)
    rb, rs = sk.hash(idx)
    np.testing.assert_array_equal(bucket.cpu().numpy().view(np.uint32).reshape(5, n), rb)
    np.testing.assert_array_equal(sign.cpu().numpy().reshape(5, n), rs)


@pytest.mark.parametrize("r,c,seed", SHAPES[:4])
@pytest.mark.parametrize("i0,n", [(0, 1 << 20), (12345678901, 300001), (0, 1), (7, 63)])
def test_hash_range_incremental_state_bit_exact(r, c, seed, i0, n):
    p = cs.cs_params_init(r, c, seed, n)
    sk = orc.SketchOracle(r, c, seed)
    bucket = torch.empty(r * n, dtype=torch.int32, device=DEV)
    sign = torch.empty(r * n, dtype=torch.int8, device=DEV)
    cs.cs_hash_debug_range(p, i0, n, bucket, sign)
    rb, rs = sk.hash(np.arange(i0, i0 + n, dtype=np.int64))
    np.testing.assert_array_equal(bucket.cpu().numpy().view(np.uint32).reshape(r, n), rb)
    np.testing.assert_array_equal(sign.cpu().numpy().reshape(r, n), rs)


# ------------------------------------------------------------------------------ accumulate
@pytest.mark.parametrize("r,c,seed", SHAPES)
@pytest.mark.parametrize("d,i0,scale", [(1_000_003, 0, 1.0), (70_001, 5_000_000_000, -0.25), (1, 9, 3.0)])
def test_accumulate_dense(r, c, seed, d, i0, scale):
    p = cs.cs_params_init(r, c, seed, d)
    sk = orc.SketchOracle(r, c, seed)
    rng = np.random.default_rng(d)
    g = (rng.standard_normal(d) * 0.01).astype(np.float32)
    g[rng.integers(0, d, size=min(d, 50))] += 1.0
    S = torch.full((r, c), 0.5, dtype=torch.float32, device=DEV)     # accumulates, does not clear
    cs.cs_sketch_accumulate(p, S, dev(g), i0=i0, scale=scale)
    ref = sk.accumulate(np.full((r, c), 0.5), g, i0=i0, scale=scale)
    assert_cells_close(S.cpu().numpy(), ref, terms_per_cell=d / c)


def test_accumulate_empty_is_noop():
    p = cs.cs_params_init(5, 64, 1)
    S = torch.ones(5, 64, dtype=torch.float32, device=DEV)
    cs.cs_sketch_accumulate(p, S, torch.empty(0, dtype=torch.float32, device=DEV))
    assert (S == 1).all()


@pytest.mark.parametrize("W", [1, 3, 33])
def test_accumulate_batch(W):
    r, c, seed, d = 5, 1 << 12, 11, 200_003
    p = cs.cs_params_init(r, c, seed, d)
    sk = orc.SketchOracle(r, c, seed)
    rng = np.random.default_rng(W)
    gs = [(rng.standard_normal(d) * 0.01).astype(np.float32) for _ in range(W)]
    S_w = [torch.zeros(r, c, dtype=torch.float32, device=DEV) for _ in range(W)]
    cs.cs_sketch_accumulate_batch(p, S_w, [dev(g) for g in gs], i0=17, scale=0.5)
    for w in range(W):
        assert_cells_close(S_w[w].cpu().numpy(), sk.sketch(gs[w], i0=17, scale=0.5), what=f"worker {w}")


@pytest.mark.parametrize("W", [1, 2, 3, 5, 8, 13, 16, 32, 37])
@pytest.mark.parametrize("r,c,seed,d,i0", [(5, 1 << 12, 11, 200_003, (1 << 45) + 17), (7, 1 << 15, 5, 1_000_003, 0),
                                           (3, 1000, 9, 50_001, 3), (5, 1 << 10, 2, 1000, 0),
                                           (3, 64, 3, 2_000_003, 5),       # d / c = 31 250: thinned lists
                                           (15, 180_000, 4, 400_003, 1 << 40),    # a sketch shape of Table 1
                                           (7, 40, 6, 100_003, 0), (7, 40, 6, 784, 0),   # App. E's sketch
                                           (5, 100, 8, 300_001, 7), (1, 100, 8, 300_001, 7),
                                           (3, 32, 5, 70_001, 0),          # table in LDS
                                           (15, 127, 2, 50_001, 9)])       # the largest LDS table (61 KB)
@pytest.mark.parametrize("lds_table", [True, False])
def test_accumulate_bundle(W, r, c, seed, d, i0, lds_table):
    if W > 8 and d > 500_000:
        pytest.skip("covered by the smaller shapes")
    p = cs.cs_params_init(r, c, seed, d)
    if not lds_table:
        if c > 128 or r * c > 2048:
            pytest.skip("not a table that would get a workgroup-private copy anyway")
        p.flags = binding.CS_FLAG_NO_LDS_TABLE
    sk = orc.SketchOracle(r, c, seed)
    rng = np.random.default_rng(W * 1000 + r)
    gs = [(rng.standard_normal(d) * 0.01).astype(np.float32) for _ in range(W)]
    for g in gs:
        g[rng.integers(0, d, size=20)] += 1.0
    G = cs.CS_BUNDLE_GROUP
    n = cs.cs_bundle_floats(p, W)
    assert n == -(-W // G) * r * c * G
    T = torch.full((n,), 0.25, dtype=torch.float32, device=DEV)    # accumulates into T
    cs.cs_sketch_accumulate_bundle(p, T, [dev(g) for g in gs], i0=i0, scale=0.5)
    Th = T.cpu().numpy().reshape(-1, r, c, G)
    tables = [Th[w // G, :, :, w % G] for w in range(W)]
    for w in range(W):
        ref = sk.accumulate(np.full((r, c), 0.25), gs[w], i0=i0, scale=0.5)
        assert_cells_close(tables[w], ref, what=f"worker {w}", terms_per_cell=d / c)
    if W % G:                      # padding slots of the last group are never written
        assert (Th[-1, :, :, W % G:] == 0.25).all()
        T.view(-1, r, c, G)[-1, :, :, W % G:] = 0.0
    # merge of the bundle = (1/W) sum of the workers' tables
    dst0 = rng.standard_normal((r, c)).astype(np.float32)
    dst = dev(dst0)
    cs.cs_bundle_merge(p, dst, T, W, alpha=1.0 / W, beta=0.5)
    ref = orc.merge(tables, alpha=1.0 / W, beta=0.5, dst=dst0)
    assert_cells_close(dst.cpu().numpy(), ref)
    cs.cs_bundle_zero(p, T, W)
    assert (T == 0).all()


@pytest.mark.parametrize("W", [1, 3, 8, 13, 32])
@pytest.mark.parametrize("r,c,seed,d,i0,listed", [
    (5, 1 << 12, 11, 200_003, (1 << 45) + 17, True),      # visit lists, power-of-two columns
    (7, 1 << 15, 5, 1_000_003, 0, True),
    (5, 180_000, 41, 6_500_003, 1 << 40, True),           # visit lists for any column count (Table 1)
    (15, 180_000, 4, 400_003, 1 << 40, False),            # too short for such lists
    (5, 1000, 9, 50_001, 3, False),                       # worker by worker into the one table
    (7, 40, 6, 784, 0, False),                            # App. E's sketch
    (5, 1 << 12, 11, 3_000, 0, False)])                   # too short for a traversal plan
def test_accumulate_sum_of_workers(W, r, c, seed, d, i0, listed):
    """cs_sketch_accumulate_sum: the workers of one device added up as they are sketched, against
    the reference's sketch of the binary64 sum of their vectors (linearity, Sec. 3)."""
    if W > 8 and d > 2_000_000:
        pytest.skip("covered by the smaller shapes")
    p = cs.cs_params_init(r, c, seed, d)
    # which form runs: the list kernel (workers added up in registers) when every row has a list
    # that covers the vector, else the generic kernels, worker by worker into the one table
    plans = p.visit if p.c_pow2 else p.anyc
    assert all(plans[j].K > 0 and plans[j].cover >= d for j in range(r)) == listed
    sk = orc.SketchOracle(r, c, seed)
    rng = np.random.default_rng(W * 77 + r)
    gs = [(rng.standard_normal(d) * 0.01).astype(np.float32) for _ in range(W)]
    for g in gs:
        g[rng.integers(0, d, size=20)] += 1.0
    gs[0][5], gs[-1][d - 1] = np.float32(-3.0), np.float32(2.5)
    S = torch.full((r, c), 0.25, dtype=torch.float32, device=DEV)       # accumulates into S
    cs.cs_sketch_accumulate_sum(p, S, [dev(g) for g in gs], i0=i0, scale=0.5)
    gsum = np.zeros(d)
    for g in gs:
        gsum += g.astype(np.float64)
    ref = sk.accumulate(np.full((r, c), 0.25), gsum, i0=i0, scale=0.5)
    assert_cells_close(S.cpu().numpy(), ref, what=f"sum of {W} workers", terms_per_cell=W * d / c)
    # NaN and infinities of any worker reach the cells they belong to
    gs[W // 2][7] = np.nan
    gs[0][11] = np.inf
    S.fill_(0.0)
    cs.cs_sketch_accumulate_sum(p, S, [dev(g) for g in gs], i0=i0)
    got = S.cpu().numpy()
    bkt, _ = sk.hash(np.array([i0 + 7, i0 + 11]))
    for j in range(r):
        assert np.isnan(got[j, bkt[j, 0]])
        assert not np.isfinite(got[j, bkt[j, 1]])
    assert np.isfinite(got).sum() >= got.size - 2 * r


@pytest.mark.parametrize("r,c,seed,d,d_hint,W,i0", [
    (5, 180_000, 41, 6_500_000, 6_500_000, 9, 0),        # Table 1: 5 x 180 000; two groups, the second partial
    (15, 180_000, 42, 6_500_000, 6_500_000, 3, 12_345),  # Table 1: 15 x 180 000
    (5, 180_000, 43, 2_000_003, 6_500_000, 8, 1 << 40),  # a vector shorter than the list was made for
    (3, 50_021, 44, 3_000_001, 3_000_001, 2, 7),         # a prime column count
    (5, 3 << 15, 45, 5_000_000, 5_000_000, 1, 0),        # 3 * 2^15 columns
    (5, 180_000, 46, 17_000_000, 17_000_000, 1, 3)])     # long enough for the query to follow the lists too
def test_accumulate_bundle_visit_lists_for_any_column_count(r, c, seed, d, d_hint, W, i0):
    """Column counts that are not a power of two, long vectors: the update follows per-row visit
    lists (offsets whose hash advance is 0 or 1 cells modulo c) and keeps 2 or 4 running sums
    per coordinate, the second half for coordinates whose hash value wrapped past p.  Every
    worker's table against the reference, and the same call with the lists switched off."""
    p = cs.cs_params_init(r, c, seed, d_hint)
    assert all(p.anyc[j].K > 0 for j in range(r)), "no list was planned for this shape"
    # per group of 8 workers, one launch per 6 rows that keep the same number of running sums
    per_group = sum(-(-sum(1 for j in range(r) if p.anyc[j].omega == omega) // 6) for omega in (1, 2))
    assert cs.cs_bundle_update_launches(p, W, d) == per_group * -(-W // cs.CS_BUNDLE_GROUP)
    sk = orc.SketchOracle(r, c, seed)
    rng = np.random.default_rng(seed)
    gs = [(rng.standard_normal(d) * 0.01).astype(np.float32) for _ in range(W)]
    for g in gs:
        g[rng.integers(0, d, size=50)] += 1.0
    tables = _bundle_tables(p, gs, r, c, i0=i0, scale=0.5)
    for w in range(W):
        ref = sketch_in_slices_i0(sk, gs[w], i0, 0.5)
        assert_cells_close(tables[w], ref, what=f"worker {w}", terms_per_cell=d / c)
    direct = cs.CsParams.from_buffer_copy(p)
    direct.flags = binding.CS_FLAG_NO_VISIT_LIST
    assert cs.cs_bundle_update_launches(direct, W, d) == -(-W // 32)
    tables_direct = _bundle_tables(direct, gs[:1], r, c, i0=i0, scale=0.5)
    assert_cells_close(tables_direct[0], sketch_in_slices_i0(sk, gs[0], i0, 0.5), what="lists off")
    # the query follows the same lists (a lane keeps the 2 or 4 cell values a coordinate can
    # meet): bit-exact from the same table, also with NaN and infinite cells, and equal to the
    # query without lists
    T32 = rng.standard_normal((r, c)).astype(np.float32)
    T32.reshape(-1)[rng.choice(r * c, size=r * c // 50, replace=False)] = np.nan
    T32.reshape(-1)[rng.choice(r * c, size=r * c // 50, replace=False)] = -np.inf
    S = dev(T32)
    ref = estimate_in_slices_i0(sk, T32.astype(np.float64), d, i0).astype(np.float32)
    for params in (p, direct):
        est = torch.empty(d, dtype=torch.float32, device=DEV)
        n_ws = cs.cs_estimate_workspace_bytes(params, d)
        assert (n_ws > 0) == (params is p and d * (r - 1) >= 1 << 26)
        ws = torch.empty(n_ws, dtype=torch.uint8, device=DEV) if n_ws else None
        hist = torch.empty(binding.CS_TOPK_HIST_BINS, dtype=torch.int64, device=DEV)
        cs.cs_sketch_estimate(params, S, est, i0=i0, workspace=ws, hist=hist)
        got = est.cpu().numpy()
        np.testing.assert_array_equal(np.isnan(got), np.isnan(ref))
        ok = ~np.isnan(ref)
        np.testing.assert_array_equal(got[ok].view(np.uint32), ref[ok].view(np.uint32))
        want = np.bincount((got.view(np.uint32) & np.uint32(0x7FFFFFFF)) >> np.uint32(20), minlength=2048)
        np.testing.assert_array_equal(hist.cpu().numpy(), want)


def test_forged_visit_list_for_any_column_count_costs_time_not_correctness():
    """A list whose offsets do not keep a coordinate within its 2 omega cells (arbitrary gaps):
    the update sends such visits' values to memory one by one and the query gathers them from
    the table directly, so the results are still the reference's."""
    r, c, seed, d, W = 5, 180_000, 51, 17_000_000, 2
    p = cs.cs_params_init(r, c, seed, d)
    assert all(p.anyc[j].K > 0 for j in range(r))
    sk = orc.SketchOracle(r, c, seed)
    rng = np.random.default_rng(seed)
    forged = cs.CsParams.from_buffer_copy(p)
    for j in range(r):
        v = forged.anyc[j]
        gaps = [1_000_003 + 7 * j, 2_500_001, 3_000_017, 999_999]
        gaps.append(d - sum(gaps))
        v.K, v.omega, v.cover, v.gmax, v.cost, v.cost_direct = len(gaps), 1 + j % 2, d, max(gaps), 1, 2
        for k, g in enumerate(gaps):
            v.gap[k] = g
    gs = [(rng.standard_normal(d) * 0.01).astype(np.float32) for _ in range(W)]
    for w, tab in enumerate(_bundle_tables(forged, gs, r, c, i0=3, scale=1.0)):
        assert_cells_close(tab, sketch_in_slices_i0(sk, gs[w], 3, 1.0), what=f"forged list, worker {w}",
                           terms_per_cell=d / c)
    T32 = rng.standard_normal((r, c)).astype(np.float32)
    est = torch.empty(d, dtype=torch.float32, device=DEV)
    n_ws = cs.cs_estimate_workspace_bytes(forged, d)
    assert n_ws > 0
    ws = torch.empty(n_ws, dtype=torch.uint8, device=DEV)
    cs.cs_sketch_estimate(forged, dev(T32), est, i0=3, workspace=ws)
    ref = estimate_in_slices_i0(sk, T32.astype(np.float64), d, 3).astype(np.float32)
    np.testing.assert_array_equal(est.cpu().numpy(), ref)


def estimate_in_slices_i0(sk, T, d, i0):
    from concurrent.futures import ThreadPoolExecutor
    n = 1 << 20
    cuts = list(range(0, d, n))
    with ThreadPoolExecutor(max_workers=8) as pool:
        parts = list(pool.map(lambda lo: sk.estimate(T, min(n, d - lo), i0=i0 + lo), cuts))
    return np.concatenate(parts)


def sketch_in_slices_i0(sk, g, i0, scale):
    """the reference's sketch of g with global index i0 of g[0], computed slice by slice on threads"""
    from concurrent.futures import ThreadPoolExecutor
    n = 1 << 20
    cuts = list(range(0, g.size, n))
    with ThreadPoolExecutor(max_workers=8) as pool:
        parts = list(pool.map(lambda lo: sk.sketch(g[lo:lo + n], i0=i0 + lo, scale=scale), cuts))
    T = sk.zeros()
    for part in parts:
        T += part
    return T


def _bundle_tables(p, gs, r, c, i0=0, scale=1.0):
    W, G = len(gs), cs.CS_BUNDLE_GROUP
    T = torch.zeros(cs.cs_bundle_floats(p, W), dtype=torch.float32, device=DEV)
    cs.cs_sketch_accumulate_bundle(p, T, [dev(g) for g in gs], i0=i0, scale=scale)
    Th = T.cpu().numpy().reshape(-1, r, c, G)
    return [Th[w // G, :, :, w % G] for w in range(W)]


@pytest.mark.parametrize("W", [1, 2, 3, 8, 12, 13, 70])    # 12: a narrow last group; 70: two launches
def test_accumulate_bundle_every_traversal(W):
    """The same vectors through the visit-list update (the default when a list exists), the
    stride walk (list switched off by flag), a forged list whose offsets do not keep a lane
    within its cells (every such visit takes the kernel's one-by-one fallback), and vectors
    shorter and longer than the length the list was built for: all against the reference."""
    import ctypes
    r, c, seed, d = 5, 1 << 12, 11, 200_003
    P = (1 << 61) - 1
    p = cs.cs_params_init(r, c, seed, d)
    assert all(p.visit[j].K > 0 for j in range(r))
    sk = orc.SketchOracle(r, c, seed)
    rng = np.random.default_rng(W)
    gs = [(rng.standard_normal(d) * 0.01).astype(np.float32) for _ in range(W)]
    for g in gs:
        g[rng.integers(0, d, size=20)] -= 1.0
    refs = [sk.sketch(g, i0=5, scale=2.0) for g in gs]

    def check(params, what):
        for w, tab in enumerate(_bundle_tables(params, gs, r, c, i0=5, scale=2.0)):
            assert_cells_close(tab, refs[w], what=f"{what}, worker {w}", terms_per_cell=d / c)

    check(p, "visit list")
    walk = binding.CsParams.from_buffer_copy(p)
    walk.flags = binding.CS_FLAG_NO_VISIT_LIST
    check(walk, "stride walk")
    forged = binding.CsParams.from_buffer_copy(p)
    g0 = 30_011
    for j in range(r):
        v = forged.visit[j]
        ctypes.memset(ctypes.byref(v), 0, ctypes.sizeof(v))
        v.K, v.ncell, v.cover, v.gmax, v.cost, v.cost_walk = 3, 2, d, d - 2 * g0, 1, 2
        v.gap[0], v.gap[3] = g0, d - 2 * g0
        v.A[0], v.As[0] = (p.a[j] * g0) % P, (p.as_[j] * g0) % P
        v.code[0] = 0b110000                      # visits 0, 1: code 0; visit 2: code 3
    check(forged, "forged list")
    # the same three sets of parameters with the workers summed as they are sketched
    # (cs_sketch_accumulate_sum): list kernel with the sums folded across lanes, the generic
    # kernels when the lists are switched off, the folded fallback of the forged list
    gsum = np.zeros(d)
    for g in gs:
        gsum += g.astype(np.float64)
    ref_sum = sk.sketch(gsum, i0=5, scale=2.0)
    for params, what in ((p, "visit list"), (walk, "lists off"), (forged, "forged list")):
        S = torch.zeros(r, c, dtype=torch.float32, device=DEV)
        cs.cs_sketch_accumulate_sum(params, S, [dev(g) for g in gs], i0=5, scale=2.0)
        assert_cells_close(S.cpu().numpy(), ref_sum, what=f"sum of workers, {what}", terms_per_cell=W * d / c)
    # shorter than planned: the list still applies; longer: the stride walk takes over
    for d2 in (d - 12_345, 4_100):
        short = [g[:d2] for g in gs]
        for w, tab in enumerate(_bundle_tables(p, short, r, c)):
            assert_cells_close(tab, sk.sketch(short[w]), what=f"d = {d2}, worker {w}",
                               terms_per_cell=d2 / c)
    pl = cs.cs_params_init(r, c, seed, d - 50_000)
    assert pl.visit[0].cover < d
    for w, tab in enumerate(_bundle_tables(pl, gs, r, c, i0=5, scale=2.0)):
        assert_cells_close(tab, refs[w], what=f"longer than planned, worker {w}", terms_per_cell=d / c)


def test_accumulate_bundle_vectors_at_any_dword_address():
    """Worker vectors need only 4-byte alignment (views into larger tensors)."""
    r, c, seed, d = 5, 1 << 12, 21, 300_001
    p = cs.cs_params_init(r, c, seed, d)
    assert any(p.visit[j].K > 0 for j in range(r))
    sk = orc.SketchOracle(r, c, seed)
    rng = np.random.default_rng(5)
    big = [(rng.standard_normal(d + 3) * 0.01).astype(np.float32) for _ in range(3)]
    views = [dev(x)[off:off + d] for off, x in zip((1, 2, 3), big)]
    assert all(v.data_ptr() % 16 != 0 for v in views)
    T = torch.zeros(cs.cs_bundle_floats(p, 3), dtype=torch.float32, device=DEV)
    cs.cs_sketch_accumulate_bundle(p, T, views)
    Th = T.cpu().numpy().reshape(-1, r, c, cs.CS_BUNDLE_GROUP)
    for w, (off, x) in enumerate(zip((1, 2, 3), big)):
        assert_cells_close(Th[0, :, :, w], sk.sketch(x[off:off + d]), what=f"worker {w}",
                           terms_per_cell=d / c)


def test_accumulate_bundle_nan_and_inf_stay_in_their_cells():
    """Device data are not validated: a NaN or an infinity in a vector must end up in exactly the
    r cells of its coordinate (as in the reference), not in neighbouring running sums."""
    r, c, seed, d, W = 5, 1 << 12, 11, 200_003, 8
    p = cs.cs_params_init(r, c, seed, d)
    assert all(p.visit[j].K > 0 for j in range(r))
    sk = orc.SketchOracle(r, c, seed)
    rng = np.random.default_rng(4)
    gs = [(rng.standard_normal(d) * 0.01).astype(np.float32) for _ in range(W)]
    gs[2][[7, 100_000]] = [np.nan, np.inf]
    gs[5][[150_000, 150_001, 199_999]] = [-np.inf, np.inf, np.nan]
    for w, tab in enumerate(_bundle_tables(p, gs, r, c)):
        with np.errstate(invalid="ignore"):
            ref = sk.sketch(gs[w])
        assert (np.isnan(tab) == np.isnan(ref)).all(), f"worker {w}: NaN cells differ"
        assert (np.isinf(tab) == np.isinf(ref)).all() and (np.sign(tab[np.isinf(ref)]) == np.sign(ref[np.isinf(ref)])).all()
        fin = np.isfinite(ref)
        assert fin.sum() >= r * c - 3 * r
        good_rows = np.where(fin, ref, 0.0)
        err = np.abs(np.where(fin, tab, 0.0) - good_rows)
        sigma = np.sqrt((good_rows ** 2).mean(axis=1, keepdims=True))
        assert (err <= 1e-5 * np.maximum(np.abs(good_rows), sigma)).all()


@pytest.mark.parametrize("r,c,seed", SHAPES[:5])
def test_accumulate_sparse_with_repeats(r, c, seed):
    p = cs.cs_params_init(r, c, seed)
    sk = orc.SketchOracle(r, c, seed)
    rng = np.random.default_rng(1)
    n = 10_007
    idx = rng.integers(0, 1 << 40, size=n)
    idx[::10] = idx[0]                                   # repeated index: values add up
    val = rng.standard_normal(n).astype(np.float32)
    S = torch.zeros(r, c, dtype=torch.float32, device=DEV)
    cs.cs_sketch_accumulate_sparse(p, S, dev(idx), dev(val), scale=-2.0)
    ref = sk.accumulate_sparse(sk.zeros(), idx, val.astype(np.float64), scale=-2.0)
    assert_cells_close(S.cpu().numpy(), ref)


# ------------------------------------------------------------------------------ table ops
@pytest.mark.parametrize("W", [1, 5, 130])
def test_merge_axpby_momentum_zero(W):
    r, c = 5, 3001
    p = cs.cs_params_init(r, c, 1)
    rng = np.random.default_rng(W)
    tabs = [rng.standard_normal((r, c)).astype(np.float32) for _ in range(W)]
    dst0 = rng.standard_normal((r, c)).astype(np.float32)
    dst = dev(dst0)
    cs.cs_sketch_merge(p, dst, [dev(t) for t in tabs], alpha=1.0 / W, beta=0.0)
    assert_cells_close(dst.cpu().numpy(), orc.merge(tabs, alpha=1.0 / W))
    dst = dev(dst0)
    cs.cs_sketch_merge(p, dst, [dev(t) for t in tabs], alpha=0.5, beta=-2.0)
    assert_cells_close(dst.cpu().numpy(), orc.merge(tabs, alpha=0.5, beta=-2.0, dst=dst0))
    # beta = 0 must not read dst (NaN there must not leak)
    dst = torch.full((r, c), float("nan"), dtype=torch.float32, device=DEV)
    cs.cs_sketch_merge(p, dst, [dev(t) for t in tabs], alpha=1.0, beta=0.0)
    assert torch.isfinite(dst).all()

    x, y = tabs[0], dst0
    yd = dev(y)
    cs.cs_sketch_axpby(p, yd, 0.75, dev(x), -1.5)
    assert_cells_close(yd.cpu().numpy(), 0.75 * x.astype(np.float64) - 1.5 * y)

    su, sv, st = dev(tabs[0]), dev(dst0), dev(tabs[-1])
    cs.cs_sketch_momentum(p, su, sv, st, 0.9)
    rho = float(np.float32(0.9))
    u_ref = rho * tabs[0].astype(np.float64) + tabs[-1]
    assert_cells_close(su.cpu().numpy(), u_ref)
    assert_cells_close(sv.cpu().numpy(), dst0.astype(np.float64) + u_ref)

    cs.cs_sketch_zero(p, su)
    assert (su == 0).all()


def test_count_nonfinite_cells():
    """the failure detector counts exactly the NaN and infinite cells (numpy's isfinite), and a
    single infinite gradient element shows up in r cells of the worker's table"""
    r, c = 5, 1 << 12
    p = cs.cs_params_init(r, c, 3, 100_003)
    rng = np.random.default_rng(0)
    T32 = rng.standard_normal((r, c)).astype(np.float32)
    T32.reshape(-1)[rng.choice(r * c, size=37, replace=False)] = np.nan
    T32.reshape(-1)[rng.choice(r * c, size=11, replace=False)] = -np.inf
    T32[0, 0] = np.float32(3.4e38)
    T32[1, 1] = np.float32(1e-45)
    count = torch.full((1,), -7, dtype=torch.int64, device=DEV)
    cs.cs_sketch_count_nonfinite(p, dev(T32), count)
    assert count.item() == int((~np.isfinite(T32)).sum())
    g = (rng.standard_normal(100_003) * 0.01).astype(np.float32)
    g[4242] = np.inf
    T = torch.zeros(cs.cs_bundle_floats(p, 1), dtype=torch.float32, device=DEV)
    cs.cs_sketch_accumulate_bundle(p, T, [dev(g)])
    S = torch.zeros(r, c, dtype=torch.float32, device=DEV)
    cs.cs_bundle_merge(p, S, T, 1, alpha=1.0, beta=0.0)
    cs.cs_sketch_count_nonfinite(p, S, count)
    assert count.item() == r


# ------------------------------------------------------------------------------ estimate
@pytest.mark.parametrize("r,c,seed", SHAPES)
@pytest.mark.parametrize("d,i0", [(1_000_003, 0), (4097, 3_000_000_000)])
def test_estimate_bit_exact_from_same_table(r, c, seed, d, i0):
    p = cs.cs_params_init(r, c, seed, d)
    sk = orc.SketchOracle(r, c, seed)
    T32 = (np.random.default_rng(seed).standard_normal((r, c))).astype(np.float32)
    S = dev(T32)
    est = torch.empty(d, dtype=torch.float32, device=DEV)
    n_ws = cs.cs_estimate_workspace_bytes(p, d)
    ws = torch.empty(n_ws, dtype=torch.uint8, device=DEV) if n_ws else None
    cs.cs_sketch_estimate(p, S, est, i0=i0, workspace=ws)
    ref = sk.estimate(T32.astype(np.float64), d, i0=i0)
    np.testing.assert_array_equal(est.cpu().numpy(), ref.astype(np.float32))
    # listed coordinates
    idx = np.random.default_rng(1).integers(i0, i0 + d, size=777)
    out = torch.empty(777, dtype=torch.float32, device=DEV)
    cs.cs_sketch_estimate_sparse(p, S, dev(idx), out)
    np.testing.assert_array_equal(out.cpu().numpy(), ref[idx - i0].astype(np.float32))


@pytest.mark.parametrize("r,c,seed,d,i0", [(5, 1 << 16, 3, (1 << 24) + 5, 7), (7, 1 << 14, 4, (1 << 24) + 4096, 0),
                                           (1, 1 << 12, 5, 1 << 24, 1)])
def test_estimate_long_vector_bit_exact(r, c, seed, d, i0):
    """Vectors of 2^24 coordinates and more: the last row's walk takes the median itself."""
    p = cs.cs_params_init(r, c, seed, d)
    sk = orc.SketchOracle(r, c, seed)
    T32 = (np.random.default_rng(seed).standard_normal((r, c))).astype(np.float32)
    est = torch.empty(d, dtype=torch.float32, device=DEV)
    n_ws = cs.cs_estimate_workspace_bytes(p, d)
    ws = torch.empty(n_ws, dtype=torch.uint8, device=DEV) if n_ws else None
    cs.cs_sketch_estimate(p, dev(T32), est, i0=i0, workspace=ws)
    ref = sk.estimate(T32.astype(np.float64), d, i0=i0)
    np.testing.assert_array_equal(est.cpu().numpy(), ref.astype(np.float32))


@pytest.mark.parametrize("r,c,seed,d,k", [(5, 1 << 16, 31, (1 << 24) + 1029, 20_000),   # counted by the kernel that writes est
                                          (5, 1 << 12, 32, 1_200_003, 1_000),          # counted by one more read of est
                                          (7, 1000, 33, 600_001, 700), (3, 64, 34, 1, 1)])
def test_estimate_fills_the_first_histogram_of_the_selection(r, c, seed, d, k):
    """cs_sketch_estimate with hist: the counts of the estimates by the top 11 bits of their
    magnitude are exact (integer work on bit-exact estimates), a stale histogram is cleared, and
    the selection that is handed the histogram returns what the selection without it returns."""
    p = cs.cs_params_init(r, c, seed, d)
    sk = orc.SketchOracle(r, c, seed)
    T32 = (np.random.default_rng(seed).standard_normal((r, c)) * 0.01).astype(np.float32)
    T32.reshape(-1)[::17] *= 64.0                     # a few octaves of magnitudes
    est = torch.empty(d, dtype=torch.float32, device=DEV)
    hist = torch.full((binding.CS_TOPK_HIST_BINS,), 12345, dtype=torch.int64, device=DEV)
    n_ws = cs.cs_estimate_workspace_bytes(p, d)
    ws = torch.empty(n_ws, dtype=torch.uint8, device=DEV) if n_ws else None
    cs.cs_sketch_estimate(p, dev(T32), est, i0=0, workspace=ws, hist=hist)
    ref = sk.estimate(T32.astype(np.float64), d).astype(np.float32)
    np.testing.assert_array_equal(est.cpu().numpy(), ref)
    want = np.bincount((ref.view(np.uint32) & np.uint32(0x7FFFFFFF)) >> np.uint32(20), minlength=2048)
    np.testing.assert_array_equal(hist.cpu().numpy(), want)
    tws = torch.empty(cs.cs_topk_workspace_bytes(d, k), dtype=torch.uint8, device=DEV)
    out = []
    for h in (hist, None):
        idx = torch.empty(k, dtype=torch.int64, device=DEV)
        val = torch.empty(k, dtype=torch.float32, device=DEV)
        cs.cs_heavy_hitters_topk(est, k, idx, val, tws, hist=h)
        out.append((idx.cpu().numpy(), val.cpu().numpy()))
    np.testing.assert_array_equal(out[0][0], out[1][0])
    np.testing.assert_array_equal(out[0][1].view(np.uint32), out[1][1].view(np.uint32))
    np.testing.assert_array_equal(out[0][0], orc.topk_threshold(ref, k))


@pytest.mark.parametrize("r,c,seed,d", [(5, 1 << 12, 21, 300_007),          # median pass over stored rows
                                        (7, 1 << 10, 22, (1 << 24) + 33),  # median inside the last row's walk
                                        (5, 1000, 23, 50_001),             # one thread per coordinate
                                        (15, 180, 24, 20_003), (3, 64, 25, 4_099)])
def test_estimate_with_nan_and_infinite_cells(r, c, seed, d):
    """Alg. 4's estimate when the table holds NaN and infinities (a diverged run): the median is
    the middle of the r signed cells after a sort, and with a NaN among them the sort's own
    sequence of comparisons decides what ends up in the middle.  The device makes the comparisons
    the reference's insertion sort makes, so NaN appears in exactly the same estimates and every
    other estimate is equal bit for bit (signed zeros included)."""
    p = cs.cs_params_init(r, c, seed, d)
    sk = orc.SketchOracle(r, c, seed)
    rng = np.random.default_rng(seed)
    T32 = rng.standard_normal((r, c)).astype(np.float32)
    flat = T32.reshape(-1)
    n = flat.size
    for value, share in [(np.nan, 0.08), (np.inf, 0.05), (-np.inf, 0.05), (0.0, 0.05), (-0.0, 0.05)]:
        flat[rng.choice(n, size=max(1, int(share * n)), replace=False)] = value
    S = dev(T32)
    est = torch.empty(d, dtype=torch.float32, device=DEV)
    n_ws = cs.cs_estimate_workspace_bytes(p, d)
    ws = torch.empty(n_ws, dtype=torch.uint8, device=DEV) if n_ws else None
    cs.cs_sketch_estimate(p, S, est, i0=0, workspace=ws)
    ref = sk.estimate(T32.astype(np.float64), d).astype(np.float32)
    got = est.cpu().numpy()
    assert np.isnan(ref).any() and np.isinf(ref).any()

    def same(a, b, what):
        np.testing.assert_array_equal(np.isnan(a), np.isnan(b), err_msg=what)
        ok = ~np.isnan(b)
        np.testing.assert_array_equal(a[ok].view(np.uint32), b[ok].view(np.uint32), err_msg=what)

    same(got, ref, "all coordinates")
    idx = rng.integers(0, d, size=5000)
    out = torch.empty(idx.size, dtype=torch.float32, device=DEV)
    cs.cs_sketch_estimate_sparse(p, S, dev(idx), out)
    same(out.cpu().numpy(), ref[idx], "listed coordinates")


# ------------------------------------------------------------------------------ top-k
def run_topk(est32, k):
    d = est32.size
    est = dev(est32)
    idx = torch.empty(k, dtype=torch.int64, device=DEV)
    val = torch.empty(k, dtype=torch.float32, device=DEV)
    ws = torch.empty(cs.cs_topk_workspace_bytes(d, k), dtype=torch.uint8, device=DEV)
    ws.fill_(0xAB)      # contents on entry must not matter
    cs.cs_heavy_hitters_topk(est, k, idx, val, ws)
    return idx.cpu().numpy(), val.cpu().numpy()


@pytest.mark.parametrize("d,k", [(1, 1), (5, 5), (1000, 1), (1023, 37), (1025, 1025), (4096, 256),
                                 (1_000_003, 1000), (1_000_003, 999_999), (5_000_011, 50_000)])
@pytest.mark.parametrize("kind", ["gauss", "ties", "zeros"])
def test_topk_exact(d, k, kind):
    rng = np.random.default_rng(d + k)
    if kind == "gauss":
        est = (rng.standard_normal(d) * 0.01).astype(np.float32)
    elif kind == "ties":                       # heavy ties, both signs, signed zeros
        est = (np.round(rng.standard_normal(d) * 3) / 4).astype(np.float32)
        est[::7] *= -1
    else:
        est = np.zeros(d, dtype=np.float32)
        est[1::2] = -0.0
    want = orc.topk_threshold(est, k) if d > (1 << 18) else orc.topk(est, k)
    idx, val = run_topk(est, k)
    np.testing.assert_array_equal(idx, want)
    np.testing.assert_array_equal(val.view(np.uint32), est[want].view(np.uint32))


@pytest.mark.parametrize("case", ["spread", "one block full of heavy entries", "unaligned", "all in one bin",
                                  "k a few per cent of d", "k a few per cent of d, heavy tail"])
def test_topk_candidate_list_and_five_pass_form_agree(case):
    """With room for a candidate list in the workspace the selection reads est twice, without it
    five times; both must return the reference's selection.  Covered: the ordinary case, a
    stretch of heavy entries longer than one block can stage (the list is abandoned on the
    device and the five-pass form takes over), an input at an odd dword address, and
    magnitudes that all fall into the bin of the k-th largest (the list overflows as a whole)."""
    rng = np.random.default_rng(len(case))
    d, k = 20_000_003, 30_000
    est = (rng.standard_normal(d) * 0.01).astype(np.float32)
    if case == "one block full of heavy entries":
        est[7_000_000:7_009_000] = rng.uniform(0.5, 1.0, size=9000).astype(np.float32)
    elif case == "all in one bin":
        est = rng.uniform(1.0, 1.05, size=d).astype(np.float32) * rng.choice([-1.0, 1.0], size=d).astype(np.float32)
    elif case == "unaligned":
        d, k = 700_001, 500
        est = est[:d].copy()
    elif case.startswith("k a few per cent of d"):
        k = 1_200_000                                  # 6 % of d: the tightly sized list (3 k + 65 536 entries)
        if case.endswith("heavy tail"):
            est = (rng.standard_t(2.5, size=d) * 0.01).astype(np.float32)
    want = orc.topk_threshold(est, k)
    base = torch.empty(d + 1, dtype=torch.float32, device=DEV)
    off = 1 if case == "unaligned" else 0
    view = base[off:off + d]
    view.copy_(dev(est))
    full = cs.cs_topk_workspace_bytes(d, k)
    bare = cs.cs_topk_workspace_bytes(1, 1)            # the fixed part alone: no list
    assert full > bare + 12 * (2 * k + 4096)
    for nbytes in (full, bare):
        ws = torch.empty(nbytes, dtype=torch.uint8, device=DEV)
        ws.fill_(0x5C)
        idx = torch.full((k,), -1, dtype=torch.int64, device=DEV)
        val = torch.empty(k, dtype=torch.float32, device=DEV)
        cs.cs_heavy_hitters_topk(view, k, idx, val, ws)
        np.testing.assert_array_equal(idx.cpu().numpy(), want)
        np.testing.assert_array_equal(val.cpu().numpy().view(np.uint32), est[want].view(np.uint32))


def test_topk_extreme_values_and_unaligned_input():
    d, k = 100_003, 10
    est = (np.random.default_rng(0).standard_normal(d)).astype(np.float32)
    est[17] = np.float32(3.4e38)
    est[99_999] = -np.float32(3.4e38)
    est[5] = np.float32(1e-45)                  # subnormal: smallest positive key
    base = torch.empty(d + 1, dtype=torch.float32, device=DEV)
    base[1:] = dev(est)
    view = base[1:]                             # 4-byte aligned only
    idx = torch.empty(k, dtype=torch.int64, device=DEV)
    val = torch.empty(k, dtype=torch.float32, device=DEV)
    ws = torch.empty(cs.cs_topk_workspace_bytes(d, k), dtype=torch.uint8, device=DEV)
    cs.cs_heavy_hitters_topk(view, k, idx, val, ws)
    want = orc.topk(est, k)
    np.testing.assert_array_equal(idx.cpu().numpy(), want)
    assert 17 in want and 99_999 in want


@pytest.mark.parametrize("n,k", [(1, 1), (600, 50), (3_600_000, 100_000), (5000, 5000)])
def test_select_exact_topk(n, k):
    rng = np.random.default_rng(n + k)
    cand = np.sort(rng.choice(10**8, n, replace=False)).astype(np.int64)
    x = (np.round(rng.standard_normal(n) * 50) / 50).astype(np.float32)      # ties
    idx = torch.empty(k, dtype=torch.int64, device=DEV)
    val = torch.empty(k, dtype=torch.float32, device=DEV)
    ws = torch.empty(cs.cs_topk_workspace_bytes(n, k), dtype=torch.uint8, device=DEV)
    cs.cs_select_exact_topk(dev(cand), dev(x), k, idx, val, ws)
    if n > (1 << 18):
        pos = orc.topk_threshold(x, k)
        want_idx, want_val = cand[pos], x[pos]
    else:
        want_idx, want_val = orc.select_exact_topk(cand, x, k)
    np.testing.assert_array_equal(idx.cpu().numpy(), want_idx)
    np.testing.assert_array_equal(val.cpu().numpy(), np.asarray(want_val, dtype=np.float32))


# ------------------------------------------------------------------------------ gather / feedback
@pytest.mark.parametrize("W", [1, 4, 70])
def test_gather_exact(W):
    d, k = 300_007, 5000
    rng = np.random.default_rng(W)
    vecs = [rng.standard_normal(d).astype(np.float32) for _ in range(W)]
    idx = np.sort(rng.choice(d, k, replace=False))
    out = torch.empty(k, dtype=torch.float32, device=DEV)
    cs.cs_gather_exact([dev(v) for v in vecs], dev(idx), out, alpha=1.0 / W)
    ref = orc.gather_exact(vecs, idx, 1.0 / W)
    scale = 1.0 / np.sqrt(W)
    assert_values_close(out.cpu().numpy(), ref, scale)


def test_feedback_removes_estimated_values():
    r, c, seed, d, k = 5, 1 << 12, 21, 1 << 16, 300
    p = cs.cs_params_init(r, c, seed, d)
    sk = orc.SketchOracle(r, c, seed)
    rng = np.random.default_rng(2)
    T32 = rng.standard_normal((r, c)).astype(np.float32)
    idx = np.sort(rng.choice(d, k, replace=False))
    S = dev(T32)
    val = torch.empty(k, dtype=torch.float32, device=DEV)
    cs.cs_sketch_feedback(p, S, dev(idx), val)
    T = T32.astype(np.float64)
    ref_val = sk.estimate_sparse(T, idx)
    np.testing.assert_array_equal(val.cpu().numpy(), ref_val.astype(np.float32))
    sk.accumulate_sparse(T, idx, ref_val, scale=-1.0)
    assert_cells_close(S.cpu().numpy(), T)


# ------------------------------------------------------------------------------ HEAVYMIX
@pytest.mark.parametrize("r,c,seed,d,k,planted", [
    (5, 1 << 12, 31, 200_003, 100, 12),
    (7, 1 << 15, 32, 3_000_001, 1000, 40),
    (5, 1 << 15, 190304489, 10_000_000, 2000, 0),
    (3, 64, 33, 5_000, 5_000, 3),            # k = d: everything is selected
    (1, 1 << 10, 34, 70_000, 1, 1),
])
def test_heavymix_l2_estimate_and_selection(r, c, seed, d, k, planted):
    """Alg. 1 on the device against the reference: the norm estimate from the same fp32 table
    (binary64 sums: equal to rounding order), then the threshold split and the seeded fill on
    the same binary32 estimates and the same threshold, which must agree index by index."""
    p = cs.cs_params_init(r, c, seed, d)
    sk = orc.SketchOracle(r, c, seed)
    rng = np.random.default_rng(seed)
    g = (rng.standard_normal(d) * 0.01).astype(np.float32)
    where = rng.choice(d, planted, replace=False)
    g[where] = (rng.uniform(0.5, 1.0, planted) * rng.choice([-1.0, 1.0], planted)).astype(np.float32)
    S = torch.zeros(r, c, dtype=torch.float32, device=DEV)
    cs.cs_sketch_accumulate(p, S, dev(g))
    out = torch.empty(1 + r, dtype=torch.float64, device=DEV)
    cs.cs_sketch_l2sq(p, S, out)
    ref_l2, ref_rows = orc.l2sq_estimate(ref_table_from_device(S))
    got = out.cpu().numpy()
    np.testing.assert_allclose(got[1:], ref_rows, rtol=1e-12)
    np.testing.assert_allclose(got[0], ref_l2, rtol=1e-12)
    true = float(g.astype(np.float64) @ g.astype(np.float64))
    if c >= 1 << 12:
        assert 0.5 * true <= got[0] <= 1.5 * true                      # Alg. 1 step 1

    est = torch.empty(d, dtype=torch.float32, device=DEV)
    ws_e = torch.empty(cs.cs_estimate_workspace_bytes(p, d), dtype=torch.uint8, device=DEV)
    cs.cs_sketch_estimate(p, S, est, workspace=ws_e if ws_e.numel() else None)
    est_h = est.cpu().numpy()
    ws = torch.empty(cs.cs_topk_workspace_bytes(d, k), dtype=torch.uint8, device=DEV)
    idx = torch.empty(k, dtype=torch.int64, device=DEV)
    val = torch.empty(k, dtype=torch.float32, device=DEV)
    n_heavy = torch.full((1,), -1, dtype=torch.int64, device=DEV)
    # the sketch's own threshold, one so small that more than k pass, one so large that none does
    for l2sq in (float(got[0]), 1e-12, 1e12):
        l2 = torch.tensor([l2sq], dtype=torch.float64, device=DEV)
        for rng_seed in (7, (1 << 64) - 1):
            cs.cs_heavymix_select(est, k, l2 if l2sq != float(got[0]) else out, rng_seed, idx, val,
                                  n_heavy, ws)
            ref_idx, ref_heavy = orc.heavymix_select(est_h, k, l2sq, rng_seed)
            np.testing.assert_array_equal(idx.cpu().numpy(), ref_idx)
            np.testing.assert_array_equal(val.cpu().numpy(), est_h[ref_idx])
            assert int(n_heavy.item()) == ref_heavy
        if l2sq == float(got[0]) and planted and c >= 1 << 12 and k < d:
            # the heavy ones are planted coordinates: those whose square reaches l2sq / k
            heavy = ref_idx[est_h[ref_idx].astype(np.float64) ** 2 >= l2sq / k]
            assert 0 < ref_heavy == heavy.size and set(heavy.tolist()) <= set(where.tolist())
            clear = where[g[where].astype(np.float64) ** 2 >= 1.5 * l2sq / k]
            assert set(clear.tolist()) <= set(heavy.tolist())
        if l2sq == 1e12:
            assert ref_heavy == 0
    # without the optional outputs
    cs.cs_heavymix_select(est, k, out, 7, idx, None, None, ws)
    np.testing.assert_array_equal(idx.cpu().numpy(), orc.heavymix_select(est_h, k, float(got[0]), 7)[0])


# ------------------------------------------------------------------------------ 16-bit sketches
@pytest.mark.parametrize("fmt,name", [(0, "bf16"), (1, "f16")])
def test_quantize16_bit_exact_and_merge(fmt, name):
    """binary32 -> 16 bits on the device equals the reference pattern for pattern (random
    values over the whole exponent range, every special value, ties), dequantisation is exact,
    and the merge of a quantised bundle equals the reference merge of the dequantised tables."""
    rng = np.random.default_rng(fmt)
    special = np.array([0.0, -0.0, 1.0, -2.5, np.inf, -np.inf, 1 + 2.0 ** -8, 1 + 3 * 2.0 ** -8,
                        1 + 2.0 ** -11, 1 + 3 * 2.0 ** -11, 65504.0, 65520.0, 3.4e38, 2.0 ** -24,
                        2.0 ** -25, 1e-40, -1e-40, 6e-8], dtype=np.float32)
    x = np.concatenate([
        special,
        (rng.standard_normal(300_000) * 10.0 ** rng.uniform(-12, 12, 300_000)).astype(np.float32),
        rng.integers(0, 1 << 32, 300_000, dtype=np.uint64).astype(np.uint32).view(np.float32)])
    q = torch.empty(x.size, dtype=torch.int16, device=DEV)
    cs.cs_quantize16(dev(x), q, fmt)
    got = q.cpu().numpy().view(np.uint16)
    want = orc.quantize16(x, name)
    ok = ~np.isnan(x)
    np.testing.assert_array_equal(got[ok], want[ok])
    assert np.isnan(orc.dequantize16(got[~ok], name)).all()              # NaN stays NaN
    back = torch.empty(x.size, dtype=torch.float32, device=DEV)
    cs.cs_dequantize16(q, back, fmt)
    np.testing.assert_array_equal(back.cpu().numpy()[ok].astype(np.float64), orc.dequantize16(want[ok], name))

    r, c, seed, d, W = 5, 1 << 12, 11, 100_003, 13
    p = cs.cs_params_init(r, c, seed, d)
    gs = [(rng.standard_normal(d) * 0.01).astype(np.float32) for _ in range(W)]
    T = torch.zeros(cs.cs_bundle_floats(p, W), dtype=torch.float32, device=DEV)
    cs.cs_sketch_accumulate_bundle(p, T, [dev(g) for g in gs])
    T16 = torch.empty(T.numel(), dtype=torch.int16, device=DEV)
    cs.cs_quantize16(T, T16, fmt)
    G = cs.CS_BUNDLE_GROUP
    Th = T.cpu().numpy().reshape(-1, r, c, G)
    tables16 = [orc.dequantize16(orc.quantize16(Th[w // G, :, :, w % G], name), name).reshape(r, c)
                for w in range(W)]
    dst0 = rng.standard_normal((r, c)).astype(np.float32)
    dst = dev(dst0)
    cs.cs_bundle_merge16(p, dst, T16, W, fmt, alpha=1.0 / W, beta=0.25)
    assert_cells_close(dst.cpu().numpy(), orc.merge(tables16, alpha=1.0 / W, beta=0.25, dst=dst0))
    # what 16 bits cost: a value moves by at most half a unit in the last place, 2^-9 (bf16) or 2^-12 (f16) of itself
    exact = orc.merge([Th[w // G, :, :, w % G] for w in range(W)], alpha=1.0 / W)
    cs.cs_bundle_merge16(p, dst, T16, W, fmt, alpha=1.0 / W, beta=0.0)
    err = np.abs(dst.cpu().numpy() - exact).max() / np.abs(exact).max()
    assert err < (2.0 ** -8 if fmt == 0 else 2.0 ** -11)


@pytest.mark.parametrize("W,d,offset", [(1, 1, 0), (3, 1_000_003, 0), (2, 4096, 1), (40, 70_001, 0)])
def test_probe_stream_read_adds_up_everything_it_reads(W, d, offset):
    """The measurement aid reads every element exactly once: its sum equals the exact sum."""
    rng = np.random.default_rng(d)
    xs = [rng.integers(-8, 9, size=d + offset).astype(np.float32) for _ in range(W)]   # exact in fp32
    vecs = [dev(x)[offset:] for x in xs]                  # offset 1: not 16-byte aligned
    out = torch.full((1,), 3.0, dtype=torch.float32, device=DEV)
    cs.cs_probe_stream_read(vecs, out)
    assert out.item() == 3.0 + sum(float(x[offset:].astype(np.float64).sum()) for x in xs)
