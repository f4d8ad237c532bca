"""The path on a vector of more than 2^32 coordinates (17 GB of fp32): every index, offset and
count inside the kernels has to be 64 bits wide, and nothing at the sizes of the benchmark
configurations (d <= 10^8) would notice if one were not.

The reference cannot sketch 4.3 G coordinates in a test's time, so the vector is zero except for
three dense windows of noise (the start, around 2^31, from below 2^32 to the ragged end) and 30 000
planted heavy coordinates spread over the whole range: the reference sketches exactly the
non-zero part (zeros add nothing to any cell), while the device walks all 4.3 G coordinates.
A coordinate whose index were truncated to 32 bits anywhere would land in the wrong cell, read
the wrong estimate or come out of the selection with the wrong index."""
import numpy as np
import pytest
import torch

from oracle import cs_oracle as orc
from paper_1903_04488_amd import binding as B
from paper_1903_04488_amd.pipeline import HotPath
from parity_util import assert_cells_close, estimate_sparse_in_slices

pytestmark = pytest.mark.gpu
DEV = "cuda:0"

D = (1 << 32) + (1 << 20) + 77
HALF = 1 << 21
WINDOWS = [(0, 1 << 22), ((1 << 31) - HALF, (1 << 31) + HALF), ((1 << 32) - HALF, D)]
EDGES = np.array([0, (1 << 31) - 1, 1 << 31, (1 << 31) + 1, (1 << 32) - 1, 1 << 32, (1 << 32) + 1, D - 1],
                 dtype=np.int64)


def in_a_window(idx):
    inside = np.zeros(idx.shape, dtype=bool)
    for lo, hi in WINDOWS:
        inside |= (idx >= lo) & (idx < hi)
    return inside


def test_vector_of_more_than_two_to_the_32_coordinates(progress):
    r, c, k, seed = 5, 1 << 20, 20_000, 20260101
    torch.cuda.empty_cache()          # blocks that earlier tests left in torch's cache count as used
    free, _ = torch.cuda.mem_get_info()
    if free < 130 * (1 << 30):
        pytest.skip("needs 130 GB of free device memory")
    rng = np.random.default_rng(seed)
    gen = torch.Generator(device=DEV)
    gen.manual_seed(seed)
    g = torch.zeros(D, dtype=torch.float32, device=DEV)
    for lo, hi in WINDOWS:
        g[lo:hi] = 0.01 * torch.randn(hi - lo, generator=gen, device=DEV)
    planted = np.unique(np.concatenate([rng.integers(0, D, 30_000), EDGES]))
    val = (rng.uniform(0.5, 1.0, planted.size) * rng.choice([-1.0, 1.0], planted.size)).astype(np.float32)
    val[np.isin(planted, EDGES)] = np.float32(2.0) * np.sign(val[np.isin(planted, EDGES)])
    g[torch.from_numpy(planted).to(DEV)] = torch.from_numpy(val).to(DEV)
    progress(f"[d = 2^32 + {D - (1 << 32)}] input on the device")

    # ---- reference: the sketch of the non-zero part
    sk = orc.SketchOracle(r, c, seed)
    T = sk.zeros()
    for lo, hi in WINDOWS:
        part = g[lo:hi].cpu().numpy()
        for s in range(0, hi - lo, 1 << 20):             # i0 of every slice given explicitly
            T += sk.sketch(part[s:s + (1 << 20)], i0=lo + s)
    outside = ~in_a_window(planted)
    sk.accumulate_sparse(T, planted[outside], val[outside].astype(np.float64))
    progress("reference table done")

    # ---- device: update, merge
    hp = HotPath(D, 1, r, c, k, seed, device=DEV)
    progress("traversal plan and buffers done")
    hp.accumulate([g])
    hp.merge()
    torch.cuda.synchronize()
    assert_cells_close(hp.worker_table(0).cpu().numpy(), T, what="worker table")
    assert_cells_close(hp.S_t.cpu().numpy(), T, what="merged table")
    progress("tables agree")

    # ---- query every coordinate; sampled comparison, bit for bit from the device's own table
    hp.estimate()
    hp.topk()
    torch.cuda.synchronize()
    table32 = hp.S_t.cpu().numpy()
    sample = np.unique(np.concatenate(
        [planted, rng.integers(0, D, 1_000_000)] +
        [np.arange(lo, lo + 4096) for lo, _ in WINDOWS] + [np.arange(hi - 4096, hi) for _, hi in WINDOWS] +
        [np.arange((1 << 32) - 70_000, (1 << 32) + 70_000)]))
    got = hp.est[torch.from_numpy(sample).to(DEV)].cpu().numpy()
    want = estimate_sparse_in_slices(sk, table32.astype(np.float64), sample).astype(np.float32)
    np.testing.assert_array_equal(got.view(np.uint32), want.view(np.uint32))
    progress(f"{sample.size} sampled estimates are the reference's, bit for bit")

    # ---- selection: properties that define it, checked over all of est on the host
    idx = hp.idx.cpu().numpy()
    at_idx = hp.est_at_idx.cpu().numpy()
    assert idx.shape == (k,) and (np.diff(idx) > 0).all() and idx[0] >= 0 and idx[-1] < D
    np.testing.assert_array_equal(at_idx.view(np.uint32),
                                  hp.est[hp.idx].cpu().numpy().view(np.uint32))
    theta = np.abs(at_idx).min()
    n_gt = n_ge = 0
    ties = []
    stage = torch.empty(1 << 28, dtype=torch.float32, pin_memory=True)
    for lo in range(0, D, 1 << 28):
        hi = min(lo + (1 << 28), D)
        stage[:hi - lo].copy_(hp.est[lo:hi])
        mag = np.abs(stage[:hi - lo].numpy())
        n_gt += int((mag > theta).sum())
        n_ge += int((mag >= theta).sum())
        ties.append(lo + np.flatnonzero(mag == theta))
    ties = np.concatenate(ties)
    assert n_gt < k <= n_ge, (n_gt, n_ge, k)
    assert int((np.abs(at_idx) > theta).sum()) == n_gt            # every larger one is selected
    chosen_ties = idx[np.abs(at_idx) == theta]
    np.testing.assert_array_equal(chosen_ties, ties[:chosen_ties.size])   # equal magnitudes: lowest index first
    assert np.isin(EDGES, idx).all()                                 # magnitude 2: always selected
    # (not every selected coordinate is a planted one: with 30 000 heavy coordinates in 2^20 columns
    # a zero coordinate shares three of its five cells with heavy ones with probability 2e-4, a
    # million such coordinates among 4.3 G -- the sketch's own error, the same in the reference)
    progress("selection is the k largest, lowest index among equals")

    # ---- second round: exact values at the selected coordinates
    hp.gather([g])
    np.testing.assert_array_equal(hp.x.cpu().numpy().view(np.uint32), g[hp.idx].cpu().numpy().view(np.uint32))
    # hash parity hook across the 2^32 boundary
    n = 4096
    i0 = (1 << 32) - n // 2
    bucket = torch.empty(r, n, dtype=torch.int32, device=DEV)
    sign = torch.empty(r, n, dtype=torch.int8, device=DEV)
    B.cs_hash_debug_range(hp.params, i0, n, bucket, sign)
    ref_b, ref_s = sk.hash(np.arange(i0, i0 + n))
    np.testing.assert_array_equal(bucket.cpu().numpy().view(np.uint32), ref_b)
    np.testing.assert_array_equal(sign.cpu().numpy(), ref_s)
