"""Tolerance rules shared by the GPU parity tests (fp32 device results vs the fp64 reference).

Cells and estimates: |gpu - ref| <= 1e-5 * max(|ref|, sigma), sigma = RMS of the reference row
(cells) or of the whole table (estimates).  A cell is a signed sum of ~d/c terms that may
cancel to nearly zero, so a purely relative bound has no meaning there; sigma is the natural
scale of one cell.  1e-5 is the tolerance the benchmark definition states (fp32 accumulation
of <= a few hundred terms in arbitrary order has relative error ~ sqrt(n) * 6e-8 of that scale).

Index sets: with theta = k-th largest reference magnitude and eps = 2e-5 * max(theta, sigma),
a device set is valid iff it has k distinct indices, contains every i with |est_i| > theta + eps
and contains no i with |est_i| < theta - eps ("equal outside near-ties").
"""
import os
from concurrent.futures import ThreadPoolExecutor

import numpy as np

REL = 1e-5

# The reference's loops are single-threaded by design.  For vectors of 10^7 .. 10^8 coordinates
# the tests call them on slices of the coordinate range from several threads (the C loops run
# without the interpreter lock) and combine the pieces: tables add up (linearity of the sketch,
# which the reference's own pins establish), estimates concatenate.  The reference's code is
# the same; only the caller splits the range.
_POOL = ThreadPoolExecutor(max_workers=max(1, min(16, os.cpu_count() or 1)))
_SLICE = 1 << 22


def _slices(d):
    return [(lo, min(lo + _SLICE, d)) for lo in range(0, d, _SLICE)]


def sketch_in_slices(sk, g, scale=1.0):
    """sk.sketch(g, scale=scale), the coordinate range cut into slices"""
    g = np.ascontiguousarray(g)
    if g.size <= _SLICE:
        return sk.sketch(g, scale=scale)
    parts = list(_POOL.map(lambda s: sk.sketch(g[s[0]:s[1]], i0=s[0], scale=scale), _slices(g.size)))
    T = sk.zeros()
    for part in parts:
        T += part
    return T


def estimate_in_slices(sk, T, d):
    """sk.estimate(T, d), the coordinate range cut into slices"""
    if d <= _SLICE:
        return sk.estimate(T, d)
    parts = list(_POOL.map(lambda s: sk.estimate(T, s[1] - s[0], i0=s[0]), _slices(d)))
    return np.concatenate(parts)


def estimate_sparse_in_slices(sk, T, idx):
    idx = np.ascontiguousarray(idx, dtype=np.int64)
    if idx.size <= (1 << 16):
        return sk.estimate_sparse(T, idx)
    cuts = np.linspace(0, idx.size, 33).astype(np.int64)
    parts = list(_POOL.map(lambda q: sk.estimate_sparse(T, idx[cuts[q]:cuts[q + 1]]), range(32)))
    return np.concatenate(parts)


def host_sum_f64(g_w):
    """sum over workers of their fp32 vectors, in binary64 on the host (worker by worker; the
    additions of one worker are spread over threads by coordinate range; device vectors come
    over through a pinned staging buffer)"""
    import torch
    d = g_w[0].numel()
    acc = np.zeros(d, dtype=np.float64)
    sl = _slices(d)
    stage = torch.empty(d, dtype=torch.float32, pin_memory=True) if g_w[0].is_cuda else None

    def add(s, h):
        acc[s[0]:s[1]] += h[s[0]:s[1]]

    for g in g_w:
        if stage is not None:
            stage.copy_(g)                     # synchronous device-to-host copy
            h = stage.numpy()
        else:
            h = g.numpy()
        if d <= _SLICE:
            acc += h
        else:
            list(_POOL.map(lambda s: add(s, h), sl))
    return acc


def table_rms_rows(T):
    return np.sqrt((np.asarray(T, dtype=np.float64) ** 2).mean(axis=1))


def assert_cells_close(gpu, ref, rel=REL, what="cells", terms_per_cell=0.0, operand_mag=None):
    """terms_per_cell: how many fp32 values were summed into one cell (d / c).  The benchmark
    configurations have at most ~100; the bound is widened by sqrt(terms / 256) beyond that,
    the growth of random-order fp32 summation error (only degenerate shapes such as c = 1).
    operand_mag: per-cell magnitude of the operands the cell was computed from, for cells that
    are the result of a cancellation (error feedback subtracts heavy values from the cell that
    held them, and two heavy values of opposite sign can share a cell: fp32 error is relative
    to what was added and subtracted, not to what is left)."""
    gpu = np.asarray(gpu, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert gpu.shape == ref.shape
    rel = rel * max(1.0, float(np.sqrt(terms_per_cell / 256.0)))
    sigma = table_rms_rows(ref)[:, None]
    mag = np.abs(ref) if operand_mag is None else np.maximum(np.abs(ref), np.abs(operand_mag))
    bound = rel * np.maximum(mag, sigma)
    err = np.abs(gpu - ref)
    worst = (err / np.maximum(bound, 1e-300)).max() if err.size else 0.0
    assert worst <= 1.0, f"{what}: worst error is {worst:.3g} x the allowed bound"
    return worst


def cancelled_cells(mag, table):
    """Cells of a state table whose value is what a cancellation left over: the largest operand
    that went through the cell (mag) is at least twice what the cell holds now (or the row's
    RMS).  Returns mag there and 0 elsewhere.  An estimate is one of the r cells it reads, so
    an estimate that reads such a cell carries that cell's fp32 error, which is relative to
    the operands (see assert_cells_close)."""
    table = np.abs(np.asarray(table, dtype=np.float64))
    floor = np.maximum(table, table_rms_rows(table)[:, None])
    return np.where(mag > 2.0 * floor, mag, 0.0)


def operand_scale_at(sk, cancelled, idx):
    """per listed coordinate: the largest entry of `cancelled` among the r cells it reads"""
    bkt, _ = sk.hash(np.ascontiguousarray(idx, dtype=np.int64))
    rows = np.arange(bkt.shape[0])[:, None]
    return cancelled[rows, bkt.astype(np.int64)].max(axis=0)


def operand_scale_all(sk, cancelled, d):
    """the same for every coordinate 0 .. d-1 (the reference's per-row query of the table of
    operand magnitudes, sign dropped, maximum over rows)"""
    cancelled = np.ascontiguousarray(cancelled, dtype=np.float64)
    if not cancelled.any():
        return np.zeros(d)

    def one(s):
        return np.abs(sk.row_estimates(cancelled, s[1] - s[0], i0=s[0])).max(axis=0)

    return np.concatenate(list(_POOL.map(one, _slices(d))))


def assert_values_close(gpu, ref, scale, rel=REL, what="values", operand_mag=None):
    """operand_mag: optional per-element magnitude of the operands behind a value that a
    cancellation left over (see cancelled_cells); the bound is relative to it where given."""
    gpu = np.asarray(gpu, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert gpu.shape == ref.shape
    mag = np.abs(ref) if operand_mag is None else np.maximum(np.abs(ref), operand_mag)
    bound = rel * np.maximum(mag, scale)
    err = np.abs(gpu - ref)
    worst = (err / np.maximum(bound, 1e-300)).max() if err.size else 0.0
    assert worst <= 1.0, f"{what}: worst error is {worst:.3g} x the allowed bound"
    return worst


def assert_valid_topk(gpu_idx, ref_est, k, sigma, what="top-k"):
    """Returns the number of indices in which the device set differs from the reference's own
    selection (0 when there is no near-tie at the threshold)."""
    gpu_idx = np.asarray(gpu_idx, dtype=np.int64)
    mag = np.abs(np.asarray(ref_est, dtype=np.float64))
    assert gpu_idx.shape == (k,), f"{what}: wrong length"
    assert (np.diff(gpu_idx) > 0).all(), f"{what}: not strictly ascending"
    assert gpu_idx.min() >= 0 and gpu_idx.max() < mag.size
    theta = np.partition(mag, mag.size - k)[mag.size - k]
    eps = 2e-5 * max(theta, sigma)
    chosen = np.zeros(mag.size, dtype=bool)
    chosen[gpu_idx] = True
    must = mag > theta + eps
    never = mag < theta - eps
    assert not (must & ~chosen).any(), f"{what}: misses {int((must & ~chosen).sum())} clear heavy hitters"
    assert not (never & chosen).any(), f"{what}: selects {int((never & chosen).sum())} clearly light coordinates"
    ref_sel = (mag > theta)
    return int((chosen & ~ref_sel & (mag != theta)).sum())
