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
import numpy as np

REL = 1e-5


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


def assert_values_close(gpu, ref, scale, rel=REL, what="values"):
    gpu = np.asarray(gpu, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert gpu.shape == ref.shape
    bound = rel * np.maximum(np.abs(ref), scale)
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
