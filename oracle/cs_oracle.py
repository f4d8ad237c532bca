"""Count Sketch / Sketched-SGD reference ("oracle") -- TEST INFRASTRUCTURE, NOT THE PRODUCT.

Plain, slow, single-threaded CPU code in fp64 that computes what the data-parallel
hot path of Sketched-SGD computes, step by step, in the paper's order and notation:

    Alg. 4 (App. C)   init / update / estimate of a Count Sketch
    Sec. 3, App. C    mergeability: S(g1) + S(g2) = S(g1 + g2)
    Alg. 3 (Sec. 5.1) worker sketches -> (1/W) sum -> recover top-k -> second round of
                      exact values; momentum u <- m u + g and error accumulation v <- v + u,
                      here held as their sketches (linear images), see SketchSpaceState
    Sec. 5.2          every coordinate is queried and the largest estimates are chosen
    Alg. 1 (Sec. 4)   HEAVYMIX: l2 estimate from the sketch, threshold split, random fill

Only tests, the smoke check and the benchmark's cpu_baseline leg may import this module.
It imports nothing from the HIP package and the HIP package imports nothing from here.
The inner loops live in cs_oracle.c (compiled with gcc); everything that has a textbook
routine (sort, sum, fancy indexing) is written with numpy.

Every function here is pinned by tests/test_oracle_pins.py to something other than
itself (dense-matrix product on tiny inputs, linearity, closed-form row variance, AMS
special case, planted-sparse recovery, numpy's stable argsort, a dense-state twin of the
sketch-space state; for HEAVYMIX: the exact norm of sparse vectors, the paper's (1 +- 0.5)
band, a brute-force split, the uniformity of the fill and the k/d contraction of Lemma 1).
Nothing in this file is "parity unpinned"; the one free choice
(the value fed back in sketch space, SketchSpaceState.feedback) is a documented reading,
pinned internally by the dense-state twin.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "cs_oracle.c")
_LIB = os.path.join(_HERE, "libcs_oracle.so")

P61 = (1 << 61) - 1
MAX_R = 64


def build(force: bool = False) -> str:
    """Compile cs_oracle.c with gcc into libcs_oracle.so (next to this file)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-Wall", "-Wextra", "-shared", "-fPIC", "-o", _LIB, _SRC]
        )
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
    return _lib


def _p(arr, ctype):
    return arr.ctypes.data_as(ctypes.POINTER(ctype))


def splitmix64(seed: int, n: int) -> np.ndarray:
    out = np.zeros(n, dtype=np.uint64)
    _load().cso_splitmix64(ctypes.c_uint64(seed), ctypes.c_int(n), _p(out, ctypes.c_uint64))
    return out


class SketchOracle:
    """Count Sketch with r rows and c columns (Alg. 4), fp64 counters, 0-based indices."""

    def __init__(self, r: int, c: int, seed: int):
        if not (1 <= r <= MAX_R) or r % 2 == 0:
            raise ValueError("r must be odd and in [1, 64] (the median of Alg. 4 needs a middle)")
        if not (1 <= c < (1 << 32)):
            raise ValueError("c must be in [1, 2^32)")
        self.r, self.c, self.seed = int(r), int(c), int(seed)
        self.a = np.zeros(r, dtype=np.uint64)
        self.b = np.zeros(r, dtype=np.uint64)
        self.as_ = np.zeros(r, dtype=np.uint64)
        self.bs = np.zeros(r, dtype=np.uint64)
        _load().cso_derive_params(
            ctypes.c_uint64(self.seed), ctypes.c_int(r),
            _p(self.a, ctypes.c_uint64), _p(self.b, ctypes.c_uint64),
            _p(self.as_, ctypes.c_uint64), _p(self.bs, ctypes.c_uint64))

    # -- plumbing ---------------------------------------------------------
    def _hp(self):
        return (ctypes.c_int(self.r), ctypes.c_uint32(self.c),
                _p(self.a, ctypes.c_uint64), _p(self.b, ctypes.c_uint64),
                _p(self.as_, ctypes.c_uint64), _p(self.bs, ctypes.c_uint64))

    def zeros(self) -> np.ndarray:
        """Alg. 4 init: the r x c table of counters, all zero."""
        return np.zeros((self.r, self.c), dtype=np.float64)

    def _check_table(self, T):
        assert T.dtype == np.float64 and T.shape == (self.r, self.c) and T.flags.c_contiguous

    # -- hashes -----------------------------------------------------------
    def hash(self, idx):
        """bucket[j, t] = h_j(idx[t]) (uint32), sign[j, t] = s_j(idx[t]) (int8, +1/-1)."""
        idx = np.ascontiguousarray(idx, dtype=np.int64)
        n = idx.size
        bucket = np.zeros((self.r, n), dtype=np.uint32)
        sign = np.zeros((self.r, n), dtype=np.int8)
        _load().cso_hash(*self._hp(), _p(idx, ctypes.c_int64), ctypes.c_int64(n),
                         _p(bucket, ctypes.c_uint32), _p(sign, ctypes.c_int8))
        return bucket, sign

    # -- update -----------------------------------------------------------
    def accumulate(self, T, g, i0: int = 0, scale: float = 1.0):
        """T[j, h_j(i0+t)] += scale * s_j(i0+t) * g[t] for every t, j (Alg. 4 update)."""
        self._check_table(T)
        g = np.ascontiguousarray(g)
        if g.dtype == np.float32:
            fn, ct = _load().cso_accumulate_f32, ctypes.c_float
        elif g.dtype == np.float64:
            fn, ct = _load().cso_accumulate_f64, ctypes.c_double
        else:
            raise TypeError("g must be float32 or float64")
        fn(*self._hp(), _p(T, ctypes.c_double), _p(g, ct), ctypes.c_int64(g.size),
           ctypes.c_int64(i0), ctypes.c_double(scale))
        return T

    def accumulate_sparse(self, T, idx, val, scale: float = 1.0):
        self._check_table(T)
        idx = np.ascontiguousarray(idx, dtype=np.int64)
        val = np.ascontiguousarray(val, dtype=np.float64)
        assert idx.size == val.size
        _load().cso_accumulate_sparse(*self._hp(), _p(T, ctypes.c_double),
                                      _p(idx, ctypes.c_int64), _p(val, ctypes.c_double),
                                      ctypes.c_int64(idx.size), ctypes.c_double(scale))
        return T

    def sketch(self, g, i0: int = 0, scale: float = 1.0):
        return self.accumulate(self.zeros(), g, i0, scale)

    # -- update with order-independent sums -------------------------------
    # Not in the paper: the same update of Alg. 4 with every contribution rounded once to a
    # multiple of 2^-frac_bits and summed as a 64-bit integer, so that the result does not
    # depend on the order of the additions and a float implementation's "reordered" can be
    # told from "wrong".  Pinned by exact rational arithmetic on small inputs and by the
    # fp64 update above on inputs that are multiples of 2^-frac_bits (tests/test_oracle_pins.py).
    @staticmethod
    def fixed_contributions(val, scale: float, frac_bits: int):
        """(q, ok): q[t] = scale * val[t] * 2^frac_bits rounded to an integer, ties to even (the
        product of two binary32 numbers and a power of two is exact in fp64); ok[t] is False,
        and q[t] = 0, where that value is not finite or not below 2^62 in magnitude."""
        val = np.asarray(val, dtype=np.float32).astype(np.float64)
        with np.errstate(invalid="ignore", over="ignore"):
            x = val * np.float64(np.float32(scale)) * np.float64(2.0) ** int(frac_bits)
            ok = np.abs(x) < 2.0 ** 62
        q = np.zeros(val.shape, dtype=np.int64)
        q[ok] = np.rint(x[ok]).astype(np.int64)
        return q, ok

    def accumulate_fixed(self, acc, g, frac_bits: int, i0: int = 0, scale: float = 1.0) -> int:
        """acc[j, h_j(i0+t)] += s_j(i0+t) * q[t] in int64; returns the number of coordinates left out."""
        g = np.asarray(g)
        idx = np.arange(i0, i0 + g.size, dtype=np.int64)
        return self.accumulate_fixed_sparse(acc, idx, g, frac_bits, scale)

    def accumulate_fixed_sparse(self, acc, idx, val, frac_bits: int, scale: float = 1.0) -> int:
        assert acc.dtype == np.int64 and acc.shape == (self.r, self.c)
        idx = np.ascontiguousarray(idx, dtype=np.int64)
        q, ok = self.fixed_contributions(val, scale, frac_bits)
        step = 1 << 20
        for t0 in range(0, idx.size, step):
            bucket, sign = self.hash(idx[t0:t0 + step])
            for j in range(self.r):
                np.add.at(acc[j], bucket[j], sign[j].astype(np.int64) * q[t0:t0 + step])
        return int(idx.size - np.count_nonzero(ok))

    def fixed_to_float(self, acc, frac_bits: int, alpha: float = 1.0) -> np.ndarray:
        """float32( float64(acc) * 2^-frac_bits * float64(alpha) ), one rounding per step."""
        cells = acc.astype(np.float64) * np.float64(2.0) ** (-int(frac_bits))
        return (cells * np.float64(np.float32(alpha))).astype(np.float32)

    # -- query ------------------------------------------------------------
    def estimate(self, T, d: int, i0: int = 0) -> np.ndarray:
        """est[t] = median_j s_j(i0+t) * T[j, h_j(i0+t)] for t in [0, d) (Alg. 4 estimate)."""
        self._check_table(T)
        est = np.zeros(d, dtype=np.float64)
        _load().cso_estimate(*self._hp(), _p(T, ctypes.c_double), ctypes.c_int64(d),
                             ctypes.c_int64(i0), _p(est, ctypes.c_double))
        return est

    def estimate_sparse(self, T, idx) -> np.ndarray:
        self._check_table(T)
        idx = np.ascontiguousarray(idx, dtype=np.int64)
        out = np.zeros(idx.size, dtype=np.float64)
        _load().cso_estimate_sparse(*self._hp(), _p(T, ctypes.c_double),
                                    _p(idx, ctypes.c_int64), ctypes.c_int64(idx.size),
                                    _p(out, ctypes.c_double))
        return out

    def row_estimates(self, T, d: int, i0: int = 0) -> np.ndarray:
        """rows[j, t] = s_j(i0+t) * T[j, h_j(i0+t)]: the r values whose median is the estimate."""
        self._check_table(T)
        rows = np.zeros((self.r, d), dtype=np.float64)
        _load().cso_row_estimates(*self._hp(), _p(T, ctypes.c_double), ctypes.c_int64(d),
                                  ctypes.c_int64(i0), _p(rows, ctypes.c_double))
        return rows


# ---------------------------------------------------------------------------
# parameter-server side: merge, selection, second round
# ---------------------------------------------------------------------------
def merge(tables, alpha: float = 1.0, beta: float = 0.0, dst=None) -> np.ndarray:
    """beta * dst + alpha * sum_w tables[w]  (Alg. 3: S_t = (1/W) sum_i S_t^i, alpha = 1/W)."""
    acc = np.zeros_like(np.asarray(tables[0], dtype=np.float64))
    for T in tables:
        acc = acc + np.asarray(T, dtype=np.float64)
    out = alpha * acc
    if dst is not None and beta != 0.0:
        out = out + beta * np.asarray(dst, dtype=np.float64)
    return out


def topk(est, k: int) -> np.ndarray:
    """Indices of the k entries of largest magnitude (Sec. 4 selects gradient elements
    by magnitude; Sec. 5.2), equal magnitudes resolved towards the lower index, returned in
    ascending index order.  Written as the definition: stable sort by descending |est|."""
    mag = np.abs(np.asarray(est, dtype=np.float64))
    order = np.argsort(-mag, kind="stable")
    return np.sort(order[:k]).astype(np.int64)


def topk_threshold(est, k: int) -> np.ndarray:
    """Same result as topk() without the full sort (for d ~ 1e8): theta = k-th largest
    magnitude; everything above theta, then the lowest-index entries equal to theta."""
    mag = np.abs(np.asarray(est, dtype=np.float64))
    d = mag.size
    theta = np.partition(mag, d - k)[d - k]
    above = np.flatnonzero(mag > theta)
    ties = np.flatnonzero(mag == theta)[: k - above.size]
    return np.sort(np.concatenate([above, ties])).astype(np.int64)


def gather_exact(vecs, idx, alpha: float = 1.0) -> np.ndarray:
    """Second round (Alg. 1 step 5, the worker-query step of Alg. 3, which keeps
    the sum): alpha * sum_w vecs[w][idx]."""
    idx = np.asarray(idx, dtype=np.int64)
    acc = np.zeros(idx.size, dtype=np.float64)
    for v in vecs:
        acc = acc + np.asarray(v)[idx].astype(np.float64)
    return alpha * acc


def select_exact_topk(cand, x, k: int):
    """Alg. 3 with P > 1 (Sec. 5.1): of the Pk candidates `cand` (ascending) with exact summed
    values `x`, keep the k of largest |x| (ties -> lower index); returns (indices ascending,
    their exact values)."""
    cand = np.asarray(cand, dtype=np.int64)
    pos = topk(np.asarray(x, dtype=np.float64), k)
    return cand[pos], np.asarray(x, dtype=np.float64)[pos]


# ---------------------------------------------------------------------------
# HEAVYMIX (Alg. 1): threshold split and random fill
# ---------------------------------------------------------------------------
def l2sq_estimate(T):
    """Alg. 1 step 1 (the squared l2 norm read off the sketch), by the AMS argument of App. C: a row's
    counters are signed sums over disjoint sets of coordinates, so the sum of their squares
    has expectation ||g||^2; the median over the r rows controls the failure probability.
    Returns (median over rows, the r row sums)."""
    rows = (np.asarray(T, dtype=np.float64) ** 2).sum(axis=1)
    return float(np.sort(rows)[rows.size // 2]), rows


def heavymix_fill_keys(rng_seed: int, d: int) -> np.ndarray:
    """The random order behind rand_l(NH) (Alg. 1 step 4): coordinate i gets the 30 top bits
    of the (i+1)-th output of the SplitMix64 generator started at rng_seed; the l non-heavy
    coordinates with the largest keys are drawn (equal keys: lower index first).  Keys of
    distinct coordinates are independent uniform draws, so this is a uniform sample without
    replacement up to the (2^-30) chance of equal keys.  SplitMix64 is written out here with
    numpy's wrapping uint64 arithmetic."""
    with np.errstate(over="ignore"):
        z = np.uint64(rng_seed) + np.arange(1, d + 1, dtype=np.uint64) * np.uint64(0x9E3779B97F4A7C15)
        z = (z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)
        z = (z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)
        z = z ^ (z >> np.uint64(31))
    return (z >> np.uint64(34)).astype(np.uint32)


def heavymix_select(est, k: int, l2sq: float, rng_seed: int):
    """Alg. 1 steps 3-4.  H = { i : est_i^2 >= l2sq / k } (the listing's comparison of est_i
    itself with l2sq / k is read as the squared form that Sec. 4's proof and Def. 2 of App. C
    use); the selection is H plus l = k - |H| coordinates drawn uniformly at random from the
    others.  The estimates are taken in binary32 (what the sketch query returns), their
    squares and the threshold in binary64.  The proof's "|H| <= k" holds for exact values
    only; if more than k estimates pass, the k largest of them are kept, ordered by the top
    30 bits of the binary32 magnitude, equal ones by lower index.
    Returns (k indices ascending, number of heavy coordinates among them)."""
    est32 = np.ascontiguousarray(est, dtype=np.float32)
    d = est32.size
    theta = np.float64(l2sq) / np.float64(k)
    heavy = est32.astype(np.float64) ** 2 >= theta
    H = np.flatnonzero(heavy)
    if H.size >= k:
        key = ((est32.view(np.uint32)[H] & np.uint32(0x7FFFFFFF)) >> np.uint32(1)).astype(np.int64)
        keep = H[np.argsort(-key, kind="stable")[:k]]
        return np.sort(keep).astype(np.int64), k
    NH = np.flatnonzero(~heavy)
    key = heavymix_fill_keys(rng_seed, d)[NH].astype(np.int64)
    fill = NH[np.argsort(-key, kind="stable")[: k - H.size]]
    return np.sort(np.concatenate([H, fill])).astype(np.int64), int(H.size)


# ---------------------------------------------------------------------------
# 16-bit sketches (Sec. 6 remarks that sketch cells can be quantised to 16 bits)
# ---------------------------------------------------------------------------
def quantize16(x, fmt: str) -> np.ndarray:
    """binary32 -> 16-bit storage, round to nearest, ties to even; returns the uint16 patterns.
    fmt "bf16": the upper half of the binary32 pattern (8 exponent bits, 7 fraction bits);
    fmt "f16": IEEE binary16 (numpy's conversion).  NaN stays NaN (quiet), overflow gives inf."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    if fmt == "f16":
        with np.errstate(over="ignore"):
            return x.astype(np.float16).view(np.uint16)
    if fmt != "bf16":
        raise ValueError(fmt)
    bits = x.view(np.uint32).astype(np.uint64)
    lower, keep = bits & np.uint64(0xFFFF), bits >> np.uint64(16)
    up = (lower > np.uint64(0x8000)) | ((lower == np.uint64(0x8000)) & ((keep & np.uint64(1)) == 1))
    out = (keep + up.astype(np.uint64)).astype(np.uint16)
    nan = np.isnan(x)
    out[nan] = ((bits[nan] >> np.uint64(16)) | np.uint64(0x0040)).astype(np.uint16)
    return out


def dequantize16(q, fmt: str) -> np.ndarray:
    """the binary64 value of every 16-bit pattern (exact)"""
    q = np.ascontiguousarray(q, dtype=np.uint16)
    if fmt == "f16":
        return q.view(np.float16).astype(np.float64)
    if fmt != "bf16":
        raise ValueError(fmt)
    return (q.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


def compression_factor(d: int, sketch_cells: int, P: int, k: int) -> float:
    """Sec. 5.3: 2d / (|S| + Pk + k)."""
    return 2.0 * d / (sketch_cells + P * k + k)


# ---------------------------------------------------------------------------
# momentum and error feedback (Alg. 3), two forms
# ---------------------------------------------------------------------------
class DenseState:
    """Alg. 3 with the W workers' u^i, v^i replaced by their means (every update of u, v is
    linear and identical on all workers, so the mean obeys the same recursion):
        u <- m u + gbar ;  v <- v + u ;  select idx from the sketch of v ;
        then subtract the fed-back values at idx.
    Exists to pin SketchSpaceState through S(v) == S_v, S(u) == S_u (linearity)."""

    def __init__(self, d: int, rho: float):
        self.u = np.zeros(d, dtype=np.float64)
        self.v = np.zeros(d, dtype=np.float64)
        self.rho = float(rho)

    def momentum(self, gbar):
        self.u = self.rho * self.u + np.asarray(gbar, dtype=np.float64)
        self.v = self.v + self.u

    def feedback(self, idx, delta_v, delta_u):
        self.v[idx] -= delta_v
        self.u[idx] -= delta_u


class DenseWorkerState:
    """Alg. 3 as printed: every worker i keeps its own dense u^i, v^i.
        u^i <- m u^i + g^i ;  v^i <- v^i + u^i ;  the sketch of v^i goes to the server ;
        the server asks for exact values of v^i at the chosen coordinates and sums them ;
        u^i, v^i <- 0 at the coordinates of the update.
    m is the fp32 value of the momentum constant, as the device receives it."""

    def __init__(self, W: int, d: int, rho: float):
        self.u = [np.zeros(d, dtype=np.float64) for _ in range(W)]
        self.v = [np.zeros(d, dtype=np.float64) for _ in range(W)]
        self.rho = float(np.float32(rho))

    def momentum(self, g_w):
        for i, g in enumerate(g_w):
            self.u[i] = self.rho * self.u[i] + np.asarray(g, dtype=np.float64)
            self.v[i] = self.v[i] + self.u[i]

    def mean_v(self):
        acc = np.zeros_like(self.v[0])
        for v in self.v:
            acc = acc + v
        return acc / len(self.v)

    def exact(self, idx):
        """second round: (1/W) sum_i v^i[idx]"""
        return gather_exact(self.v, idx, alpha=1.0 / len(self.v))

    def mask(self, idx):
        for i in range(len(self.v)):
            self.u[i][idx] = 0.0
            self.v[i][idx] = 0.0


class SketchSpaceState:
    """Momentum and error accumulation of Alg. 3 kept as sketches S_u = S(u), S_v = S(v).

    Reading (the paper keeps u, v dense on each worker; the benchmark definition asks for
    them "in sketch space"): by linearity of S,
        S_u <- rho S_u + S_t          (image of  u <- m u + g)
        S_v <- S_v + S_u              (image of  v <- v + u)
        est = estimate(S_v) ; idx = top-k |est|
        Delta = est[idx]      ; S_v <- S_v - S(Delta at idx)     (error feedback: what was
                                                                  applied leaves the residual)
        uhat = estimate(S_u, idx) ; S_u <- S_u - S(uhat at idx)  (momentum factor masking:
                                                                  zero u, v on updated coords,
                                                                  as far as a sketch can say)
    rho is the fp32 value of the momentum constant, as the device receives it."""

    def __init__(self, sk: SketchOracle, rho: float):
        self.sk = sk
        self.rho = float(np.float32(rho))
        self.S_u = sk.zeros()
        self.S_v = sk.zeros()

    def momentum(self, S_t):
        self.S_u = self.rho * self.S_u + S_t
        self.S_v = self.S_v + self.S_u

    def select(self, d: int, k: int, big: bool = False):
        est = self.sk.estimate(self.S_v, d)
        idx = topk_threshold(est, k) if big else topk(est, k)
        return est, idx

    def feedback(self, idx):
        """Returns (Delta, uhat) and removes their sketches from S_v, S_u."""
        delta = self.sk.estimate_sparse(self.S_v, idx)
        uhat = self.sk.estimate_sparse(self.S_u, idx)
        self.sk.accumulate_sparse(self.S_v, idx, delta, scale=-1.0)
        self.sk.accumulate_sparse(self.S_u, idx, uhat, scale=-1.0)
        return delta, uhat
