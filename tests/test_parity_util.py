"""The helpers that call the reference on slices of the coordinate range from several threads
(tests/parity_util.py) return what the reference returns in one call."""
import numpy as np
import torch

import parity_util as pu
from oracle import cs_oracle as orc


def test_sliced_calls_equal_whole_calls(monkeypatch):
    monkeypatch.setattr(pu, "_SLICE", 10_007)
    sk = orc.SketchOracle(5, 1 << 10, 42)
    rng = np.random.default_rng(0)
    d = 123_457
    g32 = rng.standard_normal(d).astype(np.float32)
    g64 = rng.standard_normal(d)
    for g, scale in [(g32, 1.0), (g64, 0.25)]:
        whole = sk.sketch(g, scale=scale)
        cut = pu.sketch_in_slices(sk, g, scale=scale)
        assert np.abs(whole - cut).max() <= 1e-12 * np.abs(whole).max()
    T = sk.sketch(g64)
    np.testing.assert_array_equal(pu.estimate_in_slices(sk, T, d), sk.estimate(T, d))
    idx = rng.integers(0, d, size=200_000)
    np.testing.assert_array_equal(pu.estimate_sparse_in_slices(sk, T, idx), sk.estimate_sparse(T, idx))
    vecs = [torch.from_numpy(rng.standard_normal(d).astype(np.float32)) for _ in range(3)]
    want = sum(v.numpy().astype(np.float64) for v in vecs)
    np.testing.assert_array_equal(pu.host_sum_f64(vecs), want)
