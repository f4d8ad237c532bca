"""The seeded input generators: deterministic per (config, step, worker), right shapes and
value structure.  They hold none of the method's arithmetic, so there is nothing to pin
against the paper here."""
import numpy as np
import torch

import workloads as wl


def small(cfg):
    return wl.scaled(cfg, d=1 << 16, W=3, n_heavy=64 if wl.CONFIGS[cfg].n_heavy else 0)


def test_full_size_table_matches_benchmark_definition():
    c = wl.CONFIGS
    assert (c[1].d, c[1].W, c[1].r, c[1].c, c[1].k) == (1 << 20, 4, 5, 1 << 15, 1000)
    assert (c[2].d, c[2].W, c[2].c, c[2].k) == (6_500_000, 8, 1 << 17, 5000)
    assert (c[3].d, c[3].W, c[3].c, c[3].k) == (11_000_000, 16, 1 << 18, 50_000)
    assert (c[4].d, c[4].W, c[4].c, c[4].k, c[4].steps, c[4].rho) == (10**8, 32, 1 << 20, 10**5, 10, 0.9)
    assert (c[5].d, c[5].W, c[5].r, c[5].c, c[5].k, c[5].steps) == (25_000_000, 256, 7, 1 << 19, 20_000, 20)


def test_deterministic_and_distinct_per_step_and_worker():
    for cfg in range(1, 6):
        w = wl.Workload(small(cfg))
        a = w.gradient(0, 1)
        b = wl.Workload(small(cfg)).gradient(0, 1)
        assert a.dtype == torch.float32 and a.shape == (1 << 16,)
        assert torch.equal(a, b)
        assert not torch.equal(a, w.gradient(0, 2))
        assert not torch.equal(a, w.gradient(1, 1))
        assert torch.isfinite(a).all()


def test_value_structure():
    w1 = wl.Workload(small(1))
    g = w1.gradient(0, 0).numpy()
    mask = np.ones(g.size, bool)
    mask[w1.heavy_idx.numpy()] = False
    assert abs(g[mask].std() - 0.01) < 5e-4
    heavy = np.abs(g[~mask])
    assert heavy.min() > 0.45 and heavy.max() < 1.05
    # planted values identical across workers, noise not
    g2 = w1.gradient(0, 1).numpy()
    assert np.abs(g2[~mask] - g[~mask]).max() < 0.1

    w3 = wl.Workload(small(3))
    tau = w3.tau.numpy()
    assert tau.min() >= 1e-6 * 0.999 and tau.max() <= 1e-1 * 1.001
    assert abs(np.log10(tau).mean() + 3.5) < 0.05

    w4 = wl.Workload(small(4))
    g4 = w4.gradient(2, 0).numpy()
    hv = g4[w4.heavy_idx.numpy()]
    assert 0.03 < np.abs(hv).mean() < 0.3          # Laplace(0, 0.1): E|x| = 0.1

    w2 = wl.Workload(small(2))
    g2 = w2.gradient(0, 0).numpy()
    # Student-t(3) * 1e-3: heavier tails than a Gaussian of the same scale
    assert (np.abs(g2) > 5e-3).mean() > 1e-3


def test_bench_placement_choice():
    """The host logic with which bench.py picks, from probe times of successive chunks of device
    memory, the chunks that hold the input sets (sequences as measured on MI355X)."""
    import bench
    fresh = [15.46, 15.47, 15.46, 15.48, 15.46, 15.45, 15.45, 15.01, 13.93, 13.94, 13.94, 13.92]
    for n in range(1, len(fresh) + 1):
        assert bench.enough_fast_chunks(fresh[:n], 4) == (n == 12)
    assert bench.choose_chunks(fresh, 4) == [8, 9, 10, 11]
    mixed = [14.10, 14.10, 14.89, 14.87, 14.01, 14.11, 14.16, 14.08, 14.26, 14.25, 14.24, 13.96, 13.92, 14.13]
    assert not bench.enough_fast_chunks(mixed, 4)            # the four fastest are not alike
    assert bench.choose_chunks(mixed, 4) == [4, 7, 11, 12]
    alike = [44.4, 44.2, 44.3, 44.6, 44.3, 44.0, 45.0, 45.2, 45.5, 44.3, 44.0]
    assert not bench.enough_fast_chunks(alike, 2)
    assert bench.choose_chunks(alike, 2) == [0, 1]           # nothing stands out: plain order
    assert bench.choose_chunks([15.4, 13.9], 4) is None      # fewer chunks than input sets
    assert bench.choose_chunks([15.4, 13.9], 1) == [1]
