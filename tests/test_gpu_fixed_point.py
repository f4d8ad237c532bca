"""The update with order-independent sums (64-bit fixed point), through the C ABI, against the
CPU reference BIT FOR BIT: integer sums are associative, so there is no tolerance anywhere in
this file.  What the float path can only show to rounding ("reordered or wrong?") is shown
exactly here: every coordinate lands in the cell and with the sign the reference gives it.

Also the step built on it (ReproduciblePath): two runs give equal bits, a run cut in the middle,
saved and restored continues bit for bit, and its selections are valid for the reference."""
import io

import numpy as np
import pytest
import torch

import workloads as wl
from oracle import cs_oracle as orc
from paper_1903_04488_amd import binding as B
from paper_1903_04488_amd.pipeline import HotPath, ReproduciblePath
from parity_util import assert_cells_close, assert_valid_topk, estimate_in_slices

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def vector(d, seed, specials=True):
    rng = np.random.default_rng(seed)
    g = (0.01 * rng.standard_normal(d)).astype(np.float32)
    heavy = rng.choice(d, size=min(50, d), replace=False)
    g[heavy] = rng.uniform(-8, 8, heavy.size).astype(np.float32)
    if specials and d >= 16:
        # left out and counted: not finite, or scale * g * 2^F not below 2^62
        g[3], g[5], g[d - 1] = np.nan, -np.inf, np.float32(3e30)
        # exact halves of the last kept bit round to even; the smallest subnormal rounds to 0
        g[7], g[9], g[11] = np.float32(2.0 ** -41), np.float32(-3 * 2.0 ** -41), np.float32(1e-45)
    return g


@pytest.mark.parametrize("r,c,d,i0,F,scale", [
    (5, 1 << 15, (1 << 20) + 77, 0, 40, 1.0),
    (15, 180_000, 700_001, 12_345, 40, -0.5),          # the paper's widest sketch shape, any c
    (7, 40, 5_000, 1 << 33, 30, 0.3),                  # App. E's sketch, coordinates beyond 2^32
    (1, 1, 1_000, 0, 20, 1.0),
    (3, 4096, 1, 9, 62, 2.0 ** -3),                    # one coordinate, all bits fractional
])
def test_fixed_accumulate_is_bit_exact(r, c, d, i0, F, scale):
    g = vector(d, seed=r * 1000 + c % 997)
    if F == 62:
        g[:] = np.float32(0.7)
    sk = orc.SketchOracle(r, c, 4242)
    p = B.cs_params_init(r, c, 4242, d)
    acc = torch.zeros(r, c, dtype=torch.int64, device=DEV)
    dropped = torch.zeros(1, dtype=torch.int64, device=DEV)
    B.cs_fixed_accumulate(p, acc, torch.from_numpy(g).to(DEV), F, i0=i0, scale=scale, dropped=dropped)
    ref = np.zeros((r, c), dtype=np.int64)
    n_bad = sk.accumulate_fixed(ref, g, F, i0=i0, scale=scale)
    np.testing.assert_array_equal(acc.cpu().numpy(), ref)
    assert int(dropped.item()) == n_bad
    assert n_bad == (3 if d >= 16 and F != 62 else 0)
    # a second vector into the same table, without a counter
    g2 = vector(d, seed=77, specials=False)
    B.cs_fixed_accumulate(p, acc, torch.from_numpy(g2).to(DEV), F, i0=i0, scale=scale)
    assert sk.accumulate_fixed(ref, g2, F, i0=i0, scale=scale) == 0
    np.testing.assert_array_equal(acc.cpu().numpy(), ref)
    assert int(dropped.item()) == n_bad
    # conversion: same bits, alpha included
    S = torch.empty(r, c, dtype=torch.float32, device=DEV)
    for alpha in (1.0, 1.0 / 3.0):
        B.cs_fixed_to_float(p, acc, F, S, alpha=alpha)
        np.testing.assert_array_equal(S.cpu().numpy().view(np.uint32),
                                      sk.fixed_to_float(ref, F, alpha=alpha).view(np.uint32))


def test_fixed_to_float_rounds_once_per_step():
    p = B.cs_params_init(1, 4, 1, 4)
    acc = torch.tensor([[(1 << 53) + 1, -(1 << 24) - 1, 3, -(1 << 62)]], dtype=torch.int64, device=DEV)
    S = torch.empty(1, 4, dtype=torch.float32, device=DEV)
    B.cs_fixed_to_float(p, acc, 0, S)
    assert S.cpu().tolist() == [[2.0 ** 53, -(2.0 ** 24), 3.0, -(2.0 ** 62)]]
    sk = orc.SketchOracle(1, 4, 1)
    B.cs_fixed_to_float(p, acc, 7, S, alpha=0.1)
    np.testing.assert_array_equal(S.cpu().numpy().view(np.uint32),
                                  sk.fixed_to_float(acc.cpu().numpy(), 7, alpha=0.1).view(np.uint32))


@pytest.mark.parametrize("c", [1 << 12, 180_000])
def test_fixed_accumulate_sparse_is_bit_exact(c):
    r, n, F = 5, 20_000, 36
    rng = np.random.default_rng(c)
    idx = rng.integers(0, 1 << 40, n)
    idx[:500] = idx[500:1000]                          # repeated coordinates add up
    val = vector(n, seed=5)
    sk = orc.SketchOracle(r, c, 99)
    p = B.cs_params_init(r, c, 99, 1 << 20)
    acc = torch.zeros(r, c, dtype=torch.int64, device=DEV)
    dropped = torch.zeros(1, dtype=torch.int64, device=DEV)
    B.cs_fixed_accumulate_sparse(p, acc, torch.from_numpy(idx).to(DEV), torch.from_numpy(val).to(DEV),
                                 F, scale=-1.0, dropped=dropped)
    ref = np.zeros((r, c), dtype=np.int64)
    n_bad = sk.accumulate_fixed_sparse(ref, idx, val, F, scale=-1.0)
    np.testing.assert_array_equal(acc.cpu().numpy(), ref)
    assert int(dropped.item()) == n_bad == 3
    # empty list: nothing happens
    B.cs_fixed_accumulate_sparse(p, acc, torch.empty(0, dtype=torch.int64, device=DEV),
                                 torch.empty(0, dtype=torch.float32, device=DEV), F)
    np.testing.assert_array_equal(acc.cpu().numpy(), ref)


def test_workers_in_any_order_give_the_same_bits_and_agree_with_the_float_path():
    """Sums over workers are the same integer sums, so the order in which the workers arrive
    cannot matter; and the table agrees with the float path's merged table to that path's own
    tolerance (the fixed-point sum is the more accurate of the two)."""
    r, c, d, W, F = 5, 1 << 14, (1 << 21) + 13, 8, 40
    g_w = [torch.from_numpy(vector(d, seed=100 + w, specials=False)).to(DEV) for w in range(W)]
    p = B.cs_params_init(r, c, 31, d)
    tables = []
    for order in (range(W), reversed(range(W)), (3, 0, 7, 1, 6, 2, 5, 4)):
        acc = torch.zeros(r, c, dtype=torch.int64, device=DEV)
        for w in order:
            B.cs_fixed_accumulate(p, acc, g_w[w], F)
        tables.append(acc.cpu().numpy())
    np.testing.assert_array_equal(tables[0], tables[1])
    np.testing.assert_array_equal(tables[0], tables[2])
    S = torch.empty(r, c, dtype=torch.float32, device=DEV)
    B.cs_fixed_to_float(p, torch.from_numpy(tables[0]).to(DEV), F, S, alpha=1.0 / W)
    sk = orc.SketchOracle(r, c, 31)
    gsum = np.zeros(d)
    for g in g_w:
        gsum += g.cpu().numpy().astype(np.float64)
    ref = sk.sketch(gsum, scale=1.0 / W)
    # every contribution is off by at most 2^-41 and a cell holds a few hundred per worker:
    # before the rounding to binary32 the table is the reference's to 1e-9
    assert np.abs(tables[0] * 2.0 ** -F / W - ref).max() <= 1e-9
    hp = HotPath(d, W, r, c, 100, 31, device=DEV)
    hp.accumulate(g_w)
    hp.merge()
    assert_cells_close(hp.S_t.cpu().numpy(), ref, what="float path")
    assert_cells_close(S.cpu().numpy(), ref, what="fixed-point path")


def run_steps(hp, work, c, ts):
    out = []
    for t in ts:
        idx, x = hp.step([work.gradient(t, w) for w in range(c.W)])
        out.append((idx.cpu().numpy().copy(), x.cpu().numpy().copy()))
    return out


def test_reproducible_step_twice_and_resumed_bit_for_bit():
    """Six steps of the stateful path in its order-independent form: (i) run twice, every
    selection, every exact value and both state tables are equal bit for bit; (ii) cut after
    three steps, the state (S_u, S_v) saved to bytes and restored into a fresh object, the last
    three steps give the bits of the uncut run; (iii) every selection is valid for the
    reference's estimates of the reference's own state (teacher-forced as in the parity runs)."""
    c = wl.scaled(4, d=(1 << 20) + 77, W=4, c=1 << 13, k=1000, steps=6, n_heavy=300)
    work = wl.Workload(c, DEV)

    def fresh():
        return ReproduciblePath(c.d, c.W, c.r, c.c, c.k, c.hash_seed, rho=c.rho, device=DEV)

    a = fresh()
    out_a = run_steps(a, work, c, range(6))
    b = fresh()
    out_b = run_steps(b, work, c, range(6))
    for (ia, xa), (ib, xb) in zip(out_a, out_b):
        np.testing.assert_array_equal(ia, ib)
        np.testing.assert_array_equal(xa.view(np.uint32), xb.view(np.uint32))
    for name in ("S_u", "S_v", "est"):
        assert torch.equal(getattr(a, name).view(torch.int32), getattr(b, name).view(torch.int32)), name
    assert int(a.dropped.item()) == 0

    first = fresh()
    run_steps(first, work, c, range(3))
    blob = io.BytesIO()
    torch.save({"S_u": first.S_u.cpu(), "S_v": first.S_v.cpu()}, blob)
    del first
    blob.seek(0)
    saved = torch.load(blob, weights_only=True)
    second = fresh()
    second.S_u.copy_(saved["S_u"])
    second.S_v.copy_(saved["S_v"])
    out_c = run_steps(second, work, c, range(3, 6))
    for (ia, xa), (ic, xc) in zip(out_a[3:], out_c):
        np.testing.assert_array_equal(ia, ic)
        np.testing.assert_array_equal(xa.view(np.uint32), xc.view(np.uint32))
    for name in ("S_u", "S_v"):
        assert torch.equal(getattr(a, name).view(torch.int32), getattr(second, name).view(torch.int32)), name

    # (iii) against the reference, step by step
    sk = orc.SketchOracle(c.r, c.c, c.hash_seed)
    st = orc.SketchSpaceState(sk, c.rho)
    hp = fresh()
    for t in range(6):
        g_w = [work.gradient(t, w) for w in range(c.W)]
        gsum = np.zeros(c.d)
        for g in g_w:
            gsum += g.cpu().numpy().astype(np.float64)
        st.momentum(sk.sketch(gsum, scale=1.0 / c.W))
        idx, _ = hp.step(g_w)
        idx = idx.cpu().numpy()
        est_ref = estimate_in_slices(sk, st.S_v, c.d)
        sigma = float(np.sqrt((st.S_v ** 2).mean()))
        assert_valid_topk(idx, est_ref, c.k, sigma, what=f"step {t} selection")
        np.testing.assert_array_equal(idx, out_a[t][0])
        st.feedback(idx)
