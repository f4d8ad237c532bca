"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every symbol the
header declares, draws the same hash constants as the reference, and rejects bad arguments
before touching the device."""
import ctypes
import os
import re

import numpy as np
import pytest

import paper_1903_04488_amd as cs
from paper_1903_04488_amd import binding
from oracle import cs_oracle as orc

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
P = (1 << 61) - 1


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(cs.library_path()):
        from paper_1903_04488_amd.build import build_library
        build_library()
    return cs.load_library()


def test_library_exports_every_declared_symbol(lib):
    declared = set()
    for name in sorted(os.listdir(os.path.join(ROOT, "include"))):
        header = open(os.path.join(ROOT, "include", name)).read()
        header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
        declared |= set(re.findall(r"\b(cs_[a-z_0-9]+)\s*\(", header))
    assert len(declared) >= 18
    for name in declared:
        assert hasattr(lib, name), name
    assert declared == set(binding.exported_symbols())


def test_params_match_reference_draw(lib):
    for r, c, seed in [(5, 1 << 15, 190304489), (7, 1 << 19, 190304493), (15, 180000, 1), (1, 1, 0)]:
        p = cs.cs_params_init(r, c, seed)
        sk = orc.SketchOracle(r, c, seed)
        assert (p.r, p.c, p.seed) == (r, c, seed)
        assert p.c_pow2 == (1 if c & (c - 1) == 0 else 0)
        for j in range(r):
            assert p.a[j] == int(sk.a[j]) and p.b[j] == int(sk.b[j])
            assert p.as_[j] == int(sk.as_[j]) and p.bs[j] == int(sk.bs[j])


def test_traversal_plan_is_consistent(lib):
    for r, c, seed, d in [(5, 1 << 20, 190304492, 10**8), (5, 1 << 15, 190304489, 1 << 20),
                          (7, 1000, 3, 0), (5, 1 << 17, 9, 100)]:
        p = cs.cs_params_init(r, c, seed, d)
        for j in range(r):
            pl = p.plan[j]
            assert pl.D >= 1 and pl.lanes in (16, 32, 64) and 0 <= pl.scan_steps <= 4
            if d:
                assert pl.D <= max(d // 8, 1)      # at least 8 lanes have work
            assert pl.AD == (p.a[j] * pl.D) % P
            assert pl.ADs == (p.as_[j] * pl.D) % P
            if p.c_pow2:
                # scan_steps covers the longest run of neighbouring lanes in one bucket
                arc = (1 << 61) // c
                Au = (pl.AD * arc) % P
                A1 = min(Au, P - Au)
                longest = (arc - 1) // A1 + 1 if A1 else 1 << 60
                assert (1 << pl.scan_steps) >= min(longest, 16)


@pytest.mark.parametrize("r,c,seed,d", [(5, 1 << 15, 190304489, 1 << 20), (7, 1 << 19, 190304493, 25_000_000),
                                        (5, 1 << 12, 11, 200_003), (3, 64, 3, 5_000_000),
                                        (5, 1000, 9, 50_001), (5, 1 << 15, 2, 1000), (5, 1 << 15, 2, 0)])
def test_visit_list_is_consistent(lib, r, c, seed, d):
    """The visit list of the bundle update: starts at offset 0, gaps tile [0, d_hint) exactly,
    the hash advances belong to the gaps, and -- the property the kernel's running sums rest
    on -- moving any coordinate by any listed offset advances its bucket by fewer than ncell
    cells (checked with Python integers on random coordinates and on coordinates chosen to sit
    at the edges of a cell)."""
    p = cs.cs_params_init(r, c, seed, d)
    rng = np.random.default_rng(seed)
    pow2 = c & (c - 1) == 0
    for j in range(r):
        v = p.visit[j]
        if not pow2 or d < 4096:
            assert v.K == 0
            continue
        if v.K == 0:
            continue
        assert 4 <= v.K <= binding.CS_MAX_VISITS and 2 <= v.ncell <= 4
        assert v.cover == d
        gaps = v.gaps()
        assert all(g > 0 for g in gaps) and sum(gaps) == d
        assert v.gmax == max(gaps)
        assert len(set(gaps[:-1])) <= 3            # return times of a rotation to an interval
        for q in range(4):
            assert v.A[q] == (p.a[j] * v.gap[q]) % P and v.As[q] == (p.as_[j] * v.gap[q]) % P
        a, b = int(p.a[j]), int(p.b[j])
        offsets = np.cumsum([0] + gaps[:-1]).tolist()
        # coordinates whose hash value is the first / last of a cell's arc, and random ones
        sh = 61 - (c.bit_length() - 1)
        inv_a = pow(a, P - 2, P)
        edge = []
        for cell in (0, 1, c // 2, c - 1):
            for u in ((cell << sh), ((cell + 1) << sh) - 1):          # rotated value
                x = ((u & ((1 << sh) - 1)) << (61 - sh)) | (u >> sh)  # rotate back by sh bits
                if x < P:
                    edge.append(((x - b) * inv_a) % P)
        coords = edge + rng.integers(0, 1 << 40, size=40).tolist()
        for i in coords:
            h0 = ((a * i + b) % P) % c
            for s in offsets:
                rel = ((((a * (i + s) + b) % P) % c) - h0) % c
                assert rel < v.ncell, (j, i, s, rel)
        # the list must beat the stride walk by its own estimate to be used at all
        assert v.cost > 0 and v.cost_walk > 0


@pytest.mark.parametrize("r,c,seed,d", [(5, 180_000, 41, 6_500_000), (15, 180_000, 42, 3_000_000),
                                        (3, 50_021, 44, 3_000_001), (5, 3 << 15, 45, 5_000_000),
                                        (5, 1000, 9, 50_001), (5, 1 << 15, 2, 1 << 20)])
def test_visit_list_for_any_column_count_is_consistent(lib, r, c, seed, d):
    """The visit list for column counts that are not a power of two: gaps tile [0, d_hint), and
    -- what the kernel's 2 omega running sums rest on -- moving any coordinate by any listed
    offset advances its bucket by fewer than omega cells, or by that minus p mod c when the hash
    value wrapped past p (Python integers; random coordinates and coordinates whose hash value
    sits just below p)."""
    p = cs.cs_params_init(r, c, seed, d)
    rng = np.random.default_rng(seed)
    pc = P % c
    for j in range(r):
        v = p.anyc[j]
        if c & (c - 1) == 0 or d < 65536:
            assert v.K == 0
            continue
        if v.K == 0:
            continue
        assert 4 <= v.K <= binding.CS_ANYC_MAX_VISITS and v.omega in (1, 2) and v.cover == d
        gaps = v.gaps()
        assert all(g > 0 for g in gaps) and sum(gaps) == d and v.gmax == max(gaps)
        assert v.cost > 0 and v.cost_direct > 0
        a, b = int(p.a[j]), int(p.b[j])
        inv_a = pow(a, P - 2, P)
        near_p = [((P - 1 - t - b) * inv_a) % P for t in (0, 1, 2, 1000)]   # hash value P-1-t: wraps at once
        coords = near_p + rng.integers(0, 1 << 40, size=60).tolist() + [0, 1, d - 1]
        offsets = np.cumsum([0] + gaps[:-1]).tolist()
        wrapped = 0
        for i in coords:
            h0 = ((a * i + b) % P) % c
            for s in offsets:
                t = ((((a * (i + s) + b) % P) % c) - h0) % c
                ok_plain = t < v.omega
                ok_wrap = (t + pc) % c < v.omega
                assert ok_plain or ok_wrap, (j, i, s, t)
                wrapped += (not ok_plain) and ok_wrap
        assert wrapped > 0          # the second set of sums is exercised


def test_invalid_arguments_are_rejected_without_a_gpu(lib):
    p = binding.CsParams()
    assert lib.cs_params_init(None, 5, 16, 1, 0) == -1
    for r, c in [(0, 16), (4, 16), (17, 16), (5, 0), (5, (1 << 31) + 1), (15, 1 << 29)]:
        assert lib.cs_params_init(ctypes.byref(p), r, c, 1, 0) == -1, (r, c)
    assert lib.cs_params_init(ctypes.byref(p), 5, 16, 1, -1) == -1
    assert lib.cs_params_init(ctypes.byref(p), 5, 16, 1, 0) == 0
    null = ctypes.c_void_p(0)
    fake = ctypes.c_void_p(256)      # never dereferenced: validation fails first
    assert lib.cs_sketch_accumulate(ctypes.byref(p), null, fake, 10, 0, 1.0, null) == -1
    assert lib.cs_sketch_accumulate(ctypes.byref(p), fake, fake, -1, 0, 1.0, null) == -1
    assert lib.cs_sketch_accumulate(ctypes.byref(p), fake, fake, 10, -1, 1.0, null) == -1
    assert lib.cs_sketch_accumulate(ctypes.byref(p), fake, fake, 10, 1 << 61, 1.0, null) == -1
    assert lib.cs_sketch_accumulate(ctypes.byref(p), fake, fake, 0, 0, 1.0, null) == 0   # no-op
    assert lib.cs_sketch_estimate(ctypes.byref(p), null, 10, 0, fake, null, null, 0, null) == -1
    assert lib.cs_sketch_merge(ctypes.byref(p), fake, 0.0, None, 2, 1.0, null) == -1
    assert lib.cs_heavy_hitters_topk(fake, 10, 11, null, fake, fake, fake, 1 << 20, null) == -1
    assert lib.cs_heavy_hitters_topk(fake, 10, 0, null, fake, fake, fake, 1 << 20, null) == -1
    assert lib.cs_heavy_hitters_topk(fake, 10, 5, null, fake, fake, fake, 8, null) == -2
    size = ctypes.c_size_t(0)
    assert lib.cs_topk_workspace_bytes(10, 11, ctypes.byref(size)) == -1
    assert lib.cs_topk_workspace_bytes(10, 10, ctypes.byref(size)) == 0 and size.value > 0
    bad = binding.CsParams()
    bad.r, bad.c = 4, 16
    assert lib.cs_sketch_zero(ctypes.byref(bad), fake, null) == -1
    assert lib.cs_quantize16(fake, 10, fake, 2, null) == -1
    assert lib.cs_quantize16(null, 10, fake, 0, null) == -1
    assert lib.cs_quantize16(fake, 0, fake, 0, null) == 0
    assert lib.cs_dequantize16(fake, -1, fake, 0, null) == -1
    assert lib.cs_bundle_merge16(ctypes.byref(p), fake, 0.0, ctypes.c_void_p(264), 8, 1.0, 0, null) == -1
    assert lib.cs_dense_momentum(None, None, None, 1, 10, 0.9, null) == -1
    assert lib.cs_dense_mask(None, None, 1, fake, 10, null) == -1
    assert lib.cs_probe_stream_read(None, 1, 10, fake, null) == -1
    assert lib.cs_sketch_accumulate_sum(ctypes.byref(p), null, 2, None, 10, 0, 1.0, null) == -1
    assert lib.cs_sketch_accumulate_sum(ctypes.byref(p), fake, 0, None, 10, 0, 1.0, null) == -1
    two = (ctypes.c_void_p * 2)(256, 0)
    assert lib.cs_sketch_accumulate_sum(ctypes.byref(p), fake, 2, two, 10, 0, 1.0, null) == -1   # a null vector
    assert lib.cs_sketch_accumulate_sum(ctypes.byref(p), fake, 2, two, 0, 0, 1.0, null) == 0    # no-op
    assert lib.cs_sketch_accumulate_sum(ctypes.byref(p), fake, 2, two, 10, -1, 1.0, null) == -1
    assert lib.cs_fixed_accumulate(ctypes.byref(p), fake, fake, 10, 0, 1.0, 63, null, null) == -1
    assert lib.cs_fixed_accumulate(ctypes.byref(p), fake, fake, 10, 0, 1.0, -1, null, null) == -1
    assert lib.cs_fixed_accumulate(ctypes.byref(p), null, fake, 10, 0, 1.0, 40, null, null) == -1
    assert lib.cs_fixed_accumulate(ctypes.byref(p), fake, null, 10, 0, 1.0, 40, null, null) == -1
    assert lib.cs_fixed_accumulate(ctypes.byref(p), fake, null, 0, 0, 1.0, 40, null, null) == 0   # no-op
    assert lib.cs_fixed_accumulate_sparse(ctypes.byref(p), fake, null, fake, 10, 1.0, 40, null, null) == -1
    assert lib.cs_fixed_accumulate_sparse(ctypes.byref(p), fake, null, null, 0, 1.0, 40, null, null) == 0
    assert lib.cs_fixed_to_float(ctypes.byref(p), fake, 40, 1.0, null, null) == -1
    assert lib.cs_fixed_to_float(ctypes.byref(bad), fake, 40, 1.0, fake, null) == -1
    assert lib.cs_sketch_l2sq(ctypes.byref(p), fake, null, null) == -1
    assert lib.cs_sketch_l2sq(ctypes.byref(p), fake, ctypes.c_void_p(260), null) == -1    # misaligned
    assert lib.cs_heavymix_select(fake, 10, 5, null, 1, fake, null, null, fake, 1 << 20, null) == -1
    assert lib.cs_heavymix_select(fake, 10, 11, fake, 1, fake, null, null, fake, 1 << 20, null) == -1
    assert lib.cs_heavymix_select(fake, 10, 5, fake, 1, fake, null, null, fake, 8, null) == -2


def test_update_launch_count_follows_the_grouping(lib):
    """cs_bundle_update_launches: per group of 8 workers one launch for the rows with a visit list
    (8 rows at most per launch) and one for the rows walked by stride; for other column counts
    one launch per group and up to 6 rows of equal omega with visit lists, one per 32 workers
    without; none for an empty vector."""
    for r, c, seed, d in [(5, 1 << 20, 190304492, 10**8), (5, 1 << 15, 190304489, 1 << 20),
                          (7, 1 << 19, 190304493, 25_000_000), (15, 1 << 12, 4, 3_000_000)]:
        p = cs.cs_params_init(r, c, seed, d)
        listed = sum(1 for j in range(r) if p.visit[j].K > 0 and p.visit[j].cost < p.visit[j].cost_walk)
        per_group = -(-listed // 8) + (1 if listed < r else 0)
        for W in (1, 8, 9, 32, 250):
            assert cs.cs_bundle_update_launches(p, W, d) == per_group * -(-W // 8), (r, c, W)
        assert cs.cs_bundle_update_launches(p, 8, 0) == 0
        walk = binding.CsParams.from_buffer_copy(p)
        walk.flags = binding.CS_FLAG_NO_VISIT_LIST
        assert cs.cs_bundle_update_launches(walk, 16, d) == 2
    # a column count that is not a power of two: per group of 8 workers one launch for up to 6 rows
    # that keep the same number of running sums (omega), along the rows' visit lists; one launch
    # per 32 workers without them
    for r in (5, 15):
        p = cs.cs_params_init(r, 180_000, 1, 6_500_000)
        assert all(p.anyc[j].K > 0 for j in range(r))
        per_group = sum(-(-sum(1 for j in range(r) if p.anyc[j].omega == omega) // 6) for omega in (1, 2))
        assert 1 <= per_group <= (2 if r == 5 else 4)
        for W, groups in ((1, 1), (8, 1), (9, 2), (100, 13)):
            assert cs.cs_bundle_update_launches(p, W, 6_500_000) == per_group * groups
    p = cs.cs_params_init(5, 180_000, 1, 6_500_000)
    p.flags = binding.CS_FLAG_NO_VISIT_LIST
    for W, n in ((1, 1), (32, 1), (33, 2), (100, 4)):
        assert cs.cs_bundle_update_launches(p, W, 6_500_000) == n


def test_status_strings(lib):
    assert cs.cs_status_string(0) == "ok"
    assert "invalid" in cs.cs_status_string(-1)
    assert "workspace" in cs.cs_status_string(-2)
    assert "HIP" in cs.cs_status_string(-3)


def test_binding_refuses_cpu_tensors(lib):
    import torch
    p = cs.cs_params_init(5, 16, 1)
    with pytest.raises(cs.CsError):
        cs.cs_sketch_zero(p, torch.zeros(5, 16))


def test_binding_structs_have_the_layout_of_the_header(tmp_path):
    """The ctypes mirrors of cs_params and its members have the sizes and field offsets that a C
    compiler gives the declarations in include/csketch.h."""
    import subprocess
    fields = {"cs_row_plan": ["D", "AD", "ADs", "Dw", "ADw", "ADws", "lanes", "scan_steps"],
              "cs_visit_plan": ["K", "ncell", "cover", "gmax", "cost", "cost_walk", "gap", "A", "As", "code"],
              "cs_anyc_plan": ["K", "omega", "cover", "gmax", "cost", "cost_direct", "gap"],
              "cs_params": ["r", "c", "c_pow2", "flags", "seed", "a", "b", "as", "bs", "plan", "visit", "anyc"]}
    mirror = {"cs_row_plan": binding.CsRowPlan, "cs_visit_plan": binding.CsVisitPlan,
              "cs_anyc_plan": binding.CsAnycPlan, "cs_params": binding.CsParams}
    lines = ['#include <stdio.h>', '#include <stddef.h>', '#include "csketch.h"', 'int main(void) {']
    for s, fs in fields.items():
        lines.append(f'printf("{s} %zu\\n", sizeof({s}));')
        for f in fs:
            lines.append(f'printf("{s}.{f} %zu\\n", offsetof({s}, {f}));')
    lines += ['printf("CS_MAX_R %d\\nCS_MAX_VISITS %d\\nCS_BUNDLE_GROUP %d\\n", CS_MAX_R, CS_MAX_VISITS, CS_BUNDLE_GROUP);',
              'return 0; }']
    src = tmp_path / "layout.c"
    src.write_text("\n".join(lines))
    exe = tmp_path / "layout"
    subprocess.check_call(["gcc", "-I", os.path.join(ROOT, "include"), "-o", str(exe), str(src)])
    got = dict(line.split() for line in subprocess.check_output([str(exe)], text=True).splitlines())
    for s, fs in fields.items():
        assert int(got[s]) == ctypes.sizeof(mirror[s]), s
        for f in fs:
            name = "as_" if f == "as" else f          # `as` is a Python keyword
            assert int(got[f"{s}.{f}"]) == getattr(mirror[s], name).offset, f"{s}.{f}"
    assert int(got["CS_MAX_R"]) == binding.CS_MAX_R
    assert int(got["CS_MAX_VISITS"]) == binding.CS_MAX_VISITS
    assert int(got["CS_BUNDLE_GROUP"]) == binding.CS_BUNDLE_GROUP
