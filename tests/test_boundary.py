"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every symbol the
header declares, draws the same hash constants as the reference, and rejects bad arguments
before touching the device."""
import ctypes
import os
import re

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
    header = open(os.path.join(ROOT, "include", "csketch.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(cs_[a-z_0-9]+)\s*\(", header))
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
    assert lib.cs_sketch_estimate(ctypes.byref(p), null, 10, 0, fake, null, 0, null) == -1
    assert lib.cs_sketch_merge(ctypes.byref(p), fake, 0.0, None, 2, 1.0, null) == -1
    assert lib.cs_heavy_hitters_topk(fake, 10, 11, fake, fake, fake, 1 << 20, null) == -1
    assert lib.cs_heavy_hitters_topk(fake, 10, 0, fake, fake, fake, 1 << 20, null) == -1
    assert lib.cs_heavy_hitters_topk(fake, 10, 5, fake, fake, fake, 8, null) == -2
    size = ctypes.c_size_t(0)
    assert lib.cs_topk_workspace_bytes(10, 11, ctypes.byref(size)) == -1
    assert lib.cs_topk_workspace_bytes(10, 10, ctypes.byref(size)) == 0 and size.value > 0
    bad = binding.CsParams()
    bad.r, bad.c = 4, 16
    assert lib.cs_sketch_zero(ctypes.byref(bad), fake, null) == -1


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
