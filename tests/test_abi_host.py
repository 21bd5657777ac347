"""Host-only checks of the C-ABI library: it loads, exports every symbol the
header declares, and its host logic (plans, sizes, validation) behaves.  No
kernel is launched."""
import ctypes
import os
import re

import pytest

import paper_2512_17970_amd as cg
from paper_2512_17970_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def header_symbols():
    text = open(os.path.join(ROOT, "include", "codegemm.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(codegemm_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = cg.load()
    syms = header_symbols()
    assert set(syms) == set(binding.EXPORTS)
    for s in syms:
        assert hasattr(lib, s), s


def test_status_strings():
    assert cg.codegemm_status_string(0) == "ok"
    for s in (-1, -2, -3, -4, -99):
        assert cg.codegemm_status_string(s)


def test_default_plans_are_valid_for_all_workloads():
    import synth
    for cases in synth.workloads().values():
        for c in cases:
            d = cg.Desc.make(c.B, c.K, c.N, c.v, c.m)
            p = cg.codegemm_default_plan(d)
            assert p.slots in (32, 64) and p.waves in (8, 16) and p.batch_group in (1, 2, 4)
            assert (p.slots // p.waves) * c.m <= 8
            nrb = -(-c.N // 512)
            nkt = -(-c.J // p.slots)
            assert 1 <= p.k_splits <= nkt and nrb * p.k_splits <= max(256, nrb)
            assert cg.codegemm_packed_codes_bytes(d) == nrb * nkt * p.slots * 64 * 8 * c.m
            assert cg.codegemm_workspace_bytes(d) >= c.B * p.k_splits * nrb * 512 * 4 * (nkt > 1)


def test_invalid_descriptors_are_rejected():
    for d in (cg.Desc.make(0, 512, 512, 8, 1), cg.Desc.make(1, 510, 512, 8, 1), cg.Desc.make(1, 512, 0, 8, 1),
              cg.Desc.make(1, 512, 512, 16, 1), cg.Desc.make(1, 512, 512, 8, 5), cg.Desc.make(1, 512, 512, 8, 1, b=4),
              cg.Desc.make(1, 512, 512, 8, 1, g=128), cg.Desc.make(33, 512, 512, 8, 1)):
        assert cg.codegemm_workspace_bytes(d) == 0
        assert cg.codegemm_packed_codes_bytes(d) == 0
        with pytest.raises(cg.CodegemmError):
            cg.codegemm_default_plan(d)


def test_invalid_plans_are_rejected():
    d = cg.Desc.make(1, 512, 512, 8, 2)
    for p in (cg.Plan.make(48, 16, 4), cg.Plan.make(64, 4, 4), cg.Plan.make(64, 8, 4), cg.Plan.make(32, 16, 0),
              cg.Plan.make(32, 16, 2, 3), cg.Plan.make(32, 32, 1)):
        assert cg.codegemm_workspace_bytes(d, p) == 0
    assert cg.codegemm_workspace_bytes(d, cg.Plan.make(64, 16, 4)) > 0
    d3 = cg.Desc.make(1, 512, 512, 8, 3)
    assert cg.codegemm_workspace_bytes(d3, cg.Plan.make(64, 16, 2)) == 0      # 192 KB of Psumbook does not fit
    assert cg.codegemm_workspace_bytes(d3, cg.Plan.make(32, 8, 2)) == 0       # 4 steps x 3 codebooks of code words
    assert cg.codegemm_workspace_bytes(d3, cg.Plan.make(32, 16, 2)) > 0


def test_compressed_bytes_closed_form():
    # 8192 -> 28672, v8 m2, batch 1: codes 58,720,256 + codebooks 8192 + scales 57344 + x 16384 + y 57344
    assert cg.compressed_bytes(1, 8192, 28672, 8, 2) == 58720256 + 8192 + 57344 + 16384 + 57344
