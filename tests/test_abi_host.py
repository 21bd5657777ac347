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
FIXED = 65536 + (2 << 20)        # what every workspace starts with: ticket counters, then the words of the pairwise reduction


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


def test_trace_library_exports_the_abi_and_the_trace_hook():
    """The diagnostic build exports everything codegemm.h declares plus what codegemm_trace.h declares;
    the production library does not export the trace hook."""
    from paper_2512_17970_amd import phases
    text = open(os.path.join(ROOT, "include", "codegemm_trace.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    extra = sorted(set(re.findall(r"\b(codegemm_[a-z_]+)\s*\(", text)))
    assert extra == ["codegemm_set_trace"]
    lib = ctypes.CDLL(phases.TRACE_LIB_PATH)
    for s in header_symbols() + extra:
        assert hasattr(lib, s), s
    assert not hasattr(cg.load(), "codegemm_set_trace")


def test_ablation_libraries_export_the_abi():
    """The ablation builds (parts of the batch-1 kernel compiled out, for ceiling studies) keep the whole ABI."""
    from paper_2512_17970_amd import build as cg_build
    for mask in cg_build.ABLATE_MASKS:
        path = cg_build.ablate_lib(mask)
        if not os.path.exists(path):
            pytest.skip(f"{path} not built")
        lib = ctypes.CDLL(path)
        for s in header_symbols():
            assert hasattr(lib, s), (mask, s)


def test_phases_workgroup_count_matches_the_plan():
    from paper_2512_17970_amd import phases
    d = cg.Desc.make(1, 8192, 28672, 8, 2)
    assert phases.workgroups(d, cg.Plan.make(16, 2, 4, 1)) == 224
    assert phases.workgroups(d, cg.Plan.make(8, 1, 1000, 1)) == 224 * 32
    assert phases.workgroups(cg.Desc.make(32, 4096, 14336, 8, 2), cg.Plan.make(16, 2, 2, 4)) == 28


def test_host_pack_is_the_documented_layout_and_roundtrips():
    """codegemm_pack_codes_host / codegemm_unpack_codes_host run without a GPU: checked against the
    oracle's independent description of the layout (itself pinned byte by byte in
    test_pack_layout_pin.py) and against each other."""
    import numpy as np
    from oracle.pack_layout import pack_reference
    rng = np.random.default_rng(5)
    for (N, J, v, m) in [(130, 33, 8, 1), (129, 65, 8, 2), (257, 31, 4, 3), (200, 40, 16, 4), (1, 1, 4, 2), (512, 64, 8, 2)]:
        codes = rng.integers(0, 256, size=(m, N, J), dtype=np.uint8)
        d = cg.Desc.make(1, J * v, N, v, m)
        nbytes = cg.codegemm_packed_codes_bytes(d)
        packed = np.full(nbytes + 64, 0x5A, np.uint8)
        cg.codegemm_pack_codes_host(d, codes, packed[:nbytes])
        assert np.array_equal(packed[:nbytes], pack_reference(codes))
        assert np.all(packed[nbytes:] == 0x5A)
        back = np.full_like(codes, 0x77)
        cg.codegemm_unpack_codes_host(d, packed[:nbytes], back)
        assert np.array_equal(back, codes)
    with pytest.raises(cg.CodegemmError):
        cg.codegemm_pack_codes_host(cg.Desc.make(1, 510, 512, 8, 1), np.zeros(8, np.uint8), np.zeros(8, np.uint8))


def test_large_batches_are_accepted_and_sized_by_their_largest_launch():
    """More than 32 batch rows run as consecutive launches of up to 32: the workspace is that of the larger
    of a 32-row launch and the remainder's, the default plan that of a 32-row launch."""
    d32, d70, d1 = cg.Desc.make(32, 4096, 4096, 8, 2), cg.Desc.make(70, 4096, 4096, 8, 2), cg.Desc.make(6, 4096, 4096, 8, 2)
    assert cg.codegemm_workspace_bytes(d70) == max(cg.codegemm_workspace_bytes(d32), cg.codegemm_workspace_bytes(d1))
    p70, p32 = cg.codegemm_default_plan(d70), cg.codegemm_default_plan(d32)
    assert (p70.waves, p70.row_words, p70.k_splits, p70.batch_group) == (p32.waves, p32.row_words, p32.k_splits, p32.batch_group)
    assert cg.codegemm_packed_codes_bytes(d70) == cg.codegemm_packed_codes_bytes(d32)
    assert cg.codegemm_workspace_bytes(cg.Desc.make(65536, 512, 512, 8, 1)) == 0
    assert cg.codegemm_workspace_bytes(cg.Desc.make(1, 8 << 20, 512, 8, 1)) == 0       # K beyond 2^22
    assert cg.codegemm_workspace_bytes(cg.Desc.make(1, 512, (1 << 24) + 1, 8, 1)) == 0


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
            assert p.waves in (8, 14, 16) and p.batch_group in (1, 2, 4)
            ngr = -(-c.N // 128)
            nkt = -(-c.J // 32)
            assert p.row_words in (1, 2, 4)
            rows = p.row_words * (p.waves - p.build_waves) * (32 if p.batch_group == 4 else 16)    # rows per workgroup
            nblk = -(-ngr * 128 // rows) * (-(-c.B // p.batch_group) if p.batch_group == 4 else 1)
            assert 1 <= p.k_splits <= nkt and nblk * p.k_splits <= max(256, nblk)
            assert cg.codegemm_packed_codes_bytes(d) == ngr * 128 * nkt * 32 * c.m
            assert cg.codegemm_workspace_bytes(d) >= c.B * p.k_splits * ngr * 128 * 4


def test_workspace_is_a_fixed_counter_area_plus_partial_sums():
    """64 KB of ticket counters and 2 MB of pair words at a fixed place, then B x K ranges x padded rows fp32 partial sums; a plan
    with several K ranges and more row blocks than the counter area has words is refused."""
    for (B, K, N, v, m, plan) in [(1, 8192, 8192, 8, 2, cg.Plan.make(8, 2, 8, 1)), (1, 8192, 28672, 8, 2, cg.Plan.make(16, 2, 4, 1)),
                                  (6, 4096, 1000, 4, 1, cg.Plan.make(16, 1, 5, 4)), (1, 512, 300, 8, 1, cg.Plan.make(8, 1, 1, 1))]:
        d = cg.Desc.make(B, K, N, v, m)
        nkt = -(-(K // v) // 32)
        nks = min(plan.k_splits, nkt)
        nks = -(-nkt // -(-nkt // nks))
        assert cg.codegemm_workspace_bytes(d, plan) == FIXED + B * nks * (-(-N // 128) * 128) * 4
    many_rows = cg.Desc.make(1, 512, 128 * 20000, 8, 1)               # 20000 row blocks of 128 rows
    assert cg.codegemm_workspace_bytes(many_rows, cg.Plan.make(8, 1, 2, 1)) == 0
    assert cg.codegemm_workspace_bytes(many_rows, cg.Plan.make(8, 1, 1, 1)) > 0
    assert cg.codegemm_workspace_bytes(many_rows) > 0                  # the default plan does not split K there


def test_invalid_descriptors_are_rejected():
    for d in (cg.Desc.make(0, 512, 512, 8, 1), cg.Desc.make(1, 510, 512, 8, 1), cg.Desc.make(1, 512, 0, 8, 1),
              cg.Desc.make(1, 512, 512, 32, 1), cg.Desc.make(1, 512, 512, 2, 1), cg.Desc.make(1, 512, 512, 8, 5), cg.Desc.make(1, 512, 512, 8, 1, b=4),
              cg.Desc.make(1, 512, 512, 8, 1, g=12), cg.Desc.make(1, 512, 512, 8, 1, g=4),
              cg.Desc.make(1, 512, 512, 8, 1, g=48), cg.Desc.make(1, 8 * 40, 512, 8, 1, g=128), cg.Desc.make(1, 512, 512, 8, 1, g=0),
              cg.Desc.make(65536, 512, 512, 8, 1)):
        assert cg.codegemm_workspace_bytes(d) == 0
        assert cg.codegemm_packed_codes_bytes(d) == 0
        with pytest.raises(cg.CodegemmError):
            cg.codegemm_default_plan(d)


def test_packed_scales_bytes_closed_form():
    """[NGR][NKT][groups per unit][16][8] fp16; nothing to pack for one scale per row."""
    assert cg.codegemm_packed_scales_bytes(cg.Desc.make(1, 8192, 28672, 8, 2)) == 0
    for (K, N, v, g) in [(8192, 28672, 8, 128), (8192, 28672, 8, 8), (4096, 1000, 4, 32), (4096, 130, 4, 1024), (1024, 1, 8, 512)]:
        d = cg.Desc.make(1, K, N, v, 2, g=g)
        ngr, nkt = -(-N // 128), -(-(K // v) // 32)
        assert cg.codegemm_packed_scales_bytes(d) == ngr * nkt * max(1, 32 * v // g) * 256
        assert cg.codegemm_workspace_bytes(d) > 0 and cg.codegemm_packed_codes_bytes(d) > 0
    # when g covers whole units and N is a multiple of 128 the packed array is the canonical one's size
    # times the units per group; for g <= 32 v it is exactly 2 N K / g bytes
    assert cg.codegemm_packed_scales_bytes(cg.Desc.make(1, 8192, 28672, 8, 2, g=128)) == 2 * 28672 * 8192 // 128


def test_invalid_plans_are_rejected():
    d = cg.Desc.make(1, 512, 512, 8, 2)
    for p in (cg.Plan.make(4, 1, 4), cg.Plan.make(12, 1, 4), cg.Plan.make(32, 1, 1), cg.Plan.make(16, 1, 0),
              cg.Plan.make(16, 1, 2, 3), cg.Plan.make(16, 3, 1), cg.Plan.make(8, 4, 1), cg.Plan.make(16, 4, 1, 2)):
        assert cg.codegemm_workspace_bytes(d, p) == 0
    for p in (cg.Plan.make(8, 1, 1), cg.Plan.make(16, 2, 4, 2), cg.Plan.make(8, 1, 100000, 4), cg.Plan.make(16, 4, 2)):
        assert cg.codegemm_workspace_bytes(d, p) > 0
    d3 = cg.Desc.make(4, 512, 512, 8, 3)
    assert cg.codegemm_workspace_bytes(d3, cg.Plan.make(16, 4, 1, 4)) == 0    # batched kernel: 128 accumulators need 8-wavefront workgroups
    assert cg.codegemm_workspace_bytes(d3, cg.Plan.make(8, 4, 1, 4)) > 0
    assert cg.codegemm_workspace_bytes(d3, cg.Plan.make(16, 2, 1, 4)) > 0
    assert cg.codegemm_workspace_bytes(d3, cg.Plan.make(8, 2, 1, 4)) > 0
    assert cg.codegemm_workspace_bytes(d3, cg.Plan.make(16, 1, 1, 4)) > 0
    assert cg.codegemm_workspace_bytes(d3, cg.Plan.make(16, 2, 1, 2)) == 0    # 2 rows x 3 codebooks x 16 rows per lane


def test_fp16_psumbook_plans():
    """psum_dtype = 1 needs batch rows one at a time and at most two row words; with group scales the
    16-wavefront two-row-word shape is not offered; the default plan never picks it."""
    d = cg.Desc.make(1, 4096, 4096, 8, 3)
    fp16 = binding.PSUM_FP16
    for p in (cg.Plan.make(8, 1, 2, 1, fp16), cg.Plan.make(16, 2, 4, 1, fp16), cg.Plan.make(8, 2, 1, 1, fp16)):
        assert cg.codegemm_workspace_bytes(d, p) > 0
    for p in (cg.Plan.make(16, 2, 4, 2, fp16), cg.Plan.make(16, 1, 4, 4, fp16), cg.Plan.make(16, 4, 4, 1, fp16), cg.Plan.make(8, 1, 2, 1, 2)):
        assert cg.codegemm_workspace_bytes(d, p) == 0
    dg = cg.Desc.make(1, 4096, 4096, 8, 2, g=128)
    assert cg.codegemm_workspace_bytes(dg, cg.Plan.make(16, 2, 4, 1, fp16)) == 0
    assert cg.codegemm_workspace_bytes(dg, cg.Plan.make(16, 1, 4, 1, fp16)) > 0
    assert cg.codegemm_workspace_bytes(dg, cg.Plan.make(8, 2, 4, 1, fp16)) > 0
    import synth
    for cases in synth.workloads().values():
        for c in cases:
            assert cg.codegemm_default_plan(cg.Desc.make(c.B, c.K, c.N, c.v, c.m, g=c.g)).psum_dtype == 0


def test_compressed_bytes_closed_form():
    # 8192 -> 28672, v8 m2, batch 1: codes 58,720,256 + codebooks 8192 + scales 57344 + x 16384 + y 57344
    assert cg.compressed_bytes(1, 8192, 28672, 8, 2) == 58720256 + 8192 + 57344 + 16384 + 57344


def test_grouped_launch_host_validation():
    """Sizes and refusals of the grouped launch that need no GPU."""
    d = cg.Desc.make(1, 8192, 10240, 8, 2)
    plan = cg.codegemm_default_plan(d)
    Ns = [8192, 1024, 1024]
    ws = cg.codegemm_grouped_workspace_bytes(d, plan, Ns)
    # counter area + pair-word area + one fp32 partial per K range and padded row, member by member
    pad = sum(-(-n // 128) * 128 for n in Ns)
    assert ws == FIXED + plan.k_splits * pad * 4
    assert cg.codegemm_grouped_workspace_bytes(d, None, Ns) == ws                       # NULL plan = default plan of the sum
    assert cg.codegemm_grouped_workspace_bytes(d, plan, [8192, 1024]) == 0              # heights do not add up
    assert cg.codegemm_grouped_workspace_bytes(d, plan, [8192, 1024, 512, 256, 256]) == 0   # more than four layers
    assert cg.codegemm_grouped_workspace_bytes(d, plan, [10240, 0]) == 0                # an empty layer
    d8 = cg.Desc.make(8, 8192, 10240, 8, 2)
    assert cg.codegemm_grouped_workspace_bytes(d8, cg.Plan.make(8, 1, 2, 4), Ns) == FIXED + 8 * 2 * pad * 4   # batched-kernel plan
    d64 = cg.Desc.make(64, 8192, 10240, 8, 2)
    assert cg.codegemm_grouped_workspace_bytes(d64, cg.Plan.make(8, 1, 1, 1), Ns) == 0  # more rows than one launch takes
    # ragged members are padded one by one
    d2 = cg.Desc.make(2, 1024, 130 + 129, 8, 2)
    p2 = cg.Plan.make(8, 1, 2, 2)
    assert cg.codegemm_grouped_workspace_bytes(d2, p2, [130, 129]) == FIXED + 2 * 2 * 512 * 4


def test_448_row_blocks_in_plans():
    """Heights of 7 * 2^k rows get 14-wavefront workgroups by default where those fill more compute units."""
    from paper_2512_17970_amd import phases
    for m, g in ((1, -1), (3, -1), (2, 128)):
        p = cg.codegemm_default_plan(cg.Desc.make(1, 8192, 28672, 8, m, g=g))
        # 64 blocks x 4 K ranges = 256 workgroups; with one or two codebooks 14 of 16 wavefronts own the rows and two build
        assert (p.waves - p.build_waves, p.row_words, p.k_splits) == (14, 2, 4), (m, g)
        assert p.build_waves == (2 if m <= 2 else 0)
    p = cg.codegemm_default_plan(cg.Desc.make(1, 8192, 28672, 8, 2))
    assert (p.waves, p.row_words, p.k_splits) == (16, 2, 4)                 # two codebooks, one scale per row: no gain measured
    p = cg.codegemm_default_plan(cg.Desc.make(1, 28672, 8192, 8, 2))
    assert (p.waves, p.row_words, p.k_splits) == (16, 2, 16)                # 16 x 16 = 256 already
    d = cg.Desc.make(1, 2048, 1000, 8, 2)
    assert cg.codegemm_workspace_bytes(d, cg.Plan.make(14, 2, 2, 1)) > 0
    assert cg.codegemm_workspace_bytes(d, cg.Plan.make(14, 1, 2, 1)) == 0   # only with two row words
    assert cg.codegemm_workspace_bytes(d, cg.Plan.make(14, 2, 2, 1, binding.PSUM_FP16)) == 0
    assert cg.codegemm_workspace_bytes(cg.Desc.make(8, 2048, 1000, 8, 2), cg.Plan.make(14, 2, 2, 4)) == 0
    assert cg.codegemm_workspace_bytes(cg.Desc.make(1, 2048, 1000, 8, 3), cg.Plan.make(14, 2, 2, 2)) == 0   # registers
    # build-only wavefronts: 16 wavefronts, two row words, one batch row, fp32 Psumbook, at most two codebooks
    assert cg.codegemm_workspace_bytes(d, cg.Plan.make(16, 2, 2, 1, 0, 2)) == FIXED + 2 * 1024 * 4
    assert cg.codegemm_workspace_bytes(d, cg.Plan.make(16, 1, 2, 1, 0, 2)) == 0
    assert cg.codegemm_workspace_bytes(d, cg.Plan.make(8, 2, 2, 1, 0, 2)) == 0
    assert cg.codegemm_workspace_bytes(d, cg.Plan.make(16, 2, 2, 1, 0, 1)) == 0
    assert cg.codegemm_workspace_bytes(d, cg.Plan.make(16, 2, 2, 1, binding.PSUM_FP16, 2)) == 0
    assert cg.codegemm_workspace_bytes(cg.Desc.make(2, 2048, 1000, 8, 2), cg.Plan.make(16, 2, 2, 2, 0, 2)) == 0
    assert cg.codegemm_workspace_bytes(cg.Desc.make(1, 2048, 1000, 8, 3), cg.Plan.make(16, 2, 2, 1, 0, 2)) == 0
    assert phases.workgroups(cg.Desc.make(1, 8192, 28672, 8, 2), cg.Plan.make(16, 2, 4, 1, 0, 2)) == 256
    # the batched kernel takes them with one or two row words
    d8 = cg.Desc.make(8, 2048, 1000, 8, 2)
    assert cg.codegemm_workspace_bytes(d8, cg.Plan.make(16, 1, 2, 4, 0, 2)) > 0
    assert cg.codegemm_workspace_bytes(d8, cg.Plan.make(16, 2, 2, 4, 0, 2)) > 0
    assert cg.codegemm_workspace_bytes(d8, cg.Plan.make(16, 4, 2, 4, 0, 2)) == 0
    assert cg.codegemm_workspace_bytes(d8, cg.Plan.make(8, 1, 2, 4, 0, 2)) == 0
    assert cg.codegemm_workspace_bytes(cg.Desc.make(8, 2048, 1000, 8, 3), cg.Plan.make(16, 1, 2, 4, 0, 2)) == 0
    # defaults: heights of 7 * 2^k rows at batch 4..32 get them, heights that 448 does not divide do not
    for B, want in ((4, (16, 1, 8, 2)), (8, (16, 2, 8, 2)), (16, (16, 2, 4, 2)), (32, (16, 2, 2, 2))):
        p = cg.codegemm_default_plan(cg.Desc.make(B, 4096, 14336, 8, 2))
        assert (p.waves, p.row_words, p.k_splits, p.build_waves) == want, (B, p)
    assert cg.codegemm_default_plan(cg.Desc.make(32, 14336, 4096, 8, 2)).build_waves == 0
    assert cg.codegemm_default_plan(cg.Desc.make(8, 8192, 28672, 8, 3)).build_waves == 0
    assert phases.workgroups(cg.Desc.make(1, 8192, 28672, 8, 2), cg.Plan.make(14, 2, 4, 1)) == 256
