"""GPU parity: the HIP path, called through the C-ABI, against the CPU oracle."""
import numpy as np
import pytest
import torch

import oracle
import synth
from oracle.pack_layout import pack_reference

pytestmark = pytest.mark.gpu

cg = pytest.importorskip("paper_2512_17970_amd")
from gpu_util import DeviceLayer, Guarded, check_against_oracle, dev, stream  # noqa: E402


def say(msg):
    print(msg, flush=True)


def run_case(case, plan=None, y_fp32=False, dequant=True):
    say(f"[case] {case.name} seed={case.seed} plan={plan} y_fp32={y_fp32}")
    inp = synth.generate(case)
    y_ref, T = oracle.gemm(inp.x, inp.codes, inp.codebooks, inp.scales)
    layer = DeviceLayer(inp, plan=plan, y_fp32=y_fp32)
    y = layer.gemm()
    torch.cuda.synchronize()
    rel = check_against_oracle(y.cpu().numpy(), y_ref, T, f"codegemm_gemm {case.name}")
    # second call on the same workspace: the ticket counters must have been reset
    y2 = layer.gemm()
    torch.cuda.synchronize()
    assert torch.equal(y, y2), "second call differs (workspace not left ready / not deterministic)"
    if dequant:
        yd = layer.dequant()
        torch.cuda.synchronize()
        check_against_oracle(yd.cpu().numpy(), y_ref, T, f"codegemm_dequant_gemm {case.name}")
    return rel


SMALL = [
    # K, N, v, m, B : several tiles, ragged tails in N (not a multiple of 512 or 64) and in K (not a multiple of S*v)
    (512, 512, 8, 1, 1), (512, 512, 8, 2, 1), (1032, 1000, 8, 2, 1), (520, 63, 8, 2, 1), (8, 1, 8, 1, 1),
    (4 * 131, 700, 4, 1, 1), (2048, 1537, 4, 1, 1), (776, 515, 8, 3, 1), (264, 1025, 4, 4, 1),
    (1024, 600, 8, 2, 3), (4 * 67, 130, 4, 2, 5), (1536, 2100, 8, 1, 2),
    (16 * 70, 700, 16, 4, 1), (2048, 1030, 16, 3, 1), (16 * 33, 129, 16, 1, 1), (4096, 520, 16, 2, 2), (16 * 100, 300, 16, 4, 6),
]


@pytest.mark.parametrize("K,N,v,m,B", SMALL)
def test_small_shapes_default_plan(K, N, v, m, B):
    run_case(synth.custom_case(K, N, v, m, B, seed=4242 + K + N))


@pytest.mark.parametrize("y_fp32", [False, True])
def test_tiny_config(y_fp32):
    run_case(synth.workloads()[1][0], y_fp32=y_fp32)


def plan_ok(waves, row_words, m, bg=1):
    if waves == 14:                               # 448-row blocks: gather kernel for one or two batch rows
        return row_words == 2 and bg <= 2 and bg * m <= 4
    if bg == 4:                                   # the batched kernel
        return row_words <= 2 or waves == 8
    if row_words == 4:
        return waves == 16 and bg == 1 and m <= 2
    if row_words == 2:
        return bg * m <= (8 if waves == 8 else 4)
    return True


@pytest.mark.parametrize("waves,row_words", [(8, 1), (16, 1), (8, 2), (16, 2), (16, 4), (14, 2)])
@pytest.mark.parametrize("k_splits", [1, 2, 3, 4, 1000])
@pytest.mark.parametrize("v,m", [(8, 2), (4, 1), (8, 1), (4, 2), (8, 3), (4, 4), (8, 4), (4, 3), (16, 4), (16, 3), (16, 1)])
def test_every_plan_shape(v, m, k_splits, waves, row_words):
    if not plan_ok(waves, row_words, m):
        pytest.skip("plan not offered for this m")
    case = synth.custom_case(v * 200, 1300, v, m, 1, seed=99)
    run_case(case, plan=cg.Plan.make(waves, row_words, k_splits, 1), dequant=False)


@pytest.mark.parametrize("B,bg", [(2, 1), (2, 2), (2, 4), (3, 2), (3, 4), (4, 4), (5, 4), (8, 4), (8, 1), (32, 4), (7, 2)])
@pytest.mark.parametrize("v,m,waves,row_words,k_splits", [(8, 2, 8, 1, 2), (8, 2, 16, 2, 1), (4, 1, 8, 2, 1), (8, 3, 16, 1, 2),
                                                          (8, 1, 16, 2, 3), (8, 2, 16, 1, 3), (4, 1, 16, 1, 1), (8, 1, 8, 1, 2),
                                                          (8, 3, 8, 2, 1), (4, 3, 8, 1, 3), (8, 4, 16, 1, 2), (4, 4, 8, 2, 1),
                                                          (4, 2, 8, 2, 2), (8, 2, 16, 2, 2), (8, 2, 8, 4, 1), (4, 1, 8, 4, 2),
                                                          (8, 3, 16, 2, 1), (4, 4, 8, 4, 3), (16, 4, 16, 1, 2), (16, 3, 8, 2, 1),
                                                          (16, 1, 16, 2, 2), (8, 2, 14, 2, 2), (4, 1, 14, 2, 1), (16, 2, 14, 2, 3)])
def test_batch_groups(B, bg, v, m, waves, row_words, k_splits):
    if not plan_ok(waves, row_words, m, bg):
        pytest.skip("plan not offered for this m and batch group")
    case = synth.custom_case(v * 150, 1100, v, m, B, seed=98)
    run_case(case, plan=cg.Plan.make(waves, row_words, k_splits, bg), dequant=False)


@pytest.mark.parametrize("N", [448, 449, 447, 896 + 16, 3 * 448 + 130, 1, 17, 5000])
@pytest.mark.parametrize("v,m,g,B", [(8, 2, -1, 1), (8, 2, 128, 1), (4, 1, -1, 2), (8, 3, 32, 1), (16, 4, -1, 1)])
def test_448_row_blocks(N, v, m, g, B):
    """14-wavefront workgroups own 448 rows = 3.5 granules of the packed layout: row blocks that start and
    end in the middle of a granule, with ragged last blocks on either side of a block and a granule boundary."""
    unit = max(g, v * 32)
    case = synth.custom_case(unit * 3 + (g if g > 0 else v * 5), N, v, m, B, seed=1400 + N, g=g)
    run_case(case, plan=cg.Plan.make(14, 2, 2, B), dequant=False)


@pytest.mark.parametrize("k_splits", [1, 2, 3, 1000])
@pytest.mark.parametrize("v,m,g", [(8, 2, -1), (8, 1, -1), (4, 1, -1), (16, 2, -1), (8, 2, 128), (4, 1, 32), (8, 1, 8), (16, 1, 64), (4, 2, 4)])
def test_build_only_wavefronts(v, m, g, k_splits):
    """Plans with build_waves = 2: 14 wavefronts stream, gather and own 448 rows, 2 wavefronts build every Psumbook
    one unit ahead.  Ragged N (blocks that end inside a granule), K with a ragged last unit, odd and even numbers
    of units per workgroup (1, 2, 3, 5, 11 with the K splits above)."""
    unit = max(g, v * 32)
    for N, units in ((1300, 11), (448, 1), (449, 2), (31, 5)):
        K = unit * units + (g if g > 0 else v * 7)
        case = synth.custom_case(K, N, v, m, 1, seed=1500 + N + units, g=g)
        run_case(case, plan=cg.Plan.make(16, 2, k_splits, 1, 0, 2), dequant=False)


@pytest.mark.parametrize("row_words,k_splits", [(1, 1), (1, 3), (2, 2), (2, 1000)])
@pytest.mark.parametrize("v,m,g,B", [(8, 2, -1, 4), (8, 1, -1, 8), (4, 1, -1, 5), (16, 2, -1, 3), (8, 2, 128, 32), (4, 1, 32, 6), (8, 1, 8, 4), (4, 2, 4, 7)])
def test_build_only_wavefronts_batched(v, m, g, B, row_words, k_splits):
    """The batched kernel with build_waves = 2: 14 wavefronts own 448 (896) rows, 2 build every tile's Psumbook one
    tile ahead.  Ragged batch groups, ragged N and K, one to many tiles per workgroup."""
    unit = max(g, v * 32)
    for N, units in ((1900, 7), (896, 1), (450, 2)):
        K = unit * units + (g if g > 0 else v * 9)
        case = synth.custom_case(K, N, v, m, B, seed=1600 + N + units + B, g=g)
        run_case(case, plan=cg.Plan.make(16, row_words, k_splits, 4, 0, 2), dequant=False)


def test_batched_kernel_long_ragged_k():
    """Batch groups of 4 over a long K range with a ragged last unit and a ragged last row block."""
    for (v, m, waves, rw, splits, B) in [(8, 2, 16, 1, 1, 4), (8, 2, 8, 2, 2, 9), (4, 1, 16, 1, 1, 6), (8, 1, 8, 1, 3, 4),
                                         (8, 3, 8, 1, 1, 5), (8, 4, 16, 1, 2, 8), (4, 2, 8, 2, 1, 32), (8, 2, 16, 2, 1, 7), (8, 1, 8, 4, 2, 4),
                                         (8, 4, 16, 2, 3, 12)]:
        case = synth.custom_case(v * (32 * 21 + 5), 700, v, m, B, seed=96)
        run_case(case, plan=cg.Plan.make(waves, rw, splits, 4), dequant=False)


# Normalisation groups along K (Section 2.2, Step 1).  K is a multiple of g; shapes have ragged
# row blocks, several units per workgroup and groups smaller than, equal to and larger than a unit.
GROUPED = [
    # K, N, v, m, B, g
    (1024, 600, 8, 2, 1, 128), (1024, 600, 8, 2, 1, 8), (1024, 130, 8, 2, 1, 16), (2048, 515, 8, 2, 1, 32),
    (2048, 515, 8, 2, 1, 64), (1536, 300, 8, 2, 1, 256), (2048, 257, 8, 2, 1, 512), (4096, 129, 8, 2, 1, 1024),
    (768, 1000, 4, 1, 1, 128), (512, 700, 4, 1, 1, 4), (1024, 64, 4, 1, 1, 32), (1024, 333, 4, 1, 1, 256),
    (768, 520, 8, 1, 1, 16), (768, 520, 8, 3, 1, 128), (512, 300, 4, 4, 1, 8), (1024, 260, 8, 4, 1, 64),
    (1024, 600, 8, 2, 2, 128), (1024, 600, 8, 2, 3, 32), (1024, 600, 8, 2, 4, 128), (2048, 515, 8, 2, 7, 8),
    (768, 1000, 4, 1, 5, 128), (512, 700, 4, 1, 8, 4), (768, 520, 8, 3, 6, 64), (512, 300, 4, 4, 4, 16),
    (2048, 130, 8, 1, 9, 512), (1024, 1100, 8, 2, 32, 128),
    (2048, 515, 16, 3, 1, 32), (2048, 300, 16, 4, 1, 16), (4096, 200, 16, 3, 5, 128), (2048, 700, 16, 2, 1, 1024),
]


@pytest.mark.parametrize("K,N,v,m,B,g", GROUPED)
def test_group_scales_default_plan(K, N, v, m, B, g):
    run_case(synth.custom_case(K, N, v, m, B, seed=5150 + K + N + g, g=g))


@pytest.mark.parametrize("waves,row_words,bg", [(8, 1, 1), (16, 1, 1), (8, 2, 1), (16, 2, 1), (8, 2, 2), (16, 1, 2), (16, 2, 2),
                                                (16, 1, 4), (8, 1, 4), (8, 2, 4), (16, 2, 4), (8, 4, 4), (14, 2, 1), (14, 2, 2)])
@pytest.mark.parametrize("k_splits", [1, 3])
@pytest.mark.parametrize("v,m,g", [(8, 2, 128), (8, 2, 8), (4, 1, 32), (8, 3, 64), (4, 4, 16), (8, 1, 512)])
def test_group_scales_every_plan_shape(v, m, g, k_splits, waves, row_words, bg):
    if not plan_ok(waves, row_words, m, bg):
        pytest.skip("plan not offered for this m and batch group")
    B = {1: 1, 2: 3, 4: 6}[bg]
    case = synth.custom_case(max(g, v * 32) * 5, 1300, v, m, B, seed=93, g=g)
    run_case(case, plan=cg.Plan.make(waves, row_words, k_splits, bg), dequant=False)


def fp16_plan_ok(waves, row_words, g):
    return not (g > 0 and waves == 16 and row_words == 2)


@pytest.mark.parametrize("waves,row_words", [(8, 1), (16, 1), (8, 2), (16, 2)])
@pytest.mark.parametrize("k_splits", [1, 3])
@pytest.mark.parametrize("v,m,g", [(8, 2, -1), (4, 1, -1), (8, 1, -1), (8, 3, -1), (4, 4, -1), (16, 4, -1), (16, 3, -1), (4, 2, -1),
                                   (8, 2, 128), (8, 2, 8), (4, 1, 32), (8, 3, 64), (16, 2, 256)])
def test_fp16_psumbook_every_plan_shape(v, m, g, k_splits, waves, row_words):
    """The Psumbook stored as fp16 pairs (plan field psum_dtype = 1): every partial sum carries one more
    rounding of relative size 2^-11, which the acceptance bar (relative L2 <= 1e-3, per element
    <= 1e-2 sum|terms|) has room for; checked at that bar, on ragged shapes, for every block shape."""
    if not fp16_plan_ok(waves, row_words, g):
        pytest.skip("plan not offered with an fp16 Psumbook and group scales")
    case = synth.custom_case(max(g, v * 32) * 5 + (0 if g > 0 else v * 7), 1300, v, m, 1, seed=191, g=g)
    run_case(case, plan=cg.Plan.make(waves, row_words, k_splits, 1, cg.binding.PSUM_FP16), dequant=False)


def test_fp16_psumbook_is_exact_on_integer_partial_sums():
    """+-1 codebook and small integer x: every partial sum is an integer below 2048, which fp16 holds
    exactly, so the fp16 Psumbook must give the oracle's result bit for bit (fp32 output)."""
    v, K, N = 8, 4096, 1100
    rng = np.random.default_rng(23)
    i = np.arange(256)[:, None]
    case = synth.custom_case(K, N, v, 2, 1, seed=2)
    inp = synth.generate(case)
    inp.codebooks = np.stack([np.where((i >> np.arange(v)[None, :]) & 1, 1.0, -1.0), np.where((i >> np.arange(v)[None, :]) & 1, 2.0, 0.0)]).astype(np.float16)
    inp.x = rng.integers(-8, 9, (1, K)).astype(np.float16)
    inp.scales = np.ones(N, np.float16)
    y_ref, _ = oracle.gemm(inp.x, inp.codes, inp.codebooks, inp.scales)
    for waves, rw in ((8, 2), (16, 2), (16, 1)):
        layer = DeviceLayer(inp, plan=cg.Plan.make(waves, rw, 3, 1, cg.binding.PSUM_FP16), y_fp32=True)
        y = layer.gemm()
        torch.cuda.synchronize()
        assert np.array_equal(y.cpu().numpy().astype(np.float64), y_ref)


def test_pack_scales_matches_documented_layout():
    for (K, N, v, g) in [(1024, 300, 8, 128), (1024, 300, 8, 8), (2048, 129, 8, 1024), (512, 700, 4, 4), (640, 64, 4, 128)]:
        case = synth.custom_case(K, N, v, 1, 1, seed=8, g=g)
        inp = synth.generate(case)
        desc = cg.Desc.make(1, K, N, v, 1, g=g)
        say(f"[pack_scales] {case.name}")
        nbytes = cg.codegemm_packed_scales_bytes(desc)
        J = K // v
        NGR, NKT = -(-N // 128), -(-J // 32)
        GPU = max(1, 32 * v // g)
        assert nbytes == NGR * NKT * GPU * 256
        want = np.zeros((NGR, NKT, GPU, 16, 8), np.float16)      # the layout include/codegemm.h documents
        for rg in range(NGR):
            for kt in range(NKT):
                for q in range(GPU):
                    first = kt * 32 * v + q * g
                    if first >= K:
                        continue
                    rows = np.arange(128) + 128 * rg
                    ok = rows < N
                    blockvals = np.zeros(128, np.float16)
                    blockvals[ok] = inp.scales[rows[ok], first // g]
                    want[rg, kt, q] = blockvals.reshape(16, 8)
        guard = Guarded(nbytes)
        packed = guard.t
        cg.codegemm_pack_scales(desc, dev(inp.scales), packed, stream())
        torch.cuda.synchronize()
        assert guard.intact()
        got = packed.cpu().numpy().view(np.float16).reshape(want.shape)
        assert np.array_equal(got.view(np.uint16), want.view(np.uint16))


def test_many_units_per_workgroup():
    """A long K range per workgroup: the code ring wraps many times, with a ragged last tile."""
    for (v, m, waves, rw, splits) in [(8, 2, 8, 1, 1), (8, 2, 16, 2, 2), (4, 1, 8, 2, 1), (8, 4, 16, 1, 3), (8, 3, 8, 1, 1),
                                      (8, 2, 16, 4, 1)]:
        case = synth.custom_case(v * (32 * 37 + 5), 600, v, m, 1, seed=97)
        run_case(case, plan=cg.Plan.make(waves, rw, splits, 1), dequant=False)


def test_pack_matches_documented_layout_and_roundtrips():
    for (K, N, v, m) in [(8 * 100, 700, 8, 2), (4 * 77, 513, 4, 1), (8 * 40, 64, 8, 3), (8 * 33, 1030, 8, 4)]:
        case = synth.custom_case(K, N, v, m, 1, seed=7)
        inp = synth.generate(case)
        desc = cg.Desc.make(1, K, N, v, m)
        say(f"[pack] {case.name}")
        nbytes = cg.codegemm_packed_codes_bytes(desc, None)
        want = pack_reference(inp.codes)
        assert nbytes == want.size
        codes_d = dev(inp.codes)
        gp, gb = Guarded(nbytes), Guarded(inp.codes.size)
        packed = gp.t
        packed.fill_(0xAB)
        cg.codegemm_pack_codes(desc, None, codes_d, packed, stream())
        back = gb.view(torch.uint8, codes_d.shape)
        back.fill_(0xCD)
        cg.codegemm_unpack_codes(desc, None, packed, back, stream())
        torch.cuda.synchronize()
        assert gp.intact() and gb.intact()
        assert np.array_equal(packed.cpu().numpy(), want)
        assert torch.equal(back, codes_d)
        # the host versions give the same bytes as the device kernels
        host_packed = np.full(nbytes, 0xEE, np.uint8)
        cg.codegemm_pack_codes_host(desc, inp.codes, host_packed)
        assert np.array_equal(host_packed, packed.cpu().numpy())
        host_back = np.full_like(inp.codes, 0xDD)
        cg.codegemm_unpack_codes_host(desc, packed.cpu().numpy(), host_back)
        assert np.array_equal(host_back, inp.codes)


@pytest.mark.parametrize("use_mfma", [False, True])
@pytest.mark.parametrize("K,v,m,B", [(512, 8, 2, 1), (4 * 67, 4, 1, 3), (8 * 45, 8, 3, 9), (1024, 4, 4, 2), (16 * 37, 16, 3, 2), (1024, 16, 4, 5)])
def test_psumbook_build_eq2(K, v, m, B, use_mfma):
    case = synth.custom_case(K, 8, v, m, B, seed=5)
    say(f"[psumbook] {case.name} mfma={use_mfma}")
    inp = synth.generate(case)
    P_ref = oracle.psumbook(inp.x, inp.codebooks)
    desc = cg.Desc.make(B, K, 8, v, m)
    P = torch.full((B, m, K // v, 256), float("nan"), dtype=torch.float32, device="cuda")
    cg.codegemm_psumbook_build(desc, dev(inp.x), dev(inp.codebooks), P, use_mfma, stream())
    torch.cuda.synchronize()
    got = P.cpu().numpy().astype(np.float64)
    # fp16 products are exact in fp32; v-1 fp32 additions: error <= v * 2^-24 * sum|terms|
    bound = v * 2.0 ** -24 * np.einsum("bjk,cik->bcji", np.abs(inp.x.astype(np.float64)).reshape(B, -1, v),
                                       np.abs(inp.codebooks.astype(np.float64)))
    assert np.all(np.abs(got - P_ref) <= bound + 1e-30)


def test_psumbook_one_hot_is_exact_copy_of_x():
    v, K, B = 8, 8 * 96, 2
    rng = np.random.default_rng(3)
    x = rng.standard_normal((B, K)).astype(np.float16)
    cb = np.zeros((1, 256, v), np.float16)
    cb[0, np.arange(256), np.arange(256) % v] = 1.0
    desc = cg.Desc.make(B, K, 8, v, 1)
    for use_mfma in (False, True):
        P = torch.empty((B, 1, K // v, 256), dtype=torch.float32, device="cuda")
        cg.codegemm_psumbook_build(desc, dev(x), dev(cb), P, use_mfma, stream())
        torch.cuda.synchronize()
        want = x.astype(np.float32).reshape(B, K // v, v)[:, :, np.arange(256) % v]
        assert np.array_equal(P.cpu().numpy()[:, 0], want)


@pytest.mark.parametrize("lo", [-1.0, 0.0])
def test_sign_codebook_bit_exact(lo):
    """+-1 / {0,1} codebooks with small integer x: every partial sum is an exactly
    representable integer, so the fp32 result must equal the oracle bit for bit
    whatever the summation order."""
    v, K, N, B = 8, 8192, 2100, 2
    rng = np.random.default_rng(17)
    i = np.arange(256)[:, None]
    cb = np.where((i >> np.arange(v)[None, :]) & 1, 1.0, lo).astype(np.float16)[None]
    case = synth.custom_case(K, N, v, 1, B, seed=1)
    inp = synth.generate(case)
    inp.codebooks = cb
    inp.x = rng.integers(-8, 9, (B, K)).astype(np.float16)
    inp.scales = np.ones(N, np.float16)
    y_ref, _ = oracle.gemm(inp.x, inp.codes, inp.codebooks, inp.scales)
    layer = DeviceLayer(inp, y_fp32=True)
    y = layer.gemm()
    yd = layer.dequant()
    torch.cuda.synchronize()
    assert np.array_equal(y.cpu().numpy().astype(np.float64), y_ref)
    assert np.array_equal(yd.cpu().numpy().astype(np.float64), y_ref)


def test_diagnostic_build_gives_the_same_output_and_a_monotone_timeline():
    """The trace library must compute exactly what the production library computes, and every
    workgroup must pass its phases in order."""
    from paper_2512_17970_amd import phases
    for case, plan in ((synth.custom_case(8 * 32 * 6, 1500, 8, 2, 1, seed=71), cg.Plan.make(8, 2, 3, 1)),
                       (synth.custom_case(8 * 32 * 4, 1100, 8, 2, 6, seed=72), cg.Plan.make(16, 1, 2, 4))):
        say(f"[phases] {case.name} {plan}")
        inp = synth.generate(case)
        y_ref, T = oracle.gemm(inp.x, inp.codes, inp.codebooks, inp.scales)
        layer = DeviceLayer(inp, plan=plan)
        y_prod = layer.gemm()
        torch.cuda.synchronize()
        y = layer.new_y()
        rows = phases.phase_table(torch, layer.desc, layer.plan, layer.x, layer.packed, layer.codebooks, layer.gemm_scales,
                                  y, layer.ws, layer.ws_bytes, warmup=1)
        check_against_oracle(y.cpu().numpy(), y_ref, T, f"trace build {case.name}")
        assert torch.equal(y, y_prod)
        by = {r["phase"]: r for r in rows}
        n = phases.workgroups(layer.desc, layer.plan)
        # three K ranges go through ticket and partial sums, two through the pairwise words
        tail = ["partial sums issued", "partial sums acknowledged", "ticket drawn"] if plan.k_splits == 3 else \
               ["first pair add issued", "first pair add returned", "last pair add returned"]
        for name in ("kernel entered", "first Psumbook built", "streaming loop done", "row totals staged", tail[-1]):
            assert by[name]["workgroups"] == n, name
        assert by["output stored"]["workgroups"] == n // min(plan.k_splits, -(-case.J // 32))
        order = ["kernel entered", "prologue loads issued", "first Psumbook built", "streaming loop done",
                 "row totals staged"] + tail
        means = [by[k]["mean_us"] for k in order]
        assert means == sorted(means), means
        assert 0 < by["output stored"]["max_us"] < 1000


@pytest.mark.parametrize("B,K,N,v,m,g", [(70, 1024, 600, 8, 2, -1), (33, 4 * 200, 257, 4, 1, 32), (64, 2048, 130, 16, 3, -1)])
def test_batches_above_one_launch(B, K, N, v, m, g):
    """More than 32 batch rows: consecutive launches of up to 32 rows that share the workspace."""
    run_case(synth.custom_case(K, N, v, m, B, seed=606 + B, g=g))


@pytest.mark.parametrize("fill", [0, 255, 128])
def test_constant_codes_extreme_indices(fill):
    """Every code the same index (0, 255 and 128: the ends of the table and the sign bit of the code
    byte): all lanes of a half-wavefront read one Psumbook row, and the byte-permute address assembly
    sees its extreme values.  Batch 1, 2 (code words reused for a second Psumbook) and 5 (batched kernel)."""
    for (v, m, B) in [(8, 2, 1), (4, 1, 1), (8, 3, 2), (16, 4, 1), (8, 2, 5)]:
        case = synth.custom_case(v * 32 * 9 + v * 3, 777, v, m, B, seed=400 + fill)
        inp = synth.generate(case)
        inp.codes = np.full_like(inp.codes, fill)
        say(f"[constant codes {fill}] {case.name}")
        y_ref, T = oracle.gemm(inp.x, inp.codes, inp.codebooks, inp.scales)
        layer = DeviceLayer(inp)
        y = layer.gemm()
        torch.cuda.synchronize()
        check_against_oracle(y.cpu().numpy(), y_ref, T, f"constant codes {fill} {case.name}")


def test_wide_dynamic_range_inputs():
    """Activations and centroids spread over many binades (lognormal magnitudes, up to the top of the
    fp16 range for x): fp16 x fp16 products stay exact in fp32 and the fp32 sums must still meet the
    per-element bound; fp32 output, so that nothing overflows fp16 on the way out."""
    rng = np.random.default_rng(77)
    for (v, m, B, g) in [(8, 2, 1, -1), (4, 1, 1, 32), (8, 2, 4, -1), (16, 3, 1, -1)]:
        case = synth.custom_case(v * 32 * 12, 900, v, m, B, seed=78, g=g)
        inp = synth.generate(case)
        mag = np.exp(rng.normal(0.0, 3.0, inp.x.shape)).clip(2.0 ** -14, 60000.0)
        inp.x = (np.sign(rng.standard_normal(inp.x.shape)) * mag).astype(np.float16)
        cmag = np.exp(rng.normal(-4.0, 2.5, inp.codebooks.shape)).clip(2.0 ** -20, 8.0)
        inp.codebooks = (np.sign(rng.standard_normal(inp.codebooks.shape)) * cmag).astype(np.float16)
        say(f"[dynamic range] {case.name}")
        y_ref, T = oracle.gemm(inp.x, inp.codes, inp.codebooks, inp.scales)
        layer = DeviceLayer(inp, y_fp32=True)
        y = layer.gemm()
        torch.cuda.synchronize()
        got = y.cpu().numpy().astype(np.float64)
        assert np.all(np.isfinite(got))
        assert np.all(np.abs(got - y_ref) <= 1e-5 * T + 1e-30)           # fp32 accumulation: ~K*2^-24 of sum|terms| at worst
        for b in range(case.B):
            assert np.linalg.norm(got[b] - y_ref[b]) <= 1e-3 * np.linalg.norm(y_ref[b])
        yd = layer.dequant()
        torch.cuda.synchronize()
        assert np.all(np.abs(yd.cpu().numpy().astype(np.float64) - y_ref) <= 1e-5 * T + 1e-30)


def test_random_formats_shapes_and_plans():
    """Seeded random draws over the whole supported space: format (v, m, g), shape (ragged N and K),
    batch, and launch plan (any plan the library accepts for the format)."""
    rng = np.random.default_rng(20251217)
    done = 0
    while done < 60:
        v = int(rng.choice([4, 8, 16]))
        m = int(rng.integers(1, 5))
        B = int(rng.choice([1, 1, 1, 2, 3, 4, 5, 8, 13, 32]))
        g = int(rng.choice([-1, -1, v, 2 * v, 4 * v, 128, 256, 1024]))
        if g != -1 and g < v:
            g = v
        unit = max(g, v) if g != -1 else v
        K = unit * int(rng.integers(1, max(2, 6000 // unit)))
        N = int(rng.integers(1, 1400))
        bg = 1 if B == 1 else int(rng.choice([1, 2, 4]))
        plan = cg.Plan.make(int(rng.choice([8, 16, 14])), int(rng.choice([1, 2, 4])), int(rng.choice([1, 2, 3, 5, 64])), bg)
        desc = cg.Desc.make(B, K, N, v, m, g=g)
        if cg.codegemm_workspace_bytes(desc, plan) == 0:
            continue                                  # plan not offered for this format
        run_case(synth.custom_case(K, N, v, m, B, seed=7000 + done, g=g), plan=plan, dequant=(done % 4 == 0))
        done += 1


def test_random_shapes_with_build_only_wavefronts():
    """Seeded random draws over the plans with build_waves = 2 (one or two codebooks, batch group 1 or 4):
    ragged N against the 448- and 896-row blocks, ragged K, K ranges beyond the number of units."""
    rng = np.random.default_rng(20251218)
    done = 0
    while done < 30:
        v = int(rng.choice([4, 8, 16]))
        m = int(rng.integers(1, 3))
        B = int(rng.choice([1, 1, 3, 4, 7, 12, 32]))
        g = int(rng.choice([-1, -1, v, 4 * v, 128]))
        if g != -1 and g < v:
            g = v
        unit = max(g, v) if g != -1 else v
        K = unit * int(rng.integers(1, max(2, 5000 // unit)))
        N = int(rng.integers(1, 2000))
        bg = 1 if B == 1 else 4
        plan = cg.Plan.make(16, 2 if bg == 1 else int(rng.choice([1, 2])), int(rng.choice([1, 2, 3, 7, 64])), bg, 0, 2)
        desc = cg.Desc.make(B, K, N, v, m, g=g)
        if cg.codegemm_workspace_bytes(desc, plan) == 0:
            continue                                  # plan not offered for this format
        run_case(synth.custom_case(K, N, v, m, B, seed=8000 + done, g=g), plan=plan, dequant=False)
        done += 1


def test_one_workspace_serves_calls_of_different_shapes_and_plans():
    """A workspace that went through codegemm_workspace_init once is shared by calls with different
    shapes, K-range counts and kernels, interleaved and repeated: every call leaves its ticket
    counters at zero, wherever the next call puts its own."""
    jobs = []
    for (K, N, v, m, B, plan) in [
            (2048, 1300, 8, 2, 1, cg.Plan.make(8, 2, 8, 1)), (4096, 700, 8, 2, 1, cg.Plan.make(16, 2, 16, 1)),
            (1024, 2600, 4, 1, 1, cg.Plan.make(8, 1, 3, 1)), (2048, 900, 8, 2, 6, cg.Plan.make(16, 1, 5, 4)),
            (1536, 520, 8, 1, 2, cg.Plan.make(8, 2, 6, 2)), (2048, 1300, 8, 2, 1, None)]:
        case = synth.custom_case(K, N, v, m, B, seed=7000 + len(jobs))
        inp = synth.generate(case)
        y_ref, T = oracle.gemm(inp.x, inp.codes, inp.codebooks, inp.scales)
        jobs.append((case, DeviceLayer(inp, plan=plan), y_ref, T))
    nbytes = max(L.ws_bytes for _, L, _, _ in jobs)
    ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    cg.codegemm_workspace_init(ws, nbytes, stream())
    for rnd in range(3):
        order = jobs if rnd % 2 == 0 else jobs[::-1]
        for case, L, y_ref, T in order:
            say(f"[shared workspace] round {rnd} {case.name} plan={L.plan}")
            y = L.new_y()
            cg.codegemm_gemm(L.desc, L.plan, L.x, L.packed, L.codebooks, L.gemm_scales, y, ws, nbytes, stream())
            torch.cuda.synchronize()
            check_against_oracle(y.cpu().numpy(), y_ref, T, f"shared workspace {case.name}")
    # the counter area and the words of the pairwise reduction (the first 64 KB + 2 MB of every workspace) are all zero again
    assert int(ws[:65536 + (2 << 20)].to(torch.int64).sum().item()) == 0


def test_calls_replay_correctly_from_a_hip_graph():
    """codegemm_workspace_init and codegemm_gemm only launch kernels, so they can be captured; every
    replay must give the eager result (the ticket counters are back at zero after each call), with
    eager work and synchronisations between the replays."""
    for case in (synth.custom_case(2048, 1500, 8, 2, 1, seed=61), synth.custom_case(1024, 900, 4, 1, 5, seed=62),
                 synth.custom_case(2048, 700, 8, 2, 1, seed=63, g=128)):
        say(f"[graph] {case.name}")
        inp = synth.generate(case)
        y_ref, T = oracle.gemm(inp.x, inp.codes, inp.codebooks, inp.scales)
        layer = DeviceLayer(inp)
        y_eager = layer.gemm()
        torch.cuda.synchronize()
        ys = [layer.new_y() for _ in range(3)]
        g = torch.cuda.CUDAGraph()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            with torch.cuda.graph(g, stream=side):
                cg.codegemm_workspace_init(layer.ws, layer.ws_bytes, stream())
                for y in ys:
                    layer.gemm(y, check=False)
        torch.cuda.current_stream().wait_stream(side)
        for rep in range(3):
            for y in ys:
                y.fill_(float("nan"))
            g.replay()
            layer.check_guards(f"graph replay {rep}")
            for y in ys:
                assert torch.equal(y, y_eager), f"replay {rep} differs from the eager call"
            z = layer.gemm()                              # eager work between replays, same workspace
            torch.cuda.synchronize()
            assert torch.equal(z, y_eager)
        check_against_oracle(ys[0].cpu().numpy(), y_ref, T, f"graph replay {case.name}")


def test_error_paths():
    d = cg.Desc.make(1, 512, 512, 8, 1)
    t = torch.zeros(1 << 20, dtype=torch.uint8, device="cuda")
    with pytest.raises(cg.CodegemmError):
        cg.codegemm_gemm(cg.Desc.make(1, 510, 512, 8, 1), None, t, t, t, t, t, t, 1 << 20)       # K % v
    with pytest.raises(cg.CodegemmError):
        cg.codegemm_gemm(cg.Desc.make(1, 512, 512, 32, 1), None, t, t, t, t, t, t, 1 << 20)      # v
    with pytest.raises(cg.CodegemmError):
        cg.codegemm_gemm(d, None, t, t, t, t, t, t, 16)                                          # workspace
    with pytest.raises(cg.CodegemmError):
        cg.codegemm_gemm(d, None, None, t, t, t, t, t, 1 << 20)                                  # NULL
    with pytest.raises(cg.CodegemmError):
        cg.codegemm_gemm(d, cg.Plan.make(12, 1, 4), t, t, t, t, t, t, 1 << 20)                   # plan
    for g in (12, 4, 48):                                                                        # g not v * 2^i, g < v, g not dividing K
        assert cg.codegemm_packed_scales_bytes(cg.Desc.make(1, 512 if g != 48 else 8 * 40, 512, 8, 2, g=g)) == 0
    with pytest.raises(cg.CodegemmError):
        cg.codegemm_gemm(d, None, t[1:], t, t, t, t, t, 1 << 20)                                 # alignment
