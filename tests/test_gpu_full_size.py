"""GPU parity at the full sizes of the five workload families, in the launch
configuration bench.py times (default plan), every output element against the
CPU oracle."""
import numpy as np
import pytest
import torch

import oracle
import synth

pytestmark = pytest.mark.gpu

cg = pytest.importorskip("paper_2512_17970_amd")
from gpu_util import DeviceLayer, check_against_oracle  # noqa: E402

ALL = [c for cases in synth.workloads().values() for c in cases]


@pytest.mark.parametrize("case", ALL, ids=[c.name for c in ALL])
def test_full_size_default_plan(case):
    print(f"[full] {case.name} seed={case.seed}", flush=True)
    inp = synth.generate(case)
    y_ref, T = oracle.gemm(inp.x, inp.codes, inp.codebooks, inp.scales)
    layer = DeviceLayer(inp)
    print(f"[full] plan {layer.plan}", flush=True)
    y = layer.gemm()
    torch.cuda.synchronize()
    rel = check_against_oracle(y.cpu().numpy(), y_ref, T, f"codegemm_gemm {case.name}")
    assert rel < 6e-4, f"relative L2 {rel:.2e} is above what fp16 output rounding explains"
    # bit-reproducible: a second call on the same workspace gives the same bits
    y2 = layer.gemm()
    torch.cuda.synchronize()
    assert torch.equal(y, y2)
    if case.B == 1:
        yd = layer.dequant()
        torch.cuda.synchronize()
        check_against_oracle(yd.cpu().numpy(), y_ref, T, f"codegemm_dequant_gemm {case.name}")


@pytest.mark.parametrize("B,expect", [(2, (16, 2, 4)), (4, (16, 2, 4))])
def test_small_batch_on_a_large_matrix_takes_the_batched_kernel(B, expect):
    """Default plan for 2 and 4 batch rows at 8192 -> 28672: the batched kernel with 1024-row blocks."""
    case = synth.custom_case(8192, 28672, 8, 2, B, seed=4100 + B)
    inp = synth.generate(case)
    y_ref, T = oracle.gemm(inp.x, inp.codes, inp.codebooks, inp.scales)
    layer = DeviceLayer(inp)
    assert (layer.plan.waves, layer.plan.row_words, layer.plan.batch_group) == expect, layer.plan
    y = layer.gemm()
    torch.cuda.synchronize()
    rel = check_against_oracle(y.cpu().numpy(), y_ref, T, f"batch {B} default plan")
    assert rel < 6e-4


def test_fp32_output_accuracy_at_70b_shape():
    """With fp32 output only fp32 accumulation error is left: relative L2 ~1e-6."""
    case = synth.find_case("c3_8192x28672_v8m2_b1")
    inp = synth.generate(case)
    y_ref, T = oracle.gemm(inp.x, inp.codes, inp.codebooks, inp.scales)
    layer = DeviceLayer(inp, y_fp32=True)
    y = layer.gemm()
    torch.cuda.synchronize()
    got = y.cpu().numpy().astype(np.float64)
    rel = np.linalg.norm(got - y_ref) / np.linalg.norm(y_ref)
    assert rel < 5e-6, rel
    assert np.all(np.abs(got - y_ref) <= 4e-6 * T)


def test_skewed_codes_at_70b_shape():
    """Zipf-distributed codes (the shape trained codebooks have) instead of uniform ones."""
    case = synth.find_case("c3_8192x8192_v8m2_b1")
    inp = synth.generate(case)
    inp.codes = synth.skewed_codes(case)
    y_ref, T = oracle.gemm(inp.x, inp.codes, inp.codebooks, inp.scales)
    layer = DeviceLayer(inp)
    y = layer.gemm()
    torch.cuda.synchronize()
    check_against_oracle(y.cpu().numpy(), y_ref, T, "skewed codes")


@pytest.mark.parametrize("name", ["c3_8192x8192_v8m2_b1", "c3_8192x1024_v8m2_b1", "c3_8192x28672_v8m2_b1", "c3_28672x8192_v8m2_b1",
                                  "c5_8192x28672_v8m3_b1", "c2_4096x14336_v4m1_b1", "c8_8192x28672_v8m2g128_b1"])
def test_fp16_psumbook_at_full_size(name):
    """The fp16 Psumbook option at the graded shapes, with the default block shape: the acceptance bar, and
    relative L2 below 6e-4 (fp16 rounding of the partial sums and of y together predict about 4e-4)."""
    case = synth.find_case(name)
    inp = synth.generate(case)
    y_ref, T = oracle.gemm(inp.x, inp.codes, inp.codebooks, inp.scales)
    d = cg.Desc.make(case.B, case.K, case.N, case.v, case.m, g=case.g)
    p = cg.codegemm_default_plan(d)
    waves = 16 if p.waves == 14 else p.waves            # the fp16 Psumbook pairs up 8 or 16 wavefronts
    rw = 1 if (case.g > 0 and waves == 16) else p.row_words
    plan = cg.Plan.make(waves, rw, p.k_splits, 1, cg.binding.PSUM_FP16)
    layer = DeviceLayer(inp, plan=plan)
    print(f"[fp16 psumbook] {case.name} {layer.plan}", flush=True)
    y = layer.gemm()
    torch.cuda.synchronize()
    rel = check_against_oracle(y.cpu().numpy(), y_ref, T, f"fp16 Psumbook {case.name}")
    print(f"[fp16 psumbook] relative L2 {rel:.2e}", flush=True)
    assert rel < 6e-4
    y2 = layer.gemm()
    torch.cuda.synchronize()
    assert torch.equal(y, y2)
