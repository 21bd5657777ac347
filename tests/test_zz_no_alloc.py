"""codegemm_gemm_static (the entry point that allocates nothing) against codegemm_gemm:
same kernels, same order of every sum, so the outputs must be equal bit for bit; two calls
in a row, the second on a smaller layer, then a batched and a grouped-scale call, all
sharing the library's static workspace; a layer whose workspace exceeds the limit is refused."""
import numpy as np
import pytest
import torch

import oracle
import synth

pytestmark = pytest.mark.gpu

cg = pytest.importorskip("paper_2512_17970_amd")
from gpu_util import DeviceLayer, check_against_oracle, stream  # noqa: E402


def static_call(layer):
    y = layer.new_y()
    cg.codegemm_gemm_static(layer.desc, layer.plan, layer.x, layer.packed, layer.codebooks, layer.gemm_scales, y, stream())
    layer.check_guards("codegemm_gemm_static")
    return y


def test_static_workspace_entry_point_matches_the_workspace_one():
    cases = [synth.custom_case(8 * 32 * 9, 1500, 8, 2, 1, seed=901),            # several K ranges
             synth.custom_case(8 * 32 * 3, 300, 8, 2, 1, seed=902),             # smaller, right after
             synth.custom_case(4 * 32 * 5 + 8, 700, 4, 1, 6, seed=903),         # batched kernel, ragged K
             synth.custom_case(2048, 1030, 8, 2, 2, seed=904, g=64)]            # group scales
    plans = [cg.Plan.make(8, 2, 3, 1), cg.Plan.make(8, 1, 3, 1), None, None]
    layers = []
    for case, plan in zip(cases, plans):
        print(f"[static] {case.name} plan={plan}", flush=True)
        inp = synth.generate(case)
        layer = DeviceLayer(inp, plan=plan)
        assert layer.ws_bytes <= cg.codegemm_static_workspace_limit()
        y_static = static_call(layer)
        y_ws = layer.gemm()
        torch.cuda.synchronize()
        assert torch.equal(y_static, y_ws), case.name
        y_ref, T = oracle.gemm(inp.x, inp.codes, inp.codebooks, inp.scales)
        check_against_oracle(y_static.cpu().numpy(), y_ref, T, f"codegemm_gemm_static {case.name}")
        layers.append((layer, y_ws))
    # again, in reverse order, on the workspace the other shapes left behind
    for layer, y_ws in reversed(layers):
        y_again = static_call(layer)
        torch.cuda.synchronize()
        assert torch.equal(y_again, y_ws), layer.case.name


def test_static_workspace_limit_is_enforced():
    limit = cg.codegemm_static_workspace_limit()
    assert limit == 8 << 20
    d = cg.Desc.make(32, 8 * 32 * 64, 4096, 8, 2)
    plan = cg.Plan.make(16, 1, 64, 4)
    assert cg.codegemm_workspace_bytes(d, plan) > limit
    dummy = torch.zeros(64, dtype=torch.uint8, device="cuda")
    with pytest.raises(cg.CodegemmError) as e:
        cg.codegemm_gemm_static(d, plan, dummy, dummy, dummy, dummy, dummy, stream())
    assert e.value.status == -3
    with pytest.raises(cg.CodegemmError) as e:
        cg.codegemm_gemm_static(cg.Desc.make(1, 510, 512, 8, 1), None, dummy, dummy, dummy, dummy, dummy, stream())
    assert e.value.status == -1
