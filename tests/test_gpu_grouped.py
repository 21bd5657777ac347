"""GPU parity of codegemm_gemm_grouped: several layers that share x in one launch.
Every member's y is compared with the CPU oracle (the acceptance bar) and, bit for bit,
with codegemm_gemm on that layer alone under the same plan."""
import numpy as np
import pytest
import torch

import oracle
import synth

pytestmark = pytest.mark.gpu

cg = pytest.importorskip("paper_2512_17970_amd")
from gpu_util import DeviceLayer, Guarded, check_against_oracle, dev, stream  # noqa: E402


def run_group(K, Ns, v, m, B, g, plan=None, seed=7000, y_fp32=False):
    total = sum(Ns)
    desc = cg.Desc.make(B, K, total, v, m, y_fp32=y_fp32, g=g)
    if plan is None:
        plan = cg.codegemm_default_plan(desc)
    print(f"[grouped] K={K} Ns={Ns} v={v} m={m} B={B} g={g} {plan}", flush=True)
    inps = [synth.generate(synth.custom_case(K, n, v, m, B, seed=seed + i, g=g)) for i, n in enumerate(Ns)]
    x = inps[0].x
    layers = []
    for inp in inps:
        inp.x = x                                            # the layers of a group read the same activations
        layers.append(DeviceLayer(inp, plan=plan, y_fp32=y_fp32))
    ws_bytes = cg.codegemm_grouped_workspace_bytes(desc, plan, Ns)
    assert ws_bytes > 0
    ws = Guarded(ws_bytes)
    cg.codegemm_workspace_init(ws.t, ws_bytes, stream())
    ys = [l.new_y() for l in layers]
    members = [(n, l.packed, l.codebooks, l.gemm_scales, y) for n, l, y in zip(Ns, layers, ys)]
    for rep in range(2):                                     # the second call reuses the workspace as the first left it
        cg.codegemm_gemm_grouped(desc, plan, layers[0].x, members, ws.t, ws_bytes, stream())
        torch.cuda.synchronize()
        assert ws.intact(), "bytes outside the grouped workspace were written"
        for l, y, inp in zip(layers, ys, inps):
            l.check_guards("grouped launch")
            y_ref, T = oracle.gemm(x, inp.codes, inp.codebooks, inp.scales)
            check_against_oracle(y.cpu().numpy(), y_ref, T, f"grouped member N={inp.case.N}")
            alone = l.gemm()
            torch.cuda.synchronize()
            assert torch.equal(alone, y), f"member N={inp.case.N} differs from the single-layer call (call {rep})"
    return plan


@pytest.mark.parametrize("K,Ns,v,m,B,g", [
    (1024, (512, 128, 128), 8, 2, 1, -1),          # q, k, v of a small block
    (1024, (384, 384), 8, 2, 1, -1),               # gate and up
    (1000, (200, 72, 136, 8), 8, 1, 1, -1),        # four members, ragged N and K
    (2048, (640, 256), 4, 1, 2, -1),               # two batch rows
    (1024, (520, 130, 130), 8, 2, 1, 128),         # group scales
    (2048, (300, 300), 16, 3, 1, 32),
    (512, (4096,), 8, 2, 1, -1),                   # a group of one
])
def test_grouped_small(K, Ns, v, m, B, g):
    run_group(K, list(Ns), v, m, B, g)


@pytest.mark.parametrize("waves,row_words,k_splits,psum,build", [(8, 1, 3, 0, 0), (16, 1, 2, 0, 0), (16, 2, 4, 0, 0), (8, 2, 1, 0, 0), (8, 1, 2, 1, 0),
                                                                  (14, 2, 3, 0, 0), (16, 2, 3, 0, 2), (16, 2, 1, 0, 2)])
def test_grouped_plans(waves, row_words, k_splits, psum, build):
    """Explicit plans: block heights of 128..512 rows, with and without a split of K, members whose
    heights are not multiples of the block, fp16 Psumbook."""
    plan = cg.Plan.make(waves, row_words, k_splits, 1, psum, build)
    run_group(2048, [700, 130, 260], 8, 2, 1, -1, plan=plan, seed=7100 + waves + row_words)


@pytest.mark.parametrize("K,Ns,v,m,B,g,plan", [
    (1024, (512, 200, 130), 8, 2, 4, -1, None),
    (2048, (700, 260), 8, 2, 7, -1, (8, 1, 3, 4)),         # ragged batch group, K split
    (1024, (1100, 1030), 8, 2, 8, -1, (16, 2, 2, 4)),      # 1024-row blocks
    (2048, (300, 520, 8), 4, 1, 32, 128, None),            # group scales, a full launch of batch rows
    (1024, (384, 384), 16, 3, 5, -1, None),
    (2048, (900, 450, 130), 8, 2, 6, -1, (16, 1, 2, 4, 0, 2)),     # 14 gathering + 2 building wavefronts
    (1024, (1000, 896), 4, 1, 8, 32, (16, 2, 1, 4, 0, 2)),
])
def test_grouped_batched_kernel(K, Ns, v, m, B, g, plan):
    """Groups through the batched kernel (4 batch rows per pass)."""
    pl = run_group(K, list(Ns), v, m, B, g, plan=None if plan is None else cg.Plan.make(*plan), seed=7200 + B)
    assert pl.batch_group == 4, pl


@pytest.mark.parametrize("plan", [(8, 1, 4, 1), (16, 2, 4, 2), (16, 2, 2, 1)])
def test_grouped_and_single_calls_agree_across_reduction_protocols(plan):
    """Two or four K ranges are combined pairwise through 64-bit words when the words of the launch fit into their
    fixed area, else by ticket and partial sums.  Here each member alone fits and the group does not (two batch
    rows, 2 x 3 x 8 bytes per padded row with four ranges): the bits must agree all the same."""
    Ns = [40000, 40000] if plan[2] == 4 else [70000, 70000]
    run_group(1024, Ns, 8, 1, 2, -1, plan=cg.Plan.make(*plan), seed=7300)


def test_grouped_null_plan_is_the_default_plan_of_the_sum():
    K, Ns = 2048, [900, 300, 300]
    desc = cg.Desc.make(1, K, sum(Ns), 8, 2)
    plan = cg.codegemm_default_plan(desc)
    inps = [synth.generate(synth.custom_case(K, n, 8, 2, 1, seed=7400 + i)) for i, n in enumerate(Ns)]
    layers = []
    for inp in inps:
        inp.x = inps[0].x
        layers.append(DeviceLayer(inp, plan=plan))
    ws_bytes = cg.codegemm_grouped_workspace_bytes(desc, None, Ns)
    assert ws_bytes == cg.codegemm_grouped_workspace_bytes(desc, plan, Ns) > 0
    ws = Guarded(ws_bytes)
    cg.codegemm_workspace_init(ws.t, ws_bytes, stream())
    out = {}
    for which in (None, plan):
        ys = [l.new_y() for l in layers]
        cg.codegemm_gemm_grouped(desc, which, layers[0].x, [(n, l.packed, l.codebooks, l.gemm_scales, y) for n, l, y in zip(Ns, layers, ys)],
                                 ws.t, ws_bytes, stream())
        torch.cuda.synchronize()
        out[which is None] = ys
    for a, b_, inp in zip(out[True], out[False], inps):
        assert torch.equal(a, b_)
        y_ref, T = oracle.gemm(inp.x, inp.codes, inp.codebooks, inp.scales)
        check_against_oracle(a.cpu().numpy(), y_ref, T, "grouped, NULL plan")
    assert ws.intact()


def test_grouped_launch_replays_from_a_hip_graph():
    """The grouped call only launches a kernel, so it can be captured; every replay gives the eager bits,
    with eager grouped and single-layer calls on the same workspace between the replays."""
    K, Ns = 2048, [700, 260, 130]
    desc = cg.Desc.make(1, K, sum(Ns), 8, 2)
    plan = cg.Plan.make(8, 2, 4, 1)
    inps = [synth.generate(synth.custom_case(K, n, 8, 2, 1, seed=7500 + i)) for i, n in enumerate(Ns)]
    layers = []
    for inp in inps:
        inp.x = inps[0].x
        layers.append(DeviceLayer(inp, plan=plan))
    ws_bytes = max(cg.codegemm_grouped_workspace_bytes(desc, plan, Ns), max(l.ws_bytes for l in layers))
    ws = Guarded(ws_bytes)
    cg.codegemm_workspace_init(ws.t, ws_bytes, stream())

    def call(ys):
        cg.codegemm_gemm_grouped(desc, plan, layers[0].x, [(n, l.packed, l.codebooks, l.gemm_scales, y) for n, l, y in zip(Ns, layers, ys)],
                                 ws.t, ws_bytes, stream())

    eager = [l.new_y() for l in layers]
    call(eager)
    torch.cuda.synchronize()
    for y, inp in zip(eager, inps):
        y_ref, T = oracle.gemm(inp.x, inp.codes, inp.codebooks, inp.scales)
        check_against_oracle(y.cpu().numpy(), y_ref, T, "grouped, eager")
    outs = [[torch.full_like(y, float("nan")) for y in eager] for _ in range(2)]
    g = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(g, stream=side):
            for ys in outs:
                call(ys)
    torch.cuda.current_stream().wait_stream(side)
    for rep in range(3):
        for ys in outs:
            for y in ys:
                y.fill_(float("nan"))
        g.replay()
        torch.cuda.synchronize()
        assert ws.intact()
        for ys in outs:
            for y, e in zip(ys, eager):
                assert torch.equal(y, e), f"replay {rep} differs from the eager grouped call"
        # eager work on the same workspace between the replays: a single layer, then the group again
        l = layers[rep % len(layers)]
        z = l.new_y()
        cg.codegemm_gemm(l.desc, plan, l.x, l.packed, l.codebooks, l.gemm_scales, z, ws.t, ws_bytes, stream())
        again = [torch.full_like(y, float("nan")) for y in eager]
        call(again)
        torch.cuda.synchronize()
        assert torch.equal(z, eager[rep % len(layers)])
        for y, e in zip(again, eager):
            assert torch.equal(y, e)


def test_grouped_fp32_output():
    run_group(1024, [256, 384], 8, 2, 1, -1, y_fp32=True)


@pytest.mark.parametrize("K,Ns,g", [(8192, (8192, 1024, 1024), -1), (8192, (28672, 28672), -1), (8192, (8192, 1024, 1024), 128),
                                    (8192, (28672, 28672), 128)])
def test_grouped_at_70b_decoder_block(K, Ns, g):
    """The q/k/v and gate/up groups of the Llama-3-70B decoder block at full size, default plan of the summed height."""
    run_group(K, list(Ns), 8, 2, 1, g, seed=7300)


def test_grouped_rejects_bad_arguments():
    desc = cg.Desc.make(1, 1024, 768, 8, 2)
    plan = cg.codegemm_default_plan(desc)
    assert cg.codegemm_grouped_workspace_bytes(desc, plan, [512, 128]) == 0            # sum != out_features
    assert cg.codegemm_grouped_workspace_bytes(desc, plan, [512, 128, 64, 32, 32]) == 0  # five members
    assert cg.codegemm_grouped_workspace_bytes(desc, plan, [512, 256]) > 0
    d64 = cg.Desc.make(64, 1024, 768, 8, 2)
    assert cg.codegemm_grouped_workspace_bytes(d64, cg.Plan.make(8, 1, 1, 4), [512, 256]) == 0   # more rows than one launch takes
    buf = torch.zeros(1 << 20, dtype=torch.uint8, device="cuda")
    with pytest.raises(cg.CodegemmError):
        cg.codegemm_gemm_grouped(desc, plan, buf, [(512, buf, buf, buf, buf), (128, buf, buf, buf, buf)], buf, buf.numel(), stream())
    with pytest.raises(cg.CodegemmError):                                                  # workspace too small
        cg.codegemm_gemm_grouped(desc, plan, buf, [(512, buf, buf, buf, buf), (256, buf, buf, buf, buf)], buf, 64, stream())
    with pytest.raises(cg.CodegemmError):                                                  # null member pointer
        cg.codegemm_gemm_grouped(desc, plan, buf, [(512, buf, None, buf, buf), (256, buf, buf, buf, buf)], buf, buf.numel(), stream())
    torch.cuda.synchronize()
