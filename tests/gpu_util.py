"""Helpers for the GPU tests: move seeded inputs to the device and call the
C-ABI through the Python binding.  No arithmetic of the method lives here."""
from __future__ import annotations

import numpy as np
import torch

import paper_2512_17970_amd as cg


def dev(a: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def stream() -> int:
    return torch.cuda.current_stream().cuda_stream


class DeviceLayer:
    """A quantized layer resident on the GPU: canonical + packed codes, workspace."""

    def __init__(self, inp, plan=None, y_fp32=False):
        c = inp.case
        self.case = c
        self.desc = cg.Desc.make(c.B, c.K, c.N, c.v, c.m, y_fp32=y_fp32, g=c.g)
        self.plan = plan if plan is not None else cg.codegemm_default_plan(self.desc)
        self.y_fp32 = y_fp32
        self.x = dev(inp.x)
        self.codes = dev(inp.codes)
        self.codebooks = dev(inp.codebooks)
        self.scales = dev(inp.scales)                      # canonical: [N] or [N][K/g]
        self.gemm_scales = self.scales                     # what codegemm_gemm takes
        if c.g > 0:
            self.gemm_scales = torch.empty(cg.codegemm_packed_scales_bytes(self.desc), dtype=torch.uint8, device="cuda")
            cg.codegemm_pack_scales(self.desc, self.scales, self.gemm_scales, stream())
        self.packed = torch.empty(cg.codegemm_packed_codes_bytes(self.desc, self.plan), dtype=torch.uint8, device="cuda")
        cg.codegemm_pack_codes(self.desc, self.plan, self.codes, self.packed, stream())
        self.ws_bytes = cg.codegemm_workspace_bytes(self.desc, self.plan)
        self.ws = torch.empty(self.ws_bytes, dtype=torch.uint8, device="cuda")
        cg.codegemm_workspace_init(self.ws, self.ws_bytes, stream())

    def new_y(self, poison=True):
        y = torch.empty((self.case.B, self.case.N), dtype=torch.float32 if self.y_fp32 else torch.float16, device="cuda")
        if poison:
            y.fill_(float("nan"))
        return y

    def gemm(self, y=None):
        y = self.new_y() if y is None else y
        cg.codegemm_gemm(self.desc, self.plan, self.x, self.packed, self.codebooks, self.gemm_scales, y,
                         self.ws, self.ws_bytes, stream())
        return y

    def dequant(self, y=None):
        y = self.new_y() if y is None else y
        cg.codegemm_dequant_gemm(self.desc, self.x, self.codes, self.codebooks, self.scales, y, stream())
        return y


def check_against_oracle(y_gpu: np.ndarray, y_ref: np.ndarray, T: np.ndarray, what: str = ""):
    """The acceptance bar: per output vector relative L2 <= 1e-3 and per element
    |error| <= 1e-2 * sum|terms|."""
    y = y_gpu.astype(np.float64)
    assert np.all(np.isfinite(y)), f"{what}: non-finite output"
    err = np.abs(y - y_ref)
    for b in range(y.shape[0]):
        denom = np.linalg.norm(y_ref[b])
        rel = np.linalg.norm(y[b] - y_ref[b]) / denom if denom > 0 else np.linalg.norm(y[b])
        assert rel <= 1e-3, f"{what}: batch row {b} relative L2 {rel:.3e} > 1e-3"
    bad = err > 1e-2 * T + 1e-30
    assert not bad.any(), f"{what}: {bad.sum()} elements exceed 1e-2*sum|terms| (max err {err.max():.3e})"
    return float(max(np.linalg.norm(y[b] - y_ref[b]) / max(np.linalg.norm(y_ref[b]), 1e-300) for b in range(y.shape[0])))
