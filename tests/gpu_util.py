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


GUARD = 4096          # bytes of canary on each side of every buffer a kernel writes
PATTERN = 0xA5


class Guarded:
    """A device buffer of `nbytes` bytes between two canary bands.  `.t` is the uint8 view the
    library sees (16-byte aligned: the allocation is, and the band is a multiple of 16)."""

    def __init__(self, nbytes: int):
        self.raw = torch.full((nbytes + 2 * GUARD,), PATTERN, dtype=torch.uint8, device="cuda")
        self.t = self.raw[GUARD:GUARD + nbytes]
        self.nbytes = nbytes

    def view(self, dtype, shape):
        return self.t.view(dtype).view(shape)

    def intact(self) -> bool:
        lo, hi = self.raw[:GUARD], self.raw[GUARD + self.nbytes:]
        return bool((lo == PATTERN).all().item()) and bool((hi == PATTERN).all().item())


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
        # Every buffer a kernel writes sits between canary bands that are checked after each call:
        # the kernels store y, the partial sums and the packed arrays through raw pointers.
        self.guards = {}
        self.gemm_scales = self.scales                     # what codegemm_gemm takes
        if c.g > 0:
            self.guards["packed scales"] = Guarded(cg.codegemm_packed_scales_bytes(self.desc))
            self.gemm_scales = self.guards["packed scales"].t
            cg.codegemm_pack_scales(self.desc, self.scales, self.gemm_scales, stream())
        self.guards["packed codes"] = Guarded(cg.codegemm_packed_codes_bytes(self.desc, self.plan))
        self.packed = self.guards["packed codes"].t
        cg.codegemm_pack_codes(self.desc, self.plan, self.codes, self.packed, stream())
        self.ws_bytes = cg.codegemm_workspace_bytes(self.desc, self.plan)
        self.guards["workspace"] = Guarded(self.ws_bytes)
        self.ws = self.guards["workspace"].t
        cg.codegemm_workspace_init(self.ws, self.ws_bytes, stream())
        self.check_guards("set-up")

    def check_guards(self, after: str):
        torch.cuda.synchronize()
        for name, g in self.guards.items():
            assert g.intact(), f"{name}: bytes outside the buffer were written ({after}, {self.case.name}, {self.plan})"

    def new_y(self, poison=True):
        dtype = torch.float32 if self.y_fp32 else torch.float16
        g = Guarded(self.case.B * self.case.N * (4 if self.y_fp32 else 2))
        y = g.view(dtype, (self.case.B, self.case.N))
        if poison:
            y.fill_(float("nan"))
        self.guards[f"y@{y.data_ptr():x}"] = g
        return y

    def _forget_other_outputs(self, y):
        for k in [k for k in self.guards if k.startswith("y@") and k != f"y@{y.data_ptr():x}"]:
            del self.guards[k]

    def gemm(self, y=None, check=True):
        """check=False: only enqueue (for calls recorded into a HIP graph, where nothing may
        synchronise); the caller runs check_guards() after the replay."""
        y = self.new_y() if y is None else y
        if check:
            self._forget_other_outputs(y)
        cg.codegemm_gemm(self.desc, self.plan, self.x, self.packed, self.codebooks, self.gemm_scales, y,
                         self.ws, self.ws_bytes, stream())
        if check:
            self.check_guards("codegemm_gemm")
        return y

    def dequant(self, y=None):
        y = self.new_y() if y is None else y
        self._forget_other_outputs(y)
        cg.codegemm_dequant_gemm(self.desc, self.x, self.codes, self.codebooks, self.scales, y, stream())
        self.check_guards("codegemm_dequant_gemm")
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
