"""Where a codegemm_gemm call spends its time: runs the call in the diagnostic build of
the library (libcodegemm_trace.so, see include/codegemm_trace.h) and turns the clock
stamps of its workgroups into a phase table.  Measurement tooling: argument marshalling
and statistics only, every step of the path still runs in the HIP kernels."""
from __future__ import annotations

import ctypes
import os
from typing import Dict, List, Optional

from . import binding

TRACE_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libcodegemm_trace.so")
SLOTS = 24
TICK_US = 0.01                                     # the stamps count a 100 MHz clock

PHASES = [  # (slot, label), in the order a workgroup passes them
    (0, "kernel entered"), (2, "prologue loads issued"), (1, "first Psumbook built"),
    (8, "unit 0 gathered"), (9, "unit 1 gathered"), (10, "unit 2 gathered"), (11, "unit 3 gathered"),
    (12, "unit 4 gathered"), (13, "unit 5 gathered"), (14, "unit 6 gathered"), (15, "last unit gathered"),
    (4, "streaming loop done"), (16, "row totals staged"), (17, "staging barrier passed"),
    (5, "partial sums issued"), (6, "partial sums acknowledged"), (7, "ticket drawn"),
    (18, "first pair add issued"), (19, "first pair add returned"), (20, "last pair add returned"), (3, "output stored"),
]


def _trace_lib() -> ctypes.CDLL:
    if not os.path.exists(TRACE_LIB_PATH):
        raise ImportError(f"{TRACE_LIB_PATH} is missing: build it with python paper_2512_17970_amd/build.py")
    lib = ctypes.CDLL(TRACE_LIB_PATH)
    vp, i, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t
    dp, pp = ctypes.POINTER(binding.Desc), ctypes.POINTER(binding.Plan)
    lib.codegemm_gemm.argtypes = [dp, pp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.codegemm_gemm.restype = i
    lib.codegemm_set_trace.argtypes = [vp]
    lib.codegemm_set_trace.restype = None
    return lib


def workgroups(desc: binding.Desc, plan: binding.Plan) -> int:
    """Workgroups of one batch group under `plan` (row blocks x K ranges)."""
    J = desc.in_features // desc.vec_len
    ngr, nkt = -(-desc.out_features // 128), -(-J // 32)
    rows = plan.row_words * (plan.waves - plan.build_waves) * (32 if plan.batch_group == 4 else 16)     # rows of one workgroup
    nblk = -(-ngr * 128 // rows)
    nks = min(plan.k_splits, nkt)
    kpw = -(-nkt // nks)
    return nblk * -(-nkt // kpw)


def phase_table(torch, desc, plan, x, packed_codes, codebooks, scales, y, workspace, workspace_bytes,
                warmup: int = 3, flush=None) -> List[Dict]:
    """Runs one traced call (after `warmup` untraced ones) on the current stream and returns,
    per phase reached, the time since the first workgroup entered the kernel: mean, min and
    max over the workgroups that reached it, in microseconds.  `flush`, if given, is a device
    tensor larger than the chip's caches that is overwritten just before the traced call, so
    that the call reads its codes from HBM (cold); without it the warm-up calls leave them in
    the memory-side cache."""
    lib = _trace_lib()
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)

    def call():
        st = lib.codegemm_gemm(ctypes.byref(desc), ctypes.byref(plan), binding._ptr(x), binding._ptr(packed_codes),
                               binding._ptr(codebooks), binding._ptr(scales), binding._ptr(y), binding._ptr(workspace),
                               workspace_bytes, stream)
        if st:
            raise binding.CodegemmError(st, "codegemm_gemm (trace build)")

    for _ in range(warmup):
        call()
    n = workgroups(desc, plan)
    stamps = torch.zeros((n, SLOTS), dtype=torch.int64, device="cuda")
    lib.codegemm_set_trace(ctypes.c_void_p(stamps.data_ptr()))
    try:
        if flush is not None:
            flush.fill_(1)
        call()
        torch.cuda.synchronize()
    finally:
        lib.codegemm_set_trace(None)
    t = stamps.cpu().numpy().astype("float64")
    t0 = t[:, 0][t[:, 0] > 0].min()
    rows = []
    for slot, label in PHASES:
        col = t[:, slot]
        ok = col > 0
        if ok.any():
            rel = (col[ok] - t0) * TICK_US
            rows.append({"slot": slot, "phase": label, "workgroups": int(ok.sum()),
                         "mean_us": float(rel.mean()), "min_us": float(rel.min()), "max_us": float(rel.max())})
    return rows
