"""ctypes binding of include/codegemm.h.  Same names as the C entry points.

Tensor arguments are anything with `.data_ptr()` (torch tensors on the GPU) or
plain integer device addresses.  `stream` is a HIP stream handle as an integer
(e.g. `torch.cuda.current_stream().cuda_stream`), 0 for the default stream.
Functions raise CodegemmError on a non-zero status.  There is no fallback: if
the library has not been built, loading fails.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

_PKG = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_PKG, "libcodegemm.so")
_lib: Optional[ctypes.CDLL] = None

FLAG_Y_FP32 = 1
PSUM_FP32, PSUM_FP16 = 0, 1

EXPORTS = [
    "codegemm_default_plan", "codegemm_workspace_bytes", "codegemm_packed_codes_bytes",
    "codegemm_workspace_init", "codegemm_pack_codes", "codegemm_unpack_codes",
    "codegemm_pack_codes_host", "codegemm_unpack_codes_host",
    "codegemm_packed_scales_bytes", "codegemm_pack_scales",
    "codegemm_psumbook_build", "codegemm_gemm", "codegemm_dequant_gemm", "codegemm_status_string",
    "codegemm_gemm_static", "codegemm_static_workspace_limit",
    "codegemm_gemm_grouped", "codegemm_grouped_workspace_bytes",
]


class CodegemmError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {codegemm_status_string(status)} ({status})")


class Desc(ctypes.Structure):
    """codegemm_desc"""
    _fields_ = [("batch", ctypes.c_int32), ("in_features", ctypes.c_int32), ("out_features", ctypes.c_int32),
                ("vec_len", ctypes.c_int32), ("num_codebooks", ctypes.c_int32), ("code_bits", ctypes.c_int32),
                ("group_size", ctypes.c_int32), ("flags", ctypes.c_int32)]

    @classmethod
    def make(cls, B: int, K: int, N: int, v: int, m: int, y_fp32: bool = False, b: int = 8, g: int = -1):
        return cls(B, K, N, v, m, b, g, FLAG_Y_FP32 if y_fp32 else 0)


class Plan(ctypes.Structure):
    """codegemm_plan"""
    _fields_ = [("waves", ctypes.c_int32), ("row_words", ctypes.c_int32), ("k_splits", ctypes.c_int32),
                ("batch_group", ctypes.c_int32), ("psum_dtype", ctypes.c_int32), ("build_waves", ctypes.c_int32),
                ("reserved", ctypes.c_int32 * 2)]

    @classmethod
    def make(cls, waves: int, row_words: int, k_splits: int, batch_group: int = 1, psum_dtype: int = 0, build_waves: int = 0):
        return cls(waves, row_words, k_splits, batch_group, psum_dtype, build_waves, (ctypes.c_int32 * 2)(0, 0))

    def __repr__(self):
        tail = ", psum_dtype=fp16" if self.psum_dtype == PSUM_FP16 else ""
        if self.build_waves:
            tail += f", build_waves={self.build_waves}"
        return (f"Plan(waves={self.waves}, row_words={self.row_words}, k_splits={self.k_splits}, "
                f"batch_group={self.batch_group}{tail})")


class GroupMember(ctypes.Structure):
    """codegemm_group_member of include/codegemm.h: one layer of a grouped launch."""
    _fields_ = [("out_features", ctypes.c_int32), ("reserved", ctypes.c_int32),
                ("packed_codes", ctypes.c_void_p), ("codebooks", ctypes.c_void_p),
                ("scales", ctypes.c_void_p), ("y", ctypes.c_void_p)]


def lib_path() -> str:
    return _LIB_PATH


def use_library(path: str) -> None:
    """Makes load() take another build of the library with the same ABI (a diagnostic build such as
    libcodegemm_ablate_<mask>.so).  Must be called before the first load()."""
    global _LIB_PATH
    if _lib is not None:
        raise RuntimeError("the library is already loaded")
    _LIB_PATH = os.path.abspath(path)


def load() -> ctypes.CDLL:
    """Loads libcodegemm.so; raises if it has not been built (no fallback exists)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise ImportError(f"{_LIB_PATH} is missing: run `python -c 'import __graft_entry__ as g; g.build()'` "
                          "(or python paper_2512_17970_amd/build.py) first; there is no CPU fallback")
    lib = ctypes.CDLL(_LIB_PATH)
    vp, i, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t
    dp, pp = ctypes.POINTER(Desc), ctypes.POINTER(Plan)
    lib.codegemm_default_plan.argtypes = [dp, pp]
    lib.codegemm_default_plan.restype = i
    lib.codegemm_workspace_bytes.argtypes = [dp, pp]
    lib.codegemm_workspace_bytes.restype = sz
    lib.codegemm_packed_codes_bytes.argtypes = [dp, pp]
    lib.codegemm_packed_codes_bytes.restype = sz
    lib.codegemm_workspace_init.argtypes = [vp, sz, vp]
    lib.codegemm_workspace_init.restype = i
    lib.codegemm_pack_codes.argtypes = [dp, pp, vp, vp, vp]
    lib.codegemm_pack_codes.restype = i
    lib.codegemm_unpack_codes.argtypes = [dp, pp, vp, vp, vp]
    lib.codegemm_unpack_codes.restype = i
    lib.codegemm_pack_codes_host.argtypes = [dp, vp, vp]
    lib.codegemm_pack_codes_host.restype = i
    lib.codegemm_unpack_codes_host.argtypes = [dp, vp, vp]
    lib.codegemm_unpack_codes_host.restype = i
    lib.codegemm_packed_scales_bytes.argtypes = [dp]
    lib.codegemm_packed_scales_bytes.restype = sz
    lib.codegemm_pack_scales.argtypes = [dp, vp, vp, vp]
    lib.codegemm_pack_scales.restype = i
    lib.codegemm_psumbook_build.argtypes = [dp, vp, vp, vp, i, vp]
    lib.codegemm_psumbook_build.restype = i
    lib.codegemm_gemm.argtypes = [dp, pp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.codegemm_gemm.restype = i
    lib.codegemm_gemm_static.argtypes = [dp, pp, vp, vp, vp, vp, vp, vp]
    lib.codegemm_gemm_static.restype = i
    lib.codegemm_gemm_grouped.argtypes = [dp, pp, vp, ctypes.POINTER(GroupMember), ctypes.c_int32, vp, sz, vp]
    lib.codegemm_gemm_grouped.restype = i
    lib.codegemm_grouped_workspace_bytes.argtypes = [dp, pp, ctypes.POINTER(ctypes.c_int32), ctypes.c_int32]
    lib.codegemm_grouped_workspace_bytes.restype = sz
    lib.codegemm_static_workspace_limit.argtypes = []
    lib.codegemm_static_workspace_limit.restype = sz
    lib.codegemm_dequant_gemm.argtypes = [dp, vp, vp, vp, vp, vp, vp]
    lib.codegemm_dequant_gemm.restype = i
    lib.codegemm_status_string.argtypes = [i]
    lib.codegemm_status_string.restype = ctypes.c_char_p
    _lib = lib
    return lib


def _ptr(t) -> ctypes.c_void_p:
    if t is None:
        return ctypes.c_void_p(0)
    if hasattr(t, "data_ptr"):
        return ctypes.c_void_p(t.data_ptr())
    return ctypes.c_void_p(int(t))


def _plan(plan: Optional[Plan]):
    return ctypes.byref(plan) if plan is not None else None


def _check(status: int, where: str) -> None:
    if status != 0:
        raise CodegemmError(status, where)


def codegemm_status_string(status: int) -> str:
    return load().codegemm_status_string(int(status)).decode()


def codegemm_default_plan(desc: Desc) -> Plan:
    plan = Plan()
    _check(load().codegemm_default_plan(ctypes.byref(desc), ctypes.byref(plan)), "codegemm_default_plan")
    return plan


def codegemm_workspace_bytes(desc: Desc, plan: Optional[Plan] = None) -> int:
    return int(load().codegemm_workspace_bytes(ctypes.byref(desc), _plan(plan)))


def codegemm_packed_codes_bytes(desc: Desc, plan: Optional[Plan] = None) -> int:
    return int(load().codegemm_packed_codes_bytes(ctypes.byref(desc), _plan(plan)))


def codegemm_workspace_init(workspace, workspace_bytes: int, stream: int = 0) -> None:
    _check(load().codegemm_workspace_init(_ptr(workspace), workspace_bytes, ctypes.c_void_p(stream)),
           "codegemm_workspace_init")


def codegemm_pack_codes(desc: Desc, plan: Optional[Plan], codes, packed, stream: int = 0) -> None:
    _check(load().codegemm_pack_codes(ctypes.byref(desc), _plan(plan), _ptr(codes), _ptr(packed),
                                      ctypes.c_void_p(stream)), "codegemm_pack_codes")


def codegemm_unpack_codes(desc: Desc, plan: Optional[Plan], packed, codes, stream: int = 0) -> None:
    _check(load().codegemm_unpack_codes(ctypes.byref(desc), _plan(plan), _ptr(packed), _ptr(codes),
                                        ctypes.c_void_p(stream)), "codegemm_unpack_codes")


def _host_ptr(a) -> ctypes.c_void_p:
    """Address of a C-contiguous uint8 numpy array (host memory)."""
    if not (a.flags["C_CONTIGUOUS"] and a.dtype.itemsize == 1):
        raise TypeError("expected a C-contiguous uint8 array")
    return ctypes.c_void_p(a.ctypes.data)


def codegemm_pack_codes_host(desc: Desc, codes, packed) -> None:
    """codes, packed: numpy uint8 arrays in host memory."""
    _check(load().codegemm_pack_codes_host(ctypes.byref(desc), _host_ptr(codes), _host_ptr(packed)),
           "codegemm_pack_codes_host")


def codegemm_unpack_codes_host(desc: Desc, packed, codes) -> None:
    _check(load().codegemm_unpack_codes_host(ctypes.byref(desc), _host_ptr(packed), _host_ptr(codes)),
           "codegemm_unpack_codes_host")


def codegemm_packed_scales_bytes(desc: Desc) -> int:
    return int(load().codegemm_packed_scales_bytes(ctypes.byref(desc)))


def codegemm_pack_scales(desc: Desc, scales, packed, stream: int = 0) -> None:
    _check(load().codegemm_pack_scales(ctypes.byref(desc), _ptr(scales), _ptr(packed), ctypes.c_void_p(stream)),
           "codegemm_pack_scales")


def codegemm_psumbook_build(desc: Desc, x, codebooks, psumbook, use_mfma: bool = False, stream: int = 0) -> None:
    _check(load().codegemm_psumbook_build(ctypes.byref(desc), _ptr(x), _ptr(codebooks), _ptr(psumbook),
                                          1 if use_mfma else 0, ctypes.c_void_p(stream)), "codegemm_psumbook_build")


def codegemm_gemm(desc: Desc, plan: Optional[Plan], x, packed_codes, codebooks, scales, y,
                  workspace, workspace_bytes: int, stream: int = 0) -> None:
    _check(load().codegemm_gemm(ctypes.byref(desc), _plan(plan), _ptr(x), _ptr(packed_codes), _ptr(codebooks),
                                _ptr(scales), _ptr(y), _ptr(workspace), workspace_bytes,
                                ctypes.c_void_p(stream)), "codegemm_gemm")


def codegemm_static_workspace_limit() -> int:
    return int(load().codegemm_static_workspace_limit())


def codegemm_gemm_static(desc: Desc, plan: Optional[Plan], x, packed_codes, codebooks, scales, y, stream: int = 0) -> None:
    _check(load().codegemm_gemm_static(ctypes.byref(desc), _plan(plan), _ptr(x), _ptr(packed_codes), _ptr(codebooks),
                                       _ptr(scales), _ptr(y), ctypes.c_void_p(stream)), "codegemm_gemm_static")


def codegemm_grouped_workspace_bytes(desc: Desc, plan: Plan, out_features) -> int:
    arr = (ctypes.c_int32 * len(out_features))(*out_features)
    return int(load().codegemm_grouped_workspace_bytes(ctypes.byref(desc), _plan(plan), arr, len(out_features)))


def codegemm_gemm_grouped(desc: Desc, plan: Plan, x, members, workspace, workspace_bytes: int, stream: int = 0) -> None:
    """members: sequence of (out_features, packed_codes, codebooks, scales, y), tensors or raw device addresses."""
    arr = (GroupMember * len(members))()
    for k, (n, packed, codebooks, scales, y) in enumerate(members):
        arr[k].out_features = n
        arr[k].reserved = 0
        arr[k].packed_codes = _ptr(packed).value
        arr[k].codebooks = _ptr(codebooks).value
        arr[k].scales = _ptr(scales).value
        arr[k].y = _ptr(y).value
    _check(load().codegemm_gemm_grouped(ctypes.byref(desc), _plan(plan), _ptr(x), arr, len(members),
                                        _ptr(workspace), workspace_bytes, ctypes.c_void_p(stream)), "codegemm_gemm_grouped")


def codegemm_dequant_gemm(desc: Desc, x, codes, codebooks, scales, y, stream: int = 0) -> None:
    _check(load().codegemm_dequant_gemm(ctypes.byref(desc), _ptr(x), _ptr(codes), _ptr(codebooks), _ptr(scales),
                                        _ptr(y), ctypes.c_void_p(stream)), "codegemm_dequant_gemm")


def compressed_bytes(B: int, K: int, N: int, v: int, m: int, g: int = -1) -> int:
    """Bytes the method must move per call: codes + codebooks + scales + x + y (fp16 y)."""
    scales = 2 * N if g == -1 else 2 * N * (K // g)
    return m * N * (K // v) + m * 256 * v * 2 + scales + 2 * B * K + 2 * B * N
