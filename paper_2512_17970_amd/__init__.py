"""MI355X-native CodeGEMM: thin Python binding over the C-ABI library libcodegemm.so.

Every computation runs in the library's HIP kernels; this package only marshals
arguments.  PyTorch is used by callers for device memory and streams.
"""
from .binding import (  # noqa: F401
    CodegemmError, Desc, Plan, lib_path, load,
    codegemm_default_plan, codegemm_workspace_bytes, codegemm_packed_codes_bytes,
    codegemm_workspace_init, codegemm_pack_codes, codegemm_unpack_codes,
    codegemm_psumbook_build, codegemm_gemm, codegemm_dequant_gemm, codegemm_status_string,
    compressed_bytes,
    codegemm_packed_scales_bytes,
    codegemm_pack_scales,
    codegemm_pack_codes_host, codegemm_unpack_codes_host,
    codegemm_gemm_static, codegemm_static_workspace_limit,
    GroupMember, codegemm_gemm_grouped, codegemm_grouped_workspace_bytes,
)
