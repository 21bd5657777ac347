"""Builds libcodegemm.so (gfx950) in-tree with hipcc.  No torch involved."""
from __future__ import annotations

import glob
import os
import subprocess

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libcodegemm.so")
TRACE_LIB = os.path.join(PKG, "libcodegemm_trace.so")   # diagnostic build: kernels stamp their phases
ABLATE_MASKS = (6, 8, 14)       # ablation builds made by default: no gather + no build, no exchange, all three
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

# Packed-FP32 instruction selection is switched off for every device compile.
# Kernel-argument preloading: the leading scalar arguments of a kernel (up to 14 dwords) arrive in
# scalar registers with the wavefront instead of being loaded from the argument segment first.
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-ffp-contract=off",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-mllvm", "-amdgpu-kernarg-preload-count=14",
         "-Wall", "-Wno-unused-command-line-argument"]


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def ablate_lib(mask: int) -> str:
    return os.path.join(PKG, f"libcodegemm_ablate_{mask}.so")


def build(verbose: bool = False, jobs: int = 8, trace: bool = False, ablate: int = 0) -> str:
    """Compiles every .hip file to an object (in parallel) and links the shared library.
    trace=True builds the diagnostic library instead (same ABI plus codegemm_set_trace;
    the gather kernels record clock stamps of their phases, see include/codegemm_trace.h).
    ablate=mask builds an ablation library (same ABI, deliberately wrong outputs: parts of the
    batch-1 gather kernel compiled out, see csrc/gemm_impl.h); only the translation units of
    that kernel are recompiled, the rest comes from the production build, which must exist."""
    out_dir = os.path.join(PKG, "_build", f"ablate_{ablate}" if ablate else ("trace" if trace else "main"))
    os.makedirs(out_dir, exist_ok=True)
    extra = ["-DCODEGEMM_TRACE"] if trace else ([f"-DCODEGEMM_ABLATE={ablate}"] if ablate else [])
    lib = ablate_lib(ablate) if ablate else (TRACE_LIB if trace else LIB)
    procs = []
    objs = []
    for src in sources():
        name = os.path.basename(src)[:-4]
        if ablate and not (name.startswith("gemm_m") and name[6:].isdigit()):
            objs.append(os.path.join(PKG, "_build", "main", name + ".o"))
            continue
        obj = os.path.join(out_dir, name + ".o")
        objs.append(obj)
        cmd = [HIPCC, *FLAGS, *extra, "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-c", src, "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        while sum(p.poll() is None for _, p in procs) >= jobs:
            for _, p in procs:
                if p.poll() is None:
                    p.wait()
                    break
    for src, p in procs:
        out, _ = p.communicate()
        lines = [l for l in out.splitlines() if "not a recognized feature" not in l]
        if p.returncode:
            raise RuntimeError(f"hipcc failed on {src}:\n" + "\n".join(lines))
        if verbose and lines:
            print("\n".join(lines))
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", lib, *objs]
    subprocess.run(cmd, check=True)
    return lib


if __name__ == "__main__":
    print(build(verbose=True))
    print(build(verbose=True, trace=True))
    for mask in ABLATE_MASKS:
        print(build(verbose=True, ablate=mask))
