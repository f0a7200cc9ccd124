"""Builds libtbik.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree.

    python -m paper_2511_17826_amd.build

hipcc cross-compiles without a GPU.  Object files go to ``paper_2511_17826_amd/_build/``,
the library to ``paper_2511_17826_amd/libtbik.so``.
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
BUILD = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libtbik.so")

SOURCES = ["tbik_api.hip", "gemm_reference.hip", "gemm_tiled.hip", "gemm_f32.hip", "gemm_fp8.hip", "gemm_mxfp4.hip", "gemm_mxfp6.hip", "combine.hip", "activation.hip", "rmsnorm.hip", "row_reduce.hip",
           "attention.hip"]

# -ffp-contract=off: a tree addition or an RMSNorm multiply must never be fused into an FMA.
# packed-fp32 ops are switched off for the device pass (known-bad forms on the test machines).
# -amdgpu-mfma-vgpr-form: MFMA accumulators are allocated as ordinary VGPRs, so the tree additions (VALU) work
# on them in place and the allocator parks the cold stash levels in AGPRs instead of spilling to scratch.
FLAGS = ["--offload-arch=gfx950", "-mllvm", "-amdgpu-mfma-vgpr-form", "-O3", "-std=c++17", "-fPIC", "-ffp-contract=off", "-fno-fast-math",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wall", "-Wno-unused-command-line-argument",
         "-Wno-unknown-attributes", "-Wno-inline-asm"]


def _hipcc() -> str:
    for c in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if c and (os.path.sep not in c or os.path.exists(c)):
            return c
    raise RuntimeError("hipcc not found")


def _compile(src: str, extra) -> str:
    obj = os.path.join(BUILD, os.path.splitext(src)[0] + ".o")
    cmd = [_hipcc(), *FLAGS, *extra, "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    msgs = "\n".join(l for l in (r.stdout + r.stderr).splitlines() if "packed-fp32-ops" not in l and l.strip())
    if r.returncode != 0:
        raise RuntimeError("hipcc failed on %s:\n%s" % (src, msgs))
    if msgs:
        print(msgs, file=sys.stderr)
    return obj


def check_generated_code(asm_path: str, kernel_name: str = "gemm_tiled_kernel") -> None:
    """What the hand-kept bookkeeping of a kernel with direct global->LDS loads assumes about the code the compiler
    generated for it: no private-memory (scratch) traffic, whose loads and stores would share the counter that the
    kernel uses for its direct loads, and a wait state between a write of m0 and the direct load that reads it."""
    import re
    lines = [l.split(";")[0].strip() for l in open(asm_path)]      # without comments (a label line carries one)
    lines = [l for l in lines if l]
    kernel = None
    for i, l in enumerate(lines):
        if l.endswith(":") and kernel_name in l:
            kernel = l
        if l.startswith("scratch_") and kernel:
            raise RuntimeError("%s: scratch access in %s: %s" % (asm_path, kernel, l))
        if re.match(r"s_\w+\s+m0,", l):
            j = i + 1
            while lines[j].startswith(".") or lines[j].endswith(":"):
                j += 1
            if "global_load_lds" in lines[j]:
                raise RuntimeError("%s: m0 written directly before a direct load in %s" % (asm_path, kernel))
        if l.startswith("s_endpgm"):
            kernel = None


def build(save_temps: bool = True, jobs: int = 8, defines=(), lib_path: str = LIB) -> str:
    os.makedirs(BUILD, exist_ok=True)
    extra = (["-save-temps=obj"] if save_temps else []) + ["-D" + d for d in defines]
    with ThreadPoolExecutor(max_workers=jobs) as ex:
        objs = list(ex.map(lambda s: _compile(s, extra), SOURCES))
    if save_temps:
        check_generated_code(os.path.join(BUILD, "gemm_tiled-hip-amdgcn-amd-amdhsa-gfx950.s"), "gemm_tiled_kernel")
        check_generated_code(os.path.join(BUILD, "attention-hip-amdgcn-amd-amdhsa-gfx950.s"), "attention_")
        check_generated_code(os.path.join(BUILD, "gemm_f32-hip-amdgcn-amd-amdhsa-gfx950.s"), "gemm_f32_tiled_kernel")
        check_generated_code(os.path.join(BUILD, "gemm_fp8-hip-amdgcn-amd-amdhsa-gfx950.s"), "gemm_fp8_tiled_kernel")
        check_generated_code(os.path.join(BUILD, "gemm_mxfp4-hip-amdgcn-amd-amdhsa-gfx950.s"), "gemm_mxfp4_tiled_kernel")
        check_generated_code(os.path.join(BUILD, "gemm_mxfp6-hip-amdgcn-amd-amdhsa-gfx950.s"), "gemm_mxfp6_tiled_kernel")
    cmd = [_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", lib_path, *objs]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stdout + r.stderr)
    return lib_path


if __name__ == "__main__":
    print(build())
