"""Builds libfp4mr.so (the C-ABI library of HIP kernels) in-tree for gfx950 with hipcc.

    python -m paper_2509_23202_amd.build

hipcc cross-compiles without a GPU.  Objects go to paper_2509_23202_amd/_build/, the library next to this
file, so that it travels with the source tree.
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor
from pathlib import Path

HERE = Path(__file__).resolve().parent
CSRC = HERE / "csrc"
BUILD = HERE / "_build"
LIB = HERE / "libfp4mr.so"
SOURCES = ["api.hip", "rotate_quantize.hip", "gemm_mxfp4.hip", "gemm_nvfp4.hip", "gemm_nv16.hip", "gemm_skinny.hip", "gemm_fused_decode.hip", "repack.hip", "gptq.hip", "gptq_prepare.hip", "probes.hip", "dequantize.hip"]

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
# Packed-fp32 instruction selection is switched off for all device code (a device-only target feature; the host
# pass prints a harmless "not a recognized feature" note).
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


# The rotation kernels consume every MFMA result in the vector ALU right away: letting the MFMAs write ordinary
# vector registers saves one v_accvgpr_read per value (the GEMM kernels keep their accumulators where the
# compiler puts them).
EXTRA_FLAGS = {"rotate_quantize.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form"],
               "gemm_fused_decode.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form"],
               # (dequantized fragments come out of the vector ALU: as MFMA operands they should stay in vector registers)
               "gemm_nvfp4.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form"],
               "gemm_nv16.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form"]}


def _compile(src: str) -> Path:
    obj = BUILD / (src + ".o")
    cmd = [HIPCC, *FLAGS, *EXTRA_FLAGS.get(src, []), "-I", str(HERE.parent / "include"), "-c", str(CSRC / src), "-o", str(obj)]
    r = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed for {src}:\n{err}")
    if err.strip():
        print(err, file=sys.stderr)
    return obj


def build(verbose: bool = True) -> Path:
    BUILD.mkdir(exist_ok=True)
    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES), os.cpu_count() or 1)) as ex:
        objs = list(ex.map(_compile, SOURCES))
    tmp = LIB.with_suffix(".so.tmp%d" % os.getpid())
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", str(tmp), *map(str, objs)]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stderr)
    os.replace(tmp, LIB)
    if verbose:
        print(f"built {LIB} ({LIB.stat().st_size >> 10} KiB)")
    return LIB


if __name__ == "__main__":
    build()
