"""Builds libwush.so (gfx950 only) in-tree with hipcc, and beside it libwush_probes.so, the
benchmark's measurement aids (MFMA-only and streaming kernels: not part of the layer path).

Usage: python -m paper_2512_00956_amd.build
"""
from __future__ import annotations

import os
import shutil
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libwush.so")
PROBES_SRC = os.path.join(HERE, "probes", "probes.hip")
PROBES_LIB = os.path.join(HERE, "libwush_probes.so")
SOURCES = ["wush_api.hip", "transform_quant.hip", "weight_prep.hip", "mxfp4_gemm.hip", "mxfp4_gemm_frag.hip", "build_transforms.hip", "layer_decode.hip", "gptq_prep.hip", "nvfp4_quant.hip", "nvfp4_gemm.hip", "int4_quant.hip", "w4_gemm_skinny.hip"]

HIPCC_FLAGS = [
    "-O3", "-std=c++17", "-fPIC", "--offload-arch=gfx950",
    # packed FP32 VALU ops stay disabled for every kernel of this library
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument",
]


def hipcc_path() -> str:
    p = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(p):
        raise RuntimeError("hipcc not found: the HIP library cannot be built")
    return p


def check_generated_code(hipcc: str, bdir: str) -> None:
    """The tiled MXFP4 GEMM issues its main-loop loads from inline asm; what that relies on in the
    generated code (build_checks.py) is verified on every build, with the flags of the build."""
    from .build_checks import check_gemm_frag_asm
    asm = os.path.join(bdir, "mxfp4_gemm_frag.s")
    cmd = [hipcc, *HIPCC_FLAGS, "-I", os.path.join(ROOT, "include"), "-S", "--cuda-device-only",
           os.path.join(CSRC, "mxfp4_gemm_frag.hip"), "-o", asm]
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc -S failed on mxfp4_gemm_frag.hip:\n{r.stdout}")
    with open(asm) as f:
        check_gemm_frag_asm(f.read())      # raises InvariantError


def build(verbose: bool = False) -> str:
    """Compile every kernel source and link libwush.so; returns its path."""
    hipcc = hipcc_path()
    objs = []
    procs = []
    bdir = os.path.join(HERE, "_build")
    os.makedirs(bdir, exist_ok=True)
    for src in SOURCES:
        obj = os.path.join(bdir, src.replace(".hip", ".o"))
        cmd = [hipcc, *HIPCC_FLAGS, "-I", os.path.join(ROOT, "include"), "-c", os.path.join(CSRC, src), "-o", obj]
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        objs.append(obj)
    pobj = os.path.join(bdir, "probes.o")
    pcmd = [hipcc, *HIPCC_FLAGS, "-I", os.path.join(ROOT, "include"), "-c", PROBES_SRC, "-o", pobj]
    procs.append(("probes/probes.hip", subprocess.Popen(pcmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    for src, p in procs:
        out, _ = p.communicate()
        out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l)
        if p.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}:\n{out}")
        if verbose and out.strip():
            print(out)
    check_generated_code(hipcc, bdir)
    for lib, lobjs in ((LIB, objs), (PROBES_LIB, [pobj])):
        tmp = lib + ".tmp"
        cmd = [hipcc, "-shared", "-fPIC", "--offload-arch=gfx950", *lobjs, "-o", tmp]
        r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        if r.returncode != 0:
            raise RuntimeError(f"link failed:\n{r.stdout}")
        os.replace(tmp, lib)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
    sys.exit(0)
