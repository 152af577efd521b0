"""Builds libsale.so (the C-ABI library) in-tree with hipcc for gfx950.

Usage: python -m paper_2505_24179_amd.build
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libsale.so")
SOURCES = ["api.hip", "quantize.hip", "quantize8.hip", "select.hip", "attention.hip", "calibrate.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fvisibility=default",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",   # no packed-fp32 VALU ops
    "-mllvm", "-amdgpu-mfma-vgpr-form",   # MFMA results land in VGPRs: no AGPR -> VGPR copies before the VALU work
    "-Wno-unused-command-line-argument",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
]


def _compile(src: str, extra) -> str:
    obj = os.path.join(CSRC, src.replace(".hip", ".o"))
    cmd = [HIPCC, *FLAGS, *extra, "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l and l.strip())
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed for {src}:\n{err}")
    if err:
        print(err, file=sys.stderr)
    return obj


def build(extra_flags=(), verbose: bool = True) -> str:
    with ThreadPoolExecutor(max_workers=6) as ex:
        objs = list(ex.map(lambda s: _compile(s, list(extra_flags)), SOURCES))
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", LIB]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stderr)
    if verbose:
        print("built", LIB)
    _build_c_abi_check(verbose)
    return LIB


def _build_c_abi_check(verbose: bool) -> None:
    """tests/c_abi/abi_check: a plain-C (gcc) user of include/sale.h, run by the GPU tests."""
    src = os.path.join(ROOT, "tests", "c_abi", "abi_check.c")
    if not os.path.exists(src):
        return
    exe = os.path.join(ROOT, "tests", "c_abi", "abi_check")
    rocm = os.environ.get("ROCM_PATH", "/opt/rocm")
    cmd = ["gcc", "-std=c11", "-O1", "-Wall", "-D__HIP_PLATFORM_AMD__", "-I", os.path.join(rocm, "include"),
           "-I", os.path.join(ROOT, "include"), src, "-o", exe, "-L", PKG, "-lsale", "-L", os.path.join(rocm, "lib"),
           "-lamdhip64", "-lm", "-Wl,-rpath,$ORIGIN/../../paper_2505_24179_amd", f"-Wl,-rpath,{os.path.join(rocm, 'lib')}"]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("gcc failed for abi_check.c:\n" + r.stderr)
    if verbose:
        print("built", exe)


if __name__ == "__main__":
    build(sys.argv[1:])
