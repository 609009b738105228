"""Builds libbnn_hip.so (HIP kernels + C ABI) in-tree for gfx950.

Device code is compiled by hipcc with packed-FP32 instruction selection turned
off; the host-only BatchNorm fold is compiled by g++ with floating-point
contraction off, so that its float32 expression is evaluated step by step.
"""
from __future__ import annotations

import os
import subprocess

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
INCLUDE = os.path.join(ROOT, "include")
BUILD = os.path.join(ROOT, "_build")
LIB = os.path.join(PKG, "libbnn_hip.so")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
ARCH = "gfx950"

HIP_SOURCES = ["pack_sign.hip", "xnor_gemm.hip", "xnor_gemm_mfma.hip", "xnor_gemm_mfma_shortk.hip",
               "xnor_gemm_mfma_persist.hip", "xnor_gemm_mfma_big.hip", "xnor_gemm_mfma_splitk.hip",
               "bn_sign_pack.hip", "im2col_pack.hip", "conv_implicit.hip", "conv_patch.hip", "gemm_i8_mfma.hip",
               "valu_fallbacks.hip"]
HOST_SOURCES = ["bn_fold.cpp", "api.cpp"]

HIP_FLAGS = [f"--offload-arch={ARCH}", "-O3", "-std=c++17", "-fPIC", f"-I{INCLUDE}", f"-I{CSRC}",
             "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument"]
HOST_FLAGS = ["-O2", "-std=c++17", "-fPIC", "-ffp-contract=off", "-fno-fast-math", f"-I{INCLUDE}",
              "-Wall", "-Wextra"]


def _run(cmd):
    proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    # hipcc's host pass warns that it does not know the packed-fp32 feature; harmless.
    out = "\n".join(l for l in proc.stdout.splitlines() if "packed-fp32-ops" not in l)
    if proc.returncode != 0:
        raise RuntimeError("build failed: " + " ".join(cmd) + "\n" + out)
    if out.strip():
        print(out)


def build_library(verbose: bool = False) -> str:
    """Compiles every source and links libbnn_hip.so next to this file."""
    os.makedirs(BUILD, exist_ok=True)
    objects = []
    procs = []
    for src in HIP_SOURCES:
        obj = os.path.join(BUILD, src + ".o")
        cmd = [HIPCC, *HIP_FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
        procs.append((cmd, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        objects.append(obj)
    for src in HOST_SOURCES:
        obj = os.path.join(BUILD, src + ".o")
        _run(["g++", *HOST_FLAGS, "-c", os.path.join(CSRC, src), "-o", obj])
        objects.append(obj)
    for cmd, p in procs:
        out, _ = p.communicate()
        out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l)
        if p.returncode != 0:
            raise RuntimeError("build failed: " + " ".join(cmd) + "\n" + out)
        if verbose and out.strip():
            print(out)
    _run([HIPCC, f"--offload-arch={ARCH}", "-shared", "-fPIC", *objects, "-o", LIB])
    return LIB


CLOCK_PROBE_LIB = os.path.join(PKG, "libbnn_clock_probe.so")


def build_clock_probe() -> str:
    """Compiles the benchmark's clock probe (csrc/clock_probe.hip) into a library of its own: it is a
    measurement aid that only bench.py loads, not part of the C ABI."""
    _run([HIPCC, *HIP_FLAGS, "-shared", os.path.join(CSRC, "clock_probe.hip"), "-o", CLOCK_PROBE_LIB])
    return CLOCK_PROBE_LIB


C_ABI_EXAMPLE_SRC = os.path.join(ROOT, "tests", "c_abi", "hidden_layer.cpp")
C_ABI_EXAMPLE = os.path.join(ROOT, "tests", "c_abi", "hidden_layer")


def build_c_abi_example() -> str:
    """Compiles the non-Python caller of the C ABI that the GPU tests run (tests/c_abi/hidden_layer.cpp)
    and links it against the in-tree library (found again at run time through its rpath)."""
    _run([HIPCC, f"--offload-arch={ARCH}", "-O2", "-std=c++17", f"-I{INCLUDE}", C_ABI_EXAMPLE_SRC, f"-L{PKG}",
          "-lbnn_hip", f"-Wl,-rpath,{PKG}", "-Wl,-rpath,$ORIGIN/../../paper_1602_02830_amd", "-o", C_ABI_EXAMPLE])
    return C_ABI_EXAMPLE


if __name__ == "__main__":
    print(build_library(verbose=True))
    print(build_clock_probe())
    print(build_c_abi_example())
