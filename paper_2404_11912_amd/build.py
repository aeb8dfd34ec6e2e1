"""Build libtriforce_hip.so for gfx950 with hipcc (cross-compiles without a GPU).

    python -m paper_2404_11912_amd.build
"""
from __future__ import annotations

import os
import shutil
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
INCLUDE = os.path.join(ROOT, "include")
LIB_PATH = os.path.join(PKG, "libtriforce_hip.so")

SOURCES = ["tf_api.hip", "tf_attn.hip", "tf_summarize.hip", "tf_topk_gather.hip", "tf_accept.hip", "tf_cache.hip", "tf_probe.hip"]

# packed-fp32 instructions are switched off for all device code of this library
HIP_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fno-gpu-rdc",
             "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
             "-mllvm", "-amdgpu-mfma-vgpr-form",   # MFMA accumulators stay in ordinary VGPRs
             "-Wno-unused-command-line-argument"]


def hipcc() -> str:
    exe = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(exe):
        raise RuntimeError("hipcc not found: the HIP library cannot be built")
    return exe


def build_library(verbose: bool = False, extra_flags=()) -> str:
    """Compile every HIP source and link the shared library in-tree. Always recompiles."""
    srcs = [os.path.join(CSRC, s) for s in SOURCES]
    tmp = LIB_PATH + f".{os.getpid()}.tmp"
    cmd = [hipcc(), *HIP_FLAGS, *extra_flags, "-I", INCLUDE, "-I", CSRC, "-shared", "-o", tmp, *srcs]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in res.stdout.splitlines()
                    if "packed-fp32-ops' is not a recognized feature" not in l)
    if res.returncode != 0:
        if os.path.exists(tmp):
            os.remove(tmp)
        raise RuntimeError("hipcc failed:\n" + out)
    if verbose and out.strip():
        print(out)
    os.replace(tmp, LIB_PATH)
    build_abi_check()
    return LIB_PATH


ABI_CHECK = os.path.join(PKG, "abi_check")


def build_abi_check() -> str:
    """The plain-C client of the C ABI (csrc/abi_check.c), linked against the library just built."""
    tmp = ABI_CHECK + f".{os.getpid()}.tmp"
    # (the HIP runtime's C header wants its platform macro when included from a plain C file)
    cmd = [hipcc(), "-x", "c", "-std=c99", "-O1", "-D__HIP_PLATFORM_AMD__", "-I", INCLUDE, "-I", "/opt/rocm/include",
           os.path.join(CSRC, "abi_check.c"), "-x", "none", "-o", tmp, "-L", PKG, "-l:libtriforce_hip.so",
           "-L", "/opt/rocm/lib", "-lamdhip64", "-lm", "-Wl,-rpath,$ORIGIN", "-Wl,-rpath,/opt/rocm/lib"]
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if res.returncode != 0:
        if os.path.exists(tmp):
            os.remove(tmp)
        raise RuntimeError("building abi_check failed:\n" + res.stdout)
    os.replace(tmp, ABI_CHECK)
    return ABI_CHECK


if __name__ == "__main__":
    print(build_library(verbose=True, extra_flags=sys.argv[1:]))
