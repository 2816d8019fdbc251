"""Builds libssmscan.so (HIP, gfx950 only) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libssmscan.so")
SOURCES = ["ssm_api.hip", "gemm_f32.hip", "scan.hip", "params.hip", "block.hip", "probe.hip"]
HEADERS = [os.path.join(CSRC, "ssm_internal.h"), os.path.join(CSRC, "gemm_f32_kernel.h"),
           os.path.join(CSRC, "gemm_bf16x3_kernel.h"), os.path.join(CSRC, "lookback.h"),
           os.path.join(os.path.dirname(HERE), "include", "ssm.h")]
# packed-fp32 instructions are switched off on purpose (target feature removed for device code)
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unused-command-line-argument"]


def is_stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    deps = [os.path.join(CSRC, s) for s in SOURCES] + HEADERS
    return any(os.path.getmtime(d) > t for d in deps)


def build(force: bool = True, verbose: bool = False) -> str:
    """Compile every HIP source into one shared library.  Returns its path."""
    if not force and not is_stale():
        return LIB
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    tmp = LIB + ".tmp%d" % os.getpid()
    cmd = [hipcc] + FLAGS + [os.path.join(CSRC, s) for s in SOURCES] + ["-o", tmp]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
