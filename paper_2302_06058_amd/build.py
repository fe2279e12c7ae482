"""Build step: compile the HIP sources under csrc/ into libbimask.so for gfx950."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libbimask.so")
SOURCES = ["api.hip", "mask_kernels.hip", "perm_search.hip", "perm_refine.hip", "gemm.hip", "gemm_sp24.hip", "gemm_sp24_resident.hip",
           "gemm_sp24_narrow.hip", "gemm_sp24_rowres.hip"]
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-fvisibility=hidden",
    "-Wall", "-Wextra", "-Wno-unused-parameter",
    # packed fp32 instructions stay off for every device function
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]


def build_lib(verbose: bool = False) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc] + FLAGS + [os.path.join(CSRC, s) for s in SOURCES] + ["-o", LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in res.stdout.splitlines() if "packed-fp32-ops" not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    if verbose and out.strip():
        print(out)
    return LIB


if __name__ == "__main__":
    print(build_lib(verbose="-v" in sys.argv))
