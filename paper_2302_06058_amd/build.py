"""Build step: compile the HIP sources under csrc/ into libbimask.so for gfx950."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libbimask.so")
SOURCES = ["api.hip", "mask_kernels.hip", "perm_search.hip", "perm_refine.hip", "gemm.hip", "gemm_sp24.hip", "gemm_sp24_big.hip",
           "gemm_sp24_resident.hip", "gemm_sp24_narrow.hip", "gemm_sp24_rowres.hip"]
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fvisibility=hidden",
    "-Wall", "-Wextra", "-Wno-unused-parameter",
    # packed fp32 instructions stay off for every device function
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in res.stdout.splitlines() if "packed-fp32-ops" not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    if verbose and out.strip():
        print(out)


def build_lib(verbose: bool = False, only=None) -> str:
    """Compiles every source (or, with `only`, the named ones, re-using the other objects of an
    earlier full build) and links the library.  One hipcc process per source, at most 8 at once."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(OBJ, exist_ok=True)
    srcs = list(SOURCES)
    objs = [os.path.join(OBJ, s[:-4] + ".o") for s in srcs]
    todo = [(s, o) for s, o in zip(srcs, objs) if only is None or s in only or not os.path.exists(o)]
    with ThreadPoolExecutor(max_workers=min(8, max(1, len(todo)))) as ex:
        list(ex.map(lambda so: _run([hipcc] + FLAGS + ["-c", os.path.join(CSRC, so[0]), "-o", so[1]], verbose), todo))
    _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-fvisibility=hidden"] + objs + ["-o", LIB], verbose)
    return LIB


# stand-alone measurement programs under csrc/tools/ (not part of the library): source file, extra link arguments
TOOLS = {"l2_gather_ceiling": ("l2_gather_ceiling.hip", []),
         "vendor_sparse_gemm": ("vendor_sparse_gemm.cpp", ["-L/opt/rocm/lib", "-lhipsparselt"])}
BIN = os.path.join(HERE, "bin")


def build_tools(verbose: bool = False):
    """Compiles the measurement tools into bin/ (each a self-contained HIP program with its own main)."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(BIN, exist_ok=True)
    out = []
    for t, (src, link) in TOOLS.items():
        exe = os.path.join(BIN, t)
        try:
            _run([hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
                  os.path.join(CSRC, "tools", src), "-o", exe] + link, verbose)
        except RuntimeError as e:
            if not link:
                raise
            # a context tool that needs a vendor library this machine does not have: the library itself is unaffected
            print(f"skipping tool {t}: {str(e).splitlines()[-1]}", file=sys.stderr)
            continue
        out.append(exe)
    return out


if __name__ == "__main__":
    names = [a for a in sys.argv[1:] if a.endswith(".hip")]
    if "--tools" in sys.argv:
        print("\n".join(build_tools(verbose="-v" in sys.argv)))
    else:
        print(build_lib(verbose="-v" in sys.argv, only=names or None))
