"""Host-side sanitizer runs (CPU only): the oracle's C code and the library's argument validation, each
built with -fsanitize=address,undefined into a plain executable and run on small inputs.  Nothing here
touches a GPU: every library call made by the second driver fails validation before any HIP call."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HERE = os.path.join(ROOT, "tests", "sanitize")
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:verify_asan_link_order=0:abort_on_error=0",
           UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1")


def run(cmd, **kw):
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, **kw)
    assert res.returncode == 0, " ".join(cmd) + "\n" + res.stdout[-4000:]
    return res.stdout


def test_oracle_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    exe = str(tmp_path / "oracle_san")
    run(["gcc", "-O1", "-g", "-std=c11", "-Wall", "-Wextra", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
         "-o", exe, os.path.join(ROOT, "oracle", "bimask_oracle.c"), os.path.join(HERE, "oracle_driver.c"), "-lm"])
    assert "clean" in run([exe], env=ENV)


@pytest.mark.skipif(shutil.which("hipcc") is None and not os.path.exists("/opt/rocm/bin/hipcc"), reason="no hipcc")
def test_argument_validation_under_host_sanitizers(tmp_path):
    """include/bimask.h's calls with every kind of bad argument, in a build of the library whose HOST code is
    instrumented (the device code is compiled as usual and never runs)."""
    from paper_2302_06058_amd import build as b
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host", "-fno-sanitize-recover=all"]
    # the validation path lives in api.hip; the other sources are linked as they are built for the product
    objs = []
    for s in b.SOURCES:
        o = os.path.join(b.OBJ, s[:-4] + ".o")
        if s == "api.hip" or not os.path.exists(o):
            o = str(tmp_path / (s[:-4] + ".o"))
            run([hipcc] + b.FLAGS + (san if s == "api.hip" else []) + ["-O1", "-g", "-c", os.path.join(b.CSRC, s), "-o", o])
        objs.append(o)
    exe = str(tmp_path / "api_san")
    # the driver is plain host C++: compiled and linked by the host compiler against the HIP runtime library
    drv = str(tmp_path / "api_driver.o")
    host = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all"]
    run(["g++", "-O1", "-g", "-std=c++17"] + host + ["-I", os.path.join(ROOT, "include"), "-c", os.path.join(HERE, "api_driver.cpp"), "-o", drv])
    rocm_lib = os.path.join(os.path.dirname(os.path.dirname(os.path.realpath(hipcc))), "lib")
    run(["g++"] + host + [drv] + objs + ["-L", rocm_lib, "-Wl,-rpath," + rocm_lib, "-lamdhip64", "-o", exe])
    assert "clean" in run([exe], env=ENV)
