"""Build libsolo.so (the C-ABI library of include/solo.h) with hipcc for gfx950.

Usage: python -m paper_2505_00347_amd.build [--force]
The library is built in-tree (paper_2505_00347_amd/lib/libsolo.so); object
files go to paper_2505_00347_amd/_build/.
"""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIBDIR = os.path.join(HERE, "lib")
LIB = os.path.join(LIBDIR, "libsolo.so")
PROBE = os.path.join(LIBDIR, "stream_probe")
EXAMPLE = os.path.join(LIBDIR, "solo_c_example")
SOURCES = ["solo_api.hip", "solo_step_m2.hip", "solo_step_m3.hip", "solo_step_m4.hip",
           "solo_step_m2_de.hip", "solo_step_m3_de.hip", "solo_step_m4_de.hip",
           "solo_step_big.hip", "solo_step_big_de.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
# -ffp-contract=off and IEEE divide/sqrt: the stored codes and scales depend on the exact
# rounding of every operation.  Packed-FP32 instructions are disabled on the test machines.
FLAGS = ["-O3", "--offload-arch=gfx950", "-std=c++17", "-fPIC", "-ffp-contract=off",
         "-fhip-fp32-correctly-rounded-divide-sqrt", "-fno-fast-math",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-function", "-Wno-unknown-warning-option"]


def _compile(src):
    obj = os.path.join(OBJ, src.replace(".hip", ".o"))
    subprocess.check_call([HIPCC, *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj])
    return obj


def build(force=True, verbose=False):
    os.makedirs(OBJ, exist_ok=True)
    os.makedirs(LIBDIR, exist_ok=True)
    deps = [os.path.join(CSRC, f) for f in os.listdir(CSRC)] + [
        os.path.join(HERE, "..", "include", "solo.h")]
    if not force and os.path.exists(LIB) and all(
            os.path.getmtime(LIB) >= os.path.getmtime(d) for d in deps):
        return LIB
    with ThreadPoolExecutor(len(SOURCES)) as ex:
        objs = list(ex.map(_compile, SOURCES))
    subprocess.check_call([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs])
    # stand-alone memory-ceiling probe (read / write / copy / step-shaped streams)
    subprocess.check_call([HIPCC, "-O3", "--offload-arch=gfx950", "-std=c++17",
                           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
                           "-Wno-unknown-warning-option",
                           os.path.join(CSRC, "stream_probe.hip"), "-o", PROBE])
    # a caller of the library without PyTorch (plain HIP memory and the C-ABI)
    subprocess.check_call([HIPCC, "-O2", "--offload-arch=gfx950", "-std=c++17",
                           "-Wno-unknown-warning-option", "-Wno-unused-result",
                           os.path.join(CSRC, "solo_c_example.cpp"), "-o", EXAMPLE,
                           "-L" + LIBDIR, "-lsolo", "-Wl,-rpath,$ORIGIN"])
    if verbose:
        print("built", LIB)
    return LIB


if __name__ == "__main__":
    build(force="--force" in sys.argv or True, verbose=True)
