"""Builds the in-tree shared libraries (hand-written HIP for gfx950) with hipcc:
liblags.so (the sparsifier) and libhbmcal.so (plain streaming kernels that calibrate the
benchmark's bandwidth ceiling; no method code)."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "liblags.so")
CAL_LIB = os.path.join(HERE, "libhbmcal.so")
SOURCES = ["lags_api.hip", "lags_kernels.hip", "lags_static.hip"]
HEADERS = ["lags_internal.h", os.path.join("..", "..", "include", "lags.h")]
CAL_SOURCES = ["hbm_calibrate.hip"]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-ffp-contract=off",                       # the method's acc is a product and a sum, never an fma
    "-fhip-fp32-correctly-rounded-divide-sqrt",
    "-fno-gpu-flush-denormals-to-zero",        # subnormal acc values are ordinary keys
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument",
]


def _build_one(lib, sources, headers, force, verbose):
    srcs = [os.path.join(CSRC, s) for s in sources]
    deps = srcs + [os.path.join(CSRC, h) for h in headers]
    if not force and os.path.exists(lib) and all(os.path.getmtime(lib) >= os.path.getmtime(p) for p in deps):
        return lib
    tmp = lib + ".tmp.%d" % os.getpid()
    cmd = ["hipcc", *HIPCC_FLAGS, "-o", tmp, *srcs]
    if verbose:
        print(" ".join(cmd), file=sys.stderr)
    subprocess.check_call(cmd)
    os.replace(tmp, lib)
    return lib


def build(force=True, verbose=False):
    """Compile every HIP source into the two libraries.  Returns the path of liblags.so."""
    _build_one(CAL_LIB, CAL_SOURCES, [], force, verbose)
    return _build_one(LIB, SOURCES, HEADERS, force, verbose)


if __name__ == "__main__":
    print(build(force=True, verbose=True))
