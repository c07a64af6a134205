"""Builds libbaoc.so (HIP kernels + C ABI) in-tree for gfx950 with hipcc."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libbaoc.so")
SOURCES = ["baoc_profile.hip", "baoc_sample.hip", "baoc_risk.cpp", "baoc_allocate.cpp", "baoc_partition.cpp"]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-ffp-contract=off",                                   # fused operations only where written
    "-fhip-fp32-correctly-rounded-divide-sqrt",            # the 8-bit scale L / a is an IEEE quotient
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wextra", "-Wno-unused-parameter",
]


def sources():
    return [os.path.join(CSRC, s) for s in SOURCES]


def is_stale():
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    deps = sources() + [os.path.join(CSRC, "baoc_internal.h"), os.path.join(ROOT, "include", "baoc.h")]
    return any(os.path.getmtime(d) > t for d in deps)


def build_lib(verbose=False, extra=()):
    cmd = ["hipcc", *HIPCC_FLAGS, *extra, "-I", os.path.join(ROOT, "include"), "-I", CSRC,
           "-o", LIB, *sources()]
    if verbose:
        print(" ".join(cmd))
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    build_lib(verbose=True)
