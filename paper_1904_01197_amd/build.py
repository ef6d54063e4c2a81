"""Builds libndq.so (HIP kernels + C ABI) for gfx950, in-tree."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SO = os.path.join(HERE, "libndq.so")
SOURCES = [os.path.join(HERE, "csrc", "ndq_kernels.hip")]
HEADERS = [os.path.join(HERE, "csrc", "ndq_device.hpp"), os.path.join(ROOT, "include", "ndq.h")]

HIPCC_FLAGS = [
    "-O3", "--offload-arch=gfx950", "-std=c++17", "-fPIC", "-shared",
    # every rounding is spelled out in the source: no contraction, IEEE division
    "-ffp-contract=off", "-fhip-fp32-correctly-rounded-divide-sqrt",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument",
]


def build_library(force=True, verbose=False, so=None):
    """Compiles the library with hipcc; returns the path of the shared object."""
    so = so or SO
    stale = (not os.path.exists(so)) or any(
        os.path.getmtime(p) > os.path.getmtime(so) for p in SOURCES + HEADERS)
    if force or stale:
        hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
        extra = os.environ.get("NDQ_EXTRA_HIPCC_FLAGS", "").split()
        cmd = [hipcc] + HIPCC_FLAGS + extra + ["-I", os.path.join(ROOT, "include"), "-I",
                                       os.path.join(HERE, "csrc"), "-o", so] + SOURCES
        if verbose:
            print(" ".join(cmd))
        res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        if res.returncode != 0:
            raise RuntimeError("hipcc failed:\n" + res.stdout)
    return so


def ensure_built():
    """Builds the library only if no built one is there (a fresh checkout)."""
    if not os.path.exists(SO):
        build_library(force=True)
    return SO


if __name__ == "__main__":
    print(build_library(force=True, verbose=True))
