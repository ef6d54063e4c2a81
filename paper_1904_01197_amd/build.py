"""Builds libndq.so (HIP kernels + C ABI) for gfx950, in-tree."""
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SO = os.path.join(HERE, "libndq.so")
CSRC = os.path.join(HERE, "csrc")
SOURCES = [os.path.join(CSRC, f) for f in ("ndq_encode.hip", "ndq_decode.hip", "ndq_tools.hip")]
HEADERS = [os.path.join(CSRC, "ndq_device.hpp"), os.path.join(CSRC, "ndq_host.hpp"),
           os.path.join(ROOT, "include", "ndq.h")]

HIPCC_FLAGS = [
    "-O3", "--offload-arch=gfx950", "-std=c++17", "-fPIC",
    # every rounding is spelled out in the source: no contraction, IEEE division
    "-ffp-contract=off", "-fhip-fp32-correctly-rounded-divide-sqrt",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument",
]


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd))
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + " ".join(cmd) + "\n" + res.stdout)


def build_library(force=True, verbose=False, so=None):
    """Compiles the library with hipcc (one object per source, in parallel, then
    one link); returns the path of the shared object."""
    so = so or SO
    stale = (not os.path.exists(so)) or any(
        os.path.getmtime(p) > os.path.getmtime(so) for p in SOURCES + HEADERS)
    if force or stale:
        hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
        extra = os.environ.get("NDQ_EXTRA_HIPCC_FLAGS", "").split()
        objdir = os.path.join(os.path.dirname(os.path.abspath(so)),
                              "_build_" + os.path.basename(so).replace(".", "_"))
        os.makedirs(objdir, exist_ok=True)
        inc = ["-I", os.path.join(ROOT, "include"), "-I", CSRC]
        objs = [os.path.join(objdir, os.path.basename(src) + ".o") for src in SOURCES]
        with ThreadPoolExecutor(max_workers=len(SOURCES)) as pool:
            list(pool.map(lambda so_: _run([hipcc] + HIPCC_FLAGS + extra + inc + ["-c", so_[0], "-o", so_[1]],
                                           verbose), zip(SOURCES, objs)))
        _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", so] + objs, verbose)
    return so


# Stand-alone measurement programs (no part of the library): the instruction issue rates
# the kernels' instruction choices and the benchmark's "alu" roof rest on, and the
# streaming bandwidth the memory system gives the encoders' traffic.
PROBES = ("valu_issue_probe", "hbm_stream_probe")


def build_probes(verbose=False):
    """Compiles the probes next to the library; returns their paths."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    out = []
    for name in PROBES:
        exe = os.path.join(HERE, name)
        _run([hipcc, "-O3", "--offload-arch=gfx950", "-std=c++17", "-Wno-unused-command-line-argument",
              "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
              "-o", exe, os.path.join(CSRC, name + ".hip")], verbose)
        out.append(exe)
    return out


def ensure_built():
    """Builds the library only if no built one is there (a fresh checkout)."""
    if not os.path.exists(SO):
        build_library(force=True)
    return SO


if __name__ == "__main__":
    print(build_library(force=True, verbose=True))
    print("\n".join(build_probes(verbose=True)))
