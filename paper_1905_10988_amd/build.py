"""Compile the native code (HIP, gfx950) in-tree with hipcc.

    python -m paper_1905_10988_amd.build

Two shared libraries: libnatcomp.so (the product: csrc/*.hip behind include/natcomp.h) and
libncprobe.so (csrc/probe/*.hip: bench-only kernels that measure the device's copy, read,
fill and Philox ceilings; bench.py loads it, the product never does).

hipcc cross-compiles without a GPU present.  The packed-FP32 VALU forms are switched off
for all device code with a target feature; the host pass of each file does not know that
feature and says so in a warning, which is harmless and left in the output.
"""
import glob
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libnatcomp.so")
PROBE_LIB = os.path.join(HERE, "libncprobe.so")

HIPCC_FLAGS = [
    "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-shared",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-ffp-contract=off", "-fno-fast-math", "-Wall", "-Wno-unused-command-line-argument",
]


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def probe_sources():
    return sorted(glob.glob(os.path.join(CSRC, "probe", "*.hip")))


def _headers():
    return glob.glob(os.path.join(CSRC, "*.hpp")) + [os.path.join(os.path.dirname(HERE), "include", "natcomp.h")]


def _compile(lib, srcs, force, extra_flags):
    deps = srcs + _headers()
    if not force and os.path.exists(lib) and all(os.path.getmtime(lib) >= os.path.getmtime(f) for f in deps):
        return lib
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc] + HIPCC_FLAGS + list(extra_flags) + ["-o", lib + ".tmp"] + srcs
    proc = subprocess.run(cmd, capture_output=True, text=True)
    if proc.stderr.strip():
        sys.stderr.write(proc.stderr)
    if proc.returncode != 0:
        raise RuntimeError("hipcc failed: " + " ".join(cmd))
    os.replace(lib + ".tmp", lib)
    return lib


def build(force: bool = True, extra_flags=()) -> str:
    """Build libnatcomp.so and libncprobe.so; with force=False only what is missing or older
    than a source/header.  Returns the path of libnatcomp.so."""
    _compile(PROBE_LIB, probe_sources(), force, extra_flags)
    return _compile(LIB, sources(), force, extra_flags)


if __name__ == "__main__":
    print(build(force=True))
