"""Compile the CPU oracle (plain C) into oracle/liboracle.so with gcc.

Test infrastructure only: the product never loads this library.
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "natcomp_oracle.c")
LIB = os.path.join(HERE, "liboracle.so")
SAN_LIB = os.path.join(HERE, "liboracle_san.so")


def sanitized() -> bool:
    """ORACLE_SANITIZE=1 selects a build with AddressSanitizer and UndefinedBehaviorSanitizer
    (host code only; run Python with LD_PRELOAD=$(gcc -print-file-name=libasan.so) and
    ASAN_OPTIONS=detect_leaks=0 so that the sanitizer runtime is loaded first)."""
    return os.environ.get("ORACLE_SANITIZE", "") not in ("", "0")


def build(force: bool = True) -> str:
    """Build liboracle.so (or its sanitized twin); with force=False only when missing or older
    than the source."""
    lib = SAN_LIB if sanitized() else LIB
    if not force and os.path.exists(lib) and os.path.getmtime(lib) >= os.path.getmtime(SRC):
        return lib
    opt = ["-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
           "-fno-omit-frame-pointer"] if sanitized() else ["-O2"]
    cmd = ["gcc"] + opt + ["-std=c99", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
                           "-fno-fast-math", "-Wall", "-Wextra", "-o", lib + ".tmp", SRC, "-lm"]
    subprocess.run(cmd, check=True)
    os.replace(lib + ".tmp", lib)
    return lib


if __name__ == "__main__":
    print(build(force=True))
    sys.exit(0)
