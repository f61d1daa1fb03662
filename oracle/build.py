"""Compile the C oracle (test infrastructure) into oracle/liboracle.so with gcc.

`build(sanitize=True)` (or `python oracle/build.py --sanitize`) makes an AddressSanitizer + UBSan
build, oracle/_build/liboracle_san.so, with the clang of the ROCm toolchain so that it shares one
sanitizer runtime with the sanitizer build of libtl.so; ORACLE_LIB_PATH selects it at run time.
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "ternary_oracle.c")
LIB = os.path.join(HERE, "liboracle.so")
SAN_LIB = os.path.join(HERE, "_build", "liboracle_san.so")


def build(force=True, sanitize=False):
    if sanitize:
        os.makedirs(os.path.dirname(SAN_LIB), exist_ok=True)
        clang = os.environ.get("ROCM_CLANG", "/opt/rocm/lib/llvm/bin/clang")
        cmd = [clang, "-O1", "-g", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
               "-fsanitize=address", "-fsanitize=undefined", "-fno-omit-frame-pointer", "-shared-libsan",
               "-o", SAN_LIB, SRC, "-lm"]
        subprocess.run(cmd, check=True)
        return SAN_LIB
    override = os.environ.get("ORACLE_LIB_PATH")
    if override and not force:
        return override
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= os.path.getmtime(SRC):
        return LIB
    cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
           "-o", LIB, SRC, "-lm"]
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build(sanitize="--sanitize" in sys.argv))
