"""Compile the CPU oracle (test infrastructure) into oracle/liboracle_compams.so.

Plain g++, single translation unit, IEEE arithmetic: no fast-math and no fused
multiply-add contraction, so that every fp32 operation rounds once.
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "compams_oracle.cpp")
LIB = os.path.join(HERE, "liboracle_compams.so")

FLAGS = ["-O2", "-std=c++17", "-fPIC", "-shared", "-ffp-contract=off", "-fno-fast-math",
         "-Wall", "-Wextra"]


def build(force: bool = False, sanitize: bool = False) -> str:
    lib = LIB if not sanitize else os.path.join(HERE, "liboracle_compams_asan.so")
    if (not force and os.path.exists(lib)
            and os.path.getmtime(lib) >= os.path.getmtime(SRC)):
        return lib
    # the sanitizer build stops at the first finding (no recovery), so that a test run under it fails loudly
    cmd = ["g++"] + FLAGS + (["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-g"] if sanitize else []) \
        + [SRC, "-o", lib]
    subprocess.run(cmd, check=True)
    return lib


if __name__ == "__main__":
    print(build(force=True, sanitize="--sanitize" in sys.argv))
