"""Compile the CPU oracle into oracle/libfcv2_oracle.so (test infrastructure, not the product).

build(sanitize=True) makes a second library, libfcv2_oracle_asan.so, with AddressSanitizer and
UndefinedBehaviorSanitizer in it; the CPU test suite runs the oracle's pins through it in a child process."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "fcv2_oracle.cpp")
LIB = os.path.join(HERE, "libfcv2_oracle.so")
LIB_ASAN = os.path.join(HERE, "libfcv2_oracle_asan.so")
SANITIZE = ["-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer", "-g"]


def build(force: bool = False, sanitize: bool = False) -> str:
    lib = LIB_ASAN if sanitize else LIB
    if not force and os.path.exists(lib) and os.path.getmtime(lib) >= max(
        os.path.getmtime(SRC), os.path.getmtime(os.path.join(HERE, "fcv2_oracle.h"))
    ):
        return lib
    cmd = ["g++", "-std=c++17", "-O1" if sanitize else "-O2", "-ffp-contract=off", "-fPIC", "-shared", "-Wall", "-Wextra"]
    cmd += (SANITIZE if sanitize else []) + ["-o", lib + ".tmp", SRC]
    subprocess.run(cmd, check=True, cwd=HERE)
    os.replace(lib + ".tmp", lib)
    return lib


if __name__ == "__main__":
    print(build(force="--force" in sys.argv, sanitize="--sanitize" in sys.argv))
