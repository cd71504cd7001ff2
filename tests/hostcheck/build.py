"""Compile the host-check helper: the integer/float building blocks of the kernels (csrc/fcv2_bits.h) built for
the CPU behind a C interface, so that the CPU tests can run exactly the sequences the kernels run.
Test infrastructure; nothing in the product package loads it."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
SRC = os.path.join(HERE, "fcv2_hostcheck.cpp")
DEPS = [SRC, os.path.join(ROOT, "paper_2508_03760_amd", "csrc", "fcv2_bits.h")]
SANITIZE = ["-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer", "-g"]


def lib_path(sanitize: bool = False) -> str:
    return os.path.join(HERE, "libfcv2_hostcheck_asan.so" if sanitize else "libfcv2_hostcheck.so")


def build(force: bool = False, sanitize: bool = False) -> str:
    so = lib_path(sanitize)
    if not force and os.path.exists(so) and os.path.getmtime(so) >= max(os.path.getmtime(d) for d in DEPS):
        return so
    cmd = ["g++", "-std=c++17", "-O1" if sanitize else "-O2", "-ffp-contract=off", "-fPIC", "-shared", "-Wall"]
    cmd += (SANITIZE if sanitize else []) + ["-o", so + ".tmp", SRC]
    subprocess.run(cmd, check=True, cwd=HERE)
    os.replace(so + ".tmp", so)
    return so


if __name__ == "__main__":
    print(build(force=True))
