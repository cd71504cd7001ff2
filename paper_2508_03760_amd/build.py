"""Compile libfcv2 (HIP kernels + C ABI) for gfx950 into paper_2508_03760_amd/libfcv2.so."""
import hashlib
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libfcv2.so")
SOURCES = ["fcv2_api.hip", "fcv2_quantize.hip", "fcv2_unpack.hip", "fcv2_reduce.hip", "fcv2_dispatch.hip"]
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    "-ffp-contract=off",  # the codec's arithmetic is specified step by step: no fused multiply-adds by surprise
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


def lib_path() -> str:
    return LIB


def source_digest() -> str:
    """Digest of everything the library is compiled from (sources, headers, flags)."""
    h = hashlib.sha256(" ".join(FLAGS).encode())
    inc = os.path.join(os.path.dirname(HERE), "include")
    files = [os.path.join(CSRC, f) for f in sorted(os.listdir(CSRC)) if f.endswith((".hip", ".h"))]
    files += [os.path.join(inc, f) for f in sorted(os.listdir(inc)) if f.endswith(".h")]
    for f in files:
        h.update(os.path.basename(f).encode())
        h.update(open(f, "rb").read())
    return h.hexdigest()


def is_current() -> bool:
    """True if a built library is there and was built from the sources as they are now (the digest written next to it
    at build time matches).  Content, not time stamps: a copy of the tree to another machine keeps the answer."""
    try:
        return os.path.exists(LIB) and open(LIB + ".srchash").read().strip() == source_digest()
    except OSError:
        return False


def build(verbose: bool = False) -> str:
    """Always compiles (one object per source, in parallel), links, and returns the path of the shared library."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    procs = []
    for s in SOURCES:
        obj = os.path.join(objdir, s.replace(".hip", ".o"))
        cmd = [hipcc] + FLAGS + ["-c", os.path.join(CSRC, s), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((cmd, obj, subprocess.Popen(cmd, cwd=CSRC)))
    objs = []
    for cmd, obj, p in procs:
        if p.wait() != 0:
            raise subprocess.CalledProcessError(p.returncode, cmd)
        objs.append(obj)
    link = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC"] + objs + ["-o", LIB + ".tmp"]
    if verbose:
        print(" ".join(link), flush=True)
    subprocess.run(link, check=True, cwd=CSRC)
    os.replace(LIB + ".tmp", LIB)
    with open(LIB + ".srchash", "w") as f:
        f.write(source_digest() + "\n")
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
