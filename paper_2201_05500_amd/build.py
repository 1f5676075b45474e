"""Builds libctr_sparse.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(_HERE, "csrc")
LIB = os.path.join(_HERE, "libctr_sparse.so")
SMOKE_SRC = os.path.join(CSRC, "standalone", "abi_smoke.c")   # plain C user of the ABI (no Python, no PyTorch)
SMOKE_BIN = os.path.join(_HERE, "abi_smoke")
INCLUDE = os.path.join(os.path.dirname(_HERE), "include")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-Wall",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]


def sources():
    return [os.path.join(CSRC, f) for f in sorted(os.listdir(CSRC)) if f.endswith(".hip")]


def source_hash() -> str:
    """Short hash of every kernel and host source of the library: ties a measurement to the code it was taken on."""
    import hashlib
    h = hashlib.sha256()
    for name in sorted(os.listdir(CSRC)):
        if name.endswith((".hip", ".h")):
            with open(os.path.join(CSRC, name), "rb") as f:
                h.update(name.encode() + b"\0" + f.read())
    return h.hexdigest()[:16]


def build_variant(out: str, defines, verbose: bool = False) -> str:
    """The library alone, with extra -D switches, written to `out` (for A/B measurements of the compile-time
    variants the kernels' headers document; load it with CTR_SPARSE_LIB=<out>)."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc] + HIPCC_FLAGS + ["-D" + d for d in defines] + ["-o", out] + sources()
    if verbose:
        print(" ".join(cmd))
    subprocess.check_call(cmd)
    return out


def build(verbose: bool = False) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc] + HIPCC_FLAGS + ["-o", LIB] + sources()
    if verbose:
        print(" ".join(cmd))
    subprocess.check_call(cmd)
    # the stand-alone C program: host compiler only, linked against the library just built
    rocm = os.environ.get("ROCM_PATH", "/opt/rocm")
    cc = ["gcc", "-std=gnu11", "-O2", "-Wall", "-Wextra", "-D__HIP_PLATFORM_AMD__", "-I" + INCLUDE,
          "-I" + os.path.join(rocm, "include"), SMOKE_SRC, "-o", SMOKE_BIN, "-L" + _HERE, "-lctr_sparse",
          "-L" + os.path.join(rocm, "lib"), "-lamdhip64", "-lm", "-Wl,-rpath,$ORIGIN", "-Wl,-rpath," + os.path.join(rocm, "lib")]
    if verbose:
        print(" ".join(cc))
    subprocess.check_call(cc)
    return LIB


if __name__ == "__main__":
    import argparse
    ap = argparse.ArgumentParser(description="build libctr_sparse.so, or a variant of it with extra defines")
    ap.add_argument("--define", "-D", action="append", default=[], help="NAME=VALUE, repeatable")
    ap.add_argument("--out", help="write a variant build here instead of building the in-tree library")
    a = ap.parse_args()
    print(build_variant(a.out, a.define, verbose=True) if a.out else build(verbose=True))
