"""Builds libaes_spmm.so (hipcc, gfx950) in-tree next to the sources."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libaes_spmm.so")
SOURCES = ["aes_common.cpp", "sample_build.hip", "spmm_f32.hip", "spmm_q8.hip", "quantize.hip", "gcn_layer.hip"]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-fno-gpu-rdc",
    # one rounding per written float operation; fused multiply-adds are explicit in the sources
    "-ffp-contract=off", "-fhip-fp32-correctly-rounded-divide-sqrt",
    # packed-fp32 VALU forms are kept out of the generated code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


STAMP = LIB + ".srchash"      # hash of the sources and flags the library next to it was built from


def lib_path() -> str:
    return LIB


def source_hash() -> str:
    """Hash of everything the library is built from: csrc/*, the public header, the compiler flags."""
    import hashlib
    h = hashlib.sha256(" ".join(HIPCC_FLAGS).encode())
    files = sorted(os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith((".hip", ".hpp", ".cpp", ".h")))
    for path in files + [os.path.join(ROOT, "include", "aes_spmm.h")]:
        h.update(os.path.basename(path).encode())
        with open(path, "rb") as f:
            h.update(f.read())
    return h.hexdigest()


def is_current() -> bool:
    """True if a built library is present and was built from the sources as they are now."""
    if not (os.path.exists(LIB) and os.path.exists(STAMP)):
        return False
    with open(STAMP) as f:
        return f.read().strip() == source_hash()


def _compile(hipcc: str, src: str, obj: str, verbose: bool) -> None:
    flags = [f for f in HIPCC_FLAGS if f != "-shared"]
    cmd = [hipcc] + flags + ["-I", os.path.join(ROOT, "include"), "-I", CSRC, "-x", "hip", "-c", src, "-o", obj]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)


def build(verbose: bool = False) -> str:
    """Compile every source to an object (in parallel) under _build/, then link the shared library."""
    from concurrent.futures import ThreadPoolExecutor

    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    jobs = [(os.path.join(CSRC, s), os.path.join(objdir, os.path.splitext(s)[0] + ".o")) for s in SOURCES]
    with ThreadPoolExecutor(max_workers=min(len(jobs), 8)) as pool:
        list(pool.map(lambda j: _compile(hipcc, j[0], j[1], verbose), jobs))
    link = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-fno-gpu-rdc"] + [o for _, o in jobs] + ["-o", LIB]
    if verbose:
        print(" ".join(link), flush=True)
    if os.path.exists(STAMP):
        os.remove(STAMP)
    stamp = source_hash()
    subprocess.run(link, check=True)
    with open(STAMP, "w") as f:
        f.write(stamp + "\n")
    return LIB


if __name__ == "__main__":
    build(verbose=True)
    print(LIB)
    sys.exit(0)
