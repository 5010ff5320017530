"""Compile the HIP library for gfx950 (cross-compiles without a GPU)."""
from __future__ import annotations

import glob
import hashlib
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "csrc", "ifx.hip")
LIB = os.path.join(HERE, "libifx.so")
STAMP = LIB + ".srchash"  # what the library next to it was built from

HIPCC_FLAGS = [
    "--offload-arch=gfx950",
    "-O3",
    "-std=c++17",
    "-fPIC",
    "-shared",
    # packed fp32 VALU forms are kept out of all device code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-fno-honor-nans",
    # the attention kernel pins its instruction order before register allocation
    # (sched_group_barrier); the post-RA scheduler only perturbs it (0.6 % measured)
    "-mllvm", "-enable-post-misched=false",
    # within the pinned groups the max-ILP pre-RA strategy orders a little better (0.4 % measured)
    "-mllvm", "-amdgpu-sched-strategy=max-ilp",
    "-Wall",
    "-Wno-unused-command-line-argument",
]


def source_hash() -> str:
    """A digest of everything the library is built from: the sources, the public header, the flags."""
    h = hashlib.sha256()
    files = sorted(glob.glob(os.path.join(HERE, "csrc", "*"))) + [os.path.join(os.path.dirname(HERE), "include", "ifx.h")]
    for f in files:
        h.update(os.path.basename(f).encode())
        with open(f, "rb") as fh:
            h.update(fh.read())
    h.update(" ".join(HIPCC_FLAGS).encode())
    return h.hexdigest()


def is_current() -> bool:
    """True if a built library is there and was built from the sources as they are now."""
    try:
        with open(STAMP) as f:
            return os.path.exists(LIB) and f.read().strip() == source_hash()
    except OSError:
        return False


def build_library(verbose: bool = False) -> str:
    """Run hipcc on csrc/ifx.hip and leave libifx.so (and the digest of its sources) next to this file."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, *HIPCC_FLAGS, "-o", LIB, SRC]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    # the host pass does not know the device-only target feature; that warning is noise
    err = "\n".join(l for l in res.stderr.splitlines() if "packed-fp32-ops" not in l)
    if res.returncode != 0:
        raise RuntimeError(f"hipcc failed ({res.returncode}):\n{err}")
    if verbose and err.strip():
        print(err)
    with open(STAMP, "w") as f:
        f.write(source_hash() + "\n")
    return LIB


if __name__ == "__main__":
    print(build_library(verbose=True))
