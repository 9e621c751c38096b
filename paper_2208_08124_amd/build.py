"""Builds libfmha_varlen.so (HIP, gfx950 only) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libfmha_varlen.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # the item feed's claims are single-lane atomics whose answers are needed much later:
    # the compiler's wave-wide combining of atomics would wait for them on the spot
    "-mllvm", "-amdgpu-atomic-optimizer-strategy=None",
    "-Wall", "-Wno-unused-value",
]


def sources():
    return [os.path.join(CSRC, f) for f in sorted(os.listdir(CSRC)) if f.endswith(".hip")]


ATTENTION_SOURCES = ("fmha_varlen.hip", "fwd64_kernel.h", "fwd_kernel.h", "bwd_kernels.h", "mfma_tiles.h",
                     "kernel_args.h", "item_feed.h", "schedule.h", "dropout.h")


def source_id() -> str:
    """Identifies what the attention kernels are built from: a hash over their sources and
    the compiler flags.  Measurements of them that are stored in the repository (HBM traffic
    from counter runs) carry it, so that a stored figure is never quoted for other kernels."""
    import hashlib
    h = hashlib.sha256(" ".join(HIPCC_FLAGS).encode())
    for name in ATTENTION_SOURCES:
        h.update(name.encode())
        with open(os.path.join(CSRC, name), "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()[:16]


def build(verbose: bool = False) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, *HIPCC_FLAGS, "-o", LIB, *sources()]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
