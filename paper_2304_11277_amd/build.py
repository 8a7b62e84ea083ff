"""Build libfsdp_flat.so (HIP, gfx950 only) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libfsdp_flat.so")
SOURCES = [os.path.join(CSRC, "fsdp_layout.cpp"), os.path.join(CSRC, "fsdp_kernels.hip")]
HEADERS = [os.path.join(ROOT, "include", "fsdp_flat.h")] + [
    os.path.join(CSRC, h) for h in ("fsdp_internal.h", "device_common.h", "unshard_kernels.h", "pack_kernel.h",
                                    "reduce_kernels.h", "batch_kernel.h", "elementwise_kernels.h")]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-ffp-contract=off",            # bit-exact rank-ordered sums and Adam: no fused multiply-add
    "-fno-fast-math",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",   # no packed-fp32 instructions
    "-Wall", "-Wextra", "-Wno-unused-parameter",
]


def hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.isabs(cand) and os.path.exists(cand) or not os.path.isabs(cand)):
            return cand
    return "hipcc"


def is_stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(f) > t for f in SOURCES + HEADERS)


def build_lib(force: bool = True, verbose: bool = False) -> str:
    """Compile the library.  `force=False` skips the compile when the built
    library is newer than every source."""
    if not force and not is_stale():
        return LIB
    tmp = LIB + f".tmp{os.getpid()}"
    cmd = [hipcc(), *HIPCC_FLAGS, "-x", "hip", *SOURCES, "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-o", tmp]
    if verbose:
        print(" ".join(cmd), file=sys.stderr)
    subprocess.check_call(cmd)
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build_lib(force=True, verbose=True))
