"""Build libpquant.so (HIP, gfx950) and the C pieces of the oracle in-tree."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libpquant.so")
SOURCES = ["pq_api.hip", "pq_quant.hip", "pq_gemm.hip", "pq_decode.hip", "pq_moe.hip", "pq_ffn.hip", "pq_groupwise.hip"]

HIPCC_FLAGS = [
    "-O3", "--offload-arch=gfx950", "-std=c++17", "-fPIC", "-shared",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",   # no packed-fp32 instructions
    "-ffp-contract=off",                                            # quantiser products stay un-fused
    "-Wall", "-Wno-unused-function",
]


def build(verbose: bool = True, extra_flags=(), out: str = LIB) -> str:
    srcs = [os.path.join(CSRC, s) for s in SOURCES]
    cmd = ["hipcc", *HIPCC_FLAGS, *extra_flags, "-I", os.path.join(HERE, "..", "include"), *srcs, "-o", out]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    out = "\n".join(l for l in (res.stdout + res.stderr).splitlines()
                    if "packed-fp32-ops" not in l)      # the host pass does not know the device feature
    if verbose and out.strip():
        print(out, flush=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    return out


if __name__ == "__main__":
    build(extra_flags=sys.argv[1:])
