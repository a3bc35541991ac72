"""Build the HIP routing library in-tree with hipcc for gfx950."""
from __future__ import annotations

import os
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(_HERE, "csrc")
LIB_PATH = os.path.join(_HERE, "liblaser_route.so")
SOURCES = ["api.hip", "gate.hip", "route.hip", "metrics.hip", "random.hip", "bench_helpers.hip"]

# -ffp-contract=off: the routing decisions follow a fixed binary32 operation
# order; fused multiply-adds appear only where the source writes them.
# packed-fp32-ops is switched off because the compiler-formed packed FP32
# instructions are not trusted on this hardware.
HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-ffp-contract=off", "-fno-fast-math",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument",
]


def build(verbose: bool = False) -> str:
    """Compile every source into liblaser_route.so (always recompiles)."""
    srcs = [os.path.join(CSRC, s) for s in SOURCES]
    cmd = ["hipcc", *HIPCC_FLAGS, "-o", LIB_PATH, *srcs]
    res = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in res.stderr.splitlines() if noise not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + err)
    if verbose and err.strip():
        print(err)
    return LIB_PATH


if __name__ == "__main__":
    print(build(verbose=True))
