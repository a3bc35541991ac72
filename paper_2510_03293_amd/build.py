"""Build the HIP routing library in-tree with hipcc for gfx950."""
from __future__ import annotations

import os
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(_HERE, "csrc")
LIB_PATH = os.path.join(_HERE, "liblaser_route.so")
SOURCES = ["api.hip", "gate.hip", "gate_pipeline.hip", "gate_split.hip", "route.hip", "metrics.hip", "random.hip", "bench_helpers.hip"]

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


def _run(cmd):
    res = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in res.stderr.splitlines() if noise not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + err)
    return err


def build(verbose: bool = False) -> str:
    """Compile every source into liblaser_route.so (always recompiles).  The sources are
    compiled side by side (one hipcc each, objects in a temporary folder), then linked."""
    import concurrent.futures
    import tempfile
    flags = [f for f in HIPCC_FLAGS if f != "-shared"]
    with tempfile.TemporaryDirectory(prefix="laser_build_") as tmp:
        jobs = []
        for src in SOURCES:
            obj = os.path.join(tmp, os.path.splitext(src)[0] + ".o")
            jobs.append((["hipcc", *flags, "-c", os.path.join(CSRC, src), "-o", obj], obj))
        with concurrent.futures.ThreadPoolExecutor(max_workers=min(len(jobs), os.cpu_count() or 1, 8)) as pool:
            errs = list(pool.map(_run, [cmd for cmd, _ in jobs]))
        errs.append(_run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB_PATH,
                          *[obj for _, obj in jobs]]))
    if verbose:
        text = "\n".join(e for e in errs if e.strip())
        if text:
            print(text)
    return LIB_PATH


if __name__ == "__main__":
    print(build(verbose=True))
