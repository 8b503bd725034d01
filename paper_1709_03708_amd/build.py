"""Build libpqkm.so and the microbenchmark library libpqkm_microbench.so (HIP, gfx950) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
LIB = os.path.join(HERE, "libpqkm.so")
SOURCES = [os.path.join(HERE, "csrc", "pqkm.hip")]
DEPS = SOURCES + [os.path.join(HERE, "csrc", "pqkm_kernels.h"), os.path.join(ROOT, "include", "pqkm.h"),
                  os.path.join(ROOT, "include", "pqkm_tuning.h")]
MICROBENCH_LIB = os.path.join(HERE, "libpqkm_microbench.so")          # measurement code, loaded by bench.py only
MICROBENCH_SOURCES = [os.path.join(HERE, "csrc", "microbench.hip")]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-ffp-contract=off",                      # the only fused operation is the vote's explicit fmaf
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-value",
]


def stale() -> bool:
    if not os.path.exists(LIB) or not os.path.exists(MICROBENCH_LIB):
        return True
    t = os.path.getmtime(LIB)
    if os.path.getmtime(MICROBENCH_SOURCES[0]) > os.path.getmtime(MICROBENCH_LIB):
        return True
    return any(os.path.getmtime(d) > t for d in DEPS)


def build(force: bool = True, verbose: bool = False) -> str:
    """Compile the library; returns its path.  Raises on compiler errors."""
    if not force and not stale():
        return LIB
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, *HIPCC_FLAGS, "-I", os.path.join(ROOT, "include"), "-o", LIB, *SOURCES]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if verbose or res.returncode != 0:
        print(res.stdout)
        print(res.stderr)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed: " + " ".join(cmd))
    cmd = [hipcc, *HIPCC_FLAGS, "-o", MICROBENCH_LIB, *MICROBENCH_SOURCES]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if verbose or res.returncode != 0:
        print(res.stdout)
        print(res.stderr)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed: " + " ".join(cmd))
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
