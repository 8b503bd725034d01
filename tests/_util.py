"""Shared helpers for the GPU parity tests (test infrastructure; may use the oracle)."""
from __future__ import annotations

import dataclasses
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
_T0 = time.time()


def progress(msg: str) -> None:
    """A progress line that survives pytest's capture (long tests must not look hung)."""
    line = f"[{time.time() - _T0:7.1f}s] {msg}\n"
    try:
        sys.__stderr__.write(line)
        sys.__stderr__.flush()
    except Exception:
        pass
    try:
        d = os.path.join(ROOT, "gpurun_out")
        os.makedirs(d, exist_ok=True)
        with open(os.path.join(d, "test_progress.log"), "a") as f:
            f.write(line)
    except Exception:
        pass


def workload(cfg: int, **over):
    import workloads as W

    return dataclasses.replace(W.CONFIGS[cfg], **over) if over else W.CONFIGS[cfg]


def u32(t):
    """torch int32 device tensor -> numpy uint32."""
    return t.cpu().numpy().view(np.uint32)


def rand_tables(rng, M, integer=False):
    if integer:
        return np.ascontiguousarray(rng.integers(0, 50, size=(M, 256, 256)).astype(np.float32))
    return np.ascontiguousarray((rng.random((M, 256, 256), dtype=np.float32) * 10 + 0.1).astype(np.float32))
