"""CPU oracle for the PQk-means iteration -- TEST INFRASTRUCTURE ONLY.

A ctypes binding over ``pqk_oracle.c`` (plain C, host pointers, numpy arrays).
Only ``tests/``, ``__graft_entry__.smoke()`` and ``bench.py``'s CPU-baseline
leg may import this package; the product path never does, and this package
imports nothing from the HIP side.

Function names follow the paper: tables (Sec. 2.2), assign (Eq. 5),
histogram (Eq. 7), vote (Eq. 8), update_naive (Eq. 6), fit (Alg. 1), encode / decode (Sec. 2.2).
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "pqk_oracle.c")
_LIB = os.path.join(_HERE, "libpqk_oracle.so")
L = 256


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain IEEE arithmetic, no contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c99", "-ffp-contract=off", "-fopenmp", "-shared", "-fPIC",
               "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        vp, i32, i64 = ctypes.c_void_p, ctypes.c_int, ctypes.c_int64
        lib.pqko_max_threads.restype = ctypes.c_int
        lib.pqko_set_threads.argtypes = [i32]
        lib.pqko_build_tables.argtypes = [vp, i32, i32, vp]
        lib.pqko_decode.argtypes = [vp, i32, i32, vp, i64, vp]
        lib.pqko_sdc_pairs.argtypes = [vp, vp, i64, i32, vp, vp]
        lib.pqko_assign.argtypes = [vp, i64, i32, vp, i32, vp, vp, vp]
        lib.pqko_histogram.argtypes = [vp, i64, i32, vp, i32, vp, vp]
        lib.pqko_vote.argtypes = [vp, vp, i32, i32, vp, vp]
        lib.pqko_update.argtypes = [vp, i64, i32, vp, i32, vp, vp, vp, vp]
        lib.pqko_update_naive.argtypes = [vp, i64, i32, vp, i32, vp, vp, vp]
        lib.pqko_objective.argtypes = [vp, i64, i32, vp, vp, vp]
        lib.pqko_objective.restype = ctypes.c_double
        lib.pqko_fit.argtypes = [vp, i64, i32, vp, i32, vp, i32, vp, vp, vp]
        lib.pqko_fit_until.argtypes = [vp, i64, i32, vp, i32, vp, i32, vp, vp, vp, vp]
        lib.pqko_fit_until.restype = ctypes.c_int
        lib.pqko_encode.argtypes = [vp, i64, i32, i32, vp, vp, vp]
        lib.pqko_encode.restype = None
        lib.pqko_decode_f32.argtypes = [vp, i32, i32, vp, i64, vp]
        lib.pqko_decode_f32.restype = None
        for name in ("pqko_set_threads", "pqko_build_tables", "pqko_decode", "pqko_sdc_pairs",
                     "pqko_assign", "pqko_histogram", "pqko_vote", "pqko_update",
                     "pqko_update_naive", "pqko_fit"):
            getattr(lib, name).restype = None
        _lib = lib
    return _lib


def _p(a):
    return ctypes.c_void_p(a.ctypes.data) if a is not None else ctypes.c_void_p(0)


def _chk(a, dtype, shape=None):
    a = np.ascontiguousarray(a, dtype=dtype)
    if shape is not None and tuple(a.shape) != tuple(shape):
        raise ValueError(f"expected shape {shape}, got {a.shape}")
    return a


def max_threads() -> int:
    return int(_load().pqko_max_threads())


def set_threads(n: int) -> None:
    _load().pqko_set_threads(int(n))


def build_tables(codewords) -> np.ndarray:
    """codewords [M][256][Ds] f32 -> tables [M][256][256] f32 (Sec. 2.2)."""
    cw = _chk(codewords, np.float32)
    M, l, Ds = cw.shape
    assert l == L
    tables = np.empty((M, L, L), dtype=np.float32)
    _load().pqko_build_tables(_p(cw), M, Ds, _p(tables))
    return tables


def decode(codewords, codes) -> np.ndarray:
    """codes [N][M] u8 -> reconstructed vectors [N][M*Ds] f64 (Sec. 2.2)."""
    cw = _chk(codewords, np.float32)
    M, _, Ds = cw.shape
    codes = _chk(codes, np.uint8)
    N = codes.shape[0]
    assert codes.shape == (N, M)
    out = np.empty((N, M * Ds), dtype=np.float64)
    _load().pqko_decode(_p(cw), M, Ds, _p(codes), N, _p(out))
    return out


def encode(vectors, codewords, want_dist: bool = False):
    """Sec. 2.2: vectors [N][M*Ds] f32 -> codes [N][M] u8 (and the squared distances [N][M] f32)."""
    cw = _chk(codewords, np.float32)
    M, l, Ds = cw.shape
    assert l == L
    v = _chk(vectors, np.float32)
    N = v.shape[0]
    assert v.shape == (N, M * Ds)
    codes = np.empty((N, M), dtype=np.uint8)
    d2 = np.empty((N, M), dtype=np.float32) if want_dist else None
    _load().pqko_encode(_p(v), N, M, Ds, _p(cw), _p(codes), _p(d2))
    return (codes, d2) if want_dist else codes


def decode_f32(codewords, codes) -> np.ndarray:
    """codes [N][M] u8 -> reconstructed vectors [N][M*Ds] f32 (the codewords themselves)."""
    cw = _chk(codewords, np.float32)
    M, _, Ds = cw.shape
    codes = _chk(codes, np.uint8)
    N = codes.shape[0]
    assert codes.shape == (N, M)
    out = np.empty((N, M * Ds), dtype=np.float32)
    _load().pqko_decode_f32(_p(cw), M, Ds, _p(codes), N, _p(out))
    return out


def sdc_pairs(x, y, tables) -> np.ndarray:
    """Eq. 3 for P code pairs: x, y [P][M] u8 -> [P] f32."""
    tables = _chk(tables, np.float32)
    M = tables.shape[0]
    x = _chk(x, np.uint8)
    y = _chk(y, np.uint8)
    P = x.shape[0]
    assert x.shape == (P, M) and y.shape == (P, M)
    out = np.empty(P, dtype=np.float32)
    _load().pqko_sdc_pairs(_p(x), _p(y), P, M, _p(tables), _p(out))
    return out


def assign(codes, centers, tables, want_dist: bool = True):
    """Eq. 5: -> (assign [N] i32, dist [N] f32 or None)."""
    tables = _chk(tables, np.float32)
    M = tables.shape[0]
    codes = _chk(codes, np.uint8)
    centers = _chk(centers, np.uint8)
    N, K = codes.shape[0], centers.shape[0]
    assert codes.shape == (N, M) and centers.shape == (K, M) and K >= 1
    a = np.empty(N, dtype=np.int32)
    d = np.empty(N, dtype=np.float32) if want_dist else None
    _load().pqko_assign(_p(codes), N, M, _p(centers), K, _p(tables), _p(a), _p(d))
    return a, d


def histogram(codes, assign_, K: int):
    """Eq. 7: -> (hist [K][M][256] u32, counts [K] u32)."""
    codes = _chk(codes, np.uint8)
    N, M = codes.shape
    assign_ = _chk(assign_, np.int32, (N,))
    if N and (assign_.min() < 0 or assign_.max() >= K):
        raise ValueError("assignment out of range")
    hist = np.empty((K, M, L), dtype=np.uint32)
    counts = np.empty(K, dtype=np.uint32)
    _load().pqko_histogram(_p(codes), N, M, _p(assign_), K, _p(hist), _p(counts))
    return hist, counts


def vote(hist, counts, tables, centers) -> np.ndarray:
    """Eq. 8: returns the updated copy of centers [K][M] u8."""
    tables = _chk(tables, np.float32)
    M = tables.shape[0]
    hist = _chk(hist, np.uint32)
    K = hist.shape[0]
    assert hist.shape == (K, M, L)
    counts = _chk(counts, np.uint32, (K,))
    out = _chk(centers, np.uint8, (K, M)).copy()
    _load().pqko_vote(_p(hist), _p(counts), K, M, _p(tables), _p(out))
    return out


def update(codes, assign_, tables, centers):
    """Eq. 7 + Eq. 8: -> (new centers, hist, counts)."""
    K = np.asarray(centers).shape[0]
    hist, counts = histogram(codes, assign_, K)
    return vote(hist, counts, tables, centers), hist, counts


def update_naive(codes, assign_, tables, centers, want_cost: bool = False):
    """Eq. 6 in fp64: -> new centers (and the [K][M][256] fp64 sums)."""
    tables = _chk(tables, np.float32)
    M = tables.shape[0]
    codes = _chk(codes, np.uint8)
    N = codes.shape[0]
    out = _chk(centers, np.uint8).copy()
    K = out.shape[0]
    assign_ = _chk(assign_, np.int32, (N,))
    if N and (assign_.min() < 0 or assign_.max() >= K):
        raise ValueError("assignment out of range")
    cost = np.empty((K, M, L), dtype=np.float64) if want_cost else None
    _load().pqko_update_naive(_p(codes), N, M, _p(assign_), K, _p(tables), _p(out), _p(cost))
    return (out, cost) if want_cost else out


def objective(codes, centers, assign_, tables) -> float:
    """Sum over n of the squared SD to the assigned center, in fp64."""
    tables = _chk(tables, np.float32)
    M = tables.shape[0]
    codes = _chk(codes, np.uint8)
    centers = _chk(centers, np.uint8)
    N = codes.shape[0]
    assign_ = _chk(assign_, np.int32, (N,))
    return float(_load().pqko_objective(_p(codes), N, M, _p(centers), _p(assign_), _p(tables)))


def fit(codes, tables, centers, iters: int):
    """Alg. 1 (linear scan): -> (centers, assign of the last assignment, hist, counts)."""
    tables = _chk(tables, np.float32)
    M = tables.shape[0]
    codes = _chk(codes, np.uint8)
    N = codes.shape[0]
    out = _chk(centers, np.uint8).copy()
    K = out.shape[0]
    a = np.zeros(N, dtype=np.int32)
    hist = np.zeros((K, M, L), dtype=np.uint32)
    counts = np.zeros(K, dtype=np.uint32)
    _load().pqko_fit(_p(codes), N, M, _p(tables), K, _p(out), int(iters), _p(a), _p(hist), _p(counts))
    return out, a, hist, counts


def fit_until(codes, tables, centers, max_iters: int):
    """Alg. 1 until no assignment changes (or max_iters):
    -> (centers, assign, hist, counts, stats [iters][4] = objective, changed, nonzero bins, nonempty clusters)."""
    tables = _chk(tables, np.float32)
    M = tables.shape[0]
    codes = _chk(codes, np.uint8)
    N = codes.shape[0]
    out = _chk(centers, np.uint8).copy()
    K = out.shape[0]
    a = np.zeros(N, dtype=np.int32)
    hist = np.zeros((K, M, L), dtype=np.uint32)
    counts = np.zeros(K, dtype=np.uint32)
    stats = np.zeros((max(int(max_iters), 1), 4), dtype=np.float64)
    it = _load().pqko_fit_until(_p(codes), N, M, _p(tables), K, _p(out), int(max_iters), _p(a), _p(hist),
                                _p(counts), _p(stats))
    return out, a, hist, counts, stats[:it].copy()
