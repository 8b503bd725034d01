"""Counter-based synthetic PQ codes.

The paper clusters PQ codes of SIFT1M/SIFT1B (128-D), ILSVRC and YFCC100M CNN
features (4096-D) and Deep1B (Tab. 2); none of those datasets is available, so
seeded synthetic codes of the same shape stand in for them:

* codewords ``[M][256][D/M]`` fp32 drawn from a named distribution,
* ``T`` template codes of M uniform bytes,
* code n copies a uniformly chosen template and, independently per subspace,
  replaces the subcode by a fresh uniform byte with probability ``p``
  (clustered codes => sparse per-cluster histograms, as in Tab. 3),
* initial centers are the codes at K distinct seeded indices (Alg. 1, Init()).

Every random byte is a pure function of ``(seed, stream, counter)`` through a
64-bit avalanche mixer, so any subset of a billion-code workload can be
regenerated on the host, and the same bytes can be produced on the GPU with
plain torch integer ops.  Nothing here computes a distance, a histogram or a
vote.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

_MASK = (1 << 64) - 1
_GOLD = 0x9E3779B97F4A7C15
_C1 = 0xBF58476D1CE4E5B9
_C2 = 0x94D049BB133111EB

STREAM_TEMPLATE, STREAM_PICK, STREAM_CODE, STREAM_INIT = 1, 2, 3, 4


@dataclass(frozen=True)
class Workload:
    name: str
    D: int
    M: int
    N: int
    K: int
    T: int            # number of template codes
    p: float          # per-subspace corruption probability
    iters: int
    cw_dist: str      # "normal" | "absnormal20" | "relu"
    seed: int

    @property
    def Ds(self) -> int:
        return self.D // self.M


_BASE = 170903708 * 10
CONFIGS = {
    1: Workload("tiny", 128, 4, 10_000, 100, 50, 0.3, 5, "normal", _BASE + 1),
    2: Workload("sift32", 128, 4, 1_000_000, 1_000, 2_000, 0.3, 10, "absnormal20", _BASE + 2),
    3: Workload("sift64", 128, 8, 10_000_000, 10_000, 20_000, 0.3, 5, "absnormal20", _BASE + 3),
    4: Workload("cnn", 4096, 32, 100_000_000, 10_000, 10_000, 0.2, 3, "relu", _BASE + 4),
    5: Workload("billion", 128, 4, 1_000_000_000, 100_000, 200_000, 0.3, 1, "absnormal20", _BASE + 5),
}


# ---------------------------------------------------------------- scalar / numpy mixer
def _mix_int(z: int) -> int:
    z &= _MASK
    z = ((z ^ (z >> 30)) * _C1) & _MASK
    z = ((z ^ (z >> 27)) * _C2) & _MASK
    return z ^ (z >> 31)


def _stream_key(seed: int, stream: int) -> int:
    return _mix_int(_mix_int(seed) + stream * _GOLD)


def _mix_np(z: np.ndarray) -> np.ndarray:
    z = z.astype(np.uint64, copy=True)
    z ^= z >> np.uint64(30)
    z *= np.uint64(_C1)
    z ^= z >> np.uint64(27)
    z *= np.uint64(_C2)
    z ^= z >> np.uint64(31)
    return z


def _draw_np(key: int, counter: np.ndarray) -> np.ndarray:
    """u64 draw for each counter value (uint64 array)."""
    with np.errstate(over="ignore"):
        return _mix_np(np.uint64(key) + (counter.astype(np.uint64) + np.uint64(1)) * np.uint64(_GOLD))


# ---------------------------------------------------------------- pieces
def codewords(w: Workload) -> np.ndarray:
    """[M][256][Ds] fp32 codewords from the workload's distribution."""
    rng = np.random.default_rng(w.seed)
    x = rng.standard_normal((w.M, 256, w.Ds))
    if w.cw_dist == "normal":
        pass
    elif w.cw_dist == "absnormal20":
        x = np.abs(20.0 * x)
    elif w.cw_dist == "relu":
        x = np.maximum(x, 0.0)
    else:
        raise ValueError(w.cw_dist)
    return x.astype(np.float32)


def templates(w: Workload) -> np.ndarray:
    """[T][M] uint8 template codes."""
    key = _stream_key(w.seed, STREAM_TEMPLATE)
    ctr = np.arange(w.T * w.M, dtype=np.uint64)
    return (_draw_np(key, ctr) >> np.uint64(56)).astype(np.uint8).reshape(w.T, w.M)


def _thr(w: Workload) -> int:
    return int(round(w.p * (1 << 24)))


def codes_at(w: Workload, idx: np.ndarray, tmpl: np.ndarray | None = None) -> np.ndarray:
    """Codes [len(idx)][M] uint8 for arbitrary code indices (host, numpy)."""
    idx = np.asarray(idx, dtype=np.uint64).ravel()
    tmpl = templates(w) if tmpl is None else tmpl
    kp = _stream_key(w.seed, STREAM_PICK)
    kc = _stream_key(w.seed, STREAM_CODE)
    u = _draw_np(kp, idx)
    t = ((u >> np.uint64(32)) * np.uint64(w.T)) >> np.uint64(32)
    base = tmpl[t.astype(np.int64)]                                   # [n][M]
    ctr = idx[:, None] * np.uint64(64) + np.arange(w.M, dtype=np.uint64)[None, :]
    v = _draw_np(kc, ctr)
    corrupt = (v >> np.uint64(40)) < np.uint64(_thr(w))
    fresh = ((v >> np.uint64(8)) & np.uint64(0xFF)).astype(np.uint8)
    return np.where(corrupt, fresh, base).astype(np.uint8)


def codes_numpy(w: Workload, start: int = 0, count: int | None = None, chunk: int = 1 << 20) -> np.ndarray:
    """Codes [count][M] uint8 for indices start..start+count-1 (host, chunked)."""
    count = w.N - start if count is None else count
    out = np.empty((count, w.M), dtype=np.uint8)
    tmpl = templates(w)
    for s in range(0, count, chunk):
        e = min(count, s + chunk)
        out[s:e] = codes_at(w, np.arange(start + s, start + e, dtype=np.uint64), tmpl)
    return out


# ---------------------------------------------------------------- torch (device-side) generator
def _s64(x: int) -> int:
    x &= _MASK
    return x - (1 << 64) if x >= (1 << 63) else x


def _shr_t(z, s: int):
    return (z >> s) & ((1 << (64 - s)) - 1)


def _mix_t(z):
    z = (z ^ _shr_t(z, 30)) * _s64(_C1)
    z = (z ^ _shr_t(z, 27)) * _s64(_C2)
    return z ^ _shr_t(z, 31)


def _draw_t(key: int, counter):
    return _mix_t((counter + 1) * _s64(_GOLD) + _s64(key))


def codes_torch(w: Workload, device, start: int = 0, count: int | None = None, chunk: int = 1 << 24, out=None):
    """Same bytes as :func:`codes_numpy`, produced with torch int64 ops on ``device``.

    int64 arithmetic wraps modulo 2**64, logical right shifts are emulated by
    masking, so the bit patterns equal the uint64 host computation.
    """
    import torch

    count = w.N - start if count is None else count
    if out is None:
        out = torch.empty((count, w.M), dtype=torch.uint8, device=device)
    tmpl = torch.from_numpy(templates(w)).to(device)
    kp = _stream_key(w.seed, STREAM_PICK)
    kc = _stream_key(w.seed, STREAM_CODE)
    marange = torch.arange(w.M, dtype=torch.int64, device=device)[None, :]
    thr = _thr(w)
    for s in range(0, count, chunk):
        e = min(count, s + chunk)
        idx = torch.arange(start + s, start + e, dtype=torch.int64, device=device)
        u = _draw_t(kp, idx)
        t = (_shr_t(u, 32) * w.T) >> 32
        base = tmpl[t]
        v = _draw_t(kc, idx[:, None] * 64 + marange)
        corrupt = _shr_t(v, 40) < thr
        fresh = (_shr_t(v, 8) & 0xFF).to(torch.uint8)
        out[s:e] = torch.where(corrupt, fresh, base)
        del idx, u, t, base, v, corrupt, fresh
    return out


def init_center_indices(w: Workload) -> np.ndarray:
    """K distinct code indices in seeded draw order (Alg. 1, Init(): K codes picked at random)."""
    key = _stream_key(w.seed, STREAM_INIT)
    need, got, seen, pos = w.K, [], set(), 0
    if w.K > w.N:
        raise ValueError("K > N")
    while len(got) < need:
        n = max(1024, 2 * (need - len(got)))
        u = _draw_np(key, np.arange(pos, pos + n, dtype=np.uint64))
        pos += n
        # multiply-shift into [0, N): N < 2**32 for every config here
        cand = ((u >> np.uint64(32)) * np.uint64(w.N)) >> np.uint64(32)
        for c in cand.tolist():
            if c not in seen:
                seen.add(c)
                got.append(c)
                if len(got) == need:
                    break
    return np.asarray(got, dtype=np.int64)
