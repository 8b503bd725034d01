"""ctypes marshalling for libpqkm.so.  No arithmetic of the method lives here."""
from __future__ import annotations

import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libpqkm.so")
_lib = None
L = 256


class PqkmError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: pqkm status {code} ({status_string(code)})")


def lib_path() -> str:
    return _LIB_PATH


def load():
    """Load the built library (built beforehand by __graft_entry__.build()); never falls back."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise ImportError(f"{_LIB_PATH} is missing: run `python -c 'import __graft_entry__ as g; g.build()'` first")
        # The kernels run on torch's stream with torch's device pointers, so one HIP runtime has to serve both.
        # torch ships its own copy of the runtime: imported first it is the one this library binds to; loaded the
        # other way round the process holds two runtimes and every launch of this library fails.
        import torch  # noqa: F401
        lib = ctypes.CDLL(_LIB_PATH)
        vp, i32, i64, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_size_t
        lib.pqkm_status_string.restype = ctypes.c_char_p
        lib.pqkm_status_string.argtypes = [ctypes.c_int]
        lib.pqkm_workspace_bytes.restype = sz
        lib.pqkm_workspace_bytes.argtypes = [i64, i32, i32]
        lib.pqkm_build_tables.argtypes = [vp, i32, i32, vp, vp]
        lib.pqkm_assign.argtypes = [vp, i64, i32, vp, i32, vp, vp, vp, vp, sz, vp]
        lib.pqkm_assign_noalloc.argtypes = [vp, i64, i32, vp, i32, vp, vp, vp, vp]
        lib.pqkm_index_workspace_bytes.restype = sz
        lib.pqkm_index_workspace_bytes.argtypes = [i32, i32]
        lib.pqkm_assign_indexed.argtypes = [vp, i64, i32, vp, i32, vp, vp, vp, vp, sz, vp]
        lib.pqkm_check_workspace_bytes.restype = sz
        lib.pqkm_check_workspace_bytes.argtypes = [i64, i32, i32]
        lib.pqkm_check.argtypes = [vp, i64, i32, vp, i32, vp, i32, vp, sz, vp, ctypes.POINTER(i32),
                                   ctypes.POINTER(ctypes.c_float), ctypes.POINTER(ctypes.c_float)]
        lib.pqkm_update.argtypes = [vp, i64, i32, vp, i32, vp, vp, vp, vp, vp, sz, vp]
        lib.pqkm_fit.argtypes = [vp, i64, i32, vp, i32, vp, i32, vp, vp, vp, vp, sz, vp]
        lib.pqkm_fit_until_workspace_bytes.restype = sz
        lib.pqkm_fit_until_workspace_bytes.argtypes = [i64, i32, i32]
        lib.pqkm_fit_until.argtypes = [vp, i64, i32, vp, i32, vp, i32, vp, vp, vp, vp, vp, vp, sz, vp]
        lib.pqkm_update_naive.argtypes = [vp, i64, i32, vp, i32, vp, vp, vp, vp, sz, vp]
        lib.pqkm_encode.argtypes = [vp, i64, i32, i32, vp, vp, vp]
        lib.pqkm_decode.argtypes = [vp, i64, i32, i32, vp, vp, vp]
        lib.pqkm_set_option.argtypes = [ctypes.c_char_p, i32]
        lib.pqkm_profile_read.argtypes = [ctypes.POINTER(ctypes.c_double), ctypes.POINTER(i64)]
        lib.pqkm_profile_read_steps.argtypes = [ctypes.POINTER(ctypes.c_double), ctypes.POINTER(i64)]
        for n in ("pqkm_build_tables", "pqkm_assign", "pqkm_assign_noalloc", "pqkm_assign_indexed", "pqkm_check", "pqkm_update", "pqkm_fit", "pqkm_fit_until", "pqkm_set_option",
                  "pqkm_profile_read", "pqkm_profile_read_steps", "pqkm_encode", "pqkm_decode", "pqkm_update_naive"):
            getattr(lib, n).restype = ctypes.c_int
        _lib = lib
    return _lib


def status_string(code: int) -> str:
    return load().pqkm_status_string(int(code)).decode()


def workspace_bytes(N: int, M: int, K: int) -> int:
    return int(load().pqkm_workspace_bytes(int(N), int(M), int(K)))


def _ptr(t):
    return ctypes.c_void_p(t.data_ptr()) if t is not None else ctypes.c_void_p(0)


def _stream():
    import torch

    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _need(t, dtype, shape, name):
    import torch

    if t is None:
        return
    if not isinstance(t, torch.Tensor) or not t.is_cuda or not t.is_contiguous():
        raise TypeError(f"{name}: expected a contiguous CUDA tensor")
    if t.dtype != dtype or tuple(t.shape) != tuple(shape):
        raise TypeError(f"{name}: expected {dtype} {tuple(shape)}, got {t.dtype} {tuple(t.shape)}")


def _check(code: int, where: str):
    if code != 0:
        raise PqkmError(code, where)


def _ws(workspace, N, M, K, device):
    import torch

    need = workspace_bytes(N, M, K)
    if workspace is None:
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=device)
    return workspace, workspace.numel()


def build_tables(codewords, tables=None):
    """codewords [M][256][Ds] f32 -> tables [M][256][256] f32."""
    import torch

    M, l, Ds = codewords.shape
    _need(codewords, torch.float32, (M, L, Ds), "codewords")
    if tables is None:
        tables = torch.empty((M, L, L), dtype=torch.float32, device=codewords.device)
    _need(tables, torch.float32, (M, L, L), "tables")
    _check(load().pqkm_build_tables(_ptr(codewords), M, Ds, _ptr(tables), _stream()), "pqkm_build_tables")
    return tables


def encode(vectors, codewords, codes=None):
    """vectors [N][M*Ds] f32, codewords [M][256][Ds] f32 -> codes [N][M] u8 (Sec. 2.2)."""
    import torch

    M, l, Ds = codewords.shape
    N = vectors.shape[0]
    _need(codewords, torch.float32, (M, L, Ds), "codewords")
    _need(vectors, torch.float32, (N, M * Ds), "vectors")
    if codes is None:
        codes = torch.empty((N, M), dtype=torch.uint8, device=vectors.device)
    _need(codes, torch.uint8, (N, M), "codes")
    _check(load().pqkm_encode(_ptr(vectors), N, M, Ds, _ptr(codewords), _ptr(codes), _stream()), "pqkm_encode")
    return codes


def decode(codes, codewords, vectors=None):
    """codes [N][M] u8 -> reconstructed vectors [N][M*Ds] f32 (Sec. 2.2)."""
    import torch

    M, l, Ds = codewords.shape
    N = codes.shape[0]
    _need(codewords, torch.float32, (M, L, Ds), "codewords")
    _need(codes, torch.uint8, (N, M), "codes")
    if vectors is None:
        vectors = torch.empty((N, M * Ds), dtype=torch.float32, device=codes.device)
    _need(vectors, torch.float32, (N, M * Ds), "vectors")
    _check(load().pqkm_decode(_ptr(codes), N, M, Ds, _ptr(codewords), _ptr(vectors), _stream()), "pqkm_decode")
    return vectors


def assign(codes, centers, tables, assign=None, dist=None, want_dist=True, workspace=None):
    """-> (assign [N] i32, dist [N] f32 or None)."""
    import torch

    N, M = codes.shape
    K = centers.shape[0]
    _need(codes, torch.uint8, (N, M), "codes")
    _need(centers, torch.uint8, (K, M), "centers")
    _need(tables, torch.float32, (M, L, L), "tables")
    if assign is None:
        assign = torch.empty(N, dtype=torch.int32, device=codes.device)
    if dist is None and want_dist:
        dist = torch.empty(N, dtype=torch.float32, device=codes.device)
    _need(assign, torch.int32, (N,), "assign")
    _need(dist, torch.float32, (N,), "dist")
    workspace, wb = _ws(workspace, N, M, K, codes.device)
    _check(load().pqkm_assign(_ptr(codes), N, M, _ptr(centers), K, _ptr(tables), _ptr(assign), _ptr(dist),
                              _ptr(workspace), wb, _stream()), "pqkm_assign")
    return assign, dist


def assign_indexed(codes, centers, tables, assign=None, dist=None, want_dist=True, workspace=None):
    """pqkm_assign_indexed (Alg. 1 with the table): same result as assign().  -> (assign, dist or None)."""
    import torch

    N, M = codes.shape
    K = centers.shape[0]
    _need(codes, torch.uint8, (N, M), "codes")
    _need(centers, torch.uint8, (K, M), "centers")
    _need(tables, torch.float32, (M, L, L), "tables")
    if assign is None:
        assign = torch.empty(N, dtype=torch.int32, device=codes.device)
    if dist is None and want_dist:
        dist = torch.empty(N, dtype=torch.float32, device=codes.device)
    _need(assign, torch.int32, (N,), "assign")
    _need(dist, torch.float32, (N,), "dist")
    if workspace is None:
        workspace = torch.empty(max(int(load().pqkm_index_workspace_bytes(M, K)), 256), dtype=torch.uint8,
                                device=codes.device)
    _check(load().pqkm_assign_indexed(_ptr(codes), N, M, _ptr(centers), K, _ptr(tables), _ptr(assign), _ptr(dist),
                                      _ptr(workspace), workspace.numel(), _stream()), "pqkm_assign_indexed")
    return assign, dist


def check(sample_codes, centers, tables, trials=10, workspace=None):
    """pqkm_check, Alg. 1's Check(): -> (use_index: bool, scan_ms, index_ms) on the given sample of codes."""
    import torch

    n, M = sample_codes.shape
    K = centers.shape[0]
    _need(sample_codes, torch.uint8, (n, M), "sample_codes")
    _need(centers, torch.uint8, (K, M), "centers")
    _need(tables, torch.float32, (M, L, L), "tables")
    if workspace is None:
        workspace = torch.empty(max(int(load().pqkm_check_workspace_bytes(n, M, K)), 256), dtype=torch.uint8,
                                device=sample_codes.device)
    flag, t_scan, t_index = ctypes.c_int32(0), ctypes.c_float(0), ctypes.c_float(0)
    _check(load().pqkm_check(_ptr(sample_codes), n, M, _ptr(centers), K, _ptr(tables), int(trials), _ptr(workspace),
                             workspace.numel(), _stream(), ctypes.byref(flag), ctypes.byref(t_scan),
                             ctypes.byref(t_index)), "pqkm_check")
    return bool(flag.value), t_scan.value, t_index.value


NOALLOC_SCRATCH_BYTES = 64 * 1024 * 1024


def assign_noalloc(codes, centers, tables, assign, dist=None):
    """pqkm_assign_noalloc: outputs are the caller's, the scratch is the library's static device array; raises
    PqkmError (code 5) when pqkm_workspace_bytes(N, M, K) exceeds NOALLOC_SCRATCH_BYTES.  -> (assign, dist)."""
    import torch

    N, M = codes.shape
    K = centers.shape[0]
    _need(codes, torch.uint8, (N, M), "codes")
    _need(centers, torch.uint8, (K, M), "centers")
    _need(tables, torch.float32, (M, L, L), "tables")
    _need(assign, torch.int32, (N,), "assign")
    _need(dist, torch.float32, (N,), "dist")
    _check(load().pqkm_assign_noalloc(_ptr(codes), N, M, _ptr(centers), K, _ptr(tables), _ptr(assign), _ptr(dist),
                                      _stream()), "pqkm_assign_noalloc")
    return assign, dist


def update(codes, assign, tables, centers, hist=None, counts=None, want_hist=True, workspace=None):
    """Updates ``centers`` in place; -> (centers, hist or None, counts or None)."""
    import torch

    N, M = codes.shape
    K = centers.shape[0]
    _need(codes, torch.uint8, (N, M), "codes")
    _need(assign, torch.int32, (N,), "assign")
    _need(centers, torch.uint8, (K, M), "centers")
    _need(tables, torch.float32, (M, L, L), "tables")
    if want_hist and hist is None:
        hist = torch.empty((K, M, L), dtype=torch.int32, device=codes.device)
    if want_hist and counts is None:
        counts = torch.empty(K, dtype=torch.int32, device=codes.device)
    _need(hist, torch.int32, (K, M, L), "hist")
    _need(counts, torch.int32, (K,), "counts")
    workspace, wb = _ws(workspace, N, M, K, codes.device)
    _check(load().pqkm_update(_ptr(codes), N, M, _ptr(assign), K, _ptr(tables), _ptr(centers), _ptr(hist),
                              _ptr(counts), _ptr(workspace), wb, _stream()), "pqkm_update")
    return centers, hist, counts


def update_naive(codes, assign, tables, centers, want_cost=False, workspace=None):
    """Eq. 6 by brute force, in place on ``centers``; -> (centers, cost [K][M][256] f64 or None)."""
    import torch

    N, M = codes.shape
    K = centers.shape[0]
    _need(codes, torch.uint8, (N, M), "codes")
    _need(assign, torch.int32, (N,), "assign")
    _need(centers, torch.uint8, (K, M), "centers")
    _need(tables, torch.float32, (M, L, L), "tables")
    cost = torch.empty((K, M, L), dtype=torch.float64, device=codes.device) if want_cost else None
    workspace, wb = _ws(workspace, N, M, K, codes.device)
    _check(load().pqkm_update_naive(_ptr(codes), N, M, _ptr(assign), K, _ptr(tables), _ptr(centers), _ptr(cost),
                                    _ptr(workspace), wb, _stream()), "pqkm_update_naive")
    return centers, cost


def fit(codes, tables, centers, iters, assign=None, hist=None, counts=None, workspace=None):
    """Runs ``iters`` iterations in place on ``centers``; -> (centers, assign)."""
    import torch

    N, M = codes.shape
    K = centers.shape[0]
    _need(codes, torch.uint8, (N, M), "codes")
    _need(centers, torch.uint8, (K, M), "centers")
    _need(tables, torch.float32, (M, L, L), "tables")
    if assign is None:
        assign = torch.empty(N, dtype=torch.int32, device=codes.device)
    _need(assign, torch.int32, (N,), "assign")
    _need(hist, torch.int32, (K, M, L), "hist")
    _need(counts, torch.int32, (K,), "counts")
    workspace, wb = _ws(workspace, N, M, K, codes.device)
    _check(load().pqkm_fit(_ptr(codes), N, M, _ptr(tables), K, _ptr(centers), int(iters), _ptr(assign), _ptr(hist),
                           _ptr(counts), _ptr(workspace), wb, _stream()), "pqkm_fit")
    return centers, assign


class IterStats(ctypes.Structure):
    _fields_ = [("objective", ctypes.c_double), ("changed", ctypes.c_int64), ("nonzero_bins", ctypes.c_int64),
                ("nonempty", ctypes.c_int64)]


def fit_until_workspace_bytes(N: int, M: int, K: int) -> int:
    return int(load().pqkm_fit_until_workspace_bytes(int(N), int(M), int(K)))


def fit_until(codes, tables, centers, max_iters, assign=None, hist=None, counts=None, workspace=None):
    """Iterates in place on ``centers`` until no assignment changes (blocks once per iteration);
    -> (centers, assign, list of (objective, changed, nonzero_bins, nonempty) per iteration)."""
    import torch

    N, M = codes.shape
    K = centers.shape[0]
    _need(codes, torch.uint8, (N, M), "codes")
    _need(centers, torch.uint8, (K, M), "centers")
    _need(tables, torch.float32, (M, L, L), "tables")
    if assign is None:
        assign = torch.empty(N, dtype=torch.int32, device=codes.device)
    _need(assign, torch.int32, (N,), "assign")
    _need(hist, torch.int32, (K, M, L), "hist")
    _need(counts, torch.int32, (K,), "counts")
    need = fit_until_workspace_bytes(N, M, K)
    if workspace is None:
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=codes.device)
    stats = (IterStats * max(int(max_iters), 1))()
    done = ctypes.c_int32(0)
    _check(load().pqkm_fit_until(_ptr(codes), N, M, _ptr(tables), K, _ptr(centers), int(max_iters), _ptr(assign),
                                 _ptr(hist), _ptr(counts), ctypes.cast(stats, ctypes.c_void_p), ctypes.cast(
                                     ctypes.pointer(done), ctypes.c_void_p), _ptr(workspace), workspace.numel(),
                                 _stream()), "pqkm_fit_until")
    out = [(stats[i].objective, stats[i].changed, stats[i].nonzero_bins, stats[i].nonempty) for i in range(done.value)]
    return centers, assign, out


def set_option(name: str, value: int) -> None:
    _check(load().pqkm_set_option(name.encode(), int(value)), f"pqkm_set_option({name})")


def profile_read():
    """-> (total milliseconds of the bracketed scan launches, number of launches)."""
    ms, n = ctypes.c_double(0), ctypes.c_int64(0)
    _check(load().pqkm_profile_read(ctypes.byref(ms), ctypes.byref(n)), "pqkm_profile_read")
    return ms.value, n.value


def profile_read_steps():
    """-> (total milliseconds of the bracketed whole assignment steps, their number)."""
    ms, n = ctypes.c_double(0), ctypes.c_int64(0)
    _check(load().pqkm_profile_read_steps(ctypes.byref(ms), ctypes.byref(n)), "pqkm_profile_read_steps")
    return ms.value, n.value
