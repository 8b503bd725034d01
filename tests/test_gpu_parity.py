"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle.

Bar: bit-exact for assignments, minimum distances (given identical fp32 tables), histograms,
counts and updated centers; the tables themselves within 1e-6 relative.
"""
import dataclasses
import os

import numpy as np
import pytest

from _util import progress, rand_tables, u32, workload

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def env():
    import torch

    import oracle
    import paper_1709_03708_amd as pq
    import workloads as W

    assert torch.cuda.is_available(), "gpu tests need a GPU"
    pq.load()
    return dict(torch=torch, oracle=oracle, pq=pq, W=W, dev=torch.device("cuda:0"))


def _dev(env, a):
    return env["torch"].from_numpy(np.ascontiguousarray(a)).to(env["dev"])


def _sync(env):
    env["torch"].cuda.synchronize()


# ------------------------------------------------------------------------------------ tables
@pytest.mark.parametrize("cfg,over", [(1, {}), (3, {}), (4, dict(M=8, D=1024)), (2, dict(M=3, D=21))])
def test_build_tables(env, cfg, over):
    w = workload(cfg, **over)
    cw = env["W"].codewords(w)
    got = env["pq"].build_tables(_dev(env, cw))
    _sync(env)
    ref = env["oracle"].build_tables(cw)
    got = got.cpu().numpy()
    np.testing.assert_allclose(got, ref, rtol=1e-6, atol=0)
    assert (got == ref).all()            # same fp64 operation order -> in fact identical
    for m in range(w.M):
        assert (np.diag(got[m]) == 0).all() and (got[m] == got[m].T).all()


# ------------------------------------------------------------------------------------ assign
def _check_assign(env, codes, centers, tables, **opts):
    pq, oracle = env["pq"], env["oracle"]
    for k, v in opts.items():
        pq.set_option(k, v)
    try:
        a, d = pq.assign(_dev(env, codes), _dev(env, centers), _dev(env, tables))
        _sync(env)
    finally:
        for k in opts:
            pq.set_option(k, 0)
    ra, rd = oracle.assign(codes, centers, tables)
    np.testing.assert_array_equal(a.cpu().numpy(), ra)
    np.testing.assert_array_equal(d.cpu().numpy().view(np.uint32), rd.view(np.uint32))


@pytest.mark.parametrize("M", [4, 8, 16, 32])
@pytest.mark.parametrize("N,K", [(5003, 77), (1, 1), (513, 32), (2049, 33), (300, 1000)])
def test_assign_tiled_matches_oracle(env, M, N, K):
    """Several center tiles with a ragged last tile, several workgroups with a ragged tail."""
    w = workload(1, M=M, D=32 * M, N=max(N, K), K=K, T=20)
    W = env["W"]
    codes_all = W.codes_numpy(w)
    centers = codes_all[W.init_center_indices(w)].copy()
    codes = codes_all[:N]
    tables = env["oracle"].build_tables(W.codewords(w))
    _check_assign(env, codes, centers, tables, assign_kernel=2)
    rng = np.random.default_rng(N + K + M)
    _check_assign(env, codes, centers, rand_tables(rng, M), assign_kernel=2)     # non-symmetric tables


@pytest.mark.parametrize("M", [1, 3, 4, 6, 8])
def test_assign_generic_matches_oracle(env, M):
    rng = np.random.default_rng(M)
    codes = rng.integers(0, 256, size=(3001, M), dtype=np.uint8)
    centers = rng.integers(0, 256, size=(45, M), dtype=np.uint8)
    _check_assign(env, codes, centers, rand_tables(rng, M), assign_kernel=1)


@pytest.mark.parametrize("variant", [1, 3, 5, 32, 33, 34, 35, 36, 37, 41, 44, 46, 48])
def test_assign_every_compiled_shape(env, variant):
    w = workload(1, N=9001, K=131, T=40)
    W = env["W"]
    codes = W.codes_numpy(w)
    centers = codes[W.init_center_indices(w)].copy()
    tables = env["oracle"].build_tables(W.codewords(w))
    _check_assign(env, codes, centers, tables, assign_kernel=2, scan_variant=variant)


@pytest.mark.parametrize("variant", [70, 71, 72, 73, 74, 75, 76, 80, 81, 82, 83, 84, 85, 86, 87, 88, 89, 90, 91, 92, 93, 94])
@pytest.mark.parametrize("kind,N", [("templates", 9001), ("uniform", 200003), ("uniform", 4093), ("uniform", 7),
                                    ("uniform", 1), ("one_class", 5000), ("two_classes", 6001), ("latin", 8192)])
def test_assign_regrouped_scan(env, variant, kind, N):
    """M = 4 scan over regrouped codes: the regrouping (residue groups, left-overs, holes) must not change
    any result.  Class mixes: typical, all codes in one residue class (everything left over), two classes,
    and perfectly balanced classes (no left-overs)."""
    W = env["W"]
    rng = np.random.default_rng(N + variant)
    w = workload(1, N=max(N, 200), K=131, T=40)
    allc = W.codes_numpy(w)
    centers = allc[W.init_center_indices(w)].copy()
    if kind == "templates":
        codes = allc[:N]
    else:
        codes = rng.integers(0, 256, size=(N, 4), dtype=np.uint8)
        if kind == "one_class":
            codes &= 0xFC
        elif kind == "two_classes":
            codes = (codes & 0xFC) | (rng.integers(0, 2, size=(N, 1), dtype=np.uint8) * 3)
        elif kind == "latin":
            lat = np.stack([rng.permuted(np.tile(np.arange(4, dtype=np.uint8), (N // 4, 1)), axis=1)
                            for _ in range(4)], axis=2).reshape(-1, 4)
            codes = (codes & 0xFC) | lat
    tables = env["oracle"].build_tables(W.codewords(w))
    _check_assign(env, codes, centers, tables, assign_kernel=2, scan_variant=variant)
    if variant in (70, 80, 85, 90):
        ham = np.ones((4, 256, 256), np.float32)
        for m in range(4):
            np.fill_diagonal(ham[m], 0)
        small = (codes % 3).astype(np.uint8)
        _check_assign(env, small, (centers % 3).astype(np.uint8), ham, assign_kernel=2, scan_variant=variant)
        bad = rand_tables(rng, 4)                       # non-symmetric, with NaN and infinite entries
        flat = bad.reshape(-1)
        idx = rng.choice(flat.size, flat.size // 20, replace=False)
        flat[idx[0::3]] = np.nan
        flat[idx[1::3]] = np.inf
        flat[idx[2::3]] = -np.inf
        _check_assign(env, codes, centers, bad, assign_kernel=2, scan_variant=variant)


@pytest.mark.parametrize("variant", [40, 41, 70, 71, 72, 73, 74, 75, 76, 77, 78, 80, 81, 82, 83, 84])
@pytest.mark.parametrize("kind,N", [("templates", 9001), ("uniform", 300007), ("uniform", 4093), ("uniform", 3),
                                    ("one_class", 5000), ("latin", 8192)])
def test_assign_regrouped_scan_64bit_codes(env, variant, kind, N):
    """M = 8 scan over regrouped codes (65536 residue classes, ranks from global atomics): regrouping must not
    change any result, whatever the class mix."""
    W = env["W"]
    rng = np.random.default_rng(N + variant)
    w = workload(3, N=max(N, 300), K=141, T=60)
    allc = W.codes_numpy(w)
    centers = allc[W.init_center_indices(w)].copy()
    if kind == "templates":
        codes = allc[:N]
    else:
        codes = rng.integers(0, 256, size=(N, 8), dtype=np.uint8)
        if kind == "one_class":
            codes &= 0xFC
        elif kind == "latin":
            lat = np.stack([rng.permuted(np.tile(np.arange(4, dtype=np.uint8), (N // 4, 1)), axis=1)
                            for _ in range(8)], axis=2).reshape(-1, 8)
            codes = (codes & 0xFC) | lat
    tables = env["oracle"].build_tables(W.codewords(w))
    _check_assign(env, codes, centers, tables, assign_kernel=2, scan_variant=variant)
    if variant in (70, 80):
        ham = np.ones((8, 256, 256), np.float32)
        for m in range(8):
            np.fill_diagonal(ham[m], 0)
        _check_assign(env, (codes % 3).astype(np.uint8), (centers % 3).astype(np.uint8), ham, assign_kernel=2,
                      scan_variant=variant)


def test_regrouped_scan_in_several_launches(env):
    """Scan launches smaller than N: every launch regroups its own stretch of the codes, and pqkm_fit cannot keep
    the regrouped copy between iterations (it holds one launch only)."""
    pq, oracle, W, torch = env["pq"], env["oracle"], env["W"], env["torch"]
    w = workload(2, N=300_001, K=257, T=500)
    codes = W.codes_numpy(w)
    centers = codes[W.init_center_indices(w)].copy()
    tables = oracle.build_tables(W.codewords(w))
    pq.set_option("launch_codes_log2", 17)            # 131072 codes per launch: 3 launches, the last one ragged
    try:
        a, d = pq.assign(_dev(env, codes), _dev(env, centers), _dev(env, tables))
        cen = _dev(env, centers)
        gh = torch.empty((257, 4, 256), dtype=torch.int32, device=env["dev"])
        gc = torch.empty(257, dtype=torch.int32, device=env["dev"])
        _, ga = pq.fit(_dev(env, codes), _dev(env, tables), cen, 3, hist=gh, counts=gc)
        _sync(env)
    finally:
        pq.set_option("launch_codes_log2", 26)
    ra, rd = oracle.assign(codes, centers, tables)
    np.testing.assert_array_equal(a.cpu().numpy(), ra)
    np.testing.assert_array_equal(d.cpu().numpy().view(np.uint32), rd.view(np.uint32))
    rc, rfa, rh, rcnt = oracle.fit(codes, tables, centers, 3)
    np.testing.assert_array_equal(cen.cpu().numpy(), rc)
    np.testing.assert_array_equal(ga.cpu().numpy(), rfa)
    np.testing.assert_array_equal(gh.cpu().numpy().view(np.uint32), rh)
    np.testing.assert_array_equal(gc.cpu().numpy().view(np.uint32), rcnt)


@pytest.mark.parametrize("M,variant", [(8, 0), (8, 1), (8, 2), (8, 3), (8, 4), (8, 5), (8, 6), (8, 7), (8, 10),
                                       (16, 0), (16, 1), (16, 2), (16, 3), (16, 4), (16, 6), (16, 7), (16, 10),
                                       (32, 0), (32, 1), (32, 2), (32, 3), (32, 4), (32, 5), (32, 6), (32, 10),
                                       (16, 50), (16, 51), (16, 52), (16, 53), (32, 50), (32, 51), (32, 52), (32, 53)])
def test_assign_every_compiled_shape_wide_codes(env, M, variant):
    w = workload(1, M=M, D=16 * M, N=7001, K=77, T=40)
    W = env["W"]
    codes = W.codes_numpy(w)
    centers = codes[W.init_center_indices(w)].copy()
    tables = env["oracle"].build_tables(W.codewords(w))
    _check_assign(env, codes, centers, tables, assign_kernel=2, scan_variant=variant)
    rng = np.random.default_rng(M + variant)
    _check_assign(env, codes, centers, rand_tables(rng, M), assign_kernel=2, scan_variant=variant)


@pytest.mark.parametrize("M", [16, 32])
@pytest.mark.parametrize("variant", [51, 52, 53])
@pytest.mark.parametrize("N,K", [(1, 1), (9001, 16), (4097, 1000), (300_007, 333)])
def test_assign_sliding_window_scan(env, M, variant, N, K):
    """The sliding-window scan of the wide codes (16 centers per tile, planes passing through a ring in the LDS,
    slot classes running 0..3 subspaces behind): ragged workgroups and tiles, one tile, many tiles; real tables,
    non-symmetric tables, Hamming tables (massive ties, in and across tiles and lanes) and tables with NaN and
    infinite entries; every result bit for bit."""
    W = env["W"]
    w = workload(1, M=M, D=16 * M, N=max(N, K), K=K, T=97)
    allc = W.codes_numpy(w)
    centers = allc[W.init_center_indices(w)].copy()
    codes = allc[:N]
    rng = np.random.default_rng(N + K + M + variant)
    tables = env["oracle"].build_tables(W.codewords(w))
    _check_assign(env, codes, centers, tables, assign_kernel=2, scan_variant=variant)
    if N <= 10_000:
        _check_assign(env, codes, centers, rand_tables(rng, M), assign_kernel=2, scan_variant=variant)
        ham = np.ones((M, 256, 256), np.float32)
        for m in range(M):
            np.fill_diagonal(ham[m], 0)
        _check_assign(env, (codes % 3).astype(np.uint8), (centers % 3).astype(np.uint8), ham, assign_kernel=2,
                      scan_variant=variant)
        bad = rand_tables(rng, M)
        flat = bad.reshape(-1)
        idx = rng.choice(flat.size, flat.size // 20, replace=False)
        flat[idx[0::3]] = np.nan
        flat[idx[1::3]] = np.inf
        flat[idx[2::3]] = -np.inf
        _check_assign(env, codes, centers, bad, assign_kernel=2, scan_variant=variant)


@pytest.mark.parametrize("M", [4, 8, 5, 16, 32])
def test_assign_ties_go_to_lowest_index(env, M):
    """Hamming tables: massive ties, in and across tiles and lanes."""
    rng = np.random.default_rng(7)
    tables = np.ones((M, 256, 256), np.float32)
    for m in range(M):
        np.fill_diagonal(tables[m], 0)
    codes = rng.integers(0, 3, size=(4000, M), dtype=np.uint8)
    centers = rng.integers(0, 3, size=(300, M), dtype=np.uint8)
    _check_assign(env, codes, centers, tables)
    _check_assign(env, codes, codes[:1500].copy(), tables)       # centers = codes -> distance 0, first holder


def test_assign_degenerate_inputs(env):
    pq, torch, dev = env["pq"], env["torch"], env["dev"]
    rng = np.random.default_rng(8)
    tables = rand_tables(rng, 4)
    centers = rng.integers(0, 256, size=(10, 4), dtype=np.uint8)
    # N = 0
    a, d = pq.assign(torch.empty((0, 4), dtype=torch.uint8, device=dev), _dev(env, centers), _dev(env, tables))
    assert a.numel() == 0
    # infinities: a center at infinite distance is never chosen; all-infinite -> center 0
    t2 = tables.copy()
    t2[0, :, centers[3, 0]] = np.inf
    codes = rng.integers(0, 256, size=(777, 4), dtype=np.uint8)
    _check_assign(env, codes, centers, t2)
    t3 = np.full_like(tables, np.inf)
    _check_assign(env, codes, centers, t3)
    # dist = NULL
    a, d = pq.assign(_dev(env, codes), _dev(env, centers), _dev(env, tables), want_dist=False)
    _sync(env)
    assert d is None
    np.testing.assert_array_equal(a.cpu().numpy(), env["oracle"].assign(codes, centers, tables)[0])


# ------------------------------------------------------------------------------------ indexed assignment, Check()
def _check_assign_indexed(env, codes, centers, tables):
    pq, oracle = env["pq"], env["oracle"]
    a, d = pq.assign_indexed(_dev(env, codes), _dev(env, centers), _dev(env, tables))
    _sync(env)
    ra, rd = oracle.assign(codes, centers, tables)
    np.testing.assert_array_equal(a.cpu().numpy(), ra)
    np.testing.assert_array_equal(d.cpu().numpy().view(np.uint32), rd.view(np.uint32))


@pytest.mark.parametrize("cfg,over", [(1, {}), (2, dict(N=30_001, K=1000)), (5, dict(N=20_001, K=100_000)),
                                      (3, dict(N=6_001, K=700, T=900)), (4, dict(N=1_001, K=90, T=50)),
                                      (1, dict(N=3_000, K=1)), (2, dict(N=2_000, K=300, M=2, D=64))])
def test_assign_indexed_matches_oracle(env, cfg, over):
    """Alg. 1's FindNN with the table: the bucket index over the centers must give the linear scan's result bit
    for bit (the oracle is the same pqko_assign), from toy sizes to the billion-scale configuration's 1e5 centers
    (all of them, against a stretch of its codes), for 2 to 32 subspaces."""
    W = env["W"]
    w = workload(cfg, **over)
    n_gen = max(w.N, 1)
    codes = W.codes_numpy(dataclasses.replace(w, N=n_gen)) if w.N <= 5_000_000 else None
    centers = W.codes_at(w, W.init_center_indices(w)) if w.K <= w.N else None
    if centers is None:
        # more centers than codes in this stretch: the centers are the configuration's own (drawn from all its codes)
        full = workload(cfg)
        centers = W.codes_at(full, W.init_center_indices(full))[: w.K]
    tables = env["oracle"].build_tables(W.codewords(w))
    _check_assign_indexed(env, codes, centers, tables)
    progress(f"indexed assignment cfg {cfg} {over}: bit-exact")


@pytest.mark.parametrize("M", [2, 4, 8])
def test_assign_indexed_ties_and_non_finite_tables(env, M):
    """Hamming tables (massive ties: the lowest center index must win although the walk meets the centers in
    bucket order), duplicated centers, and tables with NaN and infinite entries (bounds that are NaN prune
    nothing; +inf sums are never selected)."""
    rng = np.random.default_rng(70 + M)
    ham = np.ones((M, 256, 256), np.float32)
    for m in range(M):
        np.fill_diagonal(ham[m], 0)
    codes = rng.integers(0, 3, size=(3000, M), dtype=np.uint8)
    centers = rng.integers(0, 3, size=(200, M), dtype=np.uint8)
    _check_assign_indexed(env, codes, centers, ham)
    _check_assign_indexed(env, codes, codes[:1500].copy(), ham)
    codes = rng.integers(0, 256, size=(2000, M), dtype=np.uint8)
    centers = rng.integers(0, 256, size=(400, M), dtype=np.uint8)
    _check_assign_indexed(env, codes, centers, rand_tables(rng, M))            # non-symmetric
    _check_assign_indexed(env, codes, centers, rand_tables(rng, M, integer=True))
    for kind in ("mixed", "all_inf", "all_nan"):
        t = rand_tables(rng, M)
        flat = t.reshape(-1)
        if kind == "mixed":
            idx = rng.choice(flat.size, flat.size // 20, replace=False)
            flat[idx[0::3]] = np.nan
            flat[idx[1::3]] = np.inf
            flat[idx[2::3]] = -np.inf
        else:
            flat[:] = np.inf if kind == "all_inf" else np.nan
        _check_assign_indexed(env, codes[:500], centers, t)


def test_check_times_both_and_names_the_faster(env):
    """Check() of Alg. 1: both searches are run on the sample; the flag names the faster one."""
    pq, W, torch = env["pq"], env["W"], env["torch"]
    w = workload(2, N=20_000, K=2_000)
    codes = W.codes_numpy(w)
    centers = codes[W.init_center_indices(w)].copy()
    tables = env["oracle"].build_tables(W.codewords(w))
    use_index, t_scan, t_index = pq.check(_dev(env, codes[:4096]), _dev(env, centers), _dev(env, tables), trials=3)
    assert t_scan > 0 and t_index > 0
    assert use_index == (t_index < t_scan)
    # N = 0 is legal for the indexed assignment
    a, _ = pq.assign_indexed(torch.empty((0, 4), dtype=torch.uint8, device=env["dev"]), _dev(env, centers), _dev(env, tables))
    assert a.numel() == 0
    progress(f"Check(): scan {t_scan:.3f} ms, index {t_index:.3f} ms on 4096 codes x 2000 centers -> use_index={use_index}")


# ------------------------------------------------------------------------------------ update
@pytest.mark.parametrize("hist_kernel", [0, 1, 2, 3])
@pytest.mark.parametrize("M,K,N", [(4, 37, 3001), (8, 100, 5000), (3, 11, 700), (32, 9, 2000), (4, 70, 300_000),
                                   (8, 20_000, 200_000), (4, 1000, 50_000)])
def test_update_matches_oracle(env, M, K, N, hist_kernel):
    rng = np.random.default_rng(M * K)
    pq, oracle = env["pq"], env["oracle"]
    pq.set_option("hist_kernel", hist_kernel)
    try:
        _update_case(env, rng, M, K, N)
    finally:
        pq.set_option("hist_kernel", 0)


def _update_case(env, rng, M, K, N):
    pq, oracle = env["pq"], env["oracle"]
    for integer in (False, True):
        tables = rand_tables(rng, M, integer=integer)
        codes = rng.integers(0, 12, size=(N, M), dtype=np.uint8)
        a = rng.integers(0, K - 1, size=N).astype(np.int32)           # last cluster stays empty
        centers = rng.integers(0, 256, size=(K, M), dtype=np.uint8)
        d_cent = _dev(env, centers)
        _, hist, counts = pq.update(_dev(env, codes), _dev(env, a), _dev(env, tables), d_cent)
        _sync(env)
        rc, rh, rcnt = oracle.update(codes, a, tables, centers)
        np.testing.assert_array_equal(u32(hist), rh)
        np.testing.assert_array_equal(u32(counts), rcnt)
        np.testing.assert_array_equal(d_cent.cpu().numpy(), rc)
        assert (rc[K - 1] == centers[K - 1]).all()
        # hist / counts in the workspace
        d_cent2 = _dev(env, centers)
        pq.update(_dev(env, codes), _dev(env, a), _dev(env, tables), d_cent2, want_hist=False)
        _sync(env)
        np.testing.assert_array_equal(d_cent2.cpu().numpy(), rc)


@pytest.mark.parametrize("seed", [11, 12, 13])
def test_random_shapes_assign_then_update(env, seed):
    """Seeded random shapes, value mixes (uniform, skewed residues, few distinct subcodes) and tables (real and
    integer, i.e. many exact ties): assignment, distances, histogram, counts and new centers, all bit for bit."""
    pq, oracle = env["pq"], env["oracle"]
    rng = np.random.default_rng(seed)
    for case in range(14):
        M = int(rng.choice([4, 4, 4, 8, 8, 16, 32]))
        N = int(rng.integers(1, 300_000)) if M <= 8 else int(rng.integers(1, 40_000))
        K = int(rng.integers(1, 1200))
        kind = ("uniform", "skew", "few")[int(rng.integers(0, 3))]
        if kind == "uniform":
            codes = rng.integers(0, 256, (N, M), dtype=np.uint8)
        elif kind == "skew":
            codes = (rng.integers(0, 256, (N, M)) * rng.integers(0, 2, (N, M)) | rng.integers(0, 4, (N, 1))).astype(np.uint8)
        else:
            codes = rng.integers(0, 5, (N, M), dtype=np.uint8)
        centers = codes[rng.integers(0, N, K)].copy()
        tables = rand_tables(rng, M, integer=bool(rng.integers(0, 2)))
        progress(f"random case seed={seed} #{case}: M={M} N={N} K={K} {kind}")
        a, d = pq.assign(_dev(env, codes), _dev(env, centers), _dev(env, tables))
        d_cent = _dev(env, centers)
        _, hist, counts = pq.update(_dev(env, codes), a, _dev(env, tables), d_cent)
        _sync(env)
        ra, rd = oracle.assign(codes, centers, tables)
        rc, rh, rcnt = oracle.update(codes, ra, tables, centers)
        np.testing.assert_array_equal(a.cpu().numpy(), ra)
        np.testing.assert_array_equal(d.cpu().numpy().view(np.uint32), rd.view(np.uint32))
        np.testing.assert_array_equal(u32(hist), rh)
        np.testing.assert_array_equal(u32(counts), rcnt)
        np.testing.assert_array_equal(d_cent.cpu().numpy(), rc)
        # the same data through the fused iteration (two iterations; the oracle's whole loop)
        d_cent = _dev(env, centers)
        _, fa = pq.fit(_dev(env, codes), _dev(env, tables), d_cent, 2, hist=hist, counts=counts)
        _sync(env)
        rc, ra, rh, rcnt = oracle.fit(codes, tables, centers, 2)
        np.testing.assert_array_equal(fa.cpu().numpy(), ra)
        np.testing.assert_array_equal(u32(hist), rh)
        np.testing.assert_array_equal(u32(counts), rcnt)
        np.testing.assert_array_equal(d_cent.cpu().numpy(), rc)


@pytest.mark.parametrize("seed", [31, 32, 33])
def test_random_shapes_forced_large_input_scans(env, seed):
    """The scans that are the default only for large inputs (two lanes per code for M = 4 and M = 8, table-built
    tiles, the sliding-window scan for M = 16 and 32), forced on seeded random shapes and value mixes: one
    workgroup to a few, one tile to many, ragged everything; real and integer tables; assignment and distances bit
    for bit, then a two-iteration pqkm_fit with the same variant forced."""
    pq, oracle = env["pq"], env["oracle"]
    rng = np.random.default_rng(seed)
    choices = [(4, 80), (4, 82), (4, 84), (4, 85), (4, 86), (4, 88), (4, 89), (4, 90), (4, 93), (8, 80), (8, 82), (8, 84), (16, 50), (16, 52), (16, 53), (32, 50), (32, 51), (32, 53)]
    for case in range(12):
        M, variant = choices[int(rng.integers(0, len(choices)))]
        N = int(rng.integers(1, 120_000)) if M <= 8 else int(rng.integers(1, 40_000))
        K = int(rng.integers(1, 1500))
        kind = ("uniform", "skew", "few")[int(rng.integers(0, 3))]
        if kind == "uniform":
            codes = rng.integers(0, 256, (N, M), dtype=np.uint8)
        elif kind == "skew":
            codes = (rng.integers(0, 256, (N, M)) * rng.integers(0, 2, (N, M)) | rng.integers(0, 4, (N, 1))).astype(np.uint8)
        else:
            codes = rng.integers(0, 5, (N, M), dtype=np.uint8)
        centers = codes[rng.integers(0, N, K)].copy()
        tables = rand_tables(rng, M, integer=bool(rng.integers(0, 2)))
        progress(f"forced-scan case seed={seed} #{case}: M={M} variant={variant} N={N} K={K} {kind}")
        _check_assign(env, codes, centers, tables, assign_kernel=2, scan_variant=variant)
        torch = env["torch"]
        hist = torch.empty((K, M, 256), dtype=torch.int32, device=env["dev"])
        counts = torch.empty((K,), dtype=torch.int32, device=env["dev"])
        d_cent = _dev(env, centers)
        pq.set_option("assign_kernel", 2)
        pq.set_option("scan_variant", variant)
        try:
            _, fa = pq.fit(_dev(env, codes), _dev(env, tables), d_cent, 2, hist=hist, counts=counts)
            _sync(env)
        finally:
            pq.set_option("assign_kernel", 0)
            pq.set_option("scan_variant", 0)
        rc, ra, rh, rcnt = oracle.fit(codes, tables, centers, 2)
        np.testing.assert_array_equal(fa.cpu().numpy(), ra)
        np.testing.assert_array_equal(u32(hist), rh)
        np.testing.assert_array_equal(u32(counts), rcnt)
        np.testing.assert_array_equal(d_cent.cpu().numpy(), rc)


@pytest.mark.parametrize("M,N,K,variant", [(4, 4_700_003, 700, 85), (4, 2_500_001, 700, 89), (8, 3_100_007, 600, 80),
                                           (8, 1_300_003, 600, 70), (32, 1_700_001, 300, 53), (16, 2_300_003, 300, 51)])
def test_rounds_per_launch_do_not_change_results(env, M, N, K, variant):
    """The large scans issue their workgroups in kernel launches of one round (one workgroup per compute unit) each by
    default.  Several rounds of workgroups, a ragged last one: the assignment with one round per launch against the
    oracle on a sample of the codes, and every code bit for bit against the same scan issued two rounds per launch
    and as a single launch."""
    pq, oracle, W, torch = env["pq"], env["oracle"], env["W"], env["torch"]
    w = workload(2 if M == 4 else 3, N=N, K=K, M=M, D=16 * M)
    codes = W.codes_numpy(w)
    centers = codes[W.init_center_indices(w)].copy()
    tables = oracle.build_tables(W.codewords(w))
    d_codes, d_cent, d_tab = _dev(env, codes), _dev(env, centers), _dev(env, tables)
    res = {}
    pq.set_option("assign_kernel", 2)
    pq.set_option("scan_variant", variant)
    try:
        for rpl in (1, 2, 0):
            progress(f"rounds per launch {rpl}: M={M} N={N} K={K} variant {variant}")
            pq.set_option("scan_rounds_per_launch", rpl)
            a = torch.full((N,), -1, dtype=torch.int32, device=env["dev"])
            d = torch.full((N,), float("nan"), dtype=torch.float32, device=env["dev"])
            pq.assign(d_codes, d_cent, d_tab, assign=a, dist=d)
            _sync(env)
            res[rpl] = (a.cpu().numpy(), d.cpu().numpy())
    finally:
        pq.set_option("scan_rounds_per_launch", 1)
        pq.set_option("scan_variant", 0)
        pq.set_option("assign_kernel", 0)
    for rpl in (2, 0):
        np.testing.assert_array_equal(res[rpl][0], res[1][0])
        np.testing.assert_array_equal(res[rpl][1].view(np.uint32), res[1][1].view(np.uint32))
    rng = np.random.default_rng(N)
    pick = np.unique(np.concatenate([rng.integers(0, N, 20_000), np.arange(N - 3000, N), np.arange(3000)]))
    ra, rd = oracle.assign(np.ascontiguousarray(codes[pick]), centers, tables)
    np.testing.assert_array_equal(res[1][0][pick], ra)
    np.testing.assert_array_equal(res[1][1][pick].view(np.uint32), rd.view(np.uint32))


@pytest.mark.parametrize("seed", [21, 22])
def test_random_shapes_fused_iteration(env, seed):
    """Seeded random shapes above one round of 2048-code workgroups (M = 4, K >= 128), where pqkm_fit runs the
    regrouped scan with the scan -> histogram hand-over: three iterations against the oracle's loop."""
    pq, oracle = env["pq"], env["oracle"]
    rng = np.random.default_rng(seed)
    for case in range(4):
        N = int(rng.integers(524_289, 900_000))
        K = int(rng.integers(128, 1500))
        kind = ("uniform", "skew", "few")[int(rng.integers(0, 3))]
        if kind == "uniform":
            codes = rng.integers(0, 256, (N, 4), dtype=np.uint8)
        elif kind == "skew":
            codes = (rng.integers(0, 256, (N, 4)) * rng.integers(0, 2, (N, 4)) | rng.integers(0, 4, (N, 1))).astype(np.uint8)
        else:
            codes = rng.integers(0, 5, (N, 4), dtype=np.uint8)
        centers = codes[rng.integers(0, N, K)].copy()
        tables = rand_tables(rng, 4, integer=bool(rng.integers(0, 2)))
        progress(f"random fused case seed={seed} #{case}: N={N} K={K} {kind}")
        torch = env["torch"]
        hist = torch.empty((K, 4, 256), dtype=torch.int32, device=env["dev"])
        counts = torch.empty((K,), dtype=torch.int32, device=env["dev"])
        d_cent = _dev(env, centers)
        _, fa = pq.fit(_dev(env, codes), _dev(env, tables), d_cent, 3, hist=hist, counts=counts)
        _sync(env)
        rc, ra, rh, rcnt = oracle.fit(codes, tables, centers, 3)
        np.testing.assert_array_equal(fa.cpu().numpy(), ra)
        np.testing.assert_array_equal(u32(hist), rh)
        np.testing.assert_array_equal(u32(counts), rcnt)
        np.testing.assert_array_equal(d_cent.cpu().numpy(), rc)


def test_update_empty_input_and_big_counts(env):
    pq, oracle, torch, dev = env["pq"], env["oracle"], env["torch"], env["dev"]
    rng = np.random.default_rng(9)
    M, K = 4, 5
    tables = rand_tables(rng, M)
    centers = rng.integers(0, 256, size=(K, M), dtype=np.uint8)
    d_cent = _dev(env, centers)
    _, hist, counts = pq.update(torch.empty((0, M), dtype=torch.uint8, device=dev),
                                torch.empty(0, dtype=torch.int32, device=dev), _dev(env, tables), d_cent)
    _sync(env)
    assert u32(hist).sum() == 0 and u32(counts).sum() == 0
    np.testing.assert_array_equal(d_cent.cpu().numpy(), centers)
    # one heavy cluster: counts beyond 2**24 exercise the int -> float rounding of the vote
    N = (1 << 24) + 12345
    codes = np.zeros((N, M), np.uint8)
    codes[: N // 3] = 7
    codes[N // 3:, 1] = 200
    a = np.zeros(N, np.int32)
    a[-5:] = 3
    d_cent = _dev(env, centers)
    _, hist, counts = pq.update(_dev(env, codes), _dev(env, a), _dev(env, tables), d_cent)
    _sync(env)
    rc, rh, rcnt = oracle.update(codes, a, tables, centers)
    np.testing.assert_array_equal(u32(hist), rh)
    np.testing.assert_array_equal(u32(counts), rcnt)
    np.testing.assert_array_equal(d_cent.cpu().numpy(), rc)


def test_vote_is_fused_on_a_vote_whose_winner_depends_on_it(env):
    """Eq. 8 as read here accumulates with ONE fused multiply-add per non-zero bin.  Constructed two-bin votes
    (bin 5 holds one member, bin 9 holds h2) for which a separate multiply and add would pick another candidate,
    run through pqkm_update: the centers must be the oracle's, which is pinned to the fused reading on the CPU."""
    pq, oracle = env["pq"], env["oracle"]
    rng = np.random.default_rng(6)
    cases = []
    while len(cases) < 6:
        a1 = np.float32(rng.random() * 1000 + 1)
        a2 = np.float32(rng.random() * 10 + 0.01)
        h2 = int(rng.integers(3, 1000))
        u = np.float32(np.float32(np.float32(h2) * a2) + a1)                       # multiply, round, add, round
        f = np.float32(np.float64(h2) * np.float64(a2) + np.float64(a1))            # exact product and sum in fp64
        if f != u:
            cases.append((a1, a2, h2, f, u))
    K, M = len(cases), 1
    tables = np.full((M, 256, 256), 1e9, np.float32)
    codes, assign = [], []
    for k, (a1, a2, h2, f, u) in enumerate(cases):
        # cluster k's candidates live in columns 2k (lx) and 2k + 1 (ly) ... but one table serves all clusters, so
        # every cluster gets its own pair of member bins as well: bins 2k and 2k + 1
        jb1, jb2 = 2 * k, 2 * k + 1
        lx, ly = (100 + 2 * k + 1, 100 + 2 * k) if f < u else (100 + 2 * k, 100 + 2 * k + 1)
        tables[0, jb1, lx], tables[0, jb2, lx] = a1, a2
        tables[0, jb1, ly], tables[0, jb2, ly] = (max(f, u) if f < u else min(f, u)), 0.0
        codes += [[jb1]] + [[jb2]] * h2
        assign += [k] * (1 + h2)
    codes = np.array(codes, np.uint8)
    assign = np.array(assign, np.int32)
    cent0 = np.zeros((K, M), np.uint8)
    rc, rh, rcnt = oracle.update(codes, assign, tables, cent0)
    fused_differs = 0
    for k, (a1, a2, h2, f, u) in enumerate(cases):
        lx, ly = (100 + 2 * k + 1, 100 + 2 * k) if f < u else (100 + 2 * k, 100 + 2 * k + 1)
        assert rc[k, 0] == (lx if f < u else ly)             # the fused winner; unfused would tie -> lower index
        fused_differs += rc[k, 0] != min(lx, ly)
    assert fused_differs >= 1
    for hk in (0, 1, 2, 3):
        pq.set_option("hist_kernel", hk)
        try:
            d_cent = _dev(env, cent0)
            _, hist, counts = pq.update(_dev(env, codes), _dev(env, assign), _dev(env, tables), d_cent)
            _sync(env)
        finally:
            pq.set_option("hist_kernel", 0)
        np.testing.assert_array_equal(u32(hist), rh)
        np.testing.assert_array_equal(u32(counts), rcnt)
        np.testing.assert_array_equal(d_cent.cpu().numpy(), rc)


@pytest.mark.parametrize("M", [4, 8, 16, 32, 5])
def test_non_finite_table_entries(env, M):
    """User tables with +inf, -inf and NaN entries.  Comparisons are IEEE "<" in a sequential scan: a NaN or +inf
    sum is never selected (if none is, the result is index 0), -inf wins at the lowest index holding it.  Both
    argmins (Eq. 5 over centers, Eq. 8 over candidates) must agree with the oracle's sequential scan."""
    pq, oracle = env["pq"], env["oracle"]
    rng = np.random.default_rng(40 + M)
    N, K = 6001, 150
    codes = rng.integers(0, 256, size=(N, M), dtype=np.uint8)
    centers = rng.integers(0, 256, size=(K, M), dtype=np.uint8)
    for kind in ("nan", "mixed", "all_nan"):
        tables = rand_tables(rng, M)
        flat = tables.reshape(-1)
        if kind == "nan":
            flat[rng.choice(flat.size, flat.size // 50, replace=False)] = np.nan
        elif kind == "mixed":
            idx = rng.choice(flat.size, flat.size // 20, replace=False)
            flat[idx[0::3]] = np.nan
            flat[idx[1::3]] = np.inf
            flat[idx[2::3]] = -np.inf
        else:
            flat[:] = np.nan
        a, d = pq.assign(_dev(env, codes), _dev(env, centers), _dev(env, tables))
        _sync(env)
        ra, rd = oracle.assign(codes, centers, tables)
        np.testing.assert_array_equal(a.cpu().numpy(), ra)
        np.testing.assert_array_equal(d.cpu().numpy().view(np.uint32), rd.view(np.uint32))
        d_cent = _dev(env, centers)
        _, hist, counts = pq.update(_dev(env, codes), a, _dev(env, tables), d_cent)
        _sync(env)
        rc, rh, rcnt = oracle.update(codes, ra, tables, centers)
        np.testing.assert_array_equal(u32(hist), rh)
        np.testing.assert_array_equal(d_cent.cpu().numpy(), rc)


# ------------------------------------------------------------------------------------ Alg. 1 on the configs
def _run_config_full(env, cfg, iters, **over):
    """Every iteration compared in full: assign, dist, hist, counts, centers."""
    pq, oracle, W = env["pq"], env["oracle"], env["W"]
    w = workload(cfg, **over)
    cw = W.codewords(w)
    codes = W.codes_numpy(w)
    cent = codes[W.init_center_indices(w)].copy()
    tables_d = pq.build_tables(_dev(env, cw))
    _sync(env)
    tables = tables_d.cpu().numpy()
    np.testing.assert_allclose(tables, oracle.build_tables(cw), rtol=1e-6, atol=0)
    d_codes, d_cent = _dev(env, codes), _dev(env, cent)
    empties = 0
    for it in range(iters):
        a, d = pq.assign(d_codes, d_cent, tables_d)
        _, hist, counts = pq.update(d_codes, a, tables_d, d_cent)
        _sync(env)
        ra, rd = oracle.assign(codes, cent, tables)
        cent, rh, rcnt = oracle.update(codes, ra, tables, cent)
        np.testing.assert_array_equal(a.cpu().numpy(), ra)
        np.testing.assert_array_equal(d.cpu().numpy().view(np.uint32), rd.view(np.uint32))
        np.testing.assert_array_equal(u32(hist), rh)
        np.testing.assert_array_equal(u32(counts), rcnt)
        np.testing.assert_array_equal(d_cent.cpu().numpy(), cent)
        empties += int((rcnt == 0).sum())
        progress(f"config {cfg} iteration {it + 1}/{iters} bit-exact")
    # the same through pqkm_fit
    cent0 = codes[W.init_center_indices(w)].copy()
    d_cent = _dev(env, cent0)
    _, fa = pq.fit(d_codes, tables_d, d_cent, iters)
    _sync(env)
    rc, ra, _, _ = oracle.fit(codes, tables, cent0, iters)
    np.testing.assert_array_equal(d_cent.cpu().numpy(), rc)
    np.testing.assert_array_equal(fa.cpu().numpy(), ra)
    return empties


@pytest.mark.parametrize("N,K,kind", [(530_001, 130, "templates"), (600_007, 1000, "templates"), (540_672, 257, "skewed"),
                                      (550_003, 600, "one_class"), (525_000, 4000, "templates"),
                                      (560_001, 500, "several_launches"), (560_001, 500, "forced_owner"),
                                      (70_001, 130, "templates"), (300_007, 1000, "templates"),
                                      (4_500_000, 300, "templates"), (600_007, 1000, "four_lane"),
                                      (525_000, 4000, "four_lane"), (540_672, 257, "four_lane")])
def test_fit_files_codes_by_cluster_group(env, N, K, kind):
    """pqkm_fit with 4-byte codes at owner-path sizes: above one round of 2048-code workgroups (256 x 2048 codes) the
    regrouped scan runs and files (code, center) records by cluster group; the vote counts from those itself when
    a group has at most 16 clusters and there are at most 1024 scan workgroups, else the histogram kernel does
    (K = 4000: 32 clusters per group; N = 4.5e6: more scan workgroups).  The two smaller cases take the skewed
    scan and the separate histogram pass through the same call.  The filing scan is the one that loads its half tiles
    straight into LDS; "four_lane" forces the four-lane scan, which files the same records.  Centers, assignments, histograms and counts of the last iteration against
    the oracle, for ragged N and K, cluster sizes from empty to huge, and codes of a single residue class."""
    pq, oracle, W = env["pq"], env["oracle"], env["W"]
    rng = np.random.default_rng(N + K)
    w = workload(2, N=N, K=K)
    tables = env["oracle"].build_tables(W.codewords(w))
    if kind in ("templates", "several_launches", "forced_owner", "four_lane"):
        codes = W.codes_numpy(w)
    elif kind == "skewed":
        # nine tenths of the codes are copies of 3 codes: a few huge clusters, most groups nearly empty
        codes = rng.integers(0, 256, size=(N, 4), dtype=np.uint8)
        hot = rng.integers(0, 256, size=(3, 4), dtype=np.uint8)
        pick = rng.random(N) < 0.9
        codes[pick] = hot[rng.integers(0, 3, size=int(pick.sum()))]
    else:
        codes = (rng.integers(0, 64, size=(N, 4), dtype=np.uint8) * 4 + 1).astype(np.uint8)   # every subcode = 1 mod 4
    codes = np.ascontiguousarray(codes)
    cent0 = codes[rng.choice(N, size=K, replace=False)].copy()
    d_codes, d_tables, d_cent = _dev(env, codes), _dev(env, tables), _dev(env, cent0)
    torch = env["torch"]
    hist = torch.empty((K, 4, 256), dtype=torch.int32, device=env["dev"])
    counts = torch.empty((K,), dtype=torch.int32, device=env["dev"])
    iters = 2
    # the hand-over needs one scan launch and the automatic histogram choice: with several launches, or a forced
    # histogram kernel, the same call must fall back to the separate histogram pass
    if kind == "several_launches":
        pq.set_option("launch_codes_log2", 16)
    if kind == "forced_owner":
        pq.set_option("hist_kernel", 2)
    if kind == "four_lane":
        pq.set_option("scan_variant", 70)
    try:
        _, fa = pq.fit(d_codes, d_tables, d_cent, iters, hist=hist, counts=counts)
        _sync(env)
    finally:
        pq.set_option("launch_codes_log2", 26)
        pq.set_option("hist_kernel", 0)
        pq.set_option("scan_variant", 0)
    rc, ra, rh, rcnt = oracle.fit(codes, tables, cent0, iters)
    np.testing.assert_array_equal(fa.cpu().numpy(), ra)
    np.testing.assert_array_equal(u32(hist), rh)
    np.testing.assert_array_equal(u32(counts), rcnt)
    np.testing.assert_array_equal(d_cent.cpu().numpy(), rc)
    progress(f"fused fit N={N} K={K} {kind}: bit-exact, {int((rcnt == 0).sum())} empty clusters")


@pytest.mark.parametrize("M,N,K", [(4, 600_007, 20_000), (8, 4_300_003, 10_000), (32, 300_007, 3_000), (16, 420_001, 5_000),
                                   (4, 70_001, 20_000), (4, 2_400_003, 20_000)])
def test_fit_hands_ranks_to_the_sorted_histogram(env, M, N, K):
    """pqkm_fit at sizes where the histogram sorts the code indices by cluster (more than 255 cluster groups): the
    regrouped scans (4- and 8-byte codes) and the sliding-window scan (16, 32 bytes) count the clusters in their
    epilogue and leave every code's rank, so the update needs no counting pass and no atomics in its scatter.  The
    fifth case takes a scan without that hand-over through the same call, the last one the scan that loads its half
    tiles straight into LDS, in the shape chosen for a few rounds of workgroups.  Two iterations against the oracle's loop:
    centers, assignments, histograms, counts."""
    pq, oracle, W, torch = env["pq"], env["oracle"], env["W"], env["torch"]
    w = workload(2 if M == 4 else 3, N=N, K=K, M=M, D=16 * M)
    codes = W.codes_numpy(w)
    cent0 = codes[W.init_center_indices(w)].copy()
    tables = oracle.build_tables(W.codewords(w))
    hist = torch.empty((K, M, 256), dtype=torch.int32, device=env["dev"])
    counts = torch.empty((K,), dtype=torch.int32, device=env["dev"])
    d_cent = _dev(env, cent0)
    progress(f"fit with rank hand-over M={M} N={N} K={K}: GPU")
    _, fa = pq.fit(_dev(env, codes), _dev(env, tables), d_cent, 2, hist=hist, counts=counts)
    _sync(env)
    progress(f"fit with rank hand-over M={M} N={N} K={K}: oracle")
    rc, ra, rh, rcnt = oracle.fit(codes, tables, cent0, 2)
    np.testing.assert_array_equal(fa.cpu().numpy(), ra)
    np.testing.assert_array_equal(u32(hist), rh)
    np.testing.assert_array_equal(u32(counts), rcnt)
    np.testing.assert_array_equal(d_cent.cpu().numpy(), rc)


def test_config1_tiny_all_iterations(env):
    empties = _run_config_full(env, 1, workload(1).iters)
    assert empties > 0          # duplicate initial centers guarantee empty clusters here


def test_config2_sift32_all_iterations(env):
    _run_config_full(env, 2, workload(2).iters)


@pytest.mark.parametrize("cfg,over", [(1, {}), (2, dict(N=200_000, K=300, T=600)), (3, dict(N=50_000, K=200, T=300)),
                                      (2, dict(N=540_001, K=9_000, T=12_000))])
def test_fit_until_matches_oracle(env, cfg, over):
    """Alg. 1 with the stop condition: same number of iterations, integer statistics exact, the fp64
    objective within 1e-9 relative (it is a sum of N fp32 terms in a different order: error <= N * 2^-53),
    final centers / assignment / histogram bit-exact."""
    pq, oracle, W = env["pq"], env["oracle"], env["W"]
    w = workload(cfg, **over)
    codes = W.codes_numpy(w)
    cent0 = codes[W.init_center_indices(w)].copy()
    tables = oracle.build_tables(W.codewords(w))
    d_cent = _dev(env, cent0)
    torch = env["torch"]
    hist = torch.empty((w.K, w.M, 256), dtype=torch.int32, device=env["dev"])
    counts = torch.empty(w.K, dtype=torch.int32, device=env["dev"])
    _, a, stats = pq.fit_until(_dev(env, codes), _dev(env, tables), d_cent, 40, hist=hist, counts=counts)
    _sync(env)
    rc, ra, rh, rcnt, rstats = oracle.fit_until(codes, tables, cent0, 40)
    assert len(stats) == len(rstats) and 2 <= len(stats) < 40
    for (obj, ch, nz, ne), r in zip(stats, rstats):
        assert abs(obj - r[0]) <= 1e-9 * r[0]
        assert (ch, nz, ne) == (int(r[1]), int(r[2]), int(r[3]))
    assert stats[-1][1] == 0
    np.testing.assert_array_equal(d_cent.cpu().numpy(), rc)
    np.testing.assert_array_equal(a.cpu().numpy(), ra)
    np.testing.assert_array_equal(u32(hist), rh)
    np.testing.assert_array_equal(u32(counts), rcnt)
    # the cap is honoured, and zero iterations touch nothing
    d2 = _dev(env, cent0)
    _, _, s2 = pq.fit_until(_dev(env, codes), _dev(env, tables), d2, 2)
    assert len(s2) == 2 and s2[1][1] == int(rstats[1][1])
    d3 = _dev(env, cent0)
    _, _, s3 = pq.fit_until(_dev(env, codes), _dev(env, tables), d3, 0)
    _sync(env)
    assert s3 == [] and (d3.cpu().numpy() == cent0).all()


def _check_every_element_written_and_consistent(env, d_codes, cent, tables, a, d, label):
    """Every output element of a full-size assignment, on the host: none keeps its pre-filled value (-1 / NaN), every
    assignment names a center, and dist[n] is bit for bit Eq. 3 for (codes[n], centers[assign[n]]) -- so each
    element was written, to its own position, from its own code.  (That the center is the NEAREST one is what
    the sampled comparison against the oracle's scan checks.)"""
    oracle, torch = env["oracle"], env["torch"]
    N, K = a.numel(), cent.shape[0]
    assert int(a.min()) >= 0 and int(a.max()) < K, "an assignment was never written or is out of range"
    assert not bool(torch.isnan(d).any()), "a distance was never written"
    chunk = 50_000_000
    starts = list(range(0, N, chunk))
    if len(starts) > 24:                             # beyond 2**32 codes: the first, the last and every eighth stretch
        starts = sorted(set(starts[::8]) | {starts[0], starts[-1]})
    for n0 in starts:
        n1 = min(N, n0 + chunk)
        h_codes = d_codes[n0:n1].cpu().numpy()
        h_a = a[n0:n1].cpu().numpy()
        want = oracle.sdc_pairs(h_codes, cent[h_a], tables)
        got = d[n0:n1].cpu().numpy()
        bad = np.flatnonzero(got.view(np.uint32) != want.view(np.uint32))
        assert bad.size == 0, f"{label}: dist[{n0 + bad[0]}] is not the distance to its assigned center"
        progress(f"{label}: distances of codes {n0}..{n1} are those of their assigned centers")


def _run_config_sampled(env, cfg, n_sample, iters=1, full_first=False, **over):
    """Full-size run in the launch configuration the benchmark uses.  The assignment is checked
    on a seeded sample of codes against all K centers (with full_first, the first iteration against the
    oracle's scan over ALL codes) and, for every code, for having been written and being consistent with
    its own distance; histogram, counts and vote are checked in full by giving the GPU's assignment to the
    oracle."""
    pq, oracle, W, torch, dev = env["pq"], env["oracle"], env["W"], env["torch"], env["dev"]
    w = workload(cfg, **over)
    cw = W.codewords(w)
    tables_d = pq.build_tables(_dev(env, cw))
    _sync(env)
    tables = tables_d.cpu().numpy()
    progress(f"config {cfg}: generating {w.N} codes on the GPU")
    d_codes = W.codes_torch(w, dev)
    init = W.init_center_indices(w)
    cent = W.codes_at(w, init)
    np.testing.assert_array_equal(d_codes[torch.from_numpy(init).to(dev)].cpu().numpy(), cent)
    rng = np.random.default_rng(w.seed)
    sample = np.sort(rng.choice(w.N, size=n_sample, replace=False))
    sample[0], sample[-1] = 0, w.N - 1
    s_codes = W.codes_at(w, sample)
    np.testing.assert_array_equal(d_codes[torch.from_numpy(sample).to(dev)].cpu().numpy(), s_codes)
    d_cent = _dev(env, cent)
    ws = torch.empty(pq.workspace_bytes(w.N, w.M, w.K), dtype=torch.uint8, device=dev)
    a = torch.empty(w.N, dtype=torch.int32, device=dev)
    d = torch.empty(w.N, dtype=torch.float32, device=dev)
    hist = torch.empty((w.K, w.M, 256), dtype=torch.int32, device=dev)
    counts = torch.empty(w.K, dtype=torch.int32, device=dev)
    for it in range(iters):
        progress(f"config {cfg}: iteration {it + 1} assign on the GPU")
        a.fill_(-1)                                  # an element the scan never writes must not pass
        d.fill_(float("nan"))
        pq.assign(d_codes, d_cent, tables_d, assign=a, dist=d, workspace=ws)
        _sync(env)
        if full_first and it == 0:
            progress(f"config {cfg}: oracle scan over all {w.N} codes x {w.K} centers")
            h_codes = d_codes.cpu().numpy()
            ra, rd = oracle.assign(h_codes, cent, tables)
            del h_codes
            np.testing.assert_array_equal(a.cpu().numpy(), ra)
            np.testing.assert_array_equal(d.cpu().numpy().view(np.uint32), rd.view(np.uint32))
            del ra, rd
        else:
            progress(f"config {cfg}: oracle on {n_sample} sampled codes x {w.K} centers")
            ra, rd = oracle.assign(s_codes, cent, tables)
            idx = torch.from_numpy(sample).to(dev)
            np.testing.assert_array_equal(a[idx].cpu().numpy(), ra)
            np.testing.assert_array_equal(d[idx].cpu().numpy().view(np.uint32), rd.view(np.uint32))
            _check_every_element_written_and_consistent(env, d_codes, cent, tables, a, d, f"config {cfg} iteration {it + 1}")
        progress(f"config {cfg}: update on the GPU")
        pq.update(d_codes, a, tables_d, d_cent, hist=hist, counts=counts, workspace=ws)
        _sync(env)
        progress(f"config {cfg}: oracle histogram + vote in full")
        h_codes = d_codes.cpu().numpy()
        h_a = a.cpu().numpy()
        cent, rh, rcnt = oracle.update(h_codes, h_a, tables, cent)
        del h_codes, h_a
        np.testing.assert_array_equal(u32(counts), rcnt)
        np.testing.assert_array_equal(u32(hist), rh)
        np.testing.assert_array_equal(d_cent.cpu().numpy(), cent)
        how = "in full" if full_first and it == 0 else "sampled, every element self-consistent"
        progress(f"config {cfg}: iteration {it + 1} bit-exact (assign {how}, update full)")


def test_config3_sift64_first_iteration_full_then_sampled(env):
    """Iteration 1 against the oracle's scan over all 1e7 codes (1e11 evaluations on the host cores), iteration 2
    sampled; the update of both in full."""
    _run_config_sampled(env, 3, 100_000, iters=2, full_first=True)


def test_config4_cnn_sampled(env):
    _run_config_sampled(env, 4, 20_000, iters=1)


def test_config5_billion_sampled(env):
    _run_config_sampled(env, 5, 100_000, iters=1)


@pytest.mark.skipif(os.environ.get("PQKM_SKIP_HUGE") == "1",
                    reason="more than 2**32 codes: 60 GB of device memory, 35 GB of host memory, half a minute")
def test_more_than_2_to_32_codes(env):
    """Code indices beyond 32 bits: 65 scan launches, the atomic histogram path in chunks of 2**30 codes
    (the sorted and owner paths index codes with 32 bits and are not taken)."""
    _run_config_sampled(env, 5, 100_000, iters=1, N=(1 << 32) + 5000, K=64)


# ------------------------------------------------------------------------------------ encode / decode (Sec. 2.2)
@pytest.mark.parametrize("M,Ds,N", [(4, 32, 5003), (8, 16, 3000), (32, 128, 700), (2, 64, 1025), (3, 5, 2001), (1, 1, 300),
                                    (4, 8, 1), (2, 4, 257), (1, 200, 300)])
def test_encode_decode_match_oracle(env, M, Ds, N):
    """Bit-exact codes (every compiled subvector length and the generic kernel), including vectors that are
    codewords (distance 0, duplicated codeword -> lowest index) and integer data with many exact ties."""
    pq, oracle = env["pq"], env["oracle"]
    rng = np.random.default_rng(M * 1000 + Ds)
    cw = rng.normal(size=(M, 256, Ds)).astype(np.float32)
    cw[0, 255] = cw[0, 3]
    v = rng.normal(size=(N, M * Ds)).astype(np.float32)
    v[: min(N, 40)] = oracle.decode_f32(cw, rng.integers(0, 256, size=(min(N, 40), M), dtype=np.uint8))
    for vectors, codewords in ((v, cw), (np.rint(v * 2).astype(np.float32), np.rint(cw * 2).astype(np.float32))):
        codes = pq.encode(_dev(env, vectors), _dev(env, codewords))
        _sync(env)
        ref = oracle.encode(vectors, codewords)
        np.testing.assert_array_equal(codes.cpu().numpy(), ref)
        rec = pq.decode(codes, _dev(env, codewords))
        _sync(env)
        np.testing.assert_array_equal(rec.cpu().numpy().view(np.uint32), oracle.decode_f32(codewords, ref).view(np.uint32))


def test_encode_empty_input(env):
    pq, torch, dev = env["pq"], env["torch"], env["dev"]
    cw = torch.zeros((4, 256, 32), dtype=torch.float32, device=dev)
    assert pq.encode(torch.empty((0, 128), dtype=torch.float32, device=dev), cw).shape == (0, 4)
    assert pq.decode(torch.empty((0, 4), dtype=torch.uint8, device=dev), cw).shape == (0, 128)


# ------------------------------------------------------------------------------------ naive update (Eq. 6)
@pytest.mark.parametrize("M,K,N", [(4, 37, 3001), (8, 100, 20_000), (3, 11, 700), (4, 1000, 100_000)])
def test_update_naive_matches_oracle(env, M, K, N):
    """Integer tables: every sum is exact, so centers and cost sums equal the oracle's bit for bit whatever the
    order of the members.  Real tables: the sums agree to fp64 rounding (the member order is not fixed) and the
    centers are the oracle's except where two candidates tie to within that rounding; both equal the sparse vote's
    centers under the same rule (the paper's exactness claim, Sec. 3.2)."""
    pq, oracle = env["pq"], env["oracle"]
    rng = np.random.default_rng(M * K + 1)
    codes = rng.integers(0, 40, size=(N, M), dtype=np.uint8)
    a = rng.integers(0, K - 1, size=N).astype(np.int32)               # last cluster stays empty
    centers = rng.integers(0, 256, size=(K, M), dtype=np.uint8)
    for integer in (True, False):
        tables = rand_tables(rng, M, integer=integer)
        d_cent = _dev(env, centers)
        _, cost = pq.update_naive(_dev(env, codes), _dev(env, a), _dev(env, tables), d_cent, want_cost=True)
        _sync(env)
        got, cost = d_cent.cpu().numpy(), cost.cpu().numpy()
        rc, rcost = oracle.update_naive(codes, a, tables, centers, want_cost=True)
        assert (got[K - 1] == centers[K - 1]).all()
        if integer:
            np.testing.assert_array_equal(cost, rcost)
            np.testing.assert_array_equal(got, rc)
        else:
            np.testing.assert_allclose(cost, rcost, rtol=1e-12, atol=0)
            diff = np.argwhere(got != rc)
            for k, m in diff:                                         # only exact-tie-level differences are allowed
                assert abs(rcost[k, m, got[k, m]] - rcost[k, m, rc[k, m]]) <= 1e-12 * rcost[k, m, rc[k, m]]
            assert len(diff) <= 2
        d2 = _dev(env, centers)
        pq.update(_dev(env, codes), _dev(env, a), _dev(env, tables), d2)
        _sync(env)
        sparse = d2.cpu().numpy()
        if integer:
            np.testing.assert_array_equal(sparse, got)
        else:
            for k, m in np.argwhere(sparse != got):                    # fp32 vote vs fp64 sums: near-ties only
                assert abs(rcost[k, m, sparse[k, m]] - rcost[k, m, got[k, m]]) <= 1e-5 * rcost[k, m, got[k, m]]
