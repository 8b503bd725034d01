"""Pins for the CPU oracle: it is checked against what the paper and the
mathematics fix, never against itself.

Each test names the passage it pins and the mistake it is meant to catch.
All run on the CPU (no GPU marker).
"""
from fractions import Fraction

import numpy as np

import oracle

L = 256


# ----------------------------------------------------------------------------- helpers
def _rand_tables(rng, M, symmetric=False, integer=False):
    if integer:
        t = rng.integers(0, 50, size=(M, L, L)).astype(np.float32)
    else:
        t = rng.random((M, L, L), dtype=np.float32) * 10.0 + 0.1
    if symmetric:
        t = (t + t.transpose(0, 2, 1)) / 2
    return np.ascontiguousarray(t)


def _brute_assign_f32(codes, centers, tables):
    """Eq. 5 with Eq. 3 written out as python loops over np.float32 scalars:
    ascending m, one rounding per add, lowest k on ties."""
    N, M = codes.shape
    out = np.zeros(N, np.int32)
    dist = np.zeros(N, np.float32)
    for n in range(N):
        best, bk = np.float32(np.inf), 0
        for k in range(centers.shape[0]):
            s = tables[0, codes[n, 0], centers[k, 0]]
            for m in range(1, M):
                s = np.float32(s + tables[m, codes[n, m], centers[k, m]])
            if s < best:
                best, bk = s, k
        out[n], dist[n] = bk, best
    return out, dist


def _round_f32(r: Fraction) -> np.float32:
    """Correctly rounded (nearest-even) fp32 of an exact rational."""
    f = np.float32(float(r))
    cands = [f, np.nextafter(f, np.float32(-np.inf)), np.nextafter(f, np.float32(np.inf))]
    errs = [abs(Fraction(float(c)) - r) for c in cands]
    e = min(errs)
    win = [c for c, x in zip(cands, errs) if x == e]
    if len(win) == 1:
        return win[0]
    even = [c for c in win if (c.view(np.uint32) & 1) == 0]
    return even[0]


# ----------------------------------------------------------------------------- Sec. 2.2 tables
def test_tables_match_definition_and_structure(small_problem):
    """Sec. 2.2: A^m[i][j] is the squared distance between codewords i and j.
    Catches: missing square, wrong subspace stride, transposed codeword layout."""
    cw, tables = small_problem["cw"], small_problem["tables"]
    M, _, Ds = cw.shape
    from scipy.spatial.distance import cdist

    for m in range(M):
        ref = cdist(cw[m].astype(np.float64), cw[m].astype(np.float64), "sqeuclidean")
        np.testing.assert_allclose(tables[m], ref, rtol=1e-6, atol=0)
        assert (np.diag(tables[m]) == 0).all()
        assert (tables[m] == tables[m].T).all()
    assert (tables >= 0).all()
    # a single hand-computed entry
    d = cw[1, 3].astype(np.float64) - cw[1, 200].astype(np.float64)
    assert abs(tables[1, 3, 200] - (d * d).sum()) <= 1e-6 * (d * d).sum()


def test_tables_closed_form():
    """Codewords on a lattice: the squared distance has a closed form.
    Codeword i of subspace m is (i, 2i, 0...) * (m+1) -> A = 5 (m+1)^2 (i-j)^2."""
    M, Ds = 3, 4
    cw = np.zeros((M, L, Ds), np.float32)
    i = np.arange(L, dtype=np.float32)
    for m in range(M):
        cw[m, :, 0] = i * (m + 1)
        cw[m, :, 1] = 2 * i * (m + 1)
    t = oracle.build_tables(cw)
    ii, jj = np.meshgrid(np.arange(L), np.arange(L), indexing="ij")
    for m in range(M):
        assert (t[m] == (5.0 * (m + 1) ** 2 * (ii - jj) ** 2).astype(np.float32)).all()


# ----------------------------------------------------------------------------- Eq. 3
def test_sdc_equals_decoded_squared_distance(small_problem):
    """Eq. 3 + Sec. 2.2: SDC equals the squared Euclidean distance between the
    decoded vectors (1e-5 relative).  Decoding is redone here in numpy."""
    cw, tables, codes = small_problem["cw"], small_problem["tables"], small_problem["codes"]
    rng = np.random.default_rng(1)
    M = cw.shape[0]
    x = codes[rng.integers(0, len(codes), 4000)]
    y = rng.integers(0, 256, size=x.shape, dtype=np.uint8)
    y[:200] = x[:200]                                   # identical codes -> exactly 0
    got = oracle.sdc_pairs(x, y, tables)
    dx = np.concatenate([cw[m, x[:, m]] for m in range(M)], axis=1).astype(np.float64)
    dy = np.concatenate([cw[m, y[:, m]] for m in range(M)], axis=1).astype(np.float64)
    ref = ((dx - dy) ** 2).sum(axis=1)
    assert (got[:200] == 0).all()
    nz = ref > 0
    np.testing.assert_allclose(got[nz], ref[nz], rtol=1e-5)
    # the oracle's own decode agrees with the numpy decode
    np.testing.assert_array_equal(oracle.decode(cw, x), dx)


def test_sdc_fp32_order_is_ascending_m():
    """Reading: the running sum is fp32, added in ascending m.  A case where the
    order matters: 1e8 + 1 + 1 + ... differs between ascending and descending."""
    M = 6
    tables = np.zeros((M, L, L), np.float32)
    tables[0, 1, 2] = 1e8
    for m in range(1, M):
        tables[m, 1, 2] = 3.0
    x = np.full((1, M), 1, np.uint8)
    y = np.full((1, M), 2, np.uint8)
    got = oracle.sdc_pairs(x, y, tables)[0]
    asc = np.float32(1e8)
    for m in range(1, M):
        asc = np.float32(asc + np.float32(3.0))
    desc = np.float32(0)
    for m in range(M - 1, 0, -1):
        desc = np.float32(desc + np.float32(3.0))
    desc = np.float32(desc + np.float32(1e8))
    assert asc != desc                     # the pin has power
    assert got == asc


# ----------------------------------------------------------------------------- Eq. 5
def test_assign_brute_force_tiny_asymmetric():
    """Eq. 5 by brute force on tiny inputs, with NON-symmetric tables so that a
    swapped [code][center] index fails."""
    rng = np.random.default_rng(2)
    for M in (1, 2, 3, 5):
        tables = _rand_tables(rng, M)
        codes = rng.integers(0, 7, size=(64, M), dtype=np.uint8)
        centers = rng.integers(0, 7, size=(9, M), dtype=np.uint8)
        a, d = oracle.assign(codes, centers, tables)
        ra, rd = _brute_assign_f32(codes, centers, tables)
        np.testing.assert_array_equal(a, ra)
        np.testing.assert_array_equal(d, rd)
        # swapped orientation must differ somewhere (the pin has power)
        sa, _ = _brute_assign_f32(codes, centers, np.ascontiguousarray(tables.transpose(0, 2, 1)))
        assert (sa != ra).any()


def test_assign_m1_is_numpy_argmin():
    """M = 1: Eq. 5 is a textbook argmin over table entries (numpy's first-minimum rule)."""
    rng = np.random.default_rng(3)
    tables = _rand_tables(rng, 1)
    codes = rng.integers(0, 256, size=(500, 1), dtype=np.uint8)
    centers = rng.integers(0, 256, size=(40, 1), dtype=np.uint8)
    centers[7] = centers[3]                               # duplicate center -> tie
    a, d = oracle.assign(codes, centers, tables)
    sub = tables[0][codes[:, 0]][:, centers[:, 0]]
    np.testing.assert_array_equal(a, sub.argmin(axis=1))
    np.testing.assert_array_equal(d, sub.min(axis=1))
    assert (a != 7).all()


def test_assign_special_cases(small_problem):
    """K = 1 -> every code goes to center 0.  Centers = the codes themselves ->
    distance 0 and the lowest index holding the same code."""
    codes, tables = small_problem["codes"][:400], small_problem["tables"]
    a, _ = oracle.assign(codes, codes[5:6], tables)
    assert (a == 0).all()
    a, d = oracle.assign(codes, codes, tables)
    assert (d == 0).all()
    first = {}
    for i, c in enumerate(map(bytes, codes)):
        first.setdefault(c, i)
    np.testing.assert_array_equal(a, [first[bytes(c)] for c in codes])


def test_assign_hamming_integer_tables():
    """Integer tables A = 1 - delta: SDC is the Hamming distance between codes;
    every sum is exact, so numpy integer arithmetic is the reference, ties abound."""
    rng = np.random.default_rng(4)
    M = 8
    tables = np.ones((M, L, L), np.float32)
    for m in range(M):
        np.fill_diagonal(tables[m], 0)
    codes = rng.integers(0, 4, size=(300, M), dtype=np.uint8)
    centers = rng.integers(0, 4, size=(50, M), dtype=np.uint8)
    a, d = oracle.assign(codes, centers, tables)
    ham = (codes[:, None, :] != centers[None, :, :]).sum(axis=2)
    np.testing.assert_array_equal(a, ham.argmin(axis=1))
    np.testing.assert_array_equal(d, ham.min(axis=1).astype(np.float32))


def test_assign_matches_exact_distance_argmin(small_problem):
    """Within the fp32 error bound, Eq. 5 picks the center whose DECODED vector is
    nearest: the fp64 distance of the chosen center is within 1e-5 of the optimum."""
    cw, codes, centers, tables = (small_problem[k] for k in ("cw", "codes", "centers", "tables"))
    M = cw.shape[0]
    a, d = oracle.assign(codes, centers, tables)
    dx = np.concatenate([cw[m, codes[:, m]] for m in range(M)], axis=1).astype(np.float64)
    dc = np.concatenate([cw[m, centers[:, m]] for m in range(M)], axis=1).astype(np.float64)
    full = ((dx[:, None, :] - dc[None, :, :]) ** 2).sum(axis=2)
    opt = full.min(axis=1)
    chosen = full[np.arange(len(codes)), a]
    assert (chosen <= opt * (1 + 1e-5) + 1e-30).all()
    np.testing.assert_allclose(d, opt, rtol=1e-5, atol=1e-30)


# ----------------------------------------------------------------------------- Eq. 7
def test_histogram_definition_and_conservation(small_problem):
    """Eq. 7 by numpy bincount; sums over bins equal the cluster size; sizes sum to N."""
    codes, centers, tables = small_problem["codes"], small_problem["centers"], small_problem["tables"]
    K, M = centers.shape
    a, _ = oracle.assign(codes, centers, tables)
    hist, counts = oracle.histogram(codes, a, K)
    np.testing.assert_array_equal(counts, np.bincount(a, minlength=K))
    for m in range(M):
        ref = np.bincount(a.astype(np.int64) * 256 + codes[:, m], minlength=K * 256).reshape(K, 256)
        np.testing.assert_array_equal(hist[:, m, :], ref)
        np.testing.assert_array_equal(hist[:, m, :].sum(axis=1), counts)
    assert counts.sum() == len(codes)


# ----------------------------------------------------------------------------- Eq. 6 / Eq. 8
def _brute_update_f64(codes, a, tables, centers):
    """Eq. 6 written out: for each cluster/subspace try every l against every member."""
    K, M = centers.shape
    out = centers.copy()
    cost = np.zeros((K, M, L))
    for k in range(K):
        mem = codes[a == k]
        if len(mem) == 0:
            continue
        for m in range(M):
            c = tables[m][mem[:, m], :].astype(np.float64).sum(axis=0)   # [member j][candidate l]
            cost[k, m] = c
            out[k, m] = c.argmin()
    return out, cost


def test_vote_equals_naive_update_exact_on_integer_tables():
    """Sec. 3.2: sparse voting gives the same result as the naive method (Eq. 6).
    Integer tables make every sum exact, so equality must be bitwise.  Tables are
    NON-symmetric: reading A as [candidate][member] fails."""
    rng = np.random.default_rng(5)
    M, K, N = 3, 11, 700
    tables = _rand_tables(rng, M, integer=True)
    codes = rng.integers(0, 9, size=(N, M), dtype=np.uint8)
    a = rng.integers(0, K - 1, size=N).astype(np.int32)          # cluster K-1 stays empty
    centers = rng.integers(0, 256, size=(K, M), dtype=np.uint8)
    new, hist, counts = oracle.update(codes, a, tables, centers)
    ref, _ = _brute_update_f64(codes, a, tables, centers)
    np.testing.assert_array_equal(new, ref)
    np.testing.assert_array_equal(oracle.update_naive(codes, a, tables, centers), ref)
    assert counts[K - 1] == 0 and (new[K - 1] == centers[K - 1]).all()   # empty cluster keeps its code
    swapped, _ = _brute_update_f64(codes, a, np.ascontiguousarray(tables.transpose(0, 2, 1)), centers)
    assert (swapped != ref).any()


def test_vote_equals_naive_update_float(small_problem):
    """Same equality on real-valued tables: where the fp32 vote and the fp64 brute
    force pick different l, the fp64 cost of the vote's pick is within 1e-6 of optimal."""
    codes, centers, tables = small_problem["codes"], small_problem["centers"], small_problem["tables"]
    a, _ = oracle.assign(codes, centers, tables)
    new, _, counts = oracle.update(codes, a, tables, centers)
    ref, cost = _brute_update_f64(codes, a, tables, centers)
    naive, ncost = oracle.update_naive(codes, a, tables, centers, want_cost=True)
    np.testing.assert_array_equal(naive, ref)
    np.testing.assert_allclose(ncost, cost, rtol=1e-12)
    K, M = centers.shape
    diff = 0
    for k in range(K):
        for m in range(M):
            if counts[k] and new[k, m] != ref[k, m]:
                diff += 1
                assert cost[k, m, new[k, m]] <= cost[k, m].min() * (1 + 1e-6)
    assert diff <= 1


def test_vote_winner_is_codeword_nearest_member_mean(small_problem):
    """The minimiser of Eq. 6 is the subcodeword nearest (squared L2) to the mean of
    the decoded member subvectors:
    sum_n |c_xn - c_l|^2 = sum_n |c_xn - mean|^2 + N_k |mean - c_l|^2."""
    cw, codes, centers, tables = (small_problem[k] for k in ("cw", "codes", "centers", "tables"))
    K, M = centers.shape
    a, _ = oracle.assign(codes, centers, tables)
    new, _, counts = oracle.update(codes, a, tables, centers)
    for k in range(K):
        mem = codes[a == k]
        if len(mem) == 0:
            assert (new[k] == centers[k]).all()
            continue
        for m in range(M):
            mean = cw[m, mem[:, m]].astype(np.float64).mean(axis=0)
            d2 = ((cw[m].astype(np.float64) - mean) ** 2).sum(axis=1)
            if new[k, m] != d2.argmin():
                assert d2[new[k, m]] <= d2.min() * (1 + 1e-6) + 1e-12
    # structural special cases: a one-member cluster takes the member; a cluster whose
    # members all share a code takes that code (zero diagonal, positive off-diagonal)
    c1 = np.array([[9, 8, 7, 6], [1, 2, 3, 4], [1, 2, 3, 4], [1, 2, 3, 4]], np.uint8)
    a1 = np.array([0, 1, 1, 1], np.int32)
    new1, _, _ = oracle.update(c1, a1, tables, np.zeros((2, 4), np.uint8))
    np.testing.assert_array_equal(new1, [[9, 8, 7, 6], [1, 2, 3, 4]])


def test_vote_uses_one_fused_multiply_add_per_bin():
    """Reading: v_l accumulates in fp32 with a single-rounding fused multiply-add per
    non-zero bin, ascending bin order.  Reference: exact rational arithmetic, rounded
    to fp32 once per step.  A separate multiply-then-add differs on these inputs, and
    the second half builds a vote whose WINNER differs between the two."""
    rng = np.random.default_rng(6)
    M = 1
    tables = (rng.random((M, L, L)) * 1000 + 1).astype(np.float32)
    h = np.zeros((1, M, L), np.uint32)
    bins = [3, 17, 99, 200, 255]
    h[0, 0, bins] = [16777213, 12345679, 7, 9999991, 3]
    counts = np.array([h.sum()], np.uint32)
    new = oracle.vote(h, counts, tables, np.zeros((1, M), np.uint8))
    v_fma = np.zeros(L, np.float32)
    v_sep = np.zeros(L, np.float32)
    for l in range(L):
        acc = np.float32(0)
        sep = np.float32(0)
        for j in bins:
            hj = np.float32(h[0, 0, j])
            acc = _round_f32(Fraction(float(hj)) * Fraction(float(tables[0, j, l])) + Fraction(float(acc)))
            sep = np.float32(np.float32(hj * tables[0, j, l]) + sep)
        v_fma[l], v_sep[l] = acc, sep
    assert (v_fma != v_sep).any()
    assert new[0, 0] == int(np.argmin(v_fma))

    # A two-bin vote: bin 5 has count 1, bin 9 has count h2.  Candidate "lx" gets
    # v = fma(h2, a2, a1); candidate "ly" gets exactly max(fused, unfused) (second entry 0).
    found = 0
    for _ in range(2000):
        a1 = np.float32(rng.random() * 1000 + 1)
        a2 = np.float32(rng.random() * 10 + 0.01)
        h2 = int(rng.integers(3, 1000))
        f = _round_f32(Fraction(h2) * Fraction(float(a2)) + Fraction(float(a1)))
        u = np.float32(np.float32(np.float32(h2) * a2) + a1)
        if f == u:
            continue
        found += 1
        t = np.full((1, L, L), 1e9, np.float32)
        # index order chosen so that the unfused tie would go to the other candidate
        lx, ly = (40, 30) if f < u else (30, 40)
        t[0, 5, lx], t[0, 9, lx] = a1, a2
        t[0, 5, ly], t[0, 9, ly] = max(f, u) if f < u else min(f, u), 0.0
        hh = np.zeros((1, 1, L), np.uint32)
        hh[0, 0, 5], hh[0, 0, 9] = 1, h2
        got = oracle.vote(hh, np.array([1 + h2], np.uint32), t, np.zeros((1, 1), np.uint8))[0, 0]
        fused_winner = lx if f < u else ly         # f<u: lx strictly smaller; f>u: ly (=u) smaller
        unfused_winner = 30                        # exact tie -> lowest index
        assert fused_winner != unfused_winner
        assert got == fused_winner
        if found >= 5:
            break
    assert found >= 1


def test_vote_ties_and_zero_bins():
    """Lowest l wins ties (Hamming tables: every l outside the histogram's support
    ties); bins with zero count are skipped without changing v."""
    M = 2
    tables = np.ones((M, L, L), np.float32)
    for m in range(M):
        np.fill_diagonal(tables[m], 0)
    h = np.zeros((2, M, L), np.uint32)
    h[0, 0, [10, 20]] = [5, 5]          # tie between l=10 and l=20 -> 10
    h[0, 1, [200, 30]] = [4, 4]         # -> 30
    h[1, 0, 77] = 1
    h[1, 1, 78] = 1
    counts = np.array([10, 1], np.uint32)
    new = oracle.vote(h, counts, tables, np.zeros((2, M), np.uint8))
    np.testing.assert_array_equal(new, [[10, 30], [77, 78]])


# ----------------------------------------------------------------------------- Alg. 1
def test_fit_is_assign_then_update_and_cost_never_increases(small_problem):
    """Alg. 1: iterations of (assign; update).  Lloyd's argument (Sec. 2.1): neither
    step can increase the summed squared SD.  Evaluated here in fp64 from the tables."""
    codes, centers, tables = small_problem["codes"], small_problem["centers"], small_problem["tables"]
    M = centers.shape[1]

    def cost(cent, a):
        return sum(tables[m][codes[:, m], cent[a, m]].astype(np.float64) for m in range(M)).sum()

    cent = centers.copy()
    prev = np.inf
    for it in range(4):
        a, d = oracle.assign(codes, cent, tables)
        c_assign = cost(cent, a)
        assert c_assign <= prev * (1 + 1e-6)
        assert abs(oracle.objective(codes, cent, a, tables) - c_assign) <= 1e-6 * c_assign
        assert abs(d.astype(np.float64).sum() - c_assign) <= 1e-5 * c_assign
        cent, _, _ = oracle.update(codes, a, tables, cent)
        c_update = cost(cent, a)
        assert c_update <= c_assign * (1 + 1e-6)
        prev = c_update
    fc, fa, fh, fcnt = oracle.fit(codes, tables, centers, 4)
    np.testing.assert_array_equal(fc, cent)
    np.testing.assert_array_equal(fa, a)               # assignment of the LAST assign step
    np.testing.assert_array_equal(fcnt, np.bincount(a, minlength=len(centers)))


def test_fit_zero_iterations_and_empty_input(small_problem):
    codes, centers, tables = small_problem["codes"], small_problem["centers"], small_problem["tables"]
    fc, _, _, _ = oracle.fit(codes, tables, centers, 0)
    np.testing.assert_array_equal(fc, centers)
    a, d = oracle.assign(codes[:0], centers, tables)
    assert a.shape == (0,)
    new, hist, counts = oracle.update(codes[:0], a, tables, centers)
    np.testing.assert_array_equal(new, centers)
    assert hist.sum() == 0 and counts.sum() == 0


def test_oracle_reproduces_the_stored_config1_run():
    """Regression pin: the stored run of configuration 1 (written by tests/golden/make_golden.py,
    which calls only the oracle) is reproduced bit for bit.  The objectives in it decrease."""
    import os
    import sys

    here = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")
    sys.path.insert(0, here)
    import make_golden

    stored = [l.rstrip("\n") for l in open(os.path.join(here, "config1_fit.txt")) if not l.startswith("#")]
    assert make_golden.compute() == stored
    objs = [float(l.split()[3]) for l in stored if l.startswith("iter")]
    assert all(b <= a for a, b in zip(objs, objs[1:])) and len(objs) == 5


def test_fit_until_stops_at_the_fixed_point_and_reports_statistics(small_problem):
    """Alg. 1 with the stop condition 'no assignment changed' (Sec. 3.3 allows any condition).
    Pinned against a hand-rolled loop over the already pinned assign/update, numpy for the
    statistics, and the fixed-point property: one more iteration changes nothing."""
    codes, centers, tables = small_problem["codes"], small_problem["centers"], small_problem["tables"]
    fc, fa, fh, fcnt, stats = oracle.fit_until(codes, tables, centers, 50)
    iters = len(stats)
    assert 2 <= iters < 50                      # converges well before the cap on this problem
    cent = centers.copy()
    prev = np.full(len(codes), -1, np.int32)
    for it in range(iters):
        a, d = oracle.assign(codes, cent, tables)
        assert abs(stats[it, 0] - d.astype(np.float64).sum()) <= 1e-12 * stats[it, 0]
        assert stats[it, 1] == (a != prev).sum()
        cent, h, cnt = oracle.update(codes, a, tables, cent)
        assert stats[it, 2] == (h != 0).sum() and stats[it, 3] == (cnt != 0).sum()
        prev = a
    assert stats[0, 1] == len(codes) and stats[-1, 1] == 0 and (stats[:-1, 1] > 0).all()
    assert (np.diff(stats[:, 0]) <= 1e-9 * stats[0, 0]).all()             # Lloyd: the objective never increases
    np.testing.assert_array_equal(fc, cent)
    np.testing.assert_array_equal(fa, prev)
    # fixed point: another assignment against the final centers reproduces the assignment and the centers
    a2, _ = oracle.assign(codes, fc, tables)
    np.testing.assert_array_equal(a2, fa)
    np.testing.assert_array_equal(oracle.update(codes, a2, tables, fc)[0], fc)
    # the cap is honoured
    _, _, _, _, s2 = oracle.fit_until(codes, tables, centers, 2)
    assert len(s2) == 2 and (s2 == stats[:2]).all()


# ------------------------------------------------------------------------------------ encode / decode (Sec. 2.2)
def test_encode_is_nearest_codeword_exact_on_integer_data():
    """Integer coordinates: every difference, square and partial sum is an exactly representable integer, so the
    fp32 accumulation equals exact integer arithmetic and the result must equal numpy's integer argmin (first
    minimum = lowest index) bit for bit, whatever the summation order.  Non-square M*Ds layout catches a
    transposed subvector split."""
    rng = np.random.default_rng(21)
    M, Ds, N = 3, 5, 400
    cw = rng.integers(-20, 21, size=(M, 256, Ds)).astype(np.float32)
    v = rng.integers(-25, 26, size=(N, M * Ds)).astype(np.float32)
    codes, d2 = oracle.encode(v, cw, want_dist=True)
    vi, ci = v.astype(np.int64).reshape(N, M, Ds), cw.astype(np.int64)
    for m in range(M):
        dist = ((vi[:, m, None, :] - ci[m][None, :, :]) ** 2).sum(-1)          # [N][256] exact
        np.testing.assert_array_equal(codes[:, m], dist.argmin(1))
        np.testing.assert_array_equal(d2[:, m].astype(np.int64), dist.min(1))


def test_encode_scalar_quantiser_closed_form():
    """Ds = 1 is a scalar quantiser: the closest codeword of x is found by bisection in the sorted codewords."""
    rng = np.random.default_rng(22)
    grid = np.sort(rng.choice(np.arange(-4000, 4000), size=256, replace=False)).astype(np.float32)
    perm = rng.permutation(256)
    cw = grid[perm].reshape(1, 256, 1)
    x = (rng.integers(-5000, 5000, size=3000) + 0.25).astype(np.float32)          # never half-way between two codewords
    codes = oracle.encode(x.reshape(-1, 1), cw)[:, 0]
    pos = np.searchsorted(grid, x)
    lo, hi = np.clip(pos - 1, 0, 255), np.clip(pos, 0, 255)
    nearest = np.where(np.abs(x - grid[lo]) <= np.abs(grid[hi] - x), lo, hi)
    inv = np.empty(256, np.int64)
    inv[perm] = np.arange(256)                                                     # sorted position -> codeword index
    np.testing.assert_array_equal(codes, inv[nearest])


def test_encode_real_data_is_optimal_in_exact_arithmetic():
    """Real-valued data: the chosen codeword's exact (fp64) squared distance is within fp32 rounding of the
    exact optimum, and the reported distance equals it to fp32 accuracy."""
    rng = np.random.default_rng(23)
    M, Ds, N = 4, 32, 300
    cw = rng.normal(size=(M, 256, Ds)).astype(np.float32)
    v = rng.normal(size=(N, M * Ds)).astype(np.float32)
    codes, d2 = oracle.encode(v, cw, want_dist=True)
    v64, c64 = v.astype(np.float64).reshape(N, M, Ds), cw.astype(np.float64)
    for m in range(M):
        dist = ((v64[:, m, None, :] - c64[m][None, :, :]) ** 2).sum(-1)
        chosen = dist[np.arange(N), codes[:, m]]
        assert (chosen <= dist.min(1) * (1 + 1e-5)).all()
        np.testing.assert_allclose(d2[:, m], chosen, rtol=1e-5)


def test_encode_decode_round_trip_ties_and_accumulation():
    rng = np.random.default_rng(24)
    M, Ds = 2, 3
    cw = rng.normal(size=(M, 256, Ds)).astype(np.float32)
    cw[0, 200] = cw[0, 7]                                   # a duplicated codeword: the lower index wins
    codes = rng.integers(0, 256, size=(500, M), dtype=np.uint8)
    codes[:5, 0] = 200
    rec = oracle.decode_f32(cw, codes)
    np.testing.assert_array_equal(rec.reshape(500, M, Ds)[:, 1], cw[1][codes[:, 1]])      # decode = fetch codewords
    np.testing.assert_array_equal(rec.astype(np.float64), oracle.decode(cw, codes))
    back, d2 = oracle.encode(rec, cw, want_dist=True)
    expect = codes.copy()
    expect[expect[:, 0] == 200, 0] = 7
    np.testing.assert_array_equal(back, expect)             # a codeword encodes to itself, at distance exactly 0
    assert (d2 == 0).all()
    # the accumulation is one fused multiply-add per dimension in ascending order: vectors for which fused and
    # unfused accumulation, or ascending and descending order, give different bits (found by search, checked
    # against exact rational arithmetic rounded once per operation)
    c1 = np.zeros((1, 256, 3), np.float32)
    c1[0, 1:] = 1e6
    seen_unfused = seen_order = 0
    for trial in range(200):
        x = rng.normal(size=(1, 3)).astype(np.float32)
        _, got = oracle.encode(x, c1, want_dist=True)

        def chain(order, fused):
            acc = Fraction(0)
            for d in order:
                t = _round_f32(Fraction(float(x[0, d])) - Fraction(float(c1[0, 0, d])))
                sq = Fraction(float(t)) ** 2
                acc = Fraction(float(_round_f32(sq + acc))) if fused else \
                    Fraction(float(_round_f32(Fraction(float(_round_f32(sq))) + acc)))
            return np.float32(float(acc))

        assert got[0, 0] == chain((0, 1, 2), True)
        seen_unfused += got[0, 0] != chain((0, 1, 2), False)
        seen_order += got[0, 0] != chain((2, 1, 0), True)
    assert seen_unfused > 10 and seen_order > 10
