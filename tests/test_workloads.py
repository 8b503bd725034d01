"""Host logic of the synthetic-workload generator (no method arithmetic in it)."""
import dataclasses

import numpy as np

import workloads as W


def test_numpy_and_torch_generators_agree_bytewise():
    for cfg in (1, 2):
        w = dataclasses.replace(W.CONFIGS[cfg], N=70_001)
        a = W.codes_numpy(w, chunk=9973)
        b = W.codes_torch(w, "cpu", chunk=20_000).numpy()
        np.testing.assert_array_equal(a, b)


def test_codes_are_a_pure_function_of_the_index():
    w = W.CONFIGS[5]                                   # a billion codes: only sampled here
    idx = np.array([0, 1, 12345, 999_999_999, 500_000_000], dtype=np.int64)
    a = W.codes_at(w, idx)
    b = W.codes_numpy(w, start=999_999_990, count=10)
    np.testing.assert_array_equal(a[3], b[9])
    np.testing.assert_array_equal(W.codes_at(w, idx[::-1])[::-1], a)
    c = W.codes_torch(w, "cpu", start=12345, count=3).numpy()
    np.testing.assert_array_equal(c[0], a[2])


def test_structure_matches_the_recipe():
    w = W.CONFIGS[2]
    codes = W.codes_numpy(w, count=200_000)
    tmpl = W.templates(w)
    assert tmpl.shape == (w.T, w.M) and codes.shape == (200_000, w.M)
    # each subcode equals its template's with prob 1 - p + p/256
    tset = [set(tmpl[:, m].tolist()) for m in range(w.M)]
    all_from_templates = {bytes(t) for t in tmpl}
    exact = np.mean([bytes(c) in all_from_templates for c in codes[:20000]])
    assert abs(exact - (1 - w.p + w.p / 256) ** w.M) < 0.02
    assert all(len(s) > 200 for s in tset)
    # bytes are roughly uniform
    assert abs(codes.mean() - 127.5) < 1.0


def test_init_indices_distinct_and_seeded():
    for cfg in (1, 2, 5):
        w = W.CONFIGS[cfg]
        idx = W.init_center_indices(w)
        assert len(idx) == w.K == len(set(idx.tolist()))
        assert idx.min() >= 0 and idx.max() < w.N
        np.testing.assert_array_equal(idx, W.init_center_indices(w))
    w = dataclasses.replace(W.CONFIGS[1], N=64, K=64)
    assert sorted(W.init_center_indices(w).tolist()) == list(range(64))


def test_codeword_distributions():
    assert W.codewords(W.CONFIGS[1]).shape == (4, 256, 32)
    assert (W.codewords(W.CONFIGS[2]) >= 0).all()
    c4 = W.codewords(dataclasses.replace(W.CONFIGS[4], M=2, D=256))
    assert (c4 >= 0).all() and 0.4 < (c4 == 0).mean() < 0.6
    assert abs(W.codewords(W.CONFIGS[3]).std() - 20 * np.sqrt(1 - 2 / np.pi)) < 0.5
