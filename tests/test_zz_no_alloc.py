"""GPU: pqkm_assign_noalloc, the entry point for callers that cannot allocate (its scratch is a static device
array inside the library), against pqkm_assign on the same inputs: bit-identical assignments and distances, on two
calls in a row of which the second is smaller (the shared array keeps the first call's contents), for 4-byte codes
on the regrouped scan, for 8-byte and 32-byte codes, and the size limit."""
import numpy as np
import pytest

from _util import progress, workload

pytestmark = pytest.mark.gpu


def _case(cfg, N, K, **over):
    import torch

    import workloads as W

    dev = torch.device("cuda:0")
    w = workload(cfg, N=N, K=K, **over)
    codes = W.codes_numpy(w)
    centers = codes[W.init_center_indices(w)].copy()
    import paper_1709_03708_amd as pq

    tables = pq.build_tables(torch.from_numpy(W.codewords(w)).to(dev))
    return w, torch.from_numpy(codes).to(dev), torch.from_numpy(centers).to(dev), tables


@pytest.mark.parametrize("cfg,sizes", [(2, [(600_007, 1000), (70_001, 130)]), (2, [(9_001, 77), (300, 5)]),
                                       (2, [(1_500_000, 900), (600_007, 300)]),
                                       (3, [(200_003, 700), (5_001, 33)]), (4, [(20_001, 300), (1_000, 40)])])
def test_noalloc_assign_matches_assign_twice_in_a_row(cfg, sizes):
    import torch

    import paper_1709_03708_amd as pq

    assert torch.cuda.is_available(), "gpu tests need a GPU"
    pq.load()
    dev = torch.device("cuda:0")
    for N, K in sizes:
        w, codes, centers, tables = _case(cfg, N, K)
        assert pq.workspace_bytes(N, w.M, K) <= pq.NOALLOC_SCRATCH_BYTES
        a_ref, d_ref = pq.assign(codes, centers, tables)
        a = torch.full((N,), -1, dtype=torch.int32, device=dev)
        d = torch.full((N,), float("nan"), dtype=torch.float32, device=dev)
        pq.assign_noalloc(codes, centers, tables, a, d)
        torch.cuda.synchronize()
        assert torch.equal(a, a_ref), f"assignments differ (cfg {cfg}, N={N}, K={K})"
        assert np.array_equal(d.cpu().numpy().view(np.uint32), d_ref.cpu().numpy().view(np.uint32))
        # without distances
        a2 = torch.full((N,), -1, dtype=torch.int32, device=dev)
        pq.assign_noalloc(codes, centers, tables, a2, None)
        torch.cuda.synchronize()
        assert torch.equal(a2, a_ref)
        progress(f"noalloc assign cfg {cfg} N={N} K={K}: identical to pqkm_assign")


def test_noalloc_assign_rejects_what_its_scratch_cannot_hold():
    import torch

    import paper_1709_03708_amd as pq

    dev = torch.device("cuda:0")
    N, M, K = 3_000_000, 4, 4000
    assert pq.workspace_bytes(N, M, K) > pq.NOALLOC_SCRATCH_BYTES
    codes = torch.zeros((N, M), dtype=torch.uint8, device=dev)
    centers = torch.zeros((K, M), dtype=torch.uint8, device=dev)
    tables = torch.zeros((M, 256, 256), dtype=torch.float32, device=dev)
    a = torch.full((N,), -7, dtype=torch.int32, device=dev)
    with pytest.raises(pq.PqkmError) as e:
        pq.assign_noalloc(codes, centers, tables, a)
    assert e.value.code == 5
    torch.cuda.synchronize()
    assert int(a.min()) == -7 and int(a.max()) == -7          # nothing was launched
    # N = 0 is legal and does nothing
    pq.assign_noalloc(codes[:0], centers, tables, a[:0])
