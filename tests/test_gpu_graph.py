"""GPU: the calls only enqueue kernels on the caller's stream, so a caller may capture them in a HIP graph.

``pqkm_fit`` (tile images, regrouping or subcode words, scan, histogram path, vote; no memset nodes, no allocation, no
synchronisation; the last three cases: the M = 4 scan that loads its half tiles straight into LDS, the sliding-window scan of 32-byte codes and
the regrouped M = 8 scan, each handing ranks to the sorted-path histogram)
is captured once and replayed several times with eager work and synchronisations between the replays; every
replay must reproduce the eager result bit for bit (the eager path itself is checked against the oracle in
test_gpu_parity.py).
"""
import numpy as np
import pytest

from _util import progress, workload

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("cfg,over,iters", [(1, {}, 3), (2, dict(N=150_000, K=600), 2), (2, dict(N=600_000, K=600), 2), (3, dict(N=60_000, K=300), 2),
                                             (3, dict(N=4_300_000, K=300), 2), (2, dict(N=8_500_000, K=9_000), 2),
                                             (4, dict(N=300_000, K=3_000), 2), (3, dict(N=4_300_000, K=9_000), 2)])
def test_fit_replays_in_a_graph(cfg, over, iters):
    import torch

    import paper_1709_03708_amd as pq
    import workloads as W

    assert torch.cuda.is_available(), "gpu tests need a GPU"
    dev = torch.device("cuda:0")
    w = workload(cfg, **over)
    progress(f"graph replay: cfg {cfg} N={w.N} M={w.M} K={w.K} iters={iters}")
    codes = W.codes_torch(w, dev)
    cent0 = torch.from_numpy(W.codes_at(w, W.init_center_indices(w))).to(dev)
    tables = pq.build_tables(torch.from_numpy(W.codewords(w)).to(dev))
    ws = torch.empty(pq.workspace_bytes(w.N, w.M, w.K), dtype=torch.uint8, device=dev)

    def buffers():
        return (cent0.clone(), torch.full((w.N,), -1, dtype=torch.int32, device=dev),
                torch.zeros((w.K, w.M, 256), dtype=torch.int32, device=dev),
                torch.zeros((w.K,), dtype=torch.int32, device=dev))

    ce, ae, he, ne = buffers()
    pq.fit(codes, tables, ce, iters, assign=ae, hist=he, counts=ne, workspace=ws)     # eager (also the warm-up)
    torch.cuda.synchronize()

    cg, ag, hg, ng = buffers()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        pq.fit(codes, tables, cg, iters, assign=ag, hist=hg, counts=ng, workspace=ws)
    for rep in range(3):
        # eager work between the replays: reset the graph's buffers, scribble over the shared workspace
        cg.copy_(cent0)
        ag.fill_(-1)
        hg.zero_()
        ng.zero_()
        ws.fill_(rep + 1)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(cg, ce), f"centers differ on replay {rep}"
        assert torch.equal(ag, ae), f"assignments differ on replay {rep}"
        assert torch.equal(hg, he), f"histograms differ on replay {rep}"
        assert torch.equal(ng, ne), f"counts differ on replay {rep}"
    assert not np.array_equal(ce.cpu().numpy(), cent0.cpu().numpy())     # the iterations did move the centers
