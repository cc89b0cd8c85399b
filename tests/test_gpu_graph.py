"""The entry points only enqueue kernels on the caller's stream (no allocation, no
synchronisation, no memset), so a sequence of them can be captured into a HIP graph.
The graph is replayed several times with fresh inputs, eager work and
synchronisations between the replays, and every replay is checked against the oracle."""
import numpy as np
import pytest
import torch

import oracle
import paper_1610_03618_amd as cm
from paper_1610_03618_amd import workloads as wl

pytestmark = pytest.mark.gpu


def test_captured_hot_path_replays_match_oracle():
    N, C, H, W = 32, 24, 27, 27
    k, s = 3, 2
    n, classes = 96, 1000
    Ho, Wo = oracle.pool_out_dims(H, W, k, k, s, s, 0, 0)
    dev = torch.device("cuda:0")
    x = torch.zeros((N, C, H, W), dtype=torch.float32, device=dev)
    z = torch.zeros((n, classes), dtype=torch.float32, device=dev)
    xc = torch.empty((C, H, W, N), dtype=torch.float32, device=dev)
    pn = torch.empty((N, C, Ho, Wo), dtype=torch.float32, device=dev)
    pc = torch.empty((C, Ho, Wo, N), dtype=torch.float32, device=dev)
    an = torch.empty((N, C, Ho, Wo), dtype=torch.float32, device=dev)
    back = torch.empty((N, C, Ho, Wo), dtype=torch.float32, device=dev)
    probs = torch.empty_like(z)

    def enqueue():
        st = [cm.cnnmem_transform(x, xc, N, C, H, W, cm.NCHW, cm.CHWN),
              cm.cnnmem_pool(x, pn, N, C, H, W, cm.NCHW, cm.POOL_MAX, k, k, s, s, 0, 0),
              cm.cnnmem_pool(xc, pc, N, C, H, W, cm.CHWN, cm.POOL_MAX, k, k, s, s, 0, 0),
              cm.cnnmem_pool(x, an, N, C, H, W, cm.NCHW, cm.POOL_AVG, k, k, s, s, 0, 0),
              cm.cnnmem_transform(pc, back, N, C, Ho, Wo, cm.CHWN, cm.NCHW),
              cm.cnnmem_softmax(z, probs, n, classes)]
        assert st == [0] * 6

    enqueue()                                   # eager once (also loads the code objects before capture)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        enqueue()

    for replay in range(4):
        rng = np.random.default_rng(900 + replay)
        hx = wl.relu_normal(rng, (N, C, H, W))
        hz = wl.normal_logits(rng, n, classes, 3.0)
        x.copy_(torch.from_numpy(hx))           # eager work between replays
        z.copy_(torch.from_numpy(hz))
        for t in (xc, pn, pc, an, back, probs):
            t.fill_(-7.0)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        want_pn = oracle.pool(hx, N, C, H, W, 0, 0, k, k, s, s)
        assert np.array_equal(xc.cpu().numpy().view(np.uint32),
                              oracle.transform(hx, N, C, H, W, 0, 1).view(np.uint32)), replay
        assert np.array_equal(pn.cpu().numpy().view(np.uint32), want_pn.view(np.uint32)), replay
        assert np.array_equal(pc.cpu().numpy().view(np.uint32),
                              oracle.transform(want_pn, N, C, Ho, Wo, 0, 1).view(np.uint32)), replay
        assert np.array_equal(back.cpu().numpy().view(np.uint32), want_pn.view(np.uint32)), replay
        want_an = oracle.pool(hx, N, C, H, W, 0, 1, k, k, s, s).astype(np.float64)
        assert np.all(np.abs(an.cpu().numpy().astype(np.float64) - want_an) <= 1e-6 * np.abs(want_an)), replay
        want_p = oracle.softmax(hz).astype(np.float64)
        assert np.all(np.abs(probs.cpu().numpy().astype(np.float64) - want_p) <= np.maximum(2e-6 * want_p, 1e-7)), replay
