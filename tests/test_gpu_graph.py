"""tsa_forward under HIP graph capture: the layer queues only kernels and one device-to-device copy
on the caller's stream (no allocation, no host synchronisation, no memset node), so a caller can
record it once and replay it.  Every replay, with fresh inputs written into the captured buffers and
eager work in between, must reproduce the eager result bit for bit."""
import numpy as np
import pytest
import torch

from tests import gpu_util as gu

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def tsa():
    from paper_2602_03216_amd import binding
    binding.load_library(build_if_missing=False)
    return binding


def test_forward_replays_from_a_captured_graph(tsa):
    B, Hq, Hkv, L, d, Lq, k = 1, 4, 2, 3000, 128, 64, 700
    desc = tsa.make_desc(B, Hq, Hkv, L, d, Lq)
    r = np.random.Generator(np.random.PCG64(77))
    Q = torch.empty((B, Hq, L, d), dtype=torch.bfloat16, device=gu.DEV)
    K = torch.empty((B, Hkv, L, d), dtype=torch.bfloat16, device=gu.DEV)
    V = torch.empty_like(K)
    O = torch.empty_like(Q)
    idx = torch.empty((B, Hq, k), dtype=torch.int32, device=gu.DEV)
    ws = tsa.alloc_workspace(desc, k, gu.DEV)

    def fill():
        Q.copy_(gu.to_dev(gu.rand_bits(r, (B, Hq, L, d))))
        K.copy_(gu.to_dev(gu.rand_bits(r, (B, Hkv, L, d), 1.3)))
        V.copy_(gu.to_dev(gu.rand_bits(r, (B, Hkv, L, d))))

    fill()
    tsa.tsa_forward(desc, Q, K, V, k, O, ws, idx_out=idx)        # warm-up outside the capture
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        tsa.tsa_forward(desc, Q, K, V, k, O, ws, idx_out=idx)
    ws2 = tsa.alloc_workspace(desc, k, gu.DEV)
    for _ in range(4):
        fill()
        O.fill_(3.0)
        idx.fill_(-1)
        graph.replay()
        torch.cuda.synchronize()
        O_graph, idx_graph = O.clone(), idx.clone()
        O.fill_(5.0)
        idx.fill_(-2)
        tsa.tsa_forward(desc, Q, K, V, k, O, ws2, idx_out=idx)   # eager, on a workspace of its own
        torch.cuda.synchronize()
        assert torch.equal(idx_graph, idx)
        assert torch.equal(O_graph, O)


def test_forward_dynamic_replays_from_a_captured_graph(tsa):
    """The layer with the coverage budget decided on the device: the count changes from replay to
    replay (different inputs), the graph stays the same."""
    B, Hq, Hkv, L, d, Lq, tau_cov = 2, 4, 2, 2500, 128, 64, 0.03
    desc = tsa.make_desc(B, Hq, Hkv, L, d, Lq)
    r = np.random.Generator(np.random.PCG64(78))
    Q = torch.empty((B, Hq, L, d), dtype=torch.bfloat16, device=gu.DEV)
    K = torch.empty((B, Hkv, L, d), dtype=torch.bfloat16, device=gu.DEV)
    V = torch.empty_like(K)
    O = torch.empty_like(Q)
    kk = torch.empty((B,), dtype=torch.int32, device=gu.DEV)
    ws = tsa.alloc_forward_dynamic_workspace(desc, L, gu.DEV)

    def fill(spread):
        Q.copy_(gu.to_dev(gu.rand_bits(r, (B, Hq, L, d))))
        K.copy_(gu.to_dev(gu.rand_bits(r, (B, Hkv, L, d), spread)))     # wider keys: peakier scores, smaller count
        V.copy_(gu.to_dev(gu.rand_bits(r, (B, Hkv, L, d))))

    fill(1.0)
    tsa.tsa_forward_dynamic(desc, Q, K, V, tau_cov, L, O, ws, k_keep_out=kk)       # warm-up outside the capture
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        tsa.tsa_forward_dynamic(desc, Q, K, V, tau_cov, L, O, ws, k_keep_out=kk)
    ws2 = tsa.alloc_forward_dynamic_workspace(desc, L, gu.DEV)
    counts = []
    for spread in (1.0, 2.0, 0.5, 1.5):
        fill(spread)
        O.fill_(3.0)
        kk.fill_(-1)
        graph.replay()
        torch.cuda.synchronize()
        O_graph, kk_graph = O.clone(), kk.clone()
        O.fill_(5.0)
        kk.fill_(-2)
        tsa.tsa_forward_dynamic(desc, Q, K, V, tau_cov, L, O, ws2, k_keep_out=kk)  # eager, on a workspace of its own
        torch.cuda.synchronize()
        assert torch.equal(kk_graph, kk)
        assert torch.equal(O_graph, O)
        counts.append(kk.cpu().tolist())
    assert len({tuple(c) for c in counts}) > 1, counts       # the replays really ran with different counts
