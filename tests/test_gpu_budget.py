"""GPU parity of the Dynamic Token Coverage budget (Algorithm 1: cross-head aggregation, ascending
order, cumulative-mass threshold) against the oracle, through the C ABI.  k_keep is an integer:
it must match exactly.  Both sides form the head sum in float32 in head order; masses are float64."""
import numpy as np
import pytest
import torch

from oracle import tsa_oracle as orc
from paper_2602_03216_amd import inputs as gen
from tests import gpu_util as gu

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def tsa():
    from paper_2602_03216_amd import binding
    binding.load_library(build_if_missing=False)
    return binding


def _budget(tsa, s_np, tau):
    B, Hq, L = s_np.shape
    desc = tsa.make_desc(B, Hq, Hq, L, 128, min(64, L))
    s = torch.from_numpy(np.ascontiguousarray(s_np, dtype=np.float32)).to(gu.DEV)
    k = torch.full((B,), -5, dtype=torch.int32, device=gu.DEV)
    tsa.tsa_coverage_budget(desc, s, tau, k, tsa.alloc_workspace(desc, 1, gu.DEV))
    torch.cuda.synchronize()
    return k.cpu().numpy()


@pytest.mark.parametrize("B,Hq,L", [(1, 1, 4), (2, 3, 100), (1, 8, 5000), (3, 4, 16385), (1, 32, 70001)])
def test_budget_random_scores(tsa, B, Hq, L):
    r = np.random.Generator(np.random.PCG64(700 + L))
    s = (r.random((B, Hq, L)) ** 4).astype(np.float32)            # long tail of small scores
    for tau in (0.0, 1e-4, 0.005, 0.01, 0.2, 0.9, 1.0):
        got = _budget(tsa, s, tau)
        want = orc.coverage_budget(s, tau)
        assert np.array_equal(got, want), (tau, got, want)


def test_budget_ties_and_zeros(tsa):
    r = np.random.Generator(np.random.PCG64(9))
    # few distinct dyadic values: the threshold falls inside a run of equal tokens
    s = (r.integers(0, 5, size=(2, 4, 3000)) / 8.0).astype(np.float32)
    for tau in (0.001, 0.05, 0.25, 0.5, 0.75):
        assert np.array_equal(_budget(tsa, s, tau), orc.coverage_budget(s, tau)), tau
    # hand case of the oracle's pins
    s = np.array([[[8.0, 1.0, 5.0, 2.0]]], dtype=np.float32)
    assert [_budget(tsa, s, t)[0] for t in (0.0, 1 / 16, 1.5 / 16, 3 / 16, 3.5 / 16, 1.0)] == [4, 3, 2, 2, 1, 1]
    # uniform scores: k_sparse = ceil(tau L)
    u = np.ones((1, 3, 64), dtype=np.float32)
    assert _budget(tsa, u, 4 / 64)[0] == 60 and _budget(tsa, u, 4.5 / 64)[0] == 59


def test_budget_on_scored_workload_then_forward(tsa):
    """Scores of the 32K grouped-KV workload (cut to 8K tokens), written by the oracle's scorer and
    rounded to float32 -> the same array goes to the library's budget and to the oracle's, at the
    paper's tau = 0.005 / 0.01 and a larger one; then the layer runs with that k_keep."""
    inp = gen.make_inputs(3, L=8192)
    cfg = inp.cfg
    L, Lq = cfg["L"], cfg["last_q"]
    desc = tsa.make_desc(1, cfg["Hq"], cfg["Hkv"], L, cfg["d"], Lq)
    s_np = orc.score(orc.bf16_to_f64(inp.Q[:, :, L - Lq:, :]), orc.bf16_to_f64(inp.K), Lq).astype(np.float32)
    Q, K, V = gu.to_dev(inp.Q), gu.to_dev(inp.K), gu.to_dev(inp.V)
    ws = tsa.alloc_workspace(desc, L, gu.DEV)
    s = torch.from_numpy(s_np).to(gu.DEV)
    kk = torch.zeros(1, dtype=torch.int32, device=gu.DEV)
    for tau in (0.005, 0.01, 0.05):
        tsa.tsa_coverage_budget(desc, s, tau, kk, ws)
        torch.cuda.synchronize()
        k = int(kk.item())
        assert k == int(orc.coverage_budget(s_np, tau)[0])
        assert 1 <= k < L
        O = torch.empty_like(Q)
        idx = torch.empty((1, cfg["Hq"], k), dtype=torch.int32, device=gu.DEV)
        tsa.tsa_forward(desc, Q, K, V, k, O, tsa.alloc_workspace(desc, k, gu.DEV), idx_out=idx)
        torch.cuda.synchronize()
        # the four sink tokens survive any budget here, and exactly k rows per head are non-zero
        assert torch.all(idx[0, :, :4] == torch.arange(4, device=gu.DEV, dtype=torch.int32))
        nonzero_rows = (O[0].float().abs().sum(-1) > 0).sum(-1)
        assert torch.all(nonzero_rows <= k) and torch.all(nonzero_rows >= k - 2)
