"""GPU parity of the scoring ablation's query sets (appendix, "Token Scoring Methods": random
queries, query-only pooling) against the oracle, through the C ABI."""
import numpy as np
import pytest
import torch

from oracle import tsa_oracle as orc
from tests import gpu_util as gu

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def tsa():
    from paper_2602_03216_amd import binding
    binding.load_library(build_if_missing=False)
    return binding


def _rng(seed):
    return np.random.Generator(np.random.PCG64(seed))


@pytest.mark.parametrize("B,Hq,Hkv,L,d,n", [
    (1, 4, 2, 3000, 128, 64),
    (2, 2, 2, 1037, 64, 17),
    (1, 8, 2, 5000, 128, 128),
    (1, 2, 1, 300, 128, 1),
])
def test_random_query_scoring(tsa, B, Hq, Hkv, L, d, n):
    r = _rng(2000 + L)
    Qb, Kb = gu.rand_bits(r, (B, Hq, L, d)), gu.rand_bits(r, (B, Hkv, L, d), 1.3)
    qpos = np.sort(r.choice(L, size=n, replace=False))           # the method's random draw, made by the caller
    desc = tsa.make_desc(B, Hq, Hkv, L, d, n)
    Q, K = gu.to_dev(Qb), gu.to_dev(Kb)
    Qsel = torch.zeros((B, Hq, n, d), dtype=torch.bfloat16, device=gu.DEV)
    tsa.tsa_gather_queries(desc, Q, qpos, Qsel)
    assert np.array_equal(gu.from_dev(Qsel), Qb[:, :, qpos])
    s = torch.full((B, Hq, L), -1.0, dtype=torch.float32, device=gu.DEV)
    tsa.tsa_score_queries(desc, Qsel, qpos, K, s, tsa.alloc_workspace(desc, 1, gu.DEV))
    torch.cuda.synchronize()
    want = orc.score_queries(orc.bf16_to_f64(Qb[:, :, qpos]), qpos, orc.bf16_to_f64(Kb))
    gu.assert_scores_close(s.cpu().numpy(), want, "random-query scores")
    # keys after the last sampled position are seen by no query
    assert not s[:, :, qpos[-1] + 1:].any()


def test_repeated_positions_and_recent_queries(tsa):
    r = _rng(5)
    B, Hq, Hkv, L, d, n = 1, 2, 2, 700, 128, 6
    Qb, Kb = gu.rand_bits(r, (B, Hq, L, d)), gu.rand_bits(r, (B, Hkv, L, d))
    desc = tsa.make_desc(B, Hq, Hkv, L, d, n)
    Q, K = gu.to_dev(Qb), gu.to_dev(Kb)
    ws = tsa.alloc_workspace(desc, 1, gu.DEV)
    s = torch.empty((B, Hq, L), dtype=torch.float32, device=gu.DEV)
    Qsel = torch.empty((B, Hq, n, d), dtype=torch.bfloat16, device=gu.DEV)
    qpos = [0, 10, 10, 10, 699, 699]                            # ties are allowed, so is position 0
    tsa.tsa_gather_queries(desc, Q, qpos, Qsel)
    tsa.tsa_score_queries(desc, Qsel, qpos, K, s, ws)
    gu.assert_scores_close(s.cpu().numpy(), orc.score_queries(orc.bf16_to_f64(Qb[:, :, qpos]), qpos, orc.bf16_to_f64(Kb)))
    # the most recent queries at their own positions: bit-identical to tsa_score
    recent = list(range(L - n, L))
    s2 = torch.empty_like(s)
    tsa.tsa_gather_queries(desc, Q, recent, Qsel)
    tsa.tsa_score_queries(desc, Qsel, recent, K, s, ws)
    tsa.tsa_score(desc, Q, K, s2, ws)
    torch.cuda.synchronize()
    assert torch.equal(s, s2)


@pytest.mark.parametrize("L,d,n_pool", [(4096, 128, 1), (3001, 128, 7), (5000, 64, 64), (200, 128, 128)])
def test_query_pooling(tsa, L, d, n_pool):
    r = _rng(3000 + L)
    B, Hq, Hkv = 1, 4, 2
    Qb, Kb = gu.rand_bits(r, (B, Hq, L, d)), gu.rand_bits(r, (B, Hkv, L, d))
    desc = tsa.make_desc(B, Hq, Hkv, L, d, n_pool)
    Q, K = gu.to_dev(Qb), gu.to_dev(Kb)
    Qsel = torch.zeros((B, Hq, n_pool, d), dtype=torch.bfloat16, device=gu.DEV)
    qpos = tsa.tsa_pool_queries(desc, Q, n_pool, Qsel)
    torch.cuda.synchronize()
    want_bits, want_pos = orc.pool_queries(Qb, n_pool)
    assert qpos == want_pos.tolist()
    # the library sums in float32 (the oracle in float64): a mean that falls next to a bf16 rounding
    # boundary may land on the neighbouring bf16 value; nothing may be further off than that
    got = gu.from_dev(Qsel)
    diff = np.abs(orc.bf16_to_f64(got) - orc.bf16_to_f64(want_bits))
    ulp = np.maximum(np.abs(orc.bf16_to_f64(want_bits)), 2.0 ** -126) * 2.0 ** -7
    assert (diff <= ulp).all() and (got != want_bits).mean() < 0.02
    # scoring from the pooled rows: both sides start from the oracle's pooled rows
    s = torch.empty((B, Hq, L), dtype=torch.float32, device=gu.DEV)
    tsa.tsa_score_queries(desc, gu.to_dev(want_bits), qpos, K, s, tsa.alloc_workspace(desc, 1, gu.DEV))
    torch.cuda.synchronize()
    gu.assert_scores_close(s.cpu().numpy(), orc.score_queries(orc.bf16_to_f64(want_bits), want_pos, orc.bf16_to_f64(Kb)),
                           "pooled-query scores")


def test_rejects_bad_positions(tsa):
    desc = tsa.make_desc(1, 2, 2, 100, 128, 3)
    Q = torch.zeros((1, 2, 100, 128), dtype=torch.bfloat16, device=gu.DEV)
    Qsel = torch.zeros((1, 2, 3, 128), dtype=torch.bfloat16, device=gu.DEV)
    for bad in ([5, 4, 6], [0, 1, 100], [-1, 2, 3]):
        with pytest.raises(tsa.TsaError):
            tsa.tsa_gather_queries(desc, Q, bad, Qsel)
