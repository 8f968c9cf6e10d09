"""GPU parity of the Dynamic Token Coverage budget (Algorithm 1: cross-head aggregation, ascending
order, cumulative-mass threshold) against the oracle, through the C ABI.  k_keep is an integer.
The oracle works in float64 throughout; the library adds the heads in float32.  Where the float32
head sums are exact (scores that are multiples of 2^-20 below 1, at most 16 heads) the count must
be equal; on general scores it must lie between the oracle's counts at tau (1 +- eps), eps being
the bound on the relative error of a float32 sum of Hq non-negative terms and of the total."""
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


def _bracket(s_np, tau):
    """The oracle's counts at tau (1 + eps) and tau (1 - eps): any count in between is a correct
    answer for scores known to a relative eps.  eps: Hq - 1 float32 additions per token, 2^-24
    each, doubled for the ratio to the total."""
    eps = 2.0 * s_np.shape[1] * 2.0 ** -24
    return orc.coverage_budget(s_np, min(1.0, tau * (1 + eps))), orc.coverage_budget(s_np, tau * (1 - eps))


def _assert_in_bracket(got, s_np, tau, what=""):
    lo, hi = _bracket(s_np, tau)
    assert np.all(lo <= got) and np.all(got <= hi), (what, tau, lo.tolist(), np.asarray(got).tolist(), hi.tolist())


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
    q = 2.0 ** (24 - int(np.ceil(np.log2(max(Hq, 2)))))            # Hq values below 1 on this grid add up exactly in float32
    sq = (np.floor(s * q) / q).astype(np.float32)
    for tau in (0.0, 1e-4, 0.005, 0.01, 0.2, 0.9, 1.0):
        _assert_in_bracket(_budget(tsa, s, tau), s, tau)
        got, want = _budget(tsa, sq, tau), orc.coverage_budget(sq, tau)
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
        _assert_in_bracket(np.array([k]), s_np, tau, "scored workload")
        assert 1 <= k < L
        O = torch.empty_like(Q)
        idx = torch.empty((1, cfg["Hq"], k), dtype=torch.int32, device=gu.DEV)
        tsa.tsa_forward(desc, Q, K, V, k, O, tsa.alloc_workspace(desc, k, gu.DEV), idx_out=idx)
        torch.cuda.synchronize()
        # the four sink tokens survive any budget here, and exactly k rows per head are non-zero
        assert torch.all(idx[0, :, :4] == torch.arange(4, device=gu.DEV, dtype=torch.int32))
        nonzero_rows = (O[0].float().abs().sum(-1) > 0).sum(-1)
        assert torch.all(nonzero_rows <= k) and torch.all(nonzero_rows >= k - 2)


def _dynamic_case(tsa, B, Hq, Hkv, L, d, tau_cov, k_max, group_mode, seed, window=0):
    """Runs _dynamic_case_form with the form of the attention kernel pinned to each of the two (the layer
    with a device-side count sizes its launch for k_max, tsa_forward for the count itself, so left alone
    they may pick different forms) and once with the choice left to the library."""
    try:
        for form in (1, 2, 0):
            tsa.tsa_bench_set_attend_form(form)
            got = _dynamic_case_form(tsa, B, Hq, Hkv, L, d, tau_cov, k_max, group_mode, seed, window, form)
    finally:
        tsa.tsa_bench_set_attend_form(0)
    return got


def _dynamic_case_form(tsa, B, Hq, Hkv, L, d, tau_cov, k_max, group_mode, seed, window, form):
    """tsa_forward_dynamic against (a) the oracle's budget on the library's own scores: the count must
    lie in the oracle's bracket for those scores; (b) tsa_forward with that count, batch entry by batch
    entry: the same kernels on the same data, bit for bit (form pinned) or within the output bars."""
    r = np.random.Generator(np.random.PCG64(seed))
    Lq = min(64, L)
    Qb, Kb, Vb = gu.rand_bits(r, (B, Hq, L, d)), gu.rand_bits(r, (B, Hkv, L, d), 1.5), gu.rand_bits(r, (B, Hkv, L, d))
    Q, K, V = gu.to_dev(Qb), gu.to_dev(Kb), gu.to_dev(Vb)
    desc = tsa.make_desc(B, Hq, Hkv, L, d, Lq, group_mode=group_mode)
    Hs = Hkv if group_mode else Hq
    s = torch.empty((B, Hq, L), dtype=torch.float32, device=gu.DEV)
    tsa.tsa_score(desc, Q, K, s, tsa.alloc_workspace(desc, 1, gu.DEV))
    s_np = s.cpu().numpy()
    O = torch.full((B, Hq, L, d), 7.0, dtype=torch.bfloat16, device=gu.DEV)
    kk = torch.full((B,), -3, dtype=torch.int32, device=gu.DEV)
    idx = torch.full((B, Hs, k_max), -9, dtype=torch.int32, device=gu.DEV)
    kw = {}
    if window:      # sink + window list laid out for k_max rows: a shorter set uses its first rows
        bl = orc.lambda_block_list(k_max, 128, window, 1)
        kw = dict(block_list=torch.from_numpy(bl).to(gu.DEV), block_size=128, max_blocks_per_row=bl.shape[1])
    tsa.tsa_forward_dynamic(desc, Q, K, V, tau_cov, k_max, O, tsa.alloc_forward_dynamic_workspace(desc, k_max, gu.DEV),
                            k_keep_out=kk, idx_out=idx, **kw)
    torch.cuda.synchronize()
    got_k = kk.cpu().numpy()
    lo, hi = _bracket(s_np, tau_cov)
    assert np.all(np.minimum(lo, k_max) <= got_k) and np.all(got_k <= np.minimum(hi, k_max)), (lo, got_k, hi, k_max)
    for b in range(B):
        k = int(got_k[b])
        d1 = tsa.make_desc(1, Hq, Hkv, L, d, Lq, group_mode=group_mode)
        O1 = torch.empty((1, Hq, L, d), dtype=torch.bfloat16, device=gu.DEV)
        i1 = torch.empty((1, Hs, k), dtype=torch.int32, device=gu.DEV)
        tsa.tsa_forward(d1, Q[b:b + 1].contiguous(), K[b:b + 1].contiguous(), V[b:b + 1].contiguous(), k, O1,
                        tsa.alloc_workspace(d1, k, gu.DEV), idx_out=i1, **kw)
        torch.cuda.synchronize()
        assert torch.equal(idx[b, :, :k], i1[0]), "index sets of batch entry %d" % b
        if form:
            assert torch.equal(O[b], O1[0]), "output of batch entry %d" % b
        else:       # the two calls may have picked different forms of the attention kernel: same attention, other rounding
            gu.assert_output_close(gu.from_dev(O[b]), gu.from_dev(O1[0]), "output of batch entry %d" % b)
    return got_k


@pytest.mark.parametrize("B,Hq,Hkv,L,d,tau_cov,k_max,group_mode", [
    (1, 4, 2, 3000, 128, 0.02, 3000, 0),
    (2, 4, 2, 3000, 128, 0.04, 3000, -512),    # with a sink + 512-token window block list (negative: window)
    (3, 4, 4, 1700, 64, 0.05, 1700, 0),        # three batch entries, three different counts
    (2, 6, 2, 2500, 128, 0.01, 2500, 1),
    (2, 4, 2, 2048, 128, 0.3, 600, 0),         # the budget asks for more than k_max: clamped
    (1, 2, 2, 700, 128, 0.0, 700, 0),          # tau_cov = 0: nothing is dropped
    (1, 2, 1, 900, 64, 1.0, 900, 0),           # tau_cov = 1: a single token is kept
])
def test_forward_dynamic_equals_budget_then_forward(tsa, B, Hq, Hkv, L, d, tau_cov, k_max, group_mode):
    window = -group_mode if group_mode < 0 else 0
    got = _dynamic_case(tsa, B, Hq, Hkv, L, d, tau_cov, k_max, max(group_mode, 0), seed=4100 + L, window=window)
    print("tau_cov %.3g: k_keep %s of %d (k_max %d)" % (tau_cov, got.tolist(), L, k_max))


def test_forward_dynamic_against_the_oracle(tsa):
    """The oracle end to end: its own scores, its own budget, its own forward with that count.  The
    inputs get a margin at the k-th / (k+1)-th score of every head, and tau_cov is put halfway between
    two consecutive values of the oracle's cumulative mass, so that the count has a margin too (half a
    token's mass, some ten times the effect of the library's score error of 3e-5): the count must be
    equal, the index sets bit-exact and the outputs within the bars."""
    inp = gen.make_inputs(3, L=4096)
    cfg = inp.cfg
    B, Hq, Hkv, L, d, Lq = cfg["B"], cfg["Hq"], cfg["Hkv"], cfg["L"], cfg["d"], cfg["last_q"]
    s_ref = orc.score(orc.bf16_to_f64(inp.Q), orc.bf16_to_f64(inp.K), Lq)
    k = int(orc.coverage_budget(s_ref, 0.01)[0])
    from tests.margin import enforce_margin
    s_ref, _ = enforce_margin(inp, [k], 0)
    sl = np.sort(s_ref[0].sum(axis=0))
    cum = np.cumsum(sl / sl.sum())
    k_sparse = L - k
    tau_cov = 0.5 * (cum[k_sparse - 2] + cum[k_sparse - 1])
    assert int(orc.coverage_budget(s_ref, tau_cov)[0]) == k
    assert (cum[k_sparse - 1] - cum[k_sparse - 2]) / tau_cov > 20 * 3e-5
    desc = tsa.make_desc(B, Hq, Hkv, L, d, Lq)
    Q, K, V = gu.to_dev(inp.Q), gu.to_dev(inp.K), gu.to_dev(inp.V)
    O = torch.empty((B, Hq, L, d), dtype=torch.bfloat16, device=gu.DEV)
    kk = torch.zeros((B,), dtype=torch.int32, device=gu.DEV)
    idx = torch.zeros((B, Hq, L), dtype=torch.int32, device=gu.DEV)
    tsa.tsa_forward_dynamic(desc, Q, K, V, tau_cov, L, O, tsa.alloc_forward_dynamic_workspace(desc, L, gu.DEV),
                            k_keep_out=kk, idx_out=idx)
    torch.cuda.synchronize()
    assert int(kk[0].item()) == k
    ref = orc.forward(inp.Q, inp.K, inp.V, k, Lq)
    assert np.array_equal(idx[:, :, :k].cpu().numpy(), ref["idx"])
    gu.assert_output_close(gu.from_dev(O), ref["O"], "forward_dynamic")


def test_forward_dynamic_random_sweep(tsa):
    """Seeded sweep: 30 random shapes, thresholds, capacities, both selection modes, pooled scores."""
    r = np.random.Generator(np.random.PCG64(51))
    for i in range(30):
        B = int(r.choice([1, 2, 3])); d = int(r.choice([64, 128])); Hkv = int(r.choice([1, 2])); Hq = Hkv * int(r.choice([1, 2, 4]))
        L = int(r.integers(1, 3000)); tau = float(r.choice([0.0, 0.003, 0.02, 0.1, 0.5, 0.95, 1.0]))
        k_max = int(r.choice([L, L, max(1, L // 2), max(1, L // 7)]))
        _dynamic_case(tsa, B, Hq, Hkv, L, d, tau, k_max, int(r.integers(0, 2)), seed=5000 + i)
