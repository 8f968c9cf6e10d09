"""Pins for the CPU oracle: every function of oracle/tsa_oracle.py is checked against
something other than itself -- closed forms, hand-worked cases (tests/golden), brute
force in pure Python, and library routines (scipy softmax / logsumexp, torch SDPA and
torch's bf16 rounding) -- chosen so that a dropped term, a wrong sign or index, a
transposed operand or a wrong head mapping fails at least one of them."""
import math
import os
from fractions import Fraction

import numpy as np
import pytest
import scipy.special
import torch

from oracle import tsa_oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rng(seed):
    return np.random.Generator(np.random.PCG64(seed))


# ----------------------------------------------------------------------------- bf16

def test_bf16_widening_matches_torch():
    bits = np.arange(0, 65536, dtype=np.uint16)
    finite = ((bits >> 7) & 0xFF) != 0xFF
    bits = bits[finite]
    ours = orc.bf16_to_f64(bits)
    ref = torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(ours, ref)


def test_bf16_rounding_matches_torch_on_float32_values():
    x32 = np.concatenate([_rng(1).standard_normal(200000).astype(np.float32) * s
                          for s in (1.0, 1e-3, 1e3, 1e-30, 1e30)])
    ours = orc.f64_to_bf16(x32.astype(np.float64))
    ref = torch.from_numpy(x32).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(ours, ref)


def test_bf16_rounding_ties_and_no_double_rounding():
    # exact ties go to even; a value just above a tie that float32 cannot hold must round up
    one = 0x3F80
    assert orc.f64_to_bf16(np.array([1.0 + 2.0 ** -8]))[0] == one            # tie -> even (1.0)
    assert orc.f64_to_bf16(np.array([1.0 + 3 * 2.0 ** -8]))[0] == one + 2    # tie -> even (1 + 2^-6)
    assert orc.f64_to_bf16(np.array([1.0 + 2.0 ** -8 + 2.0 ** -40]))[0] == one + 1
    assert orc.f64_to_bf16(np.array([-(1.0 + 2.0 ** -8 + 2.0 ** -40)]))[0] == (one + 1) | 0x8000
    assert orc.f64_to_bf16(np.array([0.0, -0.0])).tolist() == [0, 0x8000]
    # round trip on every finite bf16 value
    bits = np.arange(0, 65536, dtype=np.uint16)
    bits = bits[((bits >> 7) & 0xFF) != 0xFF]
    assert np.array_equal(orc.f64_to_bf16(orc.bf16_to_f64(bits)), bits)


# ----------------------------------------------------------------------------- score

def _score_brute(Q, K, last_q, scale):
    """Pure-Python definition: Algorithm 1's proxy attention and vertical sum."""
    B, Hq, L, d = Q.shape
    g = Hq // K.shape[1]
    s = np.zeros((B, Hq, L))
    for b in range(B):
        for h in range(Hq):
            for i in range(L - last_q, L):
                logits = []
                for t in range(i + 1):
                    acc = 0.0
                    for c in range(d):
                        acc += float(Q[b, h, i, c]) * float(K[b, h // g, t, c])
                    logits.append(scale * acc)
                mx = max(logits)
                ex = [math.exp(v - mx) for v in logits]
                z = sum(ex)
                for t in range(i + 1):
                    s[b, h, t] += ex[t] / z
    return s


@pytest.mark.parametrize("B,Hq,Hkv,L,d,Lq", [(1, 2, 1, 7, 3, 3), (2, 4, 2, 9, 2, 9), (1, 3, 3, 5, 4, 1)])
def test_score_brute_force(B, Hq, Hkv, L, d, Lq):
    r = _rng(10 + L)
    Q = r.standard_normal((B, Hq, L, d))
    K = r.standard_normal((B, Hkv, L, d))
    got = orc.score(Q, K, Lq)                       # default scale must be 1/sqrt(d)
    want = _score_brute(Q, K, Lq, 1.0 / math.sqrt(d))
    assert np.allclose(got, want, rtol=0, atol=1e-13)
    got2 = orc.score(Q, K, Lq, scale=0.37)
    assert np.allclose(got2, _score_brute(Q, K, Lq, 0.37), rtol=0, atol=1e-13)


def test_score_rows_sum_to_last_q():
    r = _rng(2)
    Q = r.standard_normal((1, 4, 300, 16))
    K = r.standard_normal((1, 2, 300, 16)) * 2
    for Lq in (1, 17, 64, 300):
        s = orc.score(Q, K, Lq)
        assert np.all(s >= 0)
        assert np.allclose(s.sum(axis=-1), Lq, rtol=0, atol=1e-10)


def test_score_zero_keys_closed_form():
    # K = 0: every visible key gets 1/(i+1) from window row i, so
    # s[t] = sum_{i >= max(t, L-Lq)} 1/(i+1)
    L, Lq = 50, 12
    Q = _rng(3).standard_normal((1, 2, L, 8))
    K = np.zeros((1, 2, L, 8))
    s = orc.score(Q, K, Lq)
    want = np.array([float(sum(Fraction(1, i + 1) for i in range(max(t, L - Lq), L))) for t in range(L)])
    assert np.allclose(s[0, 0], want, atol=1e-14) and np.allclose(s[0, 1], want, atol=1e-14)


def test_score_single_query_is_a_softmax_row():
    L, d = 40, 8
    r = _rng(4)
    Q = r.standard_normal((1, 1, L, d))
    K = r.standard_normal((1, 1, L, d))
    s = orc.score(Q, K, 1)
    logits = np.array([sum(Q[0, 0, L - 1, c] * K[0, 0, t, c] for c in range(d)) for t in range(L)]) / math.sqrt(d)
    assert np.allclose(s[0, 0], scipy.special.softmax(logits), atol=1e-14)


def test_score_window_is_causal():
    # changing a key inside the window must not change what earlier window rows give to earlier keys:
    # the last key is seen only by the last query, so its score is a single softmax term <= 1
    L, Lq, d = 30, 8, 4
    r = _rng(5)
    Q = r.standard_normal((1, 1, L, d))
    K = r.standard_normal((1, 1, L, d))
    s = orc.score(Q, K, Lq)
    logits = (Q[0, 0, L - 1] @ K[0, 0].T) / math.sqrt(d)
    assert abs(s[0, 0, L - 1] - scipy.special.softmax(logits)[L - 1]) < 1e-14
    # key L-2 is seen by exactly two rows
    l2 = (Q[0, 0, L - 2] @ K[0, 0, :L - 1].T) / math.sqrt(d)
    assert abs(s[0, 0, L - 2] - scipy.special.softmax(logits)[L - 2] - scipy.special.softmax(l2)[L - 2]) < 1e-14


def test_score_queries_reduces_to_recent_query_scoring_and_brute_force():
    r = _rng(61)
    B, Hq, Hkv, L, d, n = 2, 4, 2, 37, 8, 5
    Q, K = r.standard_normal((B, Hq, L, d)), r.standard_normal((B, Hkv, L, d))
    # the most recent queries at their own positions: Algorithm 1's scorer
    assert np.allclose(orc.score_queries(Q[:, :, L - n:], np.arange(L - n, L), K), orc.score(Q, K, n), rtol=0, atol=1e-14)
    # arbitrary positions against a pure-Python loop
    qpos = np.array([3, 0, 36, 17, 17])
    Qs = Q[:, :, qpos]
    got = orc.score_queries(Qs, qpos, K, scale=0.3)
    for b in range(B):
        for h in range(Hq):
            want = [0.0] * L
            for j, pj in enumerate(qpos):
                w = [math.exp(0.3 * sum(Qs[b, h, j, c] * K[b, h // 2, t, c] for c in range(d))) for t in range(pj + 1)]
                z = sum(w)
                for t in range(pj + 1):
                    want[t] += w[t] / z
            assert np.allclose(got[b, h], want, rtol=0, atol=1e-13)
    assert np.allclose(got.sum(-1), n)                     # every query distributes a mass of one


def test_pool_queries_matches_adaptive_average_pooling():
    r = _rng(62)
    B, Hq, L, d = 1, 2, 53, 8
    from paper_2602_03216_amd import inputs as gen
    Qb = gen.f32_to_bf16_bits(r.standard_normal((B, Hq, L, d)).astype(np.float32))
    Qf = torch.from_numpy(orc.bf16_to_f64(Qb))
    for n_pool in (1, 4, 7, 53):
        bits, qpos = orc.pool_queries(Qb, n_pool)
        ref = torch.nn.functional.adaptive_avg_pool1d(Qf.reshape(B * Hq, L, d).transpose(1, 2), n_pool).transpose(1, 2)
        ref_bits = torch.from_numpy(ref.reshape(B, Hq, n_pool, d).numpy().astype(np.float32)).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
        assert np.array_equal(bits, ref_bits)
        assert qpos[-1] == L - 1 and all(qpos[j] < qpos[j + 1] for j in range(n_pool - 1))
    assert orc.pool_queries(Qb, 1)[1].tolist() == [L - 1]   # a single pooled query sees every key
    assert np.array_equal(orc.pool_queries(Qb, L)[0], Qb)   # one row per segment: the rows themselves


def test_pool_average_zero_padded():
    s = np.array([[1.0, 2.0, 4.0, 8.0, 16.0]])
    assert np.array_equal(orc.pool(s, 1), s)
    assert np.allclose(orc.pool(s, 3), np.array([[3, 7, 14, 28, 24]]) / 3.0)
    assert np.allclose(orc.pool(s, 5), np.array([[7, 15, 31, 30, 28]]) / 5.0)
    x = _rng(6).random((2, 3, 50))
    ref = torch.nn.functional.avg_pool1d(torch.from_numpy(x), 7, stride=1, padding=3,
                                         count_include_pad=True).numpy()
    assert np.allclose(orc.pool(x, 7), ref, atol=1e-15)


def test_group_scores():
    s = np.arange(2 * 6 * 4, dtype=np.float64).reshape(2, 6, 4)
    gs = orc.group_scores(s, 3)
    assert gs.shape == (2, 2, 4)
    assert np.array_equal(gs[1, 1], s[1, 3] + s[1, 4] + s[1, 5])


# ----------------------------------------------------------------------------- budget

def test_keep_count_values():
    # the sparsity sweeps of the five workloads
    assert orc.keep_count(1024, 0.75) == 256
    assert orc.keep_count(8192, 0.5) == 4096 and orc.keep_count(8192, 0.75) == 2048
    assert [orc.keep_count(32768, t) for t in (0.0, 0.5, 0.75, 0.9)] == [32768, 16384, 8192, 3277]
    assert [orc.keep_count(131072, t) for t in (0.75, 0.9)] == [32768, 13108]
    assert orc.keep_count(65536, 0.75) == 16384
    assert orc.keep_count(10, 1.0) == 1 and orc.keep_count(10, 0.0) == 10


def test_keep_count_reproduces_table4_map_sparsity():
    L = 131072
    for line in open(os.path.join(GOLDEN, "table4_map_sparsity.txt")):
        if line.startswith("#") or not line.strip():
            continue
        s_ratio, printed = [float(v) for v in line.split("|")]
        k = orc.keep_count(L, s_ratio)
        kept_pairs = k * (k + 1) // 2
        all_pairs = L * (L + 1) // 2
        assert abs(100.0 * (1 - kept_pairs / all_pairs) - printed) < 0.06


def _budget_brute(s, tau):
    """Pure-Python reading of Algorithm 1's budget steps on exact fractions."""
    B, H, L = len(s), len(s[0]), len(s[0][0])
    out = []
    for b in range(B):
        sl = [sum(Fraction(s[b][h][t]) for h in range(H)) for t in range(L)]
        tot = sum(sl)
        order = sorted(range(L), key=lambda t: (sl[t], t))
        k_sparse, cum = None, Fraction(0)
        if Fraction(tau) <= 0:
            k_sparse = 0
        else:
            for k, t in enumerate(order, start=1):
                cum += sl[t] / tot
                if cum >= Fraction(tau):
                    k_sparse = k
                    break
            if k_sparse is None:
                k_sparse = L
        out.append(max(1, L - k_sparse))
    return out


def test_coverage_budget_hand_cases_and_brute_force():
    # one head, s_l = [1, 2, 5, 8] / 16: ascending cumulative mass 1/16, 3/16, 8/16, 1
    s = np.array([[[8.0, 1.0, 5.0, 2.0]]])
    assert orc.coverage_budget(s, 0.0)[0] == 4
    assert orc.coverage_budget(s, 1 / 16)[0] == 3          # ">=": the first token alone reaches tau
    assert orc.coverage_budget(s, 1.5 / 16)[0] == 2
    assert orc.coverage_budget(s, 3 / 16)[0] == 2
    assert orc.coverage_budget(s, 3.5 / 16)[0] == 1
    assert orc.coverage_budget(s, 1.0)[0] == 1              # never fewer than one token
    # uniform scores: k_sparse = ceil(tau L)
    u = np.ones((1, 3, 64))
    assert orc.coverage_budget(u, 4 / 64)[0] == 60 and orc.coverage_budget(u, 4.5 / 64)[0] == 59
    # two heads: the sum over heads decides, not either head alone; dyadic values are exact in float32
    r = _rng(31)
    for trial in range(20):
        B, H, L = 2, 3, int(r.integers(2, 40))
        s = r.integers(0, 64, size=(B, H, L)).astype(np.float64) / 64.0
        s[:, :, 0] += 1.0                                   # a positive total
        for tau in (0.0, 1 / 128, 0.05, 0.3, 0.99):
            assert orc.coverage_budget(s, tau).tolist() == _budget_brute(s.tolist(), tau)


def test_coverage_budget_sums_the_heads_exactly():
    # head sums [1 + 2^-30, 1, 1]: the term 2^-30 survives only in a sum wider than float32.  With
    # tau = 1/3 the lightest token alone carries 1 / (3 + 2^-30) < 1/3, so two tokens are needed and one
    # is kept; a float32 head sum would see three equal tokens, reach 1/3 with one and keep two.
    s = np.array([[[1.0, 1.0, 1.0], [2.0 ** -30, 0.0, 0.0]]])
    assert _budget_brute(s.tolist(), 1 / 3) == [1]
    assert orc.coverage_budget(s, 1 / 3)[0] == 1
    assert orc.coverage_budget(s.astype(np.float32), 1 / 3)[0] == 1        # float32 INPUT, sum still exact
    # non-dyadic random scores against exact rational arithmetic (tau away from any cumulative value)
    r = _rng(77)
    for trial in range(10):
        s = r.random((1, 5, 30))
        for tau in (0.013, 0.21, 0.66):
            assert orc.coverage_budget(s, tau).tolist() == _budget_brute(s.tolist(), tau)


def test_coverage_budget_long_tail_prunes_the_tail():
    # a few heavy tokens and a long tail of mass 0.4 %: tau = 0.5 % removes exactly the tail
    L = 1000
    s = np.full((1, 2, L), 1.0)
    s[:, :, :4] = 250.0 * 249.0                             # heavy tokens
    tail_mass = (L - 4) * 2.0 / s.sum()
    k_keep = orc.coverage_budget(s, tail_mass)[0]
    assert k_keep == 4
    assert orc.coverage_budget(s, tail_mass * 1.0001)[0] == 3


# ----------------------------------------------------------------------------- select

def _select_brute(v, k):
    order = sorted(range(len(v)), key=lambda t: (-v[t], t))
    return sorted(order[:k])


def test_select_brute_force_and_ties():
    r = _rng(7)
    for trial in range(50):
        L = int(r.integers(1, 40))
        k = int(r.integers(1, L + 1))
        v = r.integers(0, 6, size=L).astype(np.float64)       # many exact ties
        idx, inv = orc.select(v[None, :], k)
        assert idx[0].tolist() == _select_brute(v.tolist(), k)
        assert np.array_equal(inv[0, idx[0]], np.arange(k))
        assert (inv[0] >= 0).sum() == k
    idx, _ = orc.select(np.array([[3.0, 1.0, 3.0, 3.0, 0.0]]), 2)
    assert idx[0].tolist() == [0, 2]
    idx, _ = orc.select(np.array([[0.5, 2.0, 2.0, 0.1]]), 1)
    assert idx[0].tolist() == [1]
    idx, inv = orc.select(np.array([[0.5, 2.0, 2.0, 0.1]]), 4)
    assert idx[0].tolist() == [0, 1, 2, 3] and inv[0].tolist() == [0, 1, 2, 3]


def test_select_shapes_and_forced_tokens():
    s = _rng(8).random((2, 3, 20))
    idx, inv = orc.select(s, 5)
    assert idx.shape == (2, 3, 5) and inv.shape == (2, 3, 20) and idx.dtype == np.int32
    assert np.all(np.diff(idx, axis=-1) > 0)
    idx, _ = orc.select(s, 5, force_first=2, force_last=1)
    assert np.all(idx[..., 0] == 0) and np.all(idx[..., 1] == 1) and np.all(idx[..., -1] == 19)
    # the two remaining slots hold the best of the unforced tokens
    for b in range(2):
        for h in range(3):
            rest = _select_brute(s[b, h, 2:19].tolist(), 2)
            assert idx[b, h, 2:4].tolist() == [t + 2 for t in rest]


# ----------------------------------------------------------------------------- compress / decompress

def test_compress_decompress_roundtrip_and_head_mapping():
    r = _rng(9)
    B, Hq, Hkv, L, d, k = 2, 4, 2, 11, 3, 5
    Q = r.integers(0, 60000, size=(B, Hq, L, d)).astype(np.uint16)
    K = r.integers(0, 60000, size=(B, Hkv, L, d)).astype(np.uint16)
    V = r.integers(0, 60000, size=(B, Hkv, L, d)).astype(np.uint16)
    idx = np.stack([np.stack([np.sort(r.choice(L, k, replace=False)) for _ in range(Hq)]) for _ in range(B)]).astype(np.int32)
    Qc, Kc, Vc = orc.compress(Q, K, V, idx, 0)
    for b in range(B):
        for h in range(Hq):
            for rr in range(k):
                assert np.array_equal(Qc[b, h, rr], Q[b, h, idx[b, h, rr]])
                assert np.array_equal(Kc[b, h, rr], K[b, h // 2, idx[b, h, rr]])
                assert np.array_equal(Vc[b, h, rr], V[b, h // 2, idx[b, h, rr]])
    O = orc.decompress(Qc, idx, L)
    for b in range(B):
        for h in range(Hq):
            mask = np.zeros(L, bool)
            mask[idx[b, h]] = True
            assert np.array_equal(O[b, h, mask], Q[b, h, mask])
            assert not O[b, h, ~mask].any()
    # group mode: one set per KV head
    gidx = idx[:, ::2]
    Qg, Kg, Vg = orc.compress(Q, K, V, gidx, 1)
    assert Kg.shape == (B, Hkv, k, d)
    assert np.array_equal(Qg[1, 3], Q[1, 3, gidx[1, 1]]) and np.array_equal(Vg[1, 1], V[1, 1, gidx[1, 1]])
    Og = orc.decompress(Qg, gidx, L)
    assert np.array_equal(Og[1, 3, gidx[1, 1]], Qg[1, 3])
    # k = L is the identity
    full = np.broadcast_to(np.arange(L, dtype=np.int32), (B, Hq, L))
    Qf, Kf, Vf = orc.compress(Q, K, V, full, 0)
    assert np.array_equal(Qf, Q) and np.array_equal(orc.decompress(Qf, full, L), Q)


def test_residual_add_matches_torch_bf16():
    r = _rng(11)
    B, Hq, L, d, k = 1, 3, 9, 4, 4
    x = orc.f64_to_bf16(r.standard_normal((B, L, Hq * d)))
    Oc = orc.f64_to_bf16(r.standard_normal((B, Hq, k, d)))
    idx = np.stack([np.sort(r.choice(L, k, replace=False)) for _ in range(Hq)])[None].astype(np.int32)
    got = orc.residual_add(x, Oc, idx)
    xt = torch.from_numpy(x.view(np.int16)).view(torch.bfloat16).clone()
    ot = torch.from_numpy(Oc.view(np.int16)).view(torch.bfloat16)
    for h in range(Hq):
        for rr in range(k):
            t = idx[0, h, rr]
            xt[0, t, h * d:(h + 1) * d] = (xt[0, t, h * d:(h + 1) * d].float() + ot[0, h, rr].float()).bfloat16()
    assert np.array_equal(got, xt.view(torch.int16).numpy().view(np.uint16))


# ----------------------------------------------------------------------------- attend

def _attend_brute(Q, K, V, scale, allowed):
    Lc, d = Q.shape
    out = np.zeros((Lc, d))
    for r in range(Lc):
        cols = [c for c in range(Lc) if allowed(r, c)]
        logits = [scale * sum(Q[r, e] * K[c, e] for e in range(d)) for c in cols]
        mx = max(logits)
        w = [math.exp(v - mx) for v in logits]
        z = sum(w)
        for wi, c in zip(w, cols):
            out[r] += (wi / z) * V[c]
    return out


def test_attend_brute_force_causal_and_gqa():
    r = _rng(12)
    B, Hq, Hk, Lc, d = 1, 4, 2, 9, 3
    Q = r.standard_normal((B, Hq, Lc, d))
    K = r.standard_normal((B, Hk, Lc, d))
    V = r.standard_normal((B, Hk, Lc, d))
    got = orc.attend(Q, K, V)
    for h in range(Hq):
        want = _attend_brute(Q[0, h], K[0, h // 2], V[0, h // 2], 1 / math.sqrt(d), lambda rr, c: c <= rr)
        assert np.allclose(got[0, h], want, atol=1e-13)


def test_attend_dense_equals_torch_sdpa():
    r = _rng(13)
    B, H, Lc, d = 2, 3, 130, 16
    Q, K, V = (r.standard_normal((B, H, Lc, d)) for _ in range(3))
    got, lse = orc.attend(Q, K, V, return_lse=True)
    ref = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(Q), torch.from_numpy(K), torch.from_numpy(V), is_causal=True).numpy()
    assert np.allclose(got, ref, atol=1e-12)
    logits = np.einsum("bhrd,bhcd->bhrc", Q, K) / math.sqrt(d)
    logits = np.where(np.tril(np.ones((Lc, Lc), bool)), logits, -np.inf)
    assert np.allclose(lse, scipy.special.logsumexp(logits, axis=-1), atol=1e-12)
    rows = np.array([0, 5, 129])
    assert np.allclose(orc.attend(Q, K, V, rows=rows), got[:, :, rows], atol=1e-14)


def test_attend_special_rows():
    r = _rng(14)
    Lc, d = 20, 5
    Q = r.standard_normal((1, 1, Lc, d))
    V = r.standard_normal((1, 1, Lc, d))
    # row 0 sees one key: its output is v_0 exactly
    K = r.standard_normal((1, 1, Lc, d))
    assert np.allclose(orc.attend(Q, K, V)[0, 0, 0], V[0, 0, 0], atol=1e-15)
    # identical keys: uniform weights -> running mean of the values
    K = np.broadcast_to(r.standard_normal((1, 1, 1, d)), (1, 1, Lc, d))
    want = np.cumsum(V[0, 0], axis=0) / np.arange(1, Lc + 1)[:, None]
    assert np.allclose(orc.attend(Q, K, V)[0, 0], want, atol=1e-13)


def test_forward_is_hard_masked_dense_attention():
    """Section 2.2, Stage 2: zero rows for unselected tokens are equivalent to a hard
    mask on the attention map -- selected rows equal dense causal attention restricted
    to the selected keys; computed here with torch SDPA and an explicit boolean mask."""
    r = _rng(15)
    B, Hq, Hkv, L, d, Lq, k = 1, 4, 2, 96, 8, 16, 37
    Qb = orc.f64_to_bf16(r.standard_normal((B, Hq, L, d)))
    Kb = orc.f64_to_bf16(r.standard_normal((B, Hkv, L, d)) * 1.5)
    Vb = orc.f64_to_bf16(r.standard_normal((B, Hkv, L, d)))
    res = orc.forward(Qb, Kb, Vb, k, Lq)
    Q, K, V = orc.bf16_to_f64(Qb), orc.bf16_to_f64(Kb), orc.bf16_to_f64(Vb)
    Kr = np.repeat(K, 2, axis=1)
    Vr = np.repeat(V, 2, axis=1)
    sel = res["inv"] >= 0                                             # [B,Hq,L]
    mask = np.tril(np.ones((L, L), bool))[None, None] & sel[:, :, None, :]
    mask |= np.eye(L, dtype=bool)[None, None]                         # keep unselected rows finite; they are discarded
    ref = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(Q), torch.from_numpy(Kr), torch.from_numpy(Vr), attn_mask=torch.from_numpy(mask)).numpy()
    O = orc.bf16_to_f64(res["O"])
    assert not O[~sel].any()
    for b in range(B):
        for h in range(Hq):
            assert np.allclose(res["Oc_exact"][b, h], ref[b, h, sel[b, h]], atol=1e-12)
    assert np.array_equal(res["O"][sel], orc.f64_to_bf16(ref[sel]))
    assert np.all(sel.sum(-1) == k)


def test_forward_keep_all_is_dense_attention():
    r = _rng(16)
    B, H, L, d = 1, 2, 40, 8
    Qb, Kb, Vb = (orc.f64_to_bf16(r.standard_normal((B, H, L, d))) for _ in range(3))
    res = orc.forward(Qb, Kb, Vb, L, 8)
    ref = torch.nn.functional.scaled_dot_product_attention(
        *(torch.from_numpy(orc.bf16_to_f64(t)) for t in (Qb, Kb, Vb)), is_causal=True).numpy()
    assert np.array_equal(res["idx"][0, 0], np.arange(L))
    assert np.array_equal(res["O"], orc.f64_to_bf16(ref))


def test_hand_cases_from_golden():
    for line in open(os.path.join(GOLDEN, "hand_cases.txt")):
        if line.startswith("#") or not line.strip():
            continue
        name, ek, s_txt, S_txt, O_txt = [p.strip() for p in line.split("|")]
        K = np.log(np.array([float(v) for v in ek.split()]))[None, None, :, None]
        Q = np.ones((1, 1, 4, 1))
        V = np.array([1.0, 2.0, 3.0, 4.0])[None, None, :, None]
        s_want = np.array([float(Fraction(v)) for v in s_txt.split()])
        S_want = [int(v) for v in S_txt.split()]
        O_want = np.array([float(Fraction(v)) for v in O_txt.split()])
        s = orc.score(Q, K, 2, scale=1.0)
        assert np.allclose(s[0, 0], s_want, atol=1e-15), name
        idx, inv = orc.select(s, 2)
        assert idx[0, 0].tolist() == S_want, name
        Qc, Kc, Vc = orc.compress(Q, K, V, idx, 0)
        Oc = orc.attend(Qc, Kc, Vc, scale=1.0)
        O = orc.decompress(Oc, idx, 4)
        assert np.allclose(O[0, 0, :, 0], O_want, atol=1e-15), name


# ----------------------------------------------------------------------------- block mask

def test_lambda_block_list_against_pair_predicate():
    Lc, Bs, W = 1000, 128, 256
    bl = orc.lambda_block_list(Lc, Bs, W, 1)
    nb = (Lc + Bs - 1) // Bs
    assert bl.shape[0] == nb
    for qb in range(nb):
        want = [kb for kb in range(nb) if kb <= qb and (kb < 1 or qb - kb <= W // Bs)]
        assert [v for v in bl[qb].tolist() if v >= 0] == want
    r = _rng(17)
    Lc, d, Bs, W = 70, 4, 8, 16
    Q, K, V = (r.standard_normal((1, 1, Lc, d)) for _ in range(3))
    bl = orc.lambda_block_list(Lc, Bs, W, 1)
    got = orc.attend(Q, K, V, block_list=bl, block_size=Bs)
    want = _attend_brute(Q[0, 0], K[0, 0], V[0, 0], 1 / math.sqrt(d),
                         lambda rr, c: c <= rr and (c // Bs < 1 or rr // Bs - c // Bs <= W // Bs))
    assert np.allclose(got[0, 0], want, atol=1e-13)
    # a window that covers everything is plain causal attention
    bl_all = orc.lambda_block_list(Lc, Bs, Lc + Bs, 1)
    assert np.allclose(orc.attend(Q, K, V, block_list=bl_all, block_size=Bs), orc.attend(Q, K, V), atol=1e-15)


def test_attend_per_head_block_lists_against_pair_predicate():
    """Per-head block lists (vertical + slash patterns): the oracle against a pure-Python loop that
    applies 'pair (r, c) is visible iff c <= r and block(c) is listed for block(r) of THIS head'."""
    from paper_2602_03216_amd import inputs as gen
    r = _rng(77)
    B, Hq, Hk, Lc, d, Bs = 1, 3, 1, 70, 4, 16
    nb = (Lc + Bs - 1) // Bs
    bl = gen.vertical_slash_block_lists(B, Hq, nb, seed=5, n_vertical=1, slash_blocks=0, n_extra=1)
    assert bl.shape[:3] == (B, Hq, nb) and any(not np.array_equal(bl[0, 0], bl[0, h]) for h in range(1, Hq))
    for h in range(Hq):
        for qb in range(nb):
            row = [int(v) for v in bl[0, h, qb] if v >= 0]
            assert row == sorted(set(row)) and row[0] == 0 and row[-1] == qb     # ascending, sink and diagonal present
    Q, K, V = r.standard_normal((B, Hq, Lc, d)), r.standard_normal((B, Hk, Lc, d)), r.standard_normal((B, Hk, Lc, d))
    got = orc.attend(Q, K, V, block_list=bl, block_size=Bs)
    for h in range(Hq):
        for row in range(Lc):
            listed = set(int(v) for v in bl[0, h, row // Bs] if v >= 0)
            vis = [c for c in range(row + 1) if c // Bs in listed]
            w = [math.exp(sum(Q[0, h, row, j] * K[0, 0, c, j] for j in range(d)) / math.sqrt(d)) for c in vis]
            z = sum(w)
            for j in range(d):
                want = sum(wi * V[0, 0, c, j] for wi, c in zip(w, vis)) / z
                assert abs(got[0, h, row, j] - want) < 1e-12
    # a shared list given per head is the same thing
    lam = orc.lambda_block_list(Lc, Bs, 16, 1)
    per_head = np.broadcast_to(lam, (B, Hq) + lam.shape).copy()
    assert np.array_equal(orc.attend(Q, K, V, block_list=lam, block_size=Bs), orc.attend(Q, K, V, block_list=per_head, block_size=Bs))


# ----------------------------------------------------------------------------- layer selection

def test_layer_drift_closed_forms_and_brute_force():
    r = _rng(41)
    h = r.standard_normal((50, 24))
    assert orc.layer_drift(h, h, 1e-6) == 0.0
    # h_out = (1 + a) h_in: every token drifts by a ||h|| / (||h|| + eps)
    a, eps = 0.25, 0.5
    norms = np.sqrt((h ** 2).sum(1))
    assert abs(orc.layer_drift(h, (1 + a) * h, eps) - np.mean(a * norms / (norms + eps))) < 1e-14
    # a single token, 3-4-5 triangle: ||(3,4)|| / (||(6,8)|| + 0) = 1/2
    assert orc.layer_drift(np.array([[6.0, 8.0]]), np.array([[9.0, 12.0]]), 0.0) == 0.5
    h2 = r.standard_normal((7, 5))
    brute = 0.0
    for t in range(7):
        num = math.sqrt(sum((h2[t, c] - h[t, c]) ** 2 for c in range(5)))
        den = math.sqrt(sum(h[t, c] ** 2 for c in range(5))) + 0.1
        brute += num / den
    assert abs(orc.layer_drift(h[:7, :5], h2, 0.1) - brute / 7) < 1e-14


def test_sparse_layers_rank_and_set():
    # R = [3, 1, 2, 4]: ranks 3/4, 1/4, 2/4, 1 -> delta = 0.5 keeps layers 1 and 2
    rank, flags = orc.sparse_layers([3.0, 1.0, 2.0, 4.0], 0.5)
    assert rank == [0.75, 0.25, 0.5, 1.0] and flags == [0, 1, 1, 0]
    # ties share the rank of the group's upper end (the indicator is <=)
    rank, flags = orc.sparse_layers([1.0, 1.0, 2.0, 2.0], 0.5)
    assert rank == [0.5, 0.5, 1.0, 1.0] and flags == [1, 1, 0, 0]
    # the C helper of the library agrees
    from paper_2602_03216_amd import binding as tsa
    r = _rng(42)
    for n in (1, 5, 32):
        d = r.random(n).astype(np.float32).tolist()
        for delta in (0.1, 0.5, 0.9):
            assert tsa.tsa_sparse_layers(d, delta) == orc.sparse_layers(d, delta)[1]
