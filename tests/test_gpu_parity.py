"""GPU parity, entry point by entry point, through the C ABI: every tsa_* call against the CPU
oracle on seeded inputs, at sizes the oracle finishes quickly that still span several tiles
and a ragged tail, plus the edge cases of each step.  Index and byte work is compared
bit-exactly; floating point within the tolerances in tests/gpu_util.py."""
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


@pytest.fixture(params=[1, 2], ids=["rows256", "rows128_split"])
def attend_form(request, tsa):
    """The attention kernel has two forms (256 query rows per workgroup; 128 rows with the keys of a tile
    split over two groups of wavefronts) and picks one per launch from the problem size.  Tests that
    take this fixture run once with each form pinned, so both meet the oracle on every shape."""
    tsa.tsa_bench_set_attend_form(request.param)
    yield request.param
    tsa.tsa_bench_set_attend_form(0)


def _rng(seed):
    return np.random.Generator(np.random.PCG64(seed))


def _ws(tsa, desc, k):
    return tsa.alloc_workspace(desc, k, gu.DEV)


# ------------------------------------------------------------------ score

@pytest.mark.parametrize("B,Hq,Hkv,L,d,Lq", [
    (1, 4, 4, 1024, 64, 64),      # workload 1 shape
    (2, 4, 2, 1500, 128, 64),     # batch, grouped KV heads, ragged length
    (1, 3, 1, 2077, 128, 17),     # odd group size, window not a multiple of the tile
    (1, 2, 2, 100, 64, 100),      # window = whole sequence
    (1, 2, 1, 33, 128, 1),        # single query
    (1, 2, 2, 5000, 128, 128),    # widest window
    (1, 8, 2, 2300, 128, 64),     # four heads per KV head (one per wavefront), several tiles per workgroup, ragged tail
    (1, 7, 1, 1500, 64, 40),      # seven heads per KV head: two rounds over the staged tiles, the second partly idle
    (1, 4, 1, 700, 128, 128),     # four heads per KV head with the widest window
    (1, 7, 1, 1030, 128, 64),     # last chunk holds only window keys
])
def test_score(tsa, B, Hq, Hkv, L, d, Lq):
    r = _rng(100 + L)
    Qb, Kb = gu.rand_bits(r, (B, Hq, L, d)), gu.rand_bits(r, (B, Hkv, L, d), 1.3)
    desc = tsa.make_desc(B, Hq, Hkv, L, d, Lq)
    s = torch.full((B, Hq, L), -1.0, dtype=torch.float32, device=gu.DEV)
    tsa.tsa_score(desc, gu.to_dev(Qb), gu.to_dev(Kb), s, _ws(tsa, desc, 1))
    torch.cuda.synchronize()
    want = orc.score(orc.bf16_to_f64(Qb), orc.bf16_to_f64(Kb), Lq)
    gu.assert_scores_close(s.cpu().numpy(), want, "score")
    assert np.allclose(s.sum(-1).cpu().numpy(), Lq, rtol=1e-4)


def test_score_custom_scale_and_determinism(tsa):
    r = _rng(7)
    B, Hq, Hkv, L, d, Lq = 1, 4, 2, 3000, 128, 64
    Qb, Kb = gu.rand_bits(r, (B, Hq, L, d)), gu.rand_bits(r, (B, Hkv, L, d))
    desc = tsa.make_desc(B, Hq, Hkv, L, d, Lq, scale=0.05)
    Q, K = gu.to_dev(Qb), gu.to_dev(Kb)
    ws = _ws(tsa, desc, 1)
    s1 = torch.empty((B, Hq, L), dtype=torch.float32, device=gu.DEV)
    s2 = torch.empty_like(s1)
    tsa.tsa_score(desc, Q, K, s1, ws)
    tsa.tsa_score(desc, Q, K, s2, ws)
    torch.cuda.synchronize()
    assert torch.equal(s1, s2)
    gu.assert_scores_close(s1.cpu().numpy(), orc.score(orc.bf16_to_f64(Qb), orc.bf16_to_f64(Kb), Lq, scale=0.05))


@pytest.mark.parametrize("pool_w", [3, 7, 33])
def test_score_pooled(tsa, pool_w):
    r = _rng(50 + pool_w)
    B, Hq, Hkv, L, d, Lq = 1, 4, 2, 1777, 128, 64
    Qb, Kb = gu.rand_bits(r, (B, Hq, L, d)), gu.rand_bits(r, (B, Hkv, L, d), 1.3)
    desc = tsa.make_desc(B, Hq, Hkv, L, d, Lq, pool_w=pool_w)
    s = torch.full((B, Hq, L), -1.0, dtype=torch.float32, device=gu.DEV)
    tsa.tsa_score(desc, gu.to_dev(Qb), gu.to_dev(Kb), s, _ws(tsa, desc, 1))
    torch.cuda.synchronize()
    want = orc.pool(orc.score(orc.bf16_to_f64(Qb), orc.bf16_to_f64(Kb), Lq), pool_w)
    gu.assert_scores_close(s.cpu().numpy(), want, "pooled score")


# ------------------------------------------------------------------ select

def _run_select(tsa, scores_np, k, **kw):
    B, Hq, L = scores_np.shape
    Hkv = kw.pop("Hkv", Hq)
    desc = tsa.make_desc(B, Hq, Hkv, L, 128, min(64, L), **kw)
    Hs = Hkv if desc.group_mode else Hq
    s = torch.from_numpy(scores_np.astype(np.float32)).to(gu.DEV)
    idx = torch.full((B, Hs, k), -7, dtype=torch.int32, device=gu.DEV)
    inv = torch.full((B, Hs, L), -7, dtype=torch.int32, device=gu.DEV)
    tsa.tsa_select(desc, s, k, idx, inv, _ws(tsa, desc, k))
    torch.cuda.synchronize()
    return idx.cpu().numpy(), inv.cpu().numpy()


@pytest.mark.parametrize("L,k", [(5, 2), (64, 1), (64, 64), (1000, 250), (1025, 1), (4097, 4097),
                                 (16384, 4096), (33000, 3300), (70001, 17500)])
def test_select_random_scores(tsa, L, k):
    s = _rng(200 + L).random((2, 3, L)).astype(np.float32)
    idx, inv = _run_select(tsa, s, k)
    widx, winv = orc.select(s, k)
    assert np.array_equal(idx, widx) and np.array_equal(inv, winv)


def test_select_exact_ties(tsa):
    idx, inv = _run_select(tsa, np.array([[[3.0, 1.0, 3.0, 3.0, 0.0]]]), 2)
    assert idx[0, 0].tolist() == [0, 2] and inv[0, 0].tolist() == [0, -1, 1, -1, -1]
    r = _rng(3)
    for L, k, levels in ((3000, 700, 4), (5000, 4999, 2), (2048, 1024, 1), (9000, 10, 3)):
        s = r.integers(0, levels, size=(1, 4, L)).astype(np.float32) * 0.25      # few distinct values, many ties
        idx, inv = _run_select(tsa, s, k)
        widx, winv = orc.select(s, k)
        assert np.array_equal(idx, widx) and np.array_equal(inv, winv)
    # rows cut into several slices (of 2048 and of 4096 tokens), ragged last slice, ties across slices
    for rows, L, k, levels in ((2, 40001, 9000, 3), (16, 70000, 20000, 5)):
        s = r.integers(0, levels, size=(1, rows, L)).astype(np.float32) * 0.25
        idx, inv = _run_select(tsa, s, k)
        widx, winv = orc.select(s, k)
        assert np.array_equal(idx, widx) and np.array_equal(inv, winv)
    # signed zeros compare equal, negative scores order correctly
    s = np.array([[[-0.0, 0.0, -1.0, 0.0, -2.0, 5.0]]], dtype=np.float32)
    idx, _ = _run_select(tsa, s, 3)
    assert idx[0, 0].tolist() == [0, 1, 5]
    idx, _ = _run_select(tsa, s, 5)
    assert idx[0, 0].tolist() == [0, 1, 2, 3, 5]


def test_select_forced_tokens_and_group_mode(tsa):
    s = _rng(5).random((1, 8, 3000)).astype(np.float32)
    idx, inv = _run_select(tsa, s, 300, force_first=4, force_last=7)
    widx, winv = orc.select(s, 300, 4, 7)
    assert np.array_equal(idx, widx) and np.array_equal(inv, winv)
    # group mode: the sets are chosen from fp32 group sums; quantise so that the sums are exact
    sq = np.round(s * 4096) / 4096
    idx, inv = _run_select(tsa, sq, 500, Hkv=2, group_mode=1)
    widx, winv = orc.select(orc.group_scores(sq.astype(np.float64), 4), 500)
    assert idx.shape == (1, 2, 500)
    assert np.array_equal(idx, widx) and np.array_equal(inv, winv)


# ------------------------------------------------------------------ compress / decompress

# k = 201 of 777 rows kept: the two-stream scatter kernel (copies driven by idx, zeros by inv);
# k = 60 and k = 700: the inv-driven kernel; both are also run without idx
@pytest.mark.parametrize("d,group_mode,k", [(128, 0, 201), (64, 0, 201), (128, 1, 201), (128, 0, 60), (64, 1, 700)])
def test_compress_decompress_bit_exact(tsa, d, group_mode, k):
    r = _rng(300 + d + group_mode + k)
    B, Hq, Hkv, L = 2, 6, 2, 777
    Qb, Kb, Vb = gu.rand_bits(r, (B, Hq, L, d)), gu.rand_bits(r, (B, Hkv, L, d)), gu.rand_bits(r, (B, Hkv, L, d))
    Hs = Hkv if group_mode else Hq
    idx_np = np.stack([np.stack([np.sort(r.choice(L, k, replace=False)) for _ in range(Hs)]) for _ in range(B)]).astype(np.int32)
    inv_np = np.full((B, Hs, L), -1, dtype=np.int32)
    for b in range(B):
        for h in range(Hs):
            inv_np[b, h, idx_np[b, h]] = np.arange(k)
    desc = tsa.make_desc(B, Hq, Hkv, L, d, 64, group_mode=group_mode)
    idx, inv = torch.from_numpy(idx_np).to(gu.DEV), torch.from_numpy(inv_np).to(gu.DEV)
    Hk = Hkv if group_mode else Hq
    Qc = torch.zeros((B, Hq, k, d), dtype=torch.bfloat16, device=gu.DEV)
    Kc = torch.zeros((B, Hk, k, d), dtype=torch.bfloat16, device=gu.DEV)
    Vc = torch.zeros_like(Kc)
    tsa.tsa_compress(desc, gu.to_dev(Qb), gu.to_dev(Kb), gu.to_dev(Vb), idx, k, Qc, Kc, Vc)
    wq, wk, wv = orc.compress(Qb, Kb, Vb, idx_np, group_mode)
    assert np.array_equal(gu.from_dev(Qc), wq) and np.array_equal(gu.from_dev(Kc), wk) and np.array_equal(gu.from_dev(Vc), wv)
    # decompress: every element written (start from garbage), unselected rows exactly zero
    O = torch.full((B, Hq, L, d), 7.0, dtype=torch.bfloat16, device=gu.DEV)
    tsa.tsa_decompress(desc, Qc, idx, inv, k, O=O)
    assert np.array_equal(gu.from_dev(O), orc.decompress(wq, idx_np, L))
    O2 = torch.full((B, Hq, L, d), 7.0, dtype=torch.bfloat16, device=gu.DEV)
    tsa.tsa_decompress(desc, Qc, None, inv, k, O=O2)                # without S_h: rows located through inv alone
    assert torch.equal(O2, O)
    # residual mode
    xb = gu.rand_bits(r, (B, L, Hq * d))
    x = gu.to_dev(xb)
    tsa.tsa_decompress(desc, Qc, idx, inv, k, residual=x)
    want = orc.residual_add(xb, wq, idx_np)
    got = gu.from_dev(x)
    diff = np.abs(orc.bf16_to_f64(got) - orc.bf16_to_f64(want))
    assert (got != want).mean() < 1e-4 and diff.max() <= 2.0 ** -6        # fp32 add vs exact add: at most one ulp, rarely
    untouched = np.ones((B, L, Hq), dtype=bool)
    for b in range(B):
        for h in range(Hq):
            untouched[b, idx_np[b, h // (Hq // Hs)], h] = False
    assert np.array_equal(got.reshape(B, L, Hq, d)[untouched], xb.reshape(B, L, Hq, d)[untouched])


def test_compress_keep_all_is_identity(tsa):
    r = _rng(11)
    B, H, L, d = 1, 2, 130, 128
    Qb = gu.rand_bits(r, (B, H, L, d))
    idx = torch.arange(L, dtype=torch.int32, device=gu.DEV).repeat(B, H, 1).contiguous()
    desc = tsa.make_desc(B, H, H, L, d, 64)
    Qc, Kc, Vc = (torch.zeros((B, H, L, d), dtype=torch.bfloat16, device=gu.DEV) for _ in range(3))
    Q = gu.to_dev(Qb)
    tsa.tsa_compress(desc, Q, Q, Q, idx, L, Qc, Kc, Vc)
    assert torch.equal(Qc, Q) and torch.equal(Kc, Q) and torch.equal(Vc, Q)


# ------------------------------------------------------------------ attend

@pytest.mark.parametrize("B,Hq,Hk,Lc,d", [
    (1, 2, 2, 1, 128), (1, 2, 2, 63, 128), (1, 2, 1, 64, 128), (1, 4, 2, 65, 64), (2, 2, 2, 128, 128),
    (1, 3, 3, 129, 128), (1, 8, 2, 300, 128), (1, 4, 4, 256, 64), (1, 9, 3, 1000, 128), (1, 2, 2, 2049, 64),
])
def test_attend_matches_oracle(tsa, attend_form, B, Hq, Hk, Lc, d):
    r = _rng(400 + Lc + d)
    Qb, Kb, Vb = gu.rand_bits(r, (B, Hq, Lc, d)), gu.rand_bits(r, (B, Hk, Lc, d)), gu.rand_bits(r, (B, Hk, Lc, d))
    desc = tsa.make_desc(B, Hq, Hk, max(Lc, 1), d, 1)
    O = torch.full((B, Hq, Lc, d), 9.0, dtype=torch.bfloat16, device=gu.DEV)
    lse = torch.zeros((B, Hq, Lc), dtype=torch.float32, device=gu.DEV)
    Vd = gu.to_dev(Vb)
    tsa.tsa_attend(desc, gu.to_dev(Qb), gu.to_dev(Kb), Vd, Lc, Hk, O, tsa.alloc_attend_workspace(desc, Lc, Hk, gu.DEV), lse)
    torch.cuda.synchronize()
    assert np.array_equal(gu.from_dev(Vd), Vb)                 # the caller's V is left alone
    want, wlse = orc.attend(orc.bf16_to_f64(Qb), orc.bf16_to_f64(Kb), orc.bf16_to_f64(Vb), return_lse=True)
    gu.assert_output_close(gu.from_dev(O), orc.f64_to_bf16(want), "attend")
    assert np.abs(lse.cpu().numpy() - wlse).max() < 2e-3
    # row 0 attends to a single key: the output is v_0 exactly
    g = Hq // Hk
    for h in range(Hq):
        assert np.array_equal(gu.from_dev(O)[0, h, 0], Vb[0, h // g, 0])


def test_attend_large_logits_and_scale(tsa, attend_form):
    r = _rng(21)
    B, H, Lc, d = 1, 2, 500, 128
    Qb, Kb, Vb = gu.rand_bits(r, (B, H, Lc, d), 4.0), gu.rand_bits(r, (B, H, Lc, d), 4.0), gu.rand_bits(r, (B, H, Lc, d))
    desc = tsa.make_desc(B, H, H, Lc, d, 1, scale=0.2)        # logits of several hundred: the running max must hold
    O = torch.empty((B, H, Lc, d), dtype=torch.bfloat16, device=gu.DEV)
    tsa.tsa_attend(desc, gu.to_dev(Qb), gu.to_dev(Kb), gu.to_dev(Vb), Lc, H, O, tsa.alloc_attend_workspace(desc, Lc, H, gu.DEV))
    want = orc.attend(orc.bf16_to_f64(Qb), orc.bf16_to_f64(Kb), orc.bf16_to_f64(Vb), scale=0.2)
    gu.assert_output_close(gu.from_dev(O), orc.f64_to_bf16(want), "attend(large logits)")


def test_attend_logits_growing_along_the_keys(tsa, attend_form):
    """Keys grow along the sequence (logit of key c about 0.066 c nats, 190 log2 units over the row):
    the running max is raised every tile or two, in the middle of the pipelined iterations, where the
    half tile that waits for its exponentials has to be shifted together with the accumulator."""
    r = _rng(23)
    B, H, Lc, d = 1, 2, 2000, 128
    u = np.ones(d) / np.sqrt(d)
    q = 6.0 * u + 0.3 * r.standard_normal((B, H, Lc, d))
    k = (np.arange(Lc)[None, None, :, None] / 8.0) * u + 0.3 * r.standard_normal((B, H, Lc, d))
    Qb, Kb, Vb = orc.f64_to_bf16(q), orc.f64_to_bf16(k), gu.rand_bits(r, (B, H, Lc, d))
    desc = tsa.make_desc(B, H, H, Lc, d, 1)
    O = torch.empty((B, H, Lc, d), dtype=torch.bfloat16, device=gu.DEV)
    lse = torch.zeros((B, H, Lc), dtype=torch.float32, device=gu.DEV)
    tsa.tsa_attend(desc, gu.to_dev(Qb), gu.to_dev(Kb), gu.to_dev(Vb), Lc, H, O, tsa.alloc_attend_workspace(desc, Lc, H, gu.DEV), lse)
    want, wlse = orc.attend(orc.bf16_to_f64(Qb), orc.bf16_to_f64(Kb), orc.bf16_to_f64(Vb), return_lse=True)
    gu.assert_output_close(gu.from_dev(O), orc.f64_to_bf16(want), "attend(growing logits)")
    assert np.abs(lse.cpu().numpy() - wlse).max() < 2e-3


# (3000, 1024): long stretches of pipelined iterations between the sink block, the window's first
# block (visited by half of the workgroup only) and the diagonal
@pytest.mark.parametrize("Lc,window,Bs", [(1000, 256, 128), (1300, 128, 128), (640, 4096, 128), (3000, 1024, 128),
                                          (1000, 256, 64), (2100, 512, 64), (1500, 512, 256), (3000, 1024, 256)])
def test_attend_block_list(tsa, attend_form, Lc, window, Bs):
    r = _rng(500 + Lc + Bs)
    B, Hq, Hk, d = 1, 4, 2, 128
    Qb, Kb, Vb = gu.rand_bits(r, (B, Hq, Lc, d)), gu.rand_bits(r, (B, Hk, Lc, d)), gu.rand_bits(r, (B, Hk, Lc, d))
    bl = orc.lambda_block_list(Lc, Bs, window, 1)
    desc = tsa.make_desc(B, Hq, Hk, Lc, d, 1)
    O = torch.empty((B, Hq, Lc, d), dtype=torch.bfloat16, device=gu.DEV)
    tsa.tsa_attend(desc, gu.to_dev(Qb), gu.to_dev(Kb), gu.to_dev(Vb), Lc, Hk, O, tsa.alloc_attend_workspace(desc, Lc, Hk, gu.DEV),
                   block_list=torch.from_numpy(bl).to(gu.DEV), block_size=Bs, max_blocks_per_row=bl.shape[1])
    want = orc.attend(orc.bf16_to_f64(Qb), orc.bf16_to_f64(Kb), orc.bf16_to_f64(Vb), block_list=bl, block_size=Bs)
    gu.assert_output_close(gu.from_dev(O), orc.f64_to_bf16(want), "attend(block list)")


# ------------------------------------------------------------------ forward

@pytest.mark.parametrize("Hq,Hkv,L,d,Lq,k,group_mode,plant", [
    (4, 2, 1111, 128, 64, 300, 0, "direction"),
    (4, 4, 700, 64, 32, 699, 0, "norm"),
    (6, 2, 900, 128, 64, 129, 1, "zipf_sink"),
    (2, 2, 257, 128, 64, 257, 0, "direction"),     # keep everything: dense causal attention
    (2, 1, 200, 64, 8, 1, 0, "norm"),              # keep a single token
])
def test_forward_small(tsa, attend_form, Hq, Hkv, L, d, Lq, k, group_mode, plant):
    from paper_2602_03216_amd import inputs as gen
    from tests.margin import enforce_margin
    cfg = dict(id=90, name="small", B=1, Hq=Hq, Hkv=Hkv, L=L, d=d, last_q=Lq, plant=plant, n_plant=20, norm_factor=3.0,
               frac_plant=0.1, boost=4.0, sink_boost=6.0, n_sink=4, zipf_a=1.2)
    inp = gen.make_inputs(cfg, seed=600 + L)
    enforce_margin(inp, [k], group_mode)            # the k-th / (k+1)-th scores are separated: one right answer
    desc = tsa.make_desc(1, Hq, Hkv, L, d, Lq, group_mode=group_mode)
    Hs = Hkv if group_mode else Hq
    O = torch.full((1, Hq, L, d), 3.0, dtype=torch.bfloat16, device=gu.DEV)
    idx = torch.zeros((1, Hs, k), dtype=torch.int32, device=gu.DEV)
    tsa.tsa_forward(desc, gu.to_dev(inp.Q), gu.to_dev(inp.K), gu.to_dev(inp.V), k, O, _ws(tsa, desc, k), idx_out=idx)
    torch.cuda.synchronize()
    ref = orc.forward(inp.Q, inp.K, inp.V, k, Lq, group_mode=group_mode)
    assert np.array_equal(idx.cpu().numpy(), ref["idx"])
    gu.assert_output_close(gu.from_dev(O), ref["O"], "forward")
    sel = ref["inv"] >= 0
    assert not gu.from_dev(O)[np.repeat(~sel, Hq // Hs, axis=1)].any()


def test_attend_random_sweep(tsa, attend_form):
    """Seeded sweep: 40 random attention problems (1 to 2600 rows, both head sizes, grouped heads, one or
    two batch entries) with no block list, a sink + window list or per-head vertical + slash lists, at
    the three block sizes: outputs within the bars of the oracle."""
    from paper_2602_03216_amd import inputs as gen
    r = _rng(41)
    for i in range(40):
        d = int(r.choice([64, 128])); Hk = int(r.choice([1, 2, 3])); Hq = Hk * int(r.choice([1, 2, 4])); B = int(r.choice([1, 1, 2]))
        Lc = int(r.integers(1, 2600)); mode = i % 3; Bs = int(r.choice([64, 128, 256]))
        Qb, Kb, Vb = gu.rand_bits(r, (B, Hq, Lc, d)), gu.rand_bits(r, (B, Hk, Lc, d)), gu.rand_bits(r, (B, Hk, Lc, d))
        kw, okw, per_head = {}, {}, 0
        if mode == 1:
            bl = orc.lambda_block_list(Lc, Bs, int(r.choice([64, 256, 700, 5000])), int(r.choice([1, 2])))
        elif mode == 2:
            bl = gen.vertical_slash_block_lists(B, Hq, (Lc + Bs - 1) // Bs, int(r.integers(1 << 30)), n_vertical=int(r.integers(0, 4)),
                                                slash_blocks=int(r.integers(0, 4)), n_extra=int(r.integers(0, 3)))
            per_head = 1
        if mode:
            kw = dict(block_list=torch.from_numpy(np.ascontiguousarray(bl)).to(gu.DEV), block_size=Bs, max_blocks_per_row=bl.shape[-1])
            okw = dict(block_list=bl, block_size=Bs)
        desc = tsa.make_desc(B, Hq, Hk, Lc, d, 1, block_list_per_head=per_head)
        O = torch.full((B, Hq, Lc, d), 9.0, dtype=torch.bfloat16, device=gu.DEV)
        tsa.tsa_attend(desc, gu.to_dev(Qb), gu.to_dev(Kb), gu.to_dev(Vb), Lc, Hk, O, tsa.alloc_attend_workspace(desc, Lc, Hk, gu.DEV), **kw)
        want = orc.attend(orc.bf16_to_f64(Qb), orc.bf16_to_f64(Kb), orc.bf16_to_f64(Vb), **okw)
        gu.assert_output_close(gu.from_dev(O), orc.f64_to_bf16(want), "attend %s" % ((B, Hq, Hk, Lc, d, mode, Bs),))


def test_select_and_budget_random_sweep(tsa):
    """Seeded sweep: 60 random shapes (1 to 140000 tokens, one to three batch entries, both selection
    modes, forced tokens) on four kinds of scores (uniform, a handful of distinct values, signed zeros
    only, a long tail with a repeated value), quantised so that float32 sums over heads are exact: index
    sets, inverse maps and budgets bit-exact against the float64 oracle."""
    r = _rng(31)
    for i in range(60):
        B = int(r.choice([1, 1, 2, 3])); Hkv = int(r.choice([1, 2, 4])); Hq = Hkv * int(r.choice([1, 2, 4])); gm = int(r.integers(0, 2))
        L = int(r.choice([r.integers(1, 300), r.integers(300, 20000), r.integers(20000, 140000)]))
        k = int(r.integers(1, L + 1)); ff = int(r.choice([0, 0, 3])); fl = int(r.choice([0, 0, 5]))
        if ff + fl > min(k, L):
            ff = fl = 0
        kind = i % 4
        if kind == 0:
            s = r.random((B, Hq, L)).astype(np.float32)
        elif kind == 1:
            s = (r.integers(0, 4, (B, Hq, L)) / 4.0).astype(np.float32)
        elif kind == 2:
            s = np.where(r.random((B, Hq, L)) < 0.5, 0.0, -0.0).astype(np.float32)
        else:
            s = (r.random((B, Hq, L)) ** 8).astype(np.float32)
            s[..., ::7] = s[..., 0:1]
        # multiples of 2^-20 below 1, at most 16 heads: the float32 sums over a group and over all
        # heads (which the library forms) are exact, so the float64 oracle must give the same answer
        s = (np.floor(s * 2.0 ** 20) / 2.0 ** 20).astype(np.float32)
        desc = tsa.make_desc(B, Hq, Hkv, L, 128, min(64, L), group_mode=gm, force_first=ff, force_last=fl)
        Hs = Hkv if gm else Hq
        sd = torch.from_numpy(s).to(gu.DEV)
        idx = torch.full((B, Hs, k), -7, dtype=torch.int32, device=gu.DEV)
        inv = torch.full((B, Hs, L), -7, dtype=torch.int32, device=gu.DEV)
        tsa.tsa_select(desc, sd, k, idx, inv, _ws(tsa, desc, k))
        sel = orc.group_scores(s.astype(np.float64), Hq // Hkv) if gm else s.astype(np.float64)
        widx, winv = orc.select(sel, k, force_first=ff, force_last=fl)
        what = (B, Hq, Hkv, gm, L, k, ff, fl, kind)
        assert np.array_equal(idx.cpu().numpy(), widx), what
        assert np.array_equal(inv.cpu().numpy(), winv), what
        if s.sum() > 0:
            tau = float(r.choice([0.0, 1e-3, 0.01, 0.3, 0.77, 1.0]))
            kk = torch.zeros(B, dtype=torch.int32, device=gu.DEV)
            tsa.tsa_coverage_budget(desc, sd, tau, kk, _ws(tsa, desc, 1))
            assert np.array_equal(kk.cpu().numpy(), orc.coverage_budget(s, tau)), (what, tau)


def _random_forward_cases(n, seed):
    r = np.random.Generator(np.random.PCG64(seed))
    cases = []
    for i in range(n):
        d = int(r.choice([64, 128]))
        Hkv = int(r.choice([1, 2, 3]))
        Hq = Hkv * int(r.choice([1, 2, 4]))
        L = int(r.integers(2, 900))
        Lq = int(min(L, r.choice([1, 8, 33, 64, 128])))
        k = int(r.integers(1, L + 1))
        cases.append((Hq, Hkv, L, d, Lq, k, int(r.integers(0, 2)), str(r.choice(["direction", "norm", "zipf_sink"])),
                      int(r.choice([1, 1, 3, 5]))))
    return cases


@pytest.mark.parametrize("Hq,Hkv,L,d,Lq,k,group_mode,plant,pool_w", _random_forward_cases(40, 20260203))
def test_forward_random_shapes(tsa, Hq, Hkv, L, d, Lq, k, group_mode, plant, pool_w):
    """Seeded sweep over ragged shapes, head groupings, window lengths, counts, both selection modes and
    pooling widths: index sets bit-exact, outputs within the bars, zero rows exact."""
    from paper_2602_03216_amd import inputs as gen
    from tests.margin import enforce_margin
    cfg = dict(id=91, name="random", B=1, Hq=Hq, Hkv=Hkv, L=L, d=d, last_q=Lq, plant=plant, n_plant=min(20, max(1, L // 4)),
               norm_factor=3.0, frac_plant=0.1, boost=4.0, sink_boost=6.0, n_sink=min(4, L), zipf_a=1.2)
    # The k-th / (k+1)-th selection scores are separated, so there is one right answer.  Pooling gives a
    # planted token's neighbours almost the token's own pooled score: a count that cuts through such a
    # run cannot be given a margin by redrawing ordinary key rows, so the count moves to the nearest one
    # that can (the draw and every other parameter of the case stay).
    for k_try in [k] + [k + s * j for j in range(1, 9) for s in (1, -1) if 1 <= k + s * j <= L]:
        inp = gen.make_inputs(cfg, seed=7000 + 13 * L + k)
        try:
            enforce_margin(inp, [k_try], group_mode, pool_w=pool_w)
        except AssertionError:
            assert pool_w > 1, "no margin without pooling"
            continue
        k = k_try
        break
    else:
        raise AssertionError("no count near %d with a margin" % k)
    desc = tsa.make_desc(1, Hq, Hkv, L, d, Lq, pool_w=pool_w, group_mode=group_mode)
    Hs = Hkv if group_mode else Hq
    O = torch.full((1, Hq, L, d), 3.0, dtype=torch.bfloat16, device=gu.DEV)
    idx = torch.zeros((1, Hs, k), dtype=torch.int32, device=gu.DEV)
    tsa.tsa_forward(desc, gu.to_dev(inp.Q), gu.to_dev(inp.K), gu.to_dev(inp.V), k, O, _ws(tsa, desc, k), idx_out=idx)
    torch.cuda.synchronize()
    ref = orc.forward(inp.Q, inp.K, inp.V, k, Lq, pool_w=pool_w, group_mode=group_mode)
    assert np.array_equal(idx.cpu().numpy(), ref["idx"])
    gu.assert_output_close(gu.from_dev(O), ref["O"], "forward")
    assert not gu.from_dev(O)[np.repeat(ref["inv"] < 0, Hq // Hs, axis=1)].any()


@pytest.mark.parametrize("B,Hq,Hkv,L,d,k,group_mode,with_blocks", [
    (1, 4, 2, 1500, 128, 700, 0, False),
    (2, 6, 2, 1203, 128, 333, 1, False),
    (1, 4, 4, 900, 64, 900, 0, False),
    (1, 4, 2, 2100, 128, 1100, 0, True),
    (3, 2, 1, 777, 64, 200, 0, True),
    (2, 4, 2, 520, 128, 1, 0, False),
])
def test_fused_path_equals_the_separate_calls(tsa, attend_form, B, Hq, Hkv, L, d, k, group_mode, with_blocks):
    """tsa_forward / tsa_compress_v_tiles + tsa_attend_fused against tsa_score -> tsa_select ->
    tsa_compress -> tsa_attend -> tsa_decompress on the same inputs: gather and scatter are copies
    and the arithmetic is the same, so every output must match bit for bit (the separate calls are
    the ones checked against the oracle above)."""
    r = _rng(900 + L)
    Lq = 64
    Q, K, V = (gu.to_dev(gu.rand_bits(r, (B, h, L, d))) for h in (Hq, Hkv, Hkv))
    desc = tsa.make_desc(B, Hq, Hkv, L, d, Lq, group_mode=group_mode)
    Hs = Hkv if group_mode else Hq
    ws = _ws(tsa, desc, k)
    bl = bl_kw = None
    kw = {}
    if with_blocks:
        bl = torch.from_numpy(orc.lambda_block_list(k, 128, 256, 1)).to(gu.DEV)
        kw = dict(block_list=bl, block_size=128, max_blocks_per_row=bl.shape[1])
    # separate calls
    s = torch.empty((B, Hq, L), dtype=torch.float32, device=gu.DEV)
    idx = torch.empty((B, Hs, k), dtype=torch.int32, device=gu.DEV)
    inv = torch.empty((B, Hs, L), dtype=torch.int32, device=gu.DEV)
    Qc = torch.empty((B, Hq, k, d), dtype=torch.bfloat16, device=gu.DEV)
    Kc = torch.empty((B, Hs, k, d), dtype=torch.bfloat16, device=gu.DEV)
    Vc, Oc, O1 = torch.empty_like(Kc), torch.empty_like(Qc), torch.full((B, Hq, L, d), 5.0, dtype=torch.bfloat16, device=gu.DEV)
    tsa.tsa_score(desc, Q, K, s, ws)
    tsa.tsa_select(desc, s, k, idx, inv, ws)
    tsa.tsa_compress(desc, Q, K, V, idx, k, Qc, Kc, Vc)
    tsa.tsa_attend(desc, Qc, Kc, Vc, k, Hs, Oc, tsa.alloc_attend_workspace(desc, k, Hs, gu.DEV), **kw)
    tsa.tsa_decompress(desc, Oc, idx, inv, k, O=O1)
    x0 = gu.to_dev(gu.rand_bits(r, (B, L, Hq * d)))
    x1, x2, x3 = x0.clone(), x0.clone(), x0.clone()
    tsa.tsa_decompress(desc, Oc, idx, inv, k, residual=x1)
    # the two fused launches on the same index sets
    Vt = tsa.alloc_attend_workspace(desc, k, Hs, gu.DEV)
    O2 = torch.full_like(O1, 7.0)
    Oc2 = torch.full_like(Oc, 7.0)
    tsa.tsa_compress_v_tiles(desc, V, idx, k, Vt)
    tsa.tsa_attend_fused(desc, Q, K, Vt, idx, inv, k, O=O2, Oc=Oc2, residual=x2, **kw)
    # the whole layer
    O3 = torch.full_like(O1, 9.0)
    idx3 = torch.empty_like(idx)
    tsa.tsa_forward(desc, Q, K, V, k, O3, ws, idx_out=idx3, residual=x3, **kw)
    torch.cuda.synchronize()
    assert torch.equal(x2, x1) and torch.equal(x3, x1) and not torch.equal(x1, x0)
    assert torch.equal(idx3, idx)
    assert torch.equal(Oc2, Oc)
    assert torch.equal(O2, O1) and torch.equal(O3, O1)


@pytest.mark.parametrize("Hq,Hk,Lc,d,Bs", [(4, 2, 1000, 128, 128), (3, 3, 1500, 64, 128), (2, 1, 2600, 128, 128),
                                           (4, 2, 1100, 128, 64), (2, 2, 1900, 64, 256)])
def test_attend_per_head_block_lists(tsa, attend_form, Hq, Hk, Lc, d, Bs):
    """Block-sparse composition with a different pattern for every head (vertical + slash), in blocks
    of 64, 128 and 256 tokens."""
    from paper_2602_03216_amd import inputs as gen
    r = _rng(1500 + Lc)
    B = 2
    Qb, Kb, Vb = gu.rand_bits(r, (B, Hq, Lc, d)), gu.rand_bits(r, (B, Hk, Lc, d)), gu.rand_bits(r, (B, Hk, Lc, d))
    bl = gen.vertical_slash_block_lists(B, Hq, (Lc + Bs - 1) // Bs, seed=Lc)
    desc = tsa.make_desc(B, Hq, Hk, Lc, d, 1, block_list_per_head=1)
    O = torch.empty((B, Hq, Lc, d), dtype=torch.bfloat16, device=gu.DEV)
    tsa.tsa_attend(desc, gu.to_dev(Qb), gu.to_dev(Kb), gu.to_dev(Vb), Lc, Hk, O, tsa.alloc_attend_workspace(desc, Lc, Hk, gu.DEV),
                   block_list=torch.from_numpy(bl).to(gu.DEV), block_size=Bs, max_blocks_per_row=bl.shape[-1])
    want = orc.attend(orc.bf16_to_f64(Qb), orc.bf16_to_f64(Kb), orc.bf16_to_f64(Vb), block_list=bl, block_size=Bs)
    gu.assert_output_close(gu.from_dev(O), orc.f64_to_bf16(want), "attend(per-head block lists)")


@pytest.mark.parametrize("Bs", [128, 64, 256])
def test_forward_with_per_head_block_lists(tsa, attend_form, Bs):
    """Token selection first, then a per-head block-sparse pattern in compacted space: the whole layer
    against the oracle's."""
    from paper_2602_03216_amd import inputs as gen
    from tests.margin import enforce_margin
    Hq, Hkv, L, d, Lq, k = 4, 2, 2000, 128, 64, 900
    cfg = dict(id=91, name="small", B=1, Hq=Hq, Hkv=Hkv, L=L, d=d, last_q=Lq, plant="direction", n_plant=20, norm_factor=3.0,
               frac_plant=0.1, boost=4.0, sink_boost=6.0, n_sink=4, zipf_a=1.2)
    inp = gen.make_inputs(cfg, seed=1234)
    enforce_margin(inp, [k], 0)
    bl = gen.vertical_slash_block_lists(1, Hq, (k + Bs - 1) // Bs, seed=9)
    desc = tsa.make_desc(1, Hq, Hkv, L, d, Lq, block_list_per_head=1)
    O = torch.full((1, Hq, L, d), 3.0, dtype=torch.bfloat16, device=gu.DEV)
    idx = torch.zeros((1, Hq, k), dtype=torch.int32, device=gu.DEV)
    tsa.tsa_forward(desc, gu.to_dev(inp.Q), gu.to_dev(inp.K), gu.to_dev(inp.V), k, O, _ws(tsa, desc, k), idx_out=idx,
                    block_list=torch.from_numpy(bl).to(gu.DEV), block_size=Bs, max_blocks_per_row=bl.shape[-1])
    torch.cuda.synchronize()
    ref = orc.forward(inp.Q, inp.K, inp.V, k, Lq, block_list=bl, block_size=Bs)
    assert np.array_equal(idx.cpu().numpy(), ref["idx"])
    gu.assert_output_close(gu.from_dev(O), ref["O"], "forward(per-head block lists)")


def test_random_small_shapes_sweep(tsa, attend_form):
    """Thirty seeded random small problems (odd lengths around the 64-key and 256-row tile edges,
    odd head counts, both head dimensions, batch > 1): attention against the oracle, and the whole
    layer against the separate calls (bit for bit) on index sets the library selected itself."""
    r = _rng(31337)
    for case in range(30):
        d = int(r.choice([64, 128]))
        Hkv = int(r.integers(1, 4))
        g = int(r.integers(1, 4))
        Hq = Hkv * g
        B = int(r.integers(1, 3))
        L = int(r.choice([1, 2, 31, 63, 64, 65, 127, 129, 255, 256, 257, 300, 511, 513, 640, 777]))
        Lq = int(min(L, r.choice([1, 7, 32, 64, 100])))
        k = int(r.integers(1, L + 1))
        group_mode = int(r.integers(0, 2))
        Qb, Kb, Vb = gu.rand_bits(r, (B, Hq, L, d)), gu.rand_bits(r, (B, Hkv, L, d)), gu.rand_bits(r, (B, Hkv, L, d))
        tag = "case %d: B=%d Hq=%d Hkv=%d L=%d d=%d Lq=%d k=%d mode=%d" % (case, B, Hq, Hkv, L, d, Lq, k, group_mode)
        desc = tsa.make_desc(B, Hq, Hkv, L, d, Lq, group_mode=group_mode)
        Q, K, V = gu.to_dev(Qb), gu.to_dev(Kb), gu.to_dev(Vb)
        # dense causal attention of the full sequence against the oracle
        O = torch.empty((B, Hq, L, d), dtype=torch.bfloat16, device=gu.DEV)
        tsa.tsa_attend(desc, Q, K, V, L, Hkv, O, tsa.alloc_attend_workspace(desc, L, Hkv, gu.DEV))
        want = orc.attend(orc.bf16_to_f64(Qb), orc.bf16_to_f64(Kb), orc.bf16_to_f64(Vb))
        gu.assert_output_close(gu.from_dev(O), orc.f64_to_bf16(want), tag)
        # the layer: fused against separate calls
        Hs = Hkv if group_mode else Hq
        ws = _ws(tsa, desc, k)
        s = torch.empty((B, Hq, L), dtype=torch.float32, device=gu.DEV)
        idx = torch.empty((B, Hs, k), dtype=torch.int32, device=gu.DEV)
        inv = torch.empty((B, Hs, L), dtype=torch.int32, device=gu.DEV)
        Qc = torch.empty((B, Hq, k, d), dtype=torch.bfloat16, device=gu.DEV)
        Kc = torch.empty((B, Hs, k, d), dtype=torch.bfloat16, device=gu.DEV)
        Vc, Oc = torch.empty_like(Kc), torch.empty_like(Qc)
        O1 = torch.full((B, Hq, L, d), 5.0, dtype=torch.bfloat16, device=gu.DEV)
        O2 = torch.full_like(O1, 7.0)
        tsa.tsa_score(desc, Q, K, s, ws)
        tsa.tsa_select(desc, s, k, idx, inv, ws)
        tsa.tsa_compress(desc, Q, K, V, idx, k, Qc, Kc, Vc)
        tsa.tsa_attend(desc, Qc, Kc, Vc, k, Hs, Oc, tsa.alloc_attend_workspace(desc, k, Hs, gu.DEV))
        tsa.tsa_decompress(desc, Oc, idx, inv, k, O=O1)
        idx2 = torch.empty_like(idx)
        tsa.tsa_forward(desc, Q, K, V, k, O2, ws, idx_out=idx2)
        torch.cuda.synchronize()
        assert torch.equal(idx2, idx) and torch.equal(O2, O1), tag
        # the selection is a valid top-k of the library's own scores: ascending, k distinct tokens,
        # nothing left out scores higher than anything kept
        sel = orc.group_scores(s.cpu().numpy().astype(np.float64), Hq // Hkv) if group_mode else s.cpu().numpy()
        got = idx.cpu().numpy()
        for b in range(B):
            for h in range(Hs):
                row = got[b, h]
                assert np.all(np.diff(row) > 0) and row[0] >= 0 and row[-1] < L, tag
                kept = np.zeros(L, dtype=bool)
                kept[row] = True
                if k < L:
                    assert sel[b, h][kept].min() >= sel[b, h][~kept].max(), tag
