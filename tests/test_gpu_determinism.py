"""Run-twice determinism and guard bands, entry point by entry point, through the C ABI.

Every output and every workspace sits between two 4 KiB guard bands inside one allocation.  Each
entry point runs twice on the same inputs: the first time its outputs and workspace are pre-filled
with one garbage byte, the second time with another.  The two results must be equal bit for bit
(nothing depends on what the buffers held before, on the order in which workgroups or atomics
arrive, or on a previous call), and every guard band must still hold its pattern (nothing is
written outside the stated shapes)."""
import numpy as np
import pytest
import torch

from oracle import tsa_oracle as orc
from paper_2602_03216_amd import inputs as gen
from tests import gpu_util as gu

pytestmark = pytest.mark.gpu

BAND = 4096
CANARY = 0xA5


@pytest.fixture(scope="module")
def tsa():
    from paper_2602_03216_amd import binding
    binding.load_library(build_if_missing=False)
    return binding


class Guarded:
    """`nbytes` of device memory between two guard bands; the payload starts 256-byte aligned."""

    def __init__(self, nbytes, fill):
        self.nbytes = int(nbytes)
        pad = (-self.nbytes) % 256
        self.raw = torch.full((BAND + self.nbytes + pad + BAND,), CANARY, dtype=torch.uint8, device=gu.DEV)
        self.raw[BAND:BAND + self.nbytes] = fill
        assert self.raw.data_ptr() % 256 == 0

    def bytes(self):
        return self.raw[BAND:BAND + self.nbytes]

    def view(self, dtype, shape):
        return self.bytes().view(dtype).view(shape)

    def intact(self):
        return bool((self.raw[:BAND] == CANARY).all().item()) and bool((self.raw[BAND + self.nbytes:] == CANARY).all().item())


def _twice(run):
    """run(fill) -> (dict of output tensors, list of Guarded); returns the outputs of the first run
    after checking them against the second."""
    first = None
    for fill in (0x3C, 0xD7):
        outs, guards = run(fill)
        torch.cuda.synchronize()
        for i, g in enumerate(guards):
            assert g.intact(), "guard band %d damaged (fill %#x)" % (i, fill)
        if first is None:
            first = {k: v.clone() for k, v in outs.items()}
        else:
            for k, v in outs.items():
                assert torch.equal(first[k].view(torch.uint8), v.view(torch.uint8)), "%s differs between two runs" % k
    return first


def _elt(dtype):
    return torch.empty((), dtype=dtype).element_size()


def _out(shape, dtype, fill):
    g = Guarded(int(np.prod(shape)) * _elt(dtype), fill)
    return g, g.view(dtype, shape)


def _ws(nbytes, fill):
    g = Guarded(max(256, nbytes), fill)
    return g, g.bytes()


CASES = [
    # B, Hq, Hkv, L, d, Lq, k, group_mode, pool_w
    (2, 4, 2, 3000, 128, 64, 700, 0, 1),
    (1, 6, 2, 20011, 128, 64, 5000, 1, 3),      # rows longer than 16384: the sliced selection kernels; pooled scores
    (3, 2, 2, 777, 64, 17, 777, 0, 1),
]


@pytest.mark.parametrize("B,Hq,Hkv,L,d,Lq,k,group_mode,pool_w", CASES)
def test_every_entry_point_twice_with_guard_bands(tsa, B, Hq, Hkv, L, d, Lq, k, group_mode, pool_w):
    r = np.random.Generator(np.random.PCG64(8800 + L))
    Q, K, V = (gu.to_dev(gu.rand_bits(r, (B, h, L, d))) for h in (Hq, Hkv, Hkv))
    desc = tsa.make_desc(B, Hq, Hkv, L, d, Lq, group_mode=group_mode, pool_w=pool_w)
    Hs = Hkv if group_mode else Hq
    ws_bytes = tsa.tsa_workspace_bytes(desc, k)

    def run_score(fill):
        gs, s = _out((B, Hq, L), torch.float32, fill)
        gw, ws = _ws(ws_bytes, fill)
        tsa.tsa_score(desc, Q, K, s, ws)
        return {"scores": s}, [gs, gw]
    s = _twice(run_score)["scores"]

    def run_budget(fill):
        gk, kk = _out((B,), torch.int32, fill)
        gw, ws = _ws(ws_bytes, fill)
        tsa.tsa_coverage_budget(desc, s, 0.02, kk, ws)
        return {"k_keep": kk}, [gk, gw]
    _twice(run_budget)

    def run_select(fill):
        gi, idx = _out((B, Hs, k), torch.int32, fill)
        gv, inv = _out((B, Hs, L), torch.int32, fill)
        gw, ws = _ws(ws_bytes, fill)
        tsa.tsa_select(desc, s, k, idx, inv, ws)
        return {"idx": idx, "inv": inv}, [gi, gv, gw]
    sel = _twice(run_select)
    idx, inv = sel["idx"], sel["inv"]

    def run_compress(fill):
        gq, Qc = _out((B, Hq, k, d), torch.bfloat16, fill)
        gk, Kc = _out((B, Hs, k, d), torch.bfloat16, fill)
        gv, Vc = _out((B, Hs, k, d), torch.bfloat16, fill)
        tsa.tsa_compress(desc, Q, K, V, idx, k, Qc, Kc, Vc)
        return {"Qc": Qc, "Kc": Kc, "Vc": Vc}, [gq, gk, gv]
    c = _twice(run_compress)

    def run_attend(fill):
        go, Oc = _out((B, Hq, k, d), torch.bfloat16, fill)
        gl, lse = _out((B, Hq, k), torch.float32, fill)
        gw, ws = _ws(tsa.tsa_attend_workspace_bytes(desc, k, Hs), fill)
        tsa.tsa_attend(desc, c["Qc"], c["Kc"], c["Vc"], k, Hs, Oc, ws, lse)
        return {"Oc": Oc, "lse": lse}, [go, gl, gw]
    Oc = _twice(run_attend)["Oc"]

    def run_decompress(fill):
        go, O = _out((B, Hq, L, d), torch.bfloat16, fill)
        tsa.tsa_decompress(desc, Oc, idx, inv, k, O=O)
        go2, O2 = _out((B, Hq, L, d), torch.bfloat16, fill)
        tsa.tsa_decompress(desc, Oc, None, inv, k, O=O2)
        return {"O": O, "O_inv_only": O2}, [go, go2]
    O_sep = _twice(run_decompress)["O"]

    x0 = gu.to_dev(gu.rand_bits(r, (B, L, Hq * d)))

    def run_residual(fill):
        gx, x = _out((B, L, Hq * d), torch.bfloat16, fill)
        x.copy_(x0)
        tsa.tsa_decompress(desc, Oc, idx, inv, k, residual=x)
        return {"x": x}, [gx]
    x_sep = _twice(run_residual)["x"]

    def run_fused(fill):
        gt, Vt = _ws(tsa.tsa_attend_workspace_bytes(desc, k, Hs), fill)
        go, O = _out((B, Hq, L, d), torch.bfloat16, fill)
        gc, Oc2 = _out((B, Hq, k, d), torch.bfloat16, fill)
        gx, x = _out((B, L, Hq * d), torch.bfloat16, fill)
        x.copy_(x0)
        tsa.tsa_compress_v_tiles(desc, V, idx, k, Vt)
        tsa.tsa_attend_fused(desc, Q, K, Vt, idx, inv, k, O=O, Oc=Oc2, residual=x)
        return {"O": O, "Oc": Oc2, "x": x}, [gt, go, gc, gx]
    f = _twice(run_fused)
    assert torch.equal(f["O"], O_sep) and torch.equal(f["Oc"], Oc) and torch.equal(f["x"], x_sep)

    def run_forward(fill):
        go, O = _out((B, Hq, L, d), torch.bfloat16, fill)
        gi, idx2 = _out((B, Hs, k), torch.int32, fill)
        gw, ws = _ws(ws_bytes, fill)
        tsa.tsa_forward(desc, Q, K, V, k, O, ws, idx_out=idx2)
        return {"O": O, "idx": idx2}, [go, gi, gw]
    fw = _twice(run_forward)
    assert torch.equal(fw["O"], O_sep) and torch.equal(fw["idx"], idx)

    def run_dynamic(fill):
        go, O = _out((B, Hq, L, d), torch.bfloat16, fill)
        gk, kk = _out((B,), torch.int32, fill)
        gi, idx2 = _out((B, Hs, L), torch.int32, fill)
        gw, ws = _ws(tsa.load_library().tsa_forward_dynamic_workspace_bytes(desc, L), fill)
        tsa.tsa_forward_dynamic(desc, Q, K, V, 0.02, L, O, ws, k_keep_out=kk, idx_out=idx2)
        torch.cuda.synchronize()
        # rows of idx_out past a batch entry's count are unspecified: compare the counted part only
        counted = torch.zeros_like(idx2)
        for b in range(B):
            n = int(kk[b].item())
            counted[b, :, :n] = idx2[b, :, :n]
        return {"O": O, "k_keep": kk, "idx": counted}, [go, gk, gi, gw]
    _twice(run_dynamic)


def test_ablation_scorers_and_drift_twice_with_guard_bands(tsa):
    r = np.random.Generator(np.random.PCG64(8899))
    B, Hq, Hkv, L, d, n = 2, 4, 2, 2500, 128, 40
    Q, K = gu.to_dev(gu.rand_bits(r, (B, Hq, L, d))), gu.to_dev(gu.rand_bits(r, (B, Hkv, L, d)))
    desc = tsa.make_desc(B, Hq, Hkv, L, d, 64)
    qpos = np.sort(r.choice(L, n, replace=False)).tolist()

    def run_gather(fill):
        gq, Qsel = _out((B, Hq, n, d), torch.bfloat16, fill)
        tsa.tsa_gather_queries(desc, Q, qpos, Qsel)
        return {"Qsel": Qsel}, [gq]
    Qsel = _twice(run_gather)["Qsel"]

    def run_score_queries(fill):
        gs, s = _out((B, Hq, L), torch.float32, fill)
        gw, ws = _ws(tsa.tsa_score_queries_workspace_bytes(desc, n), fill)
        tsa.tsa_score_queries(desc, Qsel, qpos, K, s, ws)
        return {"scores": s}, [gs, gw]
    s = _twice(run_score_queries)["scores"]
    want = orc.score_queries(orc.bf16_to_f64(gu.from_dev(Qsel)), qpos, orc.bf16_to_f64(gu.from_dev(K)))
    gu.assert_scores_close(s.cpu().numpy(), want, "general scorer, n != last_q")

    def run_pool_queries(fill):
        gq, Qp = _out((B, Hq, 5, d), torch.bfloat16, fill)
        gw, ws = _ws(tsa.load_library().tsa_pool_queries_workspace_bytes(desc, 5), fill)
        tsa.tsa_pool_queries(desc, Q, 5, Qp, ws)
        return {"Qpool": Qp}, [gq, gw]
    _twice(run_pool_queries)

    n_tok, width = 5000, 1024
    h_in = gu.to_dev(gu.rand_bits(r, (n_tok, width)))
    h_out = gu.to_dev(gu.rand_bits(r, (n_tok, width)))

    def run_drift(fill):
        gd, dr = _out((1,), torch.float32, fill)
        gw, ws = _ws(tsa.load_library().tsa_layer_drift_workspace_bytes(n_tok), fill)
        tsa.tsa_layer_drift(h_in, h_out, 1e-6, dr, ws)
        return {"drift": dr}, [gd, gw]
    _twice(run_drift)


def test_budget_is_bit_stable_on_scores_spanning_many_binades(tsa):
    """Scores from 2^-60 to 2^10 in one row, three batch entries, ten repetitions: the masses are integer
    sums, so the count cannot move from run to run, and it matches the oracle's bracket."""
    r = np.random.Generator(np.random.PCG64(99))
    B, Hq, L = 3, 8, 50021
    s_np = (2.0 ** r.uniform(-60, 10, size=(B, Hq, L))).astype(np.float32)
    desc = tsa.make_desc(B, Hq, Hq, L, 128, 64)
    s = torch.from_numpy(s_np).to(gu.DEV)
    ws = tsa.alloc_workspace(desc, 1, gu.DEV)
    for tau in (1e-6, 0.003, 0.4):
        seen = set()
        for rep in range(10):
            kk = torch.full((B,), -1, dtype=torch.int32, device=gu.DEV)
            tsa.tsa_coverage_budget(desc, s, tau, kk, ws)
            torch.cuda.synchronize()
            seen.add(tuple(kk.cpu().tolist()))
        assert len(seen) == 1, (tau, seen)
        got = np.array(next(iter(seen)))
        eps = 2.0 * Hq * 2.0 ** -24
        lo, hi = orc.coverage_budget(s_np, min(1.0, tau * (1 + eps))), orc.coverage_budget(s_np, tau * (1 - eps))
        assert np.all(lo <= got) and np.all(got <= hi), (tau, lo, got, hi)
