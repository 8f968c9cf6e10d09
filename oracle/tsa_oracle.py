"""CPU oracle for the Token Sparse Attention prefill path (test infrastructure).

This module is TEST INFRASTRUCTURE.  It is the slow, plain definition that the
HIP library is checked against.  Only the tests, the smoke check and the
benchmark's cpu_baseline leg may import it; the product path never does, and
this module imports nothing from the product package.

Everything is numpy float64 on the exact values of the bf16 inputs.  Each
function follows one passage of the paper:

  score       Algorithm 1, its first two steps: proxy attention of the most recent
              queries, then the per-head column sums (Section 2.3, Dynamic Token Coverage)
  pool        the pooling(.) of the same step (the paper does not give the
              kernel; reading: average pooling, stride 1, zero padding)
  coverage_budget  Algorithm 1, its budget steps: cross-head sum and normalisation, ascending
              order, cumulative-mass threshold tau -> k_sparse, k_keep (the dynamic budget)
  keep_count  the fixed token-sparsity ratio the paper compares its dynamic budget
              with (Table 4): a constant fraction of tokens kept
  select      Algorithm 1, its last step: per-head top-k_keep selection
  compress    Section 2.2, Stage 1 (gather rows of Q, K, V by S_h)
  attend      Section 2.2, Stage 1 last sentence: attention on the compressed
              tensors; causal, as for the decoder-only models of Section 3.1
  decompress  Section 2.2, Stage 2 (scatter into a zero-initialised tensor)
  residual_add  Section 2.2, Stage 2 last paragraph (restored output is added
              to the residual stream)
  layer_drift, sparse_layers  Section 2.4: Eq. 1 (inter-layer representation drift) and Eq. 2
              (normalised drift rank, layer set)
  forward     the five steps in the order of Figure 3

Readings taken where the paper is silent (all repeated in the design notes):
  * the scoring window is causal (query i sees keys t <= i);
  * scores are not pooled by default (pool width 1);
  * top-k ties go to the lowest token index, and S_h is emitted in ascending
    token order, so "causal" in the compacted index is causal in the original
    positions and the result is the hard mask the paper describes;
  * with grouped KV heads, each query head selects its own set (mode 0) or the
    heads of a KV group share one set chosen from their summed scores (mode 1).

Parity pins: every function here is pinned by tests/test_oracle_pins.py
(closed forms, hand-worked cases, brute force, library routines).
"""
from __future__ import annotations

import math
import numpy as np

# ----------------------------------------------------------------------------
# bf16 <-> float64 (bit patterns are carried as uint16)
# ----------------------------------------------------------------------------

def bf16_to_f64(u16: np.ndarray) -> np.ndarray:
    """Exact widening of bf16 bit patterns (uint16) to float64."""
    u = np.asarray(u16, dtype=np.uint16)
    return (u.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


def f64_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round float64 to bf16 bit patterns, round-to-nearest-even, done directly
    on the float64 value (no intermediate float32 rounding).  Finite inputs."""
    x = np.asarray(x, dtype=np.float64)
    out = np.zeros(x.shape, dtype=np.uint16)
    ax = np.abs(x)
    nz = ax > 0
    # exponent e with 2^e <= |x| < 2^(e+1); bf16 normal numbers keep 8 significant bits
    m, e = np.frexp(ax[nz])            # ax = m * 2^e, m in [0.5, 1)
    e = e - 1                          # now ax = (2m) * 2^e, 2m in [1, 2)
    e_cl = np.maximum(e, -126)         # subnormals share the exponent of the smallest normal
    ulp = np.ldexp(1.0, e_cl - 7)
    q = np.rint(ax[nz] / ulp)          # np.rint is round-half-to-even; exact since ulp is a power of two
    val = (q * ulp).astype(np.float32) # exactly representable (<= 8 significant bits)
    bits = (val.view(np.uint32) >> np.uint32(16)).astype(np.uint16)
    sign = (np.signbit(x[nz])).astype(np.uint16) << np.uint16(15)
    out[nz] = bits | sign
    out[~nz] = np.where(np.signbit(x[~nz]), np.uint16(0x8000), np.uint16(0))
    return out


# ----------------------------------------------------------------------------
# Algorithm 1: scoring
# ----------------------------------------------------------------------------

def score(Q: np.ndarray, K: np.ndarray, last_q: int, scale: float | None = None) -> np.ndarray:
    """s[b,h,t] = sum over the last `last_q` queries i of softmax_t(scale q_i.k_t)
    with the causal restriction t <= i.  Q [B,Hq,L,d], K [B,Hkv,L,d] float64.
    Only Q[..., -last_q:, :] is read, so a caller may pass just those rows; their
    positions are L - last_q .. L - 1 with L taken from K.
    Query head h reads KV head h // (Hq // Hkv).  Returns [B,Hq,L] float64."""
    K = np.asarray(K, dtype=np.float64)
    B, Hkv, L, d = K.shape
    assert 1 <= last_q <= L and Q.shape[2] >= last_q
    Q = np.asarray(Q[:, :, Q.shape[2] - last_q:, :], dtype=np.float64)
    Hq = Q.shape[1]
    assert Hq % Hkv == 0 and Q.shape == (B, Hq, last_q, d)
    g = Hq // Hkv
    if scale is None:
        scale = 1.0 / math.sqrt(d)
    s = np.zeros((B, Hq, L), dtype=np.float64)
    first = L - last_q
    pos_t = np.arange(L)
    pos_i = np.arange(first, L)
    visible = pos_t[None, :] <= pos_i[:, None]          # [last_q, L]
    for b in range(B):
        for h in range(Hq):
            x = scale * (Q[b, h] @ K[b, h // g].T)               # [last_q, L]
            x = np.where(visible, x, -np.inf)
            m = x.max(axis=1, keepdims=True)
            e = np.exp(x - m)                                     # exp(-inf) = 0 on masked entries
            p = e / e.sum(axis=1, keepdims=True)                  # rows of A-hat
            s[b, h] = p.sum(axis=0)                               # vertical sum
    return s


def score_queries(Qsel: np.ndarray, qpos, K: np.ndarray, scale: float | None = None) -> np.ndarray:
    """Token scores from an arbitrary set of scoring queries (the scoring ablation of the paper's
    appendix: randomly sampled queries, or a pooled query, in place of the most recent ones):
    s[b,h,t] = sum_j softmax_t(scale Qsel[b,h,j].k_t), query j seeing keys t <= qpos[j].
    Qsel [B,Hq,n,d], qpos [n] ints in [0, L), K [B,Hkv,L,d]; float64.  Returns [B,Hq,L]."""
    K = np.asarray(K, dtype=np.float64)
    Qsel = np.asarray(Qsel, dtype=np.float64)
    qpos = np.asarray(qpos, dtype=np.int64)
    B, Hkv, L, d = K.shape
    Hq, n = Qsel.shape[1], Qsel.shape[2]
    assert Qsel.shape == (B, Hq, n, d) and qpos.shape == (n,) and Hq % Hkv == 0
    assert qpos.min() >= 0 and qpos.max() < L
    g = Hq // Hkv
    if scale is None:
        scale = 1.0 / math.sqrt(d)
    visible = np.arange(L)[None, :] <= qpos[:, None]      # [n, L]
    s = np.zeros((B, Hq, L), dtype=np.float64)
    for b in range(B):
        for h in range(Hq):
            x = np.where(visible, scale * (Qsel[b, h] @ K[b, h // g].T), -np.inf)
            e = np.exp(x - x.max(axis=1, keepdims=True))
            s[b, h] = (e / e.sum(axis=1, keepdims=True)).sum(axis=0)
    return s


def pool_queries(Q_bits: np.ndarray, n_pool: int):
    """Query-only pooling of the scoring ablation: the L query rows of every head are cut into
    n_pool contiguous segments, segment j = rows floor(j L / n_pool) .. ceil((j+1) L / n_pool) - 1
    (the segments of adaptive average pooling), and averaged.  Q_bits [B,Hq,L,d] bf16 bit patterns.
    Returns (pooled rows as bf16 bits [B,Hq,n_pool,d], qpos [n_pool] = last row of each segment:
    a pooled query sees the keys its last member sees)."""
    B, Hq, L, d = Q_bits.shape
    assert 1 <= n_pool <= L
    Q = bf16_to_f64(Q_bits)
    out = np.zeros((B, Hq, n_pool, d), dtype=np.float64)
    qpos = np.zeros(n_pool, dtype=np.int64)
    for j in range(n_pool):
        lo = (j * L) // n_pool
        hi = -((-(j + 1) * L) // n_pool)
        out[:, :, j] = Q[:, :, lo:hi].sum(axis=2) / (hi - lo)
        qpos[j] = hi - 1
    return f64_to_bf16(out), qpos


def pool(s: np.ndarray, pool_w: int) -> np.ndarray:
    """Average pooling of width `pool_w` (odd), stride 1, zero padded, along t."""
    if pool_w == 1:
        return np.array(s, dtype=np.float64, copy=True)
    assert pool_w % 2 == 1 and pool_w >= 1
    r = pool_w // 2
    L = s.shape[-1]
    pad = np.zeros(s.shape[:-1] + (L + 2 * r,), dtype=np.float64)
    pad[..., r:r + L] = s
    out = np.zeros_like(s, dtype=np.float64)
    for u in range(pool_w):
        out += pad[..., u:u + L]
    return out / pool_w


def group_scores(s: np.ndarray, g: int) -> np.ndarray:
    """Mode-1 selection score: sum of the scores of the g query heads that share
    a KV head (the same across-head sum Algorithm 1 uses for s_l).  [B,Hq,L] -> [B,Hq/g,L]."""
    B, Hq, L = s.shape
    return s.reshape(B, Hq // g, g, L).sum(axis=2)


def keep_count(L: int, tau: float) -> int:
    """Fixed-ratio budget: drop floor(tau*L) tokens, keep the rest, at least one."""
    k_sparse = int(math.floor(float(tau) * L))
    return max(1, min(L, L - k_sparse))


def coverage_budget(s: np.ndarray, tau_cov: float) -> np.ndarray:
    """Dynamic Token Coverage budget, the budget steps of Algorithm 1 (Section 2.3): the scores
    are summed over the heads and normalised to total mass one, s_l = sum_h s_h / sum_t sum_h s_h[t];
    the tokens are put in ascending order of s_l; k_sparse is the smallest k in {0..L} whose k least
    important tokens carry a cumulative mass >= tau_cov; k_keep = L - k_sparse (at least 1).
    s [B,Hq,L]; one k_keep per batch element, int32 [B].  Everything in float64."""
    s = np.asarray(s, dtype=np.float64)
    B, Hq, L = s.shape
    out = np.empty(B, dtype=np.int32)
    for b in range(B):
        sl = s[b].sum(axis=0)
        sl = sl / sl.sum()
        order = np.argsort(sl, kind="stable")
        cum = np.cumsum(sl[order])
        if tau_cov <= 0.0:
            k_sparse = 0
        else:
            reached = np.nonzero(cum >= tau_cov)[0]
            k_sparse = int(reached[0]) + 1 if reached.size else L
        out[b] = max(1, L - k_sparse)
    return out


# ----------------------------------------------------------------------------
# Algorithm 1: top-k selection
# ----------------------------------------------------------------------------

def select(s: np.ndarray, k_keep: int, force_first: int = 0, force_last: int = 0):
    """For every leading index, the k_keep tokens of largest score; ties go to the
    lowest token index; the set is returned in ascending token order.
    Tokens t < force_first or t >= L - force_last count as score +inf.
    Returns (idx [..,k] int32, inv [..,L] int32 with inv[idx[r]] = r, else -1)."""
    s = np.asarray(s)
    L = s.shape[-1]
    assert 1 <= k_keep <= L
    flat = s.reshape(-1, L)
    idx = np.empty((flat.shape[0], k_keep), dtype=np.int32)
    inv = np.full((flat.shape[0], L), -1, dtype=np.int32)
    t = np.arange(L)
    for r in range(flat.shape[0]):
        v = flat[r].astype(np.float64, copy=True)
        if force_first > 0:
            v[:force_first] = np.inf
        if force_last > 0:
            v[L - force_last:] = np.inf
        # lexicographic order on (-score, token): np.lexsort sorts by the LAST key first
        order = np.lexsort((t, -v))
        chosen = np.sort(order[:k_keep])
        idx[r] = chosen
        inv[r, chosen] = np.arange(k_keep, dtype=np.int32)
    return idx.reshape(s.shape[:-1] + (k_keep,)), inv.reshape(s.shape)


# ----------------------------------------------------------------------------
# Stage 1: compression
# ----------------------------------------------------------------------------

def compress(Q, K, V, idx, group_mode: int = 0):
    """Row gather.  Q [B,Hq,L,d]; K,V [B,Hkv,L,d]; idx [B,Hs,k] with Hs = Hq
    (mode 0) or Hkv (mode 1).  Mode 0 returns Qc,Kc,Vc all [B,Hq,k,d] (the KV rows
    of head h // g gathered once per query head).  Mode 1 returns Qc [B,Hq,k,d]
    and Kc,Vc [B,Hkv,k,d].  Works on any dtype (bit patterns are copied)."""
    B, Hq, L, d = Q.shape
    Hkv = K.shape[1]
    g = Hq // Hkv
    k = idx.shape[-1]
    Qc = np.empty((B, Hq, k, d), dtype=Q.dtype)
    if group_mode == 0:
        assert idx.shape == (B, Hq, k)
        Kc = np.empty((B, Hq, k, d), dtype=K.dtype)
        Vc = np.empty((B, Hq, k, d), dtype=V.dtype)
        for b in range(B):
            for h in range(Hq):
                Qc[b, h] = Q[b, h, idx[b, h]]
                Kc[b, h] = K[b, h // g, idx[b, h]]
                Vc[b, h] = V[b, h // g, idx[b, h]]
    else:
        assert idx.shape == (B, Hkv, k)
        Kc = np.empty((B, Hkv, k, d), dtype=K.dtype)
        Vc = np.empty((B, Hkv, k, d), dtype=V.dtype)
        for b in range(B):
            for kv in range(Hkv):
                Kc[b, kv] = K[b, kv, idx[b, kv]]
                Vc[b, kv] = V[b, kv, idx[b, kv]]
            for h in range(Hq):
                Qc[b, h] = Q[b, h, idx[b, h // g]]
    return Qc, Kc, Vc


# ----------------------------------------------------------------------------
# Attention in the compressed space
# ----------------------------------------------------------------------------

def lambda_block_list(Lc: int, block_size: int, window: int, n_sink_blocks: int = 1) -> np.ndarray:
    """Block list of a sink + sliding-window ("Lambda") mask in compacted index
    space: query block qb visits key block kb iff kb <= qb and (kb < n_sink_blocks
    or qb - kb <= window / block_size).  Returns [nQb, max_blocks] int32, each row
    ascending and padded with -1."""
    nb = (Lc + block_size - 1) // block_size
    wb = window // block_size
    rows = []
    for qb in range(nb):
        rows.append([kb for kb in range(qb + 1) if kb < n_sink_blocks or qb - kb <= wb])
    width = max(len(r) for r in rows)
    out = np.full((nb, width), -1, dtype=np.int32)
    for qb, r in enumerate(rows):
        out[qb, :len(r)] = r
    return out


def attend(Qc, Kc, Vc, scale: float | None = None, block_list=None, block_size: int = 0,
           rows=None, return_lse: bool = False):
    """Causal softmax attention over compacted tensors, float64.
    Qc [B,Hq,Lc,d]; Kc,Vc [B,Hk,Lc,d] with Hq % Hk == 0 (head h reads h // (Hq/Hk)).
    Row r attends to columns c <= r; with a block list, additionally only to
    columns whose block c // block_size is listed for block r // block_size.
    block_list is [nQb, width] (one pattern for all heads) or [B, Hq, nQb, width]
    (one per head), rows padded with -1.
    `rows`: optional 1-D array of row numbers; then only those rows are computed
    and the result has shape [B,Hq,len(rows),d].  Returns float64 (not rounded)."""
    Qc = np.asarray(Qc, dtype=np.float64)
    Kc = np.asarray(Kc, dtype=np.float64)
    Vc = np.asarray(Vc, dtype=np.float64)
    B, Hq, Lc, d = Qc.shape
    Hk = Kc.shape[1]
    g = Hq // Hk
    if scale is None:
        scale = 1.0 / math.sqrt(d)
    rsel = np.arange(Lc) if rows is None else np.asarray(rows, dtype=np.int64)
    cols = np.arange(Lc)
    causal = cols[None, :] <= rsel[:, None]

    def block_mask(table):
        nb = (Lc + block_size - 1) // block_size
        blk_ok = np.zeros((table.shape[0], nb), dtype=bool)
        for qb in range(table.shape[0]):
            for kb in table[qb]:
                if kb >= 0:
                    blk_ok[qb, kb] = True
        return blk_ok[rsel // block_size][:, cols // block_size]

    bl = None if block_list is None else np.asarray(block_list)
    shared = causal if bl is None else (causal & block_mask(bl) if bl.ndim == 2 else None)
    out = np.zeros((B, Hq, len(rsel), d), dtype=np.float64)
    lse = np.zeros((B, Hq, len(rsel)), dtype=np.float64)
    for b in range(B):
        for h in range(Hq):
            allowed = shared if shared is not None else causal & block_mask(bl[b, h])
            y = scale * (Qc[b, h, rsel] @ Kc[b, h // g].T)
            y = np.where(allowed, y, -np.inf)
            m = y.max(axis=1, keepdims=True)
            e = np.exp(y - m)
            z = e.sum(axis=1, keepdims=True)
            out[b, h] = (e / z) @ Vc[b, h // g]
            lse[b, h] = (m + np.log(z))[:, 0]
    if return_lse:
        return out, lse
    return out


# ----------------------------------------------------------------------------
# Stage 2: decompression, residual
# ----------------------------------------------------------------------------

def decompress(Oc: np.ndarray, idx: np.ndarray, L: int) -> np.ndarray:
    """O[b,h,idx[b,hs,r],:] = Oc[b,h,r,:], every other row zero.  Any dtype."""
    B, Hq, k, d = Oc.shape
    Hs = idx.shape[1]
    g = Hq // Hs
    O = np.zeros((B, Hq, L, d), dtype=Oc.dtype)
    for b in range(B):
        for h in range(Hq):
            O[b, h, idx[b, h // g]] = Oc[b, h]
    return O


def residual_add(x_bits: np.ndarray, Oc_bits: np.ndarray, idx: np.ndarray) -> np.ndarray:
    """Residual stream update with the identity standing in for the output
    projection: x[b, t, h*d:(h+1)*d] += Oc[b,h,r,:] for t = idx[b,hs,r]; the sum is
    taken on the exact values and rounded once to bf16.  x [B,L,Hq*d] bf16 bits."""
    B, Hq, k, d = Oc_bits.shape
    Hs = idx.shape[1]
    g = Hq // Hs
    out = np.array(x_bits, dtype=np.uint16, copy=True)
    for b in range(B):
        for h in range(Hq):
            rows = idx[b, h // g]
            cur = bf16_to_f64(out[b, rows, h * d:(h + 1) * d])
            out[b, rows, h * d:(h + 1) * d] = f64_to_bf16(cur + bf16_to_f64(Oc_bits[b, h]))
    return out


# ----------------------------------------------------------------------------
# Sparse layer selection (Section 2.4)
# ----------------------------------------------------------------------------

def layer_drift(h_in: np.ndarray, h_out: np.ndarray, eps: float) -> float:
    """Eq. 1, Inter-Layer Representation Drift: mean over tokens of
    ||h_out[t] - h_in[t]||_2 / (||h_in[t]||_2 + eps).  h_in, h_out [n_tokens, width] float64."""
    h_in = np.asarray(h_in, dtype=np.float64)
    h_out = np.asarray(h_out, dtype=np.float64)
    num = np.sqrt(((h_out - h_in) ** 2).sum(axis=1))
    den = np.sqrt((h_in ** 2).sum(axis=1)) + eps
    return float((num / den).mean())


def sparse_layers(drift, delta: float = 0.5):
    """Eq. 2: normalised drift rank R^_l = (1/N) #{k : R_k <= R_l}; the layer set {l : R^_l <= delta}.
    Returns (rank list, list of 0/1 flags)."""
    n = len(drift)
    rank = [sum(1 for k in range(n) if drift[k] <= drift[l]) / n for l in range(n)]
    return rank, [1 if r <= delta else 0 for r in rank]


# ----------------------------------------------------------------------------
# Whole layer
# ----------------------------------------------------------------------------

def forward(Q_bits, K_bits, V_bits, k_keep: int, last_q: int, scale: float | None = None,
            pool_w: int = 1, group_mode: int = 0, force_first: int = 0, force_last: int = 0,
            block_list=None, block_size: int = 0):
    """score -> pool -> select -> compress -> attend -> decompress on bf16 bit
    patterns (uint16).  Returns dict with scores, idx, inv, Oc (bf16 bits),
    Oc_exact (float64) and O (bf16 bits, [B,Hq,L,d])."""
    B, Hq, L, d = Q_bits.shape
    K = bf16_to_f64(K_bits)
    g = Hq // K.shape[1]
    s = pool(score(bf16_to_f64(Q_bits[:, :, L - last_q:, :]), K, last_q, scale), pool_w)
    s_sel = group_scores(s, g) if group_mode == 1 else s
    idx, inv = select(s_sel, k_keep, force_first, force_last)
    Qc, Kc, Vc = compress(Q_bits, K_bits, V_bits, idx, group_mode)
    Oc_exact = attend(bf16_to_f64(Qc), bf16_to_f64(Kc), bf16_to_f64(Vc), scale, block_list, block_size)
    Oc = f64_to_bf16(Oc_exact)
    O = decompress(Oc, idx, L)
    return {"scores": s, "sel_scores": s_sel, "idx": idx, "inv": inv,
            "Oc": Oc, "Oc_exact": Oc_exact, "O": O}
