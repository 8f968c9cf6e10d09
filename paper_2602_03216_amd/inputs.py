"""Seeded synthetic inputs for the Token Sparse Attention prefill path.

The paper measures on long prompts run through trained decoder models; neither
the prompts nor the weights are needed for the attention hot path, only the
layer shapes and the structure the paper describes for token importance
(Section 2.1: a few important tokens, head-specific sets, a long tail; sink
tokens at the start).  This module draws N(0,1) tensors, plants per-head
important tokens, and rounds to bf16.  It contains no part of the method: no
scoring, no selection, no attention.  Both the HIP tests and the CPU oracle
read the bit patterns produced here.

All tensors are returned as numpy uint16 arrays holding bf16 bit patterns.
"""
from __future__ import annotations

import math
import os
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, field
import numpy as np

_N_THREADS = max(1, min(16, os.cpu_count() or 1))

SEED_BASE = 260203216

# name -> shape and planting recipe.  tau lists are the sparsity sweep of each workload.
CONFIGS = {
    1: dict(name="tiny_mha", B=1, Hq=4, Hkv=4, L=1024, d=64, last_q=64, taus=(0.75,),
            plant="norm", n_plant=64, norm_factor=3.0),
    2: dict(name="mha_8k", B=1, Hq=32, Hkv=32, L=8192, d=128, last_q=64, taus=(0.5, 0.75),
            plant="direction", frac_plant=0.10, boost=4.0),
    3: dict(name="gqa_32k", B=1, Hq=32, Hkv=8, L=32768, d=128, last_q=64, taus=(0.0, 0.5, 0.75, 0.9),
            plant="zipf_sink", frac_plant=0.05, boost=4.0, sink_boost=6.0, n_sink=4, zipf_a=1.2),
    4: dict(name="gqa_128k", B=1, Hq=32, Hkv=8, L=131072, d=128, last_q=64, taus=(0.75, 0.9),
            plant="zipf_sink", frac_plant=0.05, boost=4.0, sink_boost=6.0, n_sink=4, zipf_a=1.2),
    5: dict(name="stack_64k", B=1, Hq=28, Hkv=4, L=65536, d=128, last_q=64, taus=(0.75,),
            plant="zipf_sink", frac_plant=0.05, boost=4.0, sink_boost=6.0, n_sink=4, zipf_a=1.2,
            layers=4, overlap=0.30, block_size=128, window=4096),
}


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 -> bf16 bit patterns, round to nearest even (finite inputs)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(u16: np.ndarray) -> np.ndarray:
    return (np.asarray(u16, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


@dataclass
class Inputs:
    cfg: dict
    seed: int
    Q: np.ndarray            # [B,Hq,L,d] uint16 (bf16 bits)
    K: np.ndarray            # [B,Hkv,L,d]
    V: np.ndarray            # [B,Hkv,L,d]
    planted: list            # per query head: sorted int64 array of planted positions
    # what is needed to draw a key row again under the same planting rule
    directions: np.ndarray | None = None      # [Hq,d] float32 unit vectors (direction recipes)
    key_coef: np.ndarray | None = None        # [Hq,L] float32 coefficient of directions[h] added to key t
    redraws: int = 0
    extra: dict = field(default_factory=dict)


def _normal_f32(seed: int, tensor_id: int, shape) -> np.ndarray:
    """N(0,1) in float32.  Every (tensor, head) slice has its own PCG64 stream seeded from
    (seed, tensor_id, head index), so slices can be drawn by a few threads in parallel and the
    result does not depend on the number of threads."""
    out = np.empty(shape, dtype=np.float32)
    flat = out.reshape(-1, shape[-2], shape[-1])

    def fill(i):
        rng = np.random.Generator(np.random.PCG64([seed, tensor_id, i]))
        rng.standard_normal(flat.shape[1:], dtype=np.float32, out=flat[i])

    with ThreadPoolExecutor(max_workers=_N_THREADS) as pool:
        list(pool.map(fill, range(flat.shape[0])))
    return out


def _to_bf16_parallel(x: np.ndarray) -> np.ndarray:
    out = np.empty(x.shape, dtype=np.uint16)
    xf, of = x.reshape(-1, x.shape[-2], x.shape[-1]), out.reshape(-1, x.shape[-2], x.shape[-1])

    def conv(i):
        of[i] = f32_to_bf16_bits(xf[i])

    with ThreadPoolExecutor(max_workers=_N_THREADS) as pool:
        list(pool.map(conv, range(xf.shape[0])))
    return out


def _zipf_positions(rng, n, lo, hi, a):
    """n distinct positions lo + Zipf(a) - 1, truncated to < hi, in draw order."""
    got = []
    seen = set()
    for _ in range(64):
        draw = rng.zipf(a, size=4 * n).astype(np.int64) - 1 + lo
        for p in draw[draw < hi]:
            p = int(p)
            if p not in seen:
                seen.add(p)
                got.append(p)
                if len(got) == n:
                    return np.array(sorted(got), dtype=np.int64)
    return np.array(sorted(got), dtype=np.int64)


def make_inputs(cfg_id: int | dict, seed: int | None = None, layer: int = 0,
                prev_planted: list | None = None, L: int | None = None) -> Inputs:
    """Build the tensors of one workload.  `L` overrides the sequence length
    (used by tests that want the same recipe at a reduced or ragged length)."""
    cfg = dict(CONFIGS[cfg_id]) if not isinstance(cfg_id, dict) else dict(cfg_id)
    cid = cfg_id if not isinstance(cfg_id, dict) else cfg.get("id", 0)
    if L is not None:
        cfg["L"] = int(L)
    if seed is None:
        seed = SEED_BASE + 1000 * int(cid) + layer
    rng = np.random.Generator(np.random.PCG64(seed))
    B, Hq, Hkv, Ln, d = cfg["B"], cfg["Hq"], cfg["Hkv"], cfg["L"], cfg["d"]
    g = Hq // Hkv
    Lq = min(cfg["last_q"], Ln)
    cfg["last_q"] = Lq
    assert B == 1, "the recipes below are written for B = 1 (every workload of the paper's setup)"

    Q = _normal_f32(seed, 1, (B, Hq, Ln, d))
    K = _normal_f32(seed, 2, (B, Hkv, Ln, d))
    V = _normal_f32(seed, 3, (B, Hkv, Ln, d))
    planted: list = []
    directions = None
    key_coef = None
    hi = max(1, Ln - Lq)                    # planted tokens lie before the scoring window

    if cfg["plant"] == "norm":
        # key norm x factor at n_plant positions per head, positions differ per head
        n = min(cfg["n_plant"], hi)
        for h in range(Hq):
            pos = np.sort(rng.choice(hi, size=n, replace=False)).astype(np.int64)
            planted.append(pos)
            K[0, h // g, pos, :] *= np.float32(cfg["norm_factor"])
    else:
        # every query of head h gets + c u_h; planted keys get + c u_h (a logit boost of
        # c^2 / sqrt(d) = boost nats); sink keys get the larger sink_boost from every head of the group
        u = rng.standard_normal((Hq, d)).astype(np.float32)
        u /= np.linalg.norm(u, axis=1, keepdims=True)
        directions = u
        c = math.sqrt(cfg["boost"] * math.sqrt(d))
        key_coef = np.zeros((Hq, Ln), dtype=np.float32)
        n_sink = min(cfg.get("n_sink", 0), hi)
        n = max(1, int(math.floor(cfg["frac_plant"] * Ln)))
        n = min(n, max(1, hi - n_sink))
        for h in range(Hq):
            if cfg["plant"] == "direction":
                pos = np.sort(rng.choice(hi, size=n, replace=False)).astype(np.int64)
            else:
                if prev_planted is not None:
                    keep_n = int(round(cfg.get("overlap", 0.0) * n))
                    kept = rng.choice(prev_planted[h], size=min(keep_n, len(prev_planted[h])), replace=False)
                    fresh = _zipf_positions(rng, n, n_sink, hi, cfg["zipf_a"])
                    fresh = fresh[~np.isin(fresh, kept)][: n - len(kept)]
                    pos = np.unique(np.concatenate([kept, fresh])).astype(np.int64)
                else:
                    pos = _zipf_positions(rng, n, n_sink, hi, cfg["zipf_a"])
            planted.append(pos)
            key_coef[h, pos] = c
            if n_sink:
                key_coef[h, :n_sink] = cfg["sink_boost"] * math.sqrt(d) / c
            Q[0, h] += c * u[h]
        for kv in range(Hkv):
            for h in range(kv * g, (kv + 1) * g):
                nzp = np.nonzero(key_coef[h])[0]
                K[0, kv, nzp, :] += key_coef[h, nzp, None] * u[h][None, :]

    out = Inputs(cfg=cfg, seed=seed, Q=_to_bf16_parallel(Q), K=_to_bf16_parallel(K), V=_to_bf16_parallel(V),
                 planted=planted, directions=directions, key_coef=key_coef)
    if cfg["plant"] == "norm":
        out.extra["norm_factor"] = cfg["norm_factor"]
    return out


def candidate_key_rows(inp: Inputs, kv_head: int, positions: np.ndarray, n_cand: int) -> np.ndarray:
    """Fresh candidate key rows for `positions` of KV head `kv_head`: N(0,1) draws under
    the same planting rule as the original rows, rounded to bf16.  Returns bf16 bits
    [len(positions), n_cand, d].  Tests that need the k-th and (k+1)-th scores separated
    by a margin pick a replacement for each ambiguous row among these candidates and
    write it back with set_key_rows.  The stream is seeded from (seed, call counter), so a
    sequence of calls is reproducible."""
    positions = np.asarray(positions, dtype=np.int64)
    cfg = inp.cfg
    d = cfg["d"]
    g = cfg["Hq"] // cfg["Hkv"]
    inp.redraws += 1
    rng = np.random.Generator(np.random.PCG64([inp.seed, 7919, inp.redraws, kv_head]))
    rows = rng.standard_normal((positions.size, n_cand, d), dtype=np.float32)
    if cfg["plant"] == "norm":
        for h in range(kv_head * g, (kv_head + 1) * g):
            hit = np.isin(positions, inp.planted[h])
            rows[hit] *= np.float32(inp.extra["norm_factor"])
    else:
        for h in range(kv_head * g, (kv_head + 1) * g):
            rows += inp.key_coef[h, positions, None, None] * inp.directions[h][None, None, :]
    return f32_to_bf16_bits(rows)


def set_key_rows(inp: Inputs, kv_head: int, positions: np.ndarray, rows_bits: np.ndarray) -> None:
    """Overwrite key rows (bf16 bits [len(positions), d]) in place."""
    inp.K[0, kv_head, np.asarray(positions, dtype=np.int64), :] = rows_bits


def make_residual(cfg: dict, seed: int) -> np.ndarray:
    """Residual stream x [B, L, Hq*d] ~ N(0,1), bf16 bits (stack workload)."""
    rng = np.random.Generator(np.random.PCG64([seed, 104729]))
    x = rng.standard_normal((cfg["B"], cfg["L"], cfg["Hq"] * cfg["d"]), dtype=np.float32)
    return f32_to_bf16_bits(x)


def sink_window_block_list(Lc: int, block_size: int, window: int, n_sink_blocks: int = 1) -> np.ndarray:
    """Block list of the stack workload's mask in compacted index space (sink + sliding window):
    query block qb lists the first n_sink_blocks key blocks and the blocks qb - window/block_size .. qb.
    Returns [ceil(Lc / block_size), n_sink_blocks + window/block_size + 1] int32, rows ascending
    without duplicates, padded with -1."""
    nb = (Lc + block_size - 1) // block_size
    wb = window // block_size
    width = min(nb, n_sink_blocks + wb + 1)
    out = np.full((nb, width), -1, dtype=np.int32)
    for qb in range(nb):
        first = max(0, qb - wb)
        row = list(range(min(n_sink_blocks, first))) + list(range(first, qb + 1))
        out[qb, :len(row)] = row
    return out


def vertical_slash_block_lists(B: int, Hq: int, n_blocks: int, seed: int, n_vertical: int = 3, slash_blocks: int = 2,
                               n_extra: int = 2) -> np.ndarray:
    """Per-head block lists of the "vertical + slash" kind block-sparse prefill methods produce, in
    compacted index space: for head (b, h) query block qb may see (a) the first key block, (b) the
    head's own n_vertical seeded "vertical" key blocks (columns every later query sees), (c) the
    slash: the diagonal block and the slash_blocks blocks before it, (d) n_extra seeded blocks of its
    own below the diagonal.  Returns [B, Hq, n_blocks, width] int32, every row ascending, without
    duplicates, entries <= qb, padded with -1.  A stand-in for the patterns of the block-sparse
    methods the paper composes with (their pattern search is not part of this library)."""
    rng = np.random.Generator(np.random.PCG64([seed, 77]))
    width = 1 + n_vertical + slash_blocks + 1 + n_extra
    out = np.full((B, Hq, n_blocks, width), -1, dtype=np.int32)
    for b in range(B):
        for h in range(Hq):
            vertical = rng.integers(0, n_blocks, size=n_vertical)
            for qb in range(n_blocks):
                s = {0, qb}
                s.update(int(v) for v in vertical if v <= qb)
                s.update(range(max(0, qb - slash_blocks), qb + 1))
                if qb > 0:
                    s.update(int(v) for v in rng.integers(0, qb, size=n_extra))
                row = sorted(s)
                out[b, h, qb, :len(row)] = row
    return out
