"""Test helper: give the k-th / (k+1)-th score boundary a margin, so that the set of the
k largest scores is the same in any reasonable floating-point evaluation.

For every selection head and every k of the sweep, theta = sqrt(s_(k) * s_(k+1)).  Key
rows whose score lies within a relative band around some theta are replaced by fresh
draws from the input generator (same planting rule) that land on the SAME side of every
threshold of every head sharing that key row, and outside every band.  Keeping the side
keeps the number of tokens above each theta, so each theta ends up inside an empty gap.
The replacement is evaluated with the window's log-sum-exp held fixed; the next round
scores everything again with the oracle, and the loop ends when the oracle's own scores
show the margin.

With pooled scores (pool_w > 1) the selection score of token t is the mean of the raw scores of
t - w/2 .. t + w/2, so a new key row at position p moves the selection scores of all those
neighbours by (new - old) / w: a candidate is accepted when every one of them stays on its side
of every threshold and outside every band; the position to replace is chosen inside the band
token's window so that as few other band tokens as possible move with it."""
import numpy as np
import scipy.special

from oracle import tsa_oracle as orc
from paper_2602_03216_amd import inputs as gen

RHO = 2.0 ** -10        # guaranteed: s_(k) / s_(k+1) - 1 >= 2 * RHO


def _window_logits(Qw, Kh, scale, first):
    """x[i,t] = scale q_i.k_t for window rows i = first.., masked to t <= i."""
    L = Kh.shape[0]
    x = scale * (Qw @ Kh.T)
    vis = np.arange(L)[None, :] <= (first + np.arange(Qw.shape[0]))[:, None]
    return np.where(vis, x, -np.inf)


def boundary_margin(sel_scores, ks):
    worst = np.inf
    L = sel_scores.shape[-1]
    for row in sel_scores.reshape(-1, L):
        srt = np.sort(row)[::-1]
        for k in ks:
            if k < L:
                worst = min(worst, srt[k - 1] / srt[k] - 1.0)
    return worst


def enforce_margin(inp, ks, group_mode=0, rho=RHO, max_rounds=10, n_cand=64, pool_w=1):
    """Returns (selection-ready scores [B,Hq,L] float64 from the oracle (pooled if pool_w > 1),
    achieved margin).  Modifies inp.K."""
    cfg = inp.cfg
    Hq, Hkv, L, d, Lq = cfg["Hq"], cfg["Hkv"], cfg["L"], cfg["d"], cfg["last_q"]
    g = Hq // Hkv
    first = L - Lq
    scale = 1.0 / np.sqrt(d)
    ks = sorted(k for k in ks if k < L)
    Qw = orc.bf16_to_f64(inp.Q[0, :, first:, :])                       # [Hq,Lq,d]
    detect, accept = 1.5 * rho, 2.0 * rho
    Kf = orc.bf16_to_f64(inp.K)                                         # kept in step with inp.K below
    rad = pool_w // 2
    if pool_w > 1:
        max_rounds = 4 * max_rounds
    for rnd in range(max_rounds):
        s_raw = orc.score(Qw[None], Kf, Lq)
        s = orc.pool(s_raw, pool_w)
        sel = orc.group_scores(s, g) if group_mode == 1 else s
        margin = boundary_margin(sel, ks)
        if L >= 32768:
            print("  margin round %d: %.3g (target %.3g)" % (rnd, margin, 2 * rho), flush=True)
        if not ks or margin >= 2 * rho:
            return s, margin
        replaced = 0
        for kv in range(Hkv):
            heads = list(range(kv * g, (kv + 1) * g))
            Kh = Kf[0, kv]
            lse = np.stack([scipy.special.logsumexp(_window_logits(Qw[h], Kh, scale, first), axis=1) for h in heads])
            # selection rows that read this KV head, their thresholds
            rows = [sel[0, kv]] if group_mode == 1 else [sel[0, h] for h in heads]
            thetas = []
            for v in rows:
                srt = np.sort(v)[::-1]
                thetas.append(np.array([np.sqrt(srt[k - 1] * srt[k]) for k in ks]))
            thetas = np.stack(thetas)                                   # [n_rows, n_k]
            band = np.zeros(L, dtype=bool)
            for v, th in zip(rows, thetas):
                for t in th:
                    band |= np.abs(v / t - 1.0) < detect
            pos = np.nonzero(band)[0]
            if pos.size == 0:
                continue
            if pool_w > 1:
                # Neighbouring tokens share most of their pooling window and often sit in the band together,
                # on opposite sides of a threshold; a row that both windows contain moves them alike.  For
                # every band token pick the position inside its window whose own reach [p - w/2, p + w/2]
                # holds the fewest band tokens (ties: the one nearest the token), and keep the positions
                # replaced in one round at least pool_w apart so that their reaches do not overlap.
                chosen = []
                for t in pos:
                    best, best_key = None, None
                    for u in range(-rad, rad + 1):
                        q = t + u
                        if q < 0 or q >= L or any(abs(q - c) < pool_w for c in chosen):
                            continue
                        key = (int(band[max(0, q - rad):q + rad + 1].sum()), abs(u))
                        if best_key is None or key < best_key:
                            best, best_key = q, key
                    if best is not None:
                        chosen.append(best)
                pos = np.array(sorted(chosen), dtype=np.int64)
                if pos.size == 0:
                    continue
            raw_old = np.stack([s_raw[0, h, pos] for h in heads])                          # [g, n_pos]
            todo = np.arange(pos.size)
            for attempt in range(40 if pool_w == 1 else 8):
                if todo.size == 0:
                    break
                nc = max(n_cand, min(4096, 16384 // todo.size))
                cand = gen.candidate_key_rows(inp, kv, pos[todo], nc)                     # [n, c, d] bits
                cf = orc.bf16_to_f64(cand)
                # score of each candidate under each head, window log-sum-exp held fixed
                vis = (first + np.arange(Lq))[None, :] >= pos[todo][:, None]             # [n, Lq]
                sc = []
                for j, h in enumerate(heads):
                    x = scale * (cf @ Qw[h].T) - lse[j][None, None, :]                  # [n, c, Lq]
                    sc.append((np.exp(x) * vis[:, None, :]).sum(axis=2))
                # change of the selection score of every position the new row reaches: [rows, n, c]
                dlt = (np.stack(sc) - raw_old[:, todo, None]) / pool_w
                if group_mode == 1:
                    dlt = dlt.sum(axis=0, keepdims=True)
                ok = np.ones(dlt.shape[1:], dtype=bool)
                for u in range(-rad, rad + 1):
                    tpos = pos[todo] + u
                    inside = (tpos >= 0) & (tpos < L)
                    tcl = np.clip(tpos, 0, L - 1)
                    for r in range(dlt.shape[0]):
                        cur = rows[r][tcl]                                                # [n]
                        new = cur[:, None] + dlt[r]                                       # [n, c]
                        for t in thetas[r]:
                            good = ((new > t) == (cur > t)[:, None]) & (np.abs(new / t - 1.0) >= accept)
                            ok &= good | ~inside[:, None]
                has = ok.any(axis=1)
                pick = ok.argmax(axis=1)
                done = np.nonzero(has)[0]
                if done.size:
                    gen.set_key_rows(inp, kv, pos[todo[done]], cand[done, pick[done]])
                    Kf[0, kv, pos[todo[done]]] = cf[done, pick[done]]
                    replaced += done.size
                todo = todo[~has]
        if replaced == 0 and pool_w > 1:
            raise AssertionError("selection margin: no admissible replacement in round %d" % rnd)
    raise AssertionError("selection margin not reached after %d rounds" % max_rounds)
