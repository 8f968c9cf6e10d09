"""Test helper: give the k-th / (k+1)-th score boundary a margin, so that the set of the
k largest scores is the same in any reasonable floating-point evaluation.

For every selection head and every k of the sweep, theta = sqrt(s_(k) * s_(k+1)).  Key
rows whose score lies within a relative band around some theta are replaced by fresh
draws from the input generator (same planting rule) that land on the SAME side of every
threshold of every head sharing that key row, and outside every band.  Keeping the side
keeps the number of tokens above each theta, so each theta ends up inside an empty gap.
The replacement is evaluated with the window's log-sum-exp held fixed; the next round
scores everything again with the oracle, and the loop ends when the oracle's own scores
show the margin."""
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


def enforce_margin(inp, ks, group_mode=0, rho=RHO, max_rounds=10, n_cand=64):
    """Returns (scores [B,Hq,L] float64 from the oracle, achieved margin).  Modifies inp.K."""
    cfg = inp.cfg
    Hq, Hkv, L, d, Lq = cfg["Hq"], cfg["Hkv"], cfg["L"], cfg["d"], cfg["last_q"]
    g = Hq // Hkv
    first = L - Lq
    scale = 1.0 / np.sqrt(d)
    ks = sorted(k for k in ks if k < L)
    Qw = orc.bf16_to_f64(inp.Q[0, :, first:, :])                       # [Hq,Lq,d]
    detect, accept = 1.5 * rho, 2.0 * rho
    Kf = orc.bf16_to_f64(inp.K)                                         # kept in step with inp.K below
    for rnd in range(max_rounds):
        s = orc.score(Qw[None], Kf, Lq)
        sel = orc.group_scores(s, g) if group_mode == 1 else s
        margin = boundary_margin(sel, ks)
        if L >= 32768:
            print("  margin round %d: %.3g (target %.3g)" % (rnd, margin, 2 * rho), flush=True)
        if not ks or margin >= 2 * rho:
            return s, margin
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
            side = np.stack([v[pos, None] > th[None, :] for v, th in zip(rows, thetas)])   # [n_rows, n_pos, n_k]
            todo = np.arange(pos.size)
            for attempt in range(40):
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
                sc = np.stack(sc)                                                         # [g, n, c]
                if group_mode == 1:
                    sc = sc.sum(axis=0, keepdims=True)
                ok = np.ones(sc.shape[1:], dtype=bool)
                for r in range(sc.shape[0]):
                    for ki, t in enumerate(thetas[r]):
                        ok &= (sc[r] > t) == side[r, todo, ki][:, None]
                        ok &= np.abs(sc[r] / t - 1.0) >= accept
                has = ok.any(axis=1)
                pick = ok.argmax(axis=1)
                done = np.nonzero(has)[0]
                if done.size:
                    gen.set_key_rows(inp, kv, pos[todo[done]], cand[done, pick[done]])
                    Kf[0, kv, pos[todo[done]]] = cf[done, pick[done]]
                todo = todo[~has]
    raise AssertionError("selection margin not reached after %d rounds" % max_rounds)
