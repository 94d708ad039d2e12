"""A literal loop-nest evaluator of the policy forward, for tiny shapes only.

Written separately from the oracle (scalar Python floats, explicit indices, math.fsum)
so that the two can be compared as independent implementations.  Not collected by pytest.
"""
import math


def _rms(vec, gain, eps):
    ms = math.fsum(t * t for t in vec) / len(vec)
    r = math.sqrt(ms + eps)
    return [t / r * g for t, g in zip(vec, gain)]


def _matvec(W, vec):
    return [math.fsum(W[o][i] * vec[i] for i in range(len(vec))) for o in range(len(W))]


def _rot(vec, p, n_heads, hd, theta):
    out = list(vec)
    for h in range(n_heads):
        for i in range(hd // 2):
            ang = p * theta ** (-2.0 * i / hd)
            lo, hi = h * hd + i, h * hd + i + hd // 2
            out[lo] = vec[lo] * math.cos(ang) - vec[hi] * math.sin(ang)
            out[hi] = vec[hi] * math.cos(ang) + vec[lo] * math.sin(ang)
    return out


def forward_logits(cfg, Wt, rows):
    """cfg: dict(L,d,H,hd,f,V,A,theta,eps); Wt: name -> nested lists; rows: list of d-vectors.
    Returns the A action logits at the last position (whole sequence recomputed)."""
    L, d, H, hd = cfg["L"], cfg["d"], cfg["H"], cfg["hd"]
    S = len(rows)
    x = [list(r) for r in rows]
    for l in range(L):
        pre = f"layers.{l}."
        qs, ks, vs = [], [], []
        for p in range(S):
            h = _rms(x[p], Wt[pre + "attn_norm"], cfg["eps"])
            qs.append(_rot(_matvec(Wt[pre + "wq"], h), p, H, hd, cfg["theta"]))
            ks.append(_rot(_matvec(Wt[pre + "wk"], h), p, H, hd, cfg["theta"]))
            vs.append(_matvec(Wt[pre + "wv"], h))
        for p in range(S):
            o = [0.0] * d
            for hh in range(H):
                sl = range(hh * hd, (hh + 1) * hd)
                sc = [math.fsum(qs[p][j] * ks[t][j] for j in sl) / math.sqrt(hd) for t in range(p + 1)]
                m = max(sc)
                e = [math.exp(c - m) for c in sc]
                tot = math.fsum(e)
                for j in sl:
                    o[j] = math.fsum(e[t] / tot * vs[t][j] for t in range(p + 1))
            proj = _matvec(Wt[pre + "wo"], o)
            x[p] = [a + b for a, b in zip(x[p], proj)]
        for p in range(S):
            h = _rms(x[p], Wt[pre + "ffn_norm"], cfg["eps"])
            g = _matvec(Wt[pre + "w_gate"], h)
            u = _matvec(Wt[pre + "w_up"], h)
            act = [gi / (1.0 + math.exp(-gi)) * ui for gi, ui in zip(g, u)]
            dn = _matvec(Wt[pre + "w_down"], act)
            x[p] = [a + b for a, b in zip(x[p], dn)]
    h = _rms(x[S - 1], Wt["final_norm"], cfg["eps"])
    head = Wt["lm_head"][cfg["V"] - cfg["A"]:]
    return _matvec(head, h)


def greedy_rollout(cfg, Wt, rows, n_tokens):
    """Greedy autoregressive decode by full recompute; returns (tokens, logps)."""
    rows = [list(r) for r in rows]
    toks, lps = [], []
    for _ in range(n_tokens):
        z = forward_logits(cfg, Wt, rows)
        m = max(z)
        lse = m + math.log(math.fsum(math.exp(c - m) for c in z))
        t = z.index(m)
        toks.append(t)
        lps.append(z[t] - lse)
        rows.append(list(Wt["embed"][cfg["V"] - cfg["A"] + t]))
    return toks, lps
