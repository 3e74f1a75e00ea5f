"""Brute-force float64 decoder forward with explicit scalar loops (tests only).

Written separately from `oracle/` straight from the architecture's definition,
one scalar index at a time, so that an indexing, sign or transposition mistake
in the oracle shows up as a disagreement.  Only usable on tiny shapes.
"""
import math

import numpy as np


def _norm(x, g, eps):
    ms = 0.0
    for v in x:
        ms += v * v
    ms /= len(x)
    return np.array([x[i] / math.sqrt(ms + eps) * g[i] for i in range(len(x))])


def _matvec(W, x):                      # W [out, in]: y_o = sum_i W[o, i] x_i
    return np.array([float(np.dot(W[o], x)) for o in range(W.shape[0])])


def _rot(vec, pos, theta):              # one head vector of width h
    h = len(vec)
    out = np.array(vec, dtype=np.float64)
    for i in range(h // 2):
        ang = pos * theta ** (-2.0 * i / h)
        a, b = vec[i], vec[i + h // 2]
        out[i] = a * math.cos(ang) - b * math.sin(ang)
        out[i + h // 2] = b * math.cos(ang) + a * math.sin(ang)
    return out


def last_logits(w, shape, tokens):
    """Logits after the last token of `tokens`, recomputing everything."""
    W = {k: (v.double().numpy() if k != "layers" else None) for k, v in w.items()}
    Hq, Hkv, h, d, F = shape.n_heads, shape.n_kv_heads, shape.head_dim, shape.d_model, shape.d_ffn
    n = len(tokens)
    xs = [W["tok_emb"][t].copy() for t in tokens]
    for lw_t in w["layers"]:
        lw = {k: v.double().numpy() for k, v in lw_t.items()}
        Wq = lw["wqkv"][: Hq * h]
        Wk = lw["wqkv"][Hq * h: (Hq + Hkv) * h]
        Wv = lw["wqkv"][(Hq + Hkv) * h:]
        qs, ks, vs = [], [], []
        for i in range(n):
            y = _norm(xs[i], lw["attn_norm"], shape.rms_eps)
            q, k, v = _matvec(Wq, y), _matvec(Wk, y), _matvec(Wv, y)
            qs.append([_rot(q[j * h:(j + 1) * h], i, shape.rope_theta) for j in range(Hq)])
            ks.append([_rot(k[j * h:(j + 1) * h], i, shape.rope_theta) for j in range(Hkv)])
            vs.append([v[j * h:(j + 1) * h] for j in range(Hkv)])
        new_xs = []
        for i in range(n):
            att = np.zeros(Hq * h)
            for j in range(Hq):
                g = j // (Hq // Hkv)
                sc = [float(np.dot(qs[i][j], ks[m][g])) / math.sqrt(h) for m in range(i + 1)]
                mx = max(sc)
                e = [math.exp(s - mx) for s in sc]
                z = sum(e)
                for m in range(i + 1):
                    att[j * h:(j + 1) * h] += (e[m] / z) * vs[m][g]
            x1 = xs[i] + _matvec(lw["wo"], att)
            y2 = _norm(x1, lw["ffn_norm"], shape.rms_eps)
            gate = _matvec(lw["w_gate_up"][:F], y2)
            up = _matvec(lw["w_gate_up"][F:], y2)
            act = np.array([gate[c] / (1.0 + math.exp(-gate[c])) * up[c] for c in range(F)])
            new_xs.append(x1 + _matvec(lw["w_down"], act))
        xs = new_xs
    return _matvec(W["lm_head"], _norm(xs[-1], W["final_norm"], shape.rms_eps))
