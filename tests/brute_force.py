"""A second, independently written evaluation of the decoder for tiny inputs.

It deliberately uses a different formulation from the oracle: scalar Python
loops for the norm and the projections, the rotary embedding as an explicit
hd x hd rotation matrix per position, grouped-query attention by physically
repeating each KV head, the causal constraint as an explicit (L+S) x (L+S)
additive 0 / -inf matrix, and softmax by explicit exp / sum loops.  It exists
only to pin the oracle; nothing else uses it.
"""
import math

import numpy as np


def rotation_matrix(pos: int, hd: int, theta: float) -> np.ndarray:
    R = np.zeros((hd, hd))
    half = hd // 2
    for i in range(half):
        ang = pos * theta ** (-(2.0 * i) / hd)
        c, s = math.cos(ang), math.sin(ang)
        R[i, i] = c
        R[i, i + half] = -s
        R[i + half, i] = s
        R[i + half, i + half] = c
    return R


def norm_row(x, g, eps):
    d = len(x)
    ss = 0.0
    for j in range(d):
        ss += x[j] * x[j]
    r = 1.0 / math.sqrt(ss / d + eps)
    return np.array([x[j] * r * g[j] for j in range(d)])


def matvec(W, h):
    out = np.zeros(W.shape[0])
    for o in range(W.shape[0]):
        acc = 0.0
        for j in range(W.shape[1]):
            acc += W[o, j] * h[j]
        out[o] = acc
    return out


def layer(x, L, lw, k_prefix, v_prefix, cfg):
    """x: [S, d] at positions L..L+S-1; k_prefix/v_prefix: [L, Hkv, hd]."""
    S, d = x.shape
    hd, Hq, Hkv = cfg.head_dim, cfg.n_q_heads, cfg.n_kv_heads
    G = Hq // Hkv
    n = L + S
    q = np.zeros((S, Hq, hd))
    k = np.zeros((S, Hkv, hd))
    v = np.zeros((S, Hkv, hd))
    for t in range(S):
        h = norm_row(x[t], lw["attn_norm"], cfg.rms_eps)
        R = rotation_matrix(L + t, hd, cfg.rope_theta)
        qt = matvec(lw["wq"], h).reshape(Hq, hd)
        kt = matvec(lw["wk"], h).reshape(Hkv, hd)
        vt = matvec(lw["wv"], h).reshape(Hkv, hd)
        for i in range(Hq):
            q[t, i] = R @ qt[i]
        for c in range(Hkv):
            k[t, c] = R @ kt[c]
            v[t, c] = vt[c]
    K = np.concatenate([k_prefix, k], axis=0)          # [n, Hkv, hd]
    V = np.concatenate([v_prefix, v], axis=0)
    K_rep = np.repeat(K, G, axis=1)                     # [n, Hq, hd]: head i <- kv head i // G
    V_rep = np.repeat(V, G, axis=1)
    mask = np.full((n, n), -np.inf)
    for r in range(n):
        for j in range(r + 1):
            mask[r, j] = 0.0
    attn = np.zeros((S, Hq * hd))
    for i in range(Hq):
        for t in range(S):
            scores = [float(q[t, i] @ K_rep[j, i]) / math.sqrt(hd) + mask[L + t, j] for j in range(n)]
            mx = max(scores)
            w = [math.exp(s - mx) if s != -np.inf else 0.0 for s in scores]
            tot = sum(w)
            o = np.zeros(hd)
            for j in range(n):
                o += (w[j] / tot) * V_rep[j, i]
            attn[t, i * hd:(i + 1) * hd] = o
    y = np.zeros_like(x)
    for t in range(S):
        y[t] = x[t] + matvec(lw["wo"], attn[t])
    out = np.zeros_like(x)
    for t in range(S):
        h2 = norm_row(y[t], lw["mlp_norm"], cfg.rms_eps)
        gte = matvec(lw["wg"], h2)
        up = matvec(lw["wu"], h2)
        act = np.array([gte[f] / (1.0 + math.exp(-gte[f])) * up[f] for f in range(len(gte))])
        out[t] = y[t] + matvec(lw["wd"], act)
    return out, k, v


def verdict(x_last, final_norm, lm_rows, eps):
    y = norm_row(x_last, final_norm, eps)
    z = [float(sum(lm_rows[v, j] * y[j] for j in range(len(y)))) for v in range(lm_rows.shape[0])]
    mx = max(z)
    e = [math.exp(a - mx) for a in z]
    p = [a / sum(e) for a in e]
    r = max(range(len(p)), key=lambda i: (p[i], -i))
    return np.array(z), np.array(p), r, p[r]
