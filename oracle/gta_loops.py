"""Brute-force evaluation of GTA in pure Python loops (tiny inputs only).

TEST INFRASTRUCTURE ONLY; it pins oracle/gta_oracle.py and shares no code with it or with the
HIP path.  It evaluates the UN-reformulated per-head equation of Sec. 3.3,

    O_i[t] = sum_{j<=t} Softmax_j(Q_{q(i)}[t] . K_{k(i)}[j] / sqrt(d_h)) * V_i^{(t)}[j],
    V_i^{(t)}[j] = (C_{c(i)}[j] W_{P,i}) * Sigmoid(x_t W_{G,i})          (Sec. 3.2 decoder),

with nothing shared between the heads of a group, Python floats only, and explicit index
arithmetic for the group maps and for RoPE (App. B.1.1, rotate-half pairing), so that a wrong
index, sign or transposed operand in the vectorised oracle shows up as a mismatch.
"""
from __future__ import annotations

import math


def _dot_col(x_row, W, col):
    """sum_h x_row[h] * W[h][col] for a row-major matrix W[H][n]."""
    s = 0.0
    for h in range(len(x_row)):
        s += x_row[h] * W[h][col]
    return s


def _rope_vec(v, pos, base):
    d = len(v)
    half = d // 2
    out = [0.0] * d
    for j in range(half):
        ang = pos * base ** (-2.0 * j / d)
        c, s = math.cos(ang), math.sin(ang)
        out[j] = v[j] * c - v[j + half] * s
        out[j + half] = v[j + half] * c + v[j] * s
    return out


def _gate(kind, z):
    """Gate factor from the pre-activation: Sigmoid (Sec. 3.2), or Silu / ReLU^2 (ablation on the choice
    of nonlinearity), or 1 when the gate is switched off."""
    if kind is True or kind == "sigmoid":
        return 1.0 / (1.0 + math.exp(-z))
    if kind == "silu":
        return z / (1.0 + math.exp(-z))
    if kind == "relu2":
        return max(z, 0.0) ** 2
    if kind is False or kind == "off":
        return 1.0
    raise ValueError(kind)


def brute_force_sequence(x, wq, wk, wc, wg, wp, *, n_heads, n_qgroups, n_kgroups, n_cgroups,
                         head_dim, latent_dim, rope=False, rope_base=10000.0, gate=True,
                         wo=None):
    """x: T x H nested lists; weights as nested lists in the library's layouts
    (wq [H][n_q*d_h], wk [H][n_k*d_h], wc [H][n_c*d_l], wg [H][n_h*d_h], wp [n_h][d_l][d_h],
    wo [n_h*d_h][H] or None).  Returns T x (n_h*d_h) (or T x H with wo) nested lists."""
    T = len(x)
    dh, dl = head_dim, latent_dim
    heads_per_q = n_heads // n_qgroups
    q_per_k = n_qgroups // n_kgroups
    q_per_c = n_qgroups // n_cgroups
    out = [[0.0] * (n_heads * dh) for _ in range(T)]
    for i in range(n_heads):
        g = i // heads_per_q          # query / map group of head i
        kg = g // q_per_k             # key group
        cg = g // q_per_c             # latent-value group
        # per-token query, key, latent of the groups this head uses
        q = [[_dot_col(x[t], wq, g * dh + e) for e in range(dh)] for t in range(T)]
        k = [[_dot_col(x[t], wk, kg * dh + e) for e in range(dh)] for t in range(T)]
        c = [[_dot_col(x[t], wc, cg * dl + e) for e in range(dl)] for t in range(T)]
        if rope:
            q = [_rope_vec(q[t], t, rope_base) for t in range(T)]
            k = [_rope_vec(k[t], t, rope_base) for t in range(T)]
        # linear part of the decoder, C W_P, per key row
        cp = [[sum(c[j][a] * wp[i][a][e] for a in range(dl)) for e in range(dh)] for j in range(T)]
        for t in range(T):
            gt = [_gate(gate, _dot_col(x[t], wg, i * dh + e)) for e in range(dh)]
            s = [sum(q[t][e] * k[j][e] for e in range(dh)) / math.sqrt(dh) for j in range(t + 1)]
            m = max(s)
            p = [math.exp(v - m) for v in s]
            z = sum(p)
            for e in range(dh):
                acc = 0.0
                for j in range(t + 1):
                    acc += (p[j] / z) * (cp[j][e] * gt[e])      # V_i^{(t)}[j][e]
                out[t][i * dh + e] = acc
    if wo is not None:
        H = len(wo[0])
        out = [[sum(out[t][a] * wo[a][h] for a in range(n_heads * dh)) for h in range(H)]
               for t in range(T)]
    return out
