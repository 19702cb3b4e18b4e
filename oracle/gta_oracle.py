"""fp64 CPU oracle of the GTA attention forward pass (arXiv 2506.17286).

TEST INFRASTRUCTURE ONLY.  This module is the slow, plain definition that the HIP library is
checked against.  Only the test-suite, the smoke check and the benchmark's `cpu_baseline` leg may
import it; the product path never does, and it shares no code with the HIP path.

What it computes (paper notation, row-vector convention x.W):

  Sec. 3.2, input projections   Q = X W_Q, K = X W_K, C = X W_C            [N, n_q d_h] ...
  App. B.1.1                    q, k <- RoPE(q), RoPE(k); the latent value is NOT rotated
  Sec. 3.3 / App. B.1.1         A_g = causal Softmax(Q_g K_{k(g)}^T / sqrt(d_h)), one map per
                                query group g, shared by every head i with q(i) = g
  Sec. 3.3 (reformulated form)  L_g = A_g C_{c(g)}
  Sec. 3.2, value decoder       O_i = (L_{q(i)} W_{P,i}) * Sigmoid(x_t W_{G,i}), gate of row t
  Sec. 3.3                      optional U = concat_i(O_i) W_O
  App. B.1.3                    caches hold post-RoPE keys and latent values, row p = position p

Everything is float64 numpy; a matmul is used as a step, the softmax is fully materialised, and
there is no tiling, online softmax, split-K or fusion.

Readings taken where the paper is silent or inconsistent (listed again in the design notes):
  * the gate belongs to the query/output row t (prefill: one gate per row; decode: new token);
  * sigmoid is applied (the appendix drops it, the main text, abstract and ablation keep it);
  * head i uses Q_{q(i)}: only n_q distinct maps exist;
  * causal mask includes the diagonal (App. B sums k = 1..t);
  * group maps are contiguous blocks: q(i) = i // (n_h/n_q), k(g) = g // (n_q/n_k),
    c(g) = g // (n_q/n_c);
  * RoPE is the rotate-half pairing (j, j + d_h/2), theta_j = base^(-2j/d_h), positions 0-based
    per sequence; decode position = number of tokens already cached;
  * decode appends the new token's k, c first and then attends over all rows incl. itself.

Pins (tests/test_oracle_*.py): a literal per-head evaluation of the un-reformulated Sec. 3.3
equation in pure Python loops (oracle/gta_loops.py), torch's CPU scaled_dot_product_attention for
the MHA and GQA degenerate settings, closed forms (zero W_K => running mean, zero W_G => gate 1/2,
T = 1), invariants (rows of a map sum to 1, causality, decode == last prefill row, softmax shift
invariance, RoPE offset invariance) and the cache/compute ratios the paper prints.
Whether the authors' released model code resolves the ambiguities above the same way is
"parity unpinned": no implementation accompanies the paper.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Optional, Sequence

import numpy as np

CACHE_FULL = -8  # status word written for a slot whose append would exceed max_seq


@dataclass(frozen=True)
class OracleConfig:
    d_model: int          # H
    n_heads: int          # n_h
    n_qgroups: int        # n_q
    n_kgroups: int        # n_k
    n_cgroups: int        # n_c
    head_dim: int         # d_h
    latent_dim: int       # d_l
    rope: bool = False
    rope_base: float = 10000.0
    # gate nonlinearity: True / "sigmoid" (Sec. 3.2), "silu", "relu2" (the other two of the ablation on
    # the choice of nonlinearity), False / "off" => factor 1 (degenerate-case tests only)
    gate: object = True
    softmax_scale: Optional[float] = None  # None => 1/sqrt(d_h)

    def check(self) -> None:
        assert self.n_heads % self.n_qgroups == 0
        assert self.n_qgroups % self.n_kgroups == 0
        assert self.n_qgroups % self.n_cgroups == 0
        assert self.latent_dim >= self.head_dim  # Sec. 3.2: d_l >= d_h
        if self.rope:
            assert self.head_dim % 2 == 0

    @property
    def scale(self) -> float:
        return self.softmax_scale if self.softmax_scale else 1.0 / np.sqrt(self.head_dim)

    # contiguous-block group maps
    def q_of_head(self, i: int) -> int:
        return i // (self.n_heads // self.n_qgroups)

    def k_of_group(self, g: int) -> int:
        return g // (self.n_qgroups // self.n_kgroups)

    def c_of_group(self, g: int) -> int:
        return g // (self.n_qgroups // self.n_cgroups)


@dataclass
class OracleWeights:
    wq: np.ndarray                 # [H, n_q*d_h]
    wk: np.ndarray                 # [H, n_k*d_h]
    wc: np.ndarray                 # [H, n_c*d_l]
    wg: np.ndarray                 # [H, n_h*d_h]   W_{G,i} = columns [i*d_h, (i+1)*d_h)
    wp: np.ndarray                 # [n_h, d_l, d_h]
    wo: Optional[np.ndarray] = None  # [n_h*d_h, H]

    def f64(self) -> "OracleWeights":
        c = lambda a: None if a is None else np.asarray(a, dtype=np.float64)
        return OracleWeights(c(self.wq), c(self.wk), c(self.wc), c(self.wg), c(self.wp), c(self.wo))


def sigmoid(z: np.ndarray) -> np.ndarray:
    """Sigmoid(z) = 1 / (1 + exp(-z)) (Sec. 3.2), evaluated without overflow for large |z|."""
    z = np.asarray(z, dtype=np.float64)
    e = np.exp(-np.abs(z))
    return np.where(z >= 0, 1.0 / (1.0 + e), e / (1.0 + e))


def gate_factor(kind, z: np.ndarray) -> np.ndarray:
    """The factor the decoded value is multiplied by, from the gate pre-activation z = x_t W_{G,i}:
    Sigmoid(z) in the method (Sec. 3.2); the ablation on the choice of nonlinearity also trains Silu,
    z * Sigmoid(z), and ReLU^2, max(z, 0)^2."""
    if kind is True or kind == "sigmoid":
        return sigmoid(z)
    if kind == "silu":
        return np.asarray(z, dtype=np.float64) * sigmoid(z)
    if kind == "relu2":
        return np.square(np.maximum(np.asarray(z, dtype=np.float64), 0.0))
    if kind is False or kind == "off":
        return np.ones_like(np.asarray(z, dtype=np.float64))
    raise ValueError(f"unknown gate {kind!r}")


def rope_rotate(v: np.ndarray, positions: np.ndarray, base: float) -> np.ndarray:
    """Rotate-half RoPE (App. B.1.1 applies RoPE to q and k).

    v: [T, n, d_h]; positions: [T] integers.  Pair (j, j + d_h/2) is rotated by the angle
    p * base^(-2j/d_h).
    """
    v = np.asarray(v, dtype=np.float64)
    T, n, d = v.shape
    half = d // 2
    j = np.arange(half, dtype=np.float64)
    theta = base ** (-2.0 * j / d)                                   # [half]
    ang = np.asarray(positions, dtype=np.float64)[:, None] * theta[None, :]  # [T, half]
    cos = np.cos(ang)[:, None, :]
    sin = np.sin(ang)[:, None, :]
    lo, hi = v[..., :half], v[..., half:]
    out = np.empty_like(v)
    out[..., :half] = lo * cos - hi * sin
    out[..., half:] = hi * cos + lo * sin
    return out


def project_tokens(cfg: OracleConfig, w: OracleWeights, x: np.ndarray, positions: np.ndarray):
    """Sec. 3.2 projections plus App. B.1.1 RoPE for a set of tokens with given positions.

    Returns Q [T, n_q, d_h], K [T, n_k, d_h] (both rotated if cfg.rope), C [T, n_c, d_l] and the
    gate pre-activation Gpre [T, n_h, d_h].
    """
    x = np.asarray(x, dtype=np.float64)
    T = x.shape[0]
    Q = (x @ w.wq).reshape(T, cfg.n_qgroups, cfg.head_dim)
    K = (x @ w.wk).reshape(T, cfg.n_kgroups, cfg.head_dim)
    C = (x @ w.wc).reshape(T, cfg.n_cgroups, cfg.latent_dim)
    G = (x @ w.wg).reshape(T, cfg.n_heads, cfg.head_dim)
    if cfg.rope:
        Q = rope_rotate(Q, positions, cfg.rope_base)
        K = rope_rotate(K, positions, cfg.rope_base)
    return Q, K, C, G


def attention_map_rows(cfg: OracleConfig, q_rows: np.ndarray, row_pos: np.ndarray,
                       keys: np.ndarray) -> np.ndarray:
    """Materialised causal softmax rows of one group (Sec. 3.3, App. B.1.1 sum over k <= t).

    q_rows [R, d_h] are the queries at sequence positions row_pos [R]; keys [N, d_h] are the
    keys at positions 0..N-1.  Entry (r, j) is zero for j > row_pos[r].
    """
    S = (q_rows @ keys.T) * cfg.scale                                  # [R, N]
    allowed = np.arange(keys.shape[0])[None, :] <= np.asarray(row_pos)[:, None]
    S = np.where(allowed, S, -np.inf)
    S = S - S.max(axis=1, keepdims=True)
    E = np.exp(S)
    return E / E.sum(axis=1, keepdims=True)


def decode_heads(cfg: OracleConfig, w: OracleWeights, L: np.ndarray, G: np.ndarray) -> np.ndarray:
    """Sec. 3.2 value decoder on the group outputs: O_i = (L_{q(i)} W_{P,i}) * Sigmoid(Gpre_i).

    L [R, n_q, d_l], G [R, n_h, d_h] -> [R, n_h*d_h] (heads concatenated in index order), then
    the optional output projection of Sec. 3.3.
    """
    R = L.shape[0]
    O = np.empty((R, cfg.n_heads, cfg.head_dim), dtype=np.float64)
    for i in range(cfg.n_heads):
        z = L[:, cfg.q_of_head(i), :] @ w.wp[i]
        O[:, i, :] = z * gate_factor(cfg.gate, G[:, i, :])
    O = O.reshape(R, cfg.n_heads * cfg.head_dim)
    if w.wo is not None:
        O = O @ w.wo
    return O


def prefill_sequence(cfg: OracleConfig, w: OracleWeights, x: np.ndarray,
                     rows: Optional[Sequence[int]] = None, return_maps: bool = False):
    """Causal prefill of ONE sequence x [T, H].

    Returns (out, K, C[, maps]): out [R, n_h*d_h] (or [R, H] with W_O) for the requested rows
    (all rows if rows is None), K [T, n_k*d_h] post-RoPE and C [T, n_c*d_l] as they are cached.
    """
    cfg.check()
    w = w.f64()
    x = np.asarray(x, dtype=np.float64)
    T = x.shape[0]
    pos = np.arange(T)
    Q, K, C, G = project_tokens(cfg, w, x, pos)
    r = pos if rows is None else np.asarray(list(rows), dtype=np.int64)
    L = np.empty((len(r), cfg.n_qgroups, cfg.latent_dim), dtype=np.float64)
    maps = []
    for g in range(cfg.n_qgroups):
        A = attention_map_rows(cfg, Q[r, g, :], r, K[:, cfg.k_of_group(g), :])
        L[:, g, :] = A @ C[:, cfg.c_of_group(g), :]
        if return_maps:
            maps.append(A)
    out = decode_heads(cfg, w, L, G[r])
    Kf = K.reshape(T, cfg.n_kgroups * cfg.head_dim)
    Cf = C.reshape(T, cfg.n_cgroups * cfg.latent_dim)
    return (out, Kf, Cf, maps) if return_maps else (out, Kf, Cf)


def prefill(cfg: OracleConfig, w: OracleWeights, x: np.ndarray, cu_seqlens: Sequence[int]):
    """Packed varlen prefill: sequences b = tokens [cu[b], cu[b+1]) are independent."""
    outs, Ks, Cs = [], [], []
    for b in range(len(cu_seqlens) - 1):
        o, k, c = prefill_sequence(cfg, w, x[cu_seqlens[b]:cu_seqlens[b + 1]])
        outs.append(o); Ks.append(k); Cs.append(c)
    return np.concatenate(outs), np.concatenate(Ks), np.concatenate(Cs)


def cache_append(kcache: np.ndarray, ccache: np.ndarray, seq_lens: np.ndarray, status: np.ndarray,
                 slots: Sequence[int], k_new: np.ndarray, c_new: np.ndarray,
                 cu_new: Sequence[int]) -> None:
    """App. B.1.3 cache contract: rows [cu_new[b], cu_new[b+1]) go to slot slots[b] at positions
    seq_lens[slot] .. ; a sequence that would not fit writes nothing and flags its slot."""
    max_seq = kcache.shape[1]
    for b, s in enumerate(slots):
        n = cu_new[b + 1] - cu_new[b]
        p = int(seq_lens[s])
        if p + n > max_seq:
            status[s] = CACHE_FULL
            continue
        kcache[s, p:p + n, :] = k_new[cu_new[b]:cu_new[b + 1]]
        ccache[s, p:p + n, :] = c_new[cu_new[b]:cu_new[b + 1]]
        seq_lens[s] = p + n


def decode(cfg: OracleConfig, w: OracleWeights, x_new: np.ndarray, kcache: np.ndarray,
           ccache: np.ndarray, seq_lens: np.ndarray, status: np.ndarray,
           slots: Sequence[int]) -> np.ndarray:
    """One decode step (App. B.1.3): project the new token of every sequence at position
    seq_lens[slot], append its k, c, then attend over all cached rows including the new one.

    kcache [slots, max_seq, n_k*d_h] and ccache [slots, max_seq, n_c*d_l] are float64 arrays and
    are updated in place, like seq_lens.  A full slot gets CACHE_FULL and an all-zero output row.
    """
    cfg.check()
    w = w.f64()
    x_new = np.asarray(x_new, dtype=np.float64)
    B = x_new.shape[0]
    width = cfg.d_model if w.wo is not None else cfg.n_heads * cfg.head_dim
    out = np.zeros((B, width), dtype=np.float64)
    for b, s in enumerate(slots):
        p = int(seq_lens[s])
        if p + 1 > kcache.shape[1]:
            status[s] = CACHE_FULL
            continue
        Q, K, C, G = project_tokens(cfg, w, x_new[b:b + 1], np.array([p]))
        kcache[s, p, :] = K.reshape(-1)
        ccache[s, p, :] = C.reshape(-1)
        seq_lens[s] = p + 1
        n = p + 1
        Kc = kcache[s, :n, :].reshape(n, cfg.n_kgroups, cfg.head_dim)
        Cc = ccache[s, :n, :].reshape(n, cfg.n_cgroups, cfg.latent_dim)
        L = np.empty((1, cfg.n_qgroups, cfg.latent_dim), dtype=np.float64)
        for g in range(cfg.n_qgroups):
            A = attention_map_rows(cfg, Q[:, g, :], np.array([p]), Kc[:, cfg.k_of_group(g), :])
            L[:, g, :] = A @ Cc[:, cfg.c_of_group(g), :]
        out[b] = decode_heads(cfg, w, L, G)[0]
    return out
