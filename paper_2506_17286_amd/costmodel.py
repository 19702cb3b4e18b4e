"""Closed-form work counts of the GTA attention pass (paper Table 3 and App. B.1) and the
algorithmic flop / byte counters the benchmark divides by.

The paper counts multiply-accumulates over the full N x N square; the benchmark credits only the
causal lower triangle (pairs = sum_b T_b (T_b + 1) / 2) and counts 2 flops per MAC.
"""
from __future__ import annotations

from typing import Iterable


# ------------------------------------------------------------------ the paper's own counts
def gta_cache_elems_per_token(n_k: int, n_c: int, d_h: int, d_l: int) -> int:
    """Table 3 / App. B.1.3: cached elements per token per layer, n_k d_h + n_c d_l."""
    return n_k * d_h + n_c * d_l


def gqa_cache_elems_per_token(n_kv: int, d_h: int) -> int:
    """Table 3: GQA (MHA with n_kv = n_h) caches 2 n_k d_h elements per token per layer."""
    return 2 * n_kv * d_h


def gta_attention_ops(n_q: int, d_h: int, d_l: int, N: int) -> int:
    """Table 3 / App. B.1.2: n_q (d_h + d_l) N^2."""
    return n_q * (d_h + d_l) * N * N


def mha_attention_ops(n_h: int, d_h: int, N: int) -> int:
    """Table 3: 2 n_h d_h N^2 for MHA and GQA."""
    return 2 * n_h * d_h * N * N


def gta_linear_ops(H: int, n_q: int, n_k: int, n_c: int, d_h: int, d_l: int, N: int) -> int:
    """Table 3: 2 N H^2 + (n_q d_h + n_k d_h + n_c d_l + d_l) N H."""
    return 2 * N * H * H + (n_q * d_h + n_k * d_h + n_c * d_l + d_l) * N * H


# ------------------------------------------------------------------ benchmark counters
def causal_pairs(seqlens: Iterable[int]) -> int:
    return sum(int(t) * (int(t) + 1) // 2 for t in seqlens)


def prefill_flops(wl, seqlens: Iterable[int], with_wo: bool = False) -> dict:
    """Algorithmic flops of one gta_prefill call (2 per MAC, causal triangle only)."""
    seqlens = [int(t) for t in seqlens]
    tok = sum(seqlens)
    wtot = (wl.n_qgroups + wl.n_kgroups) * wl.head_dim + wl.n_cgroups * wl.latent_dim \
        + wl.n_heads * wl.head_dim
    f = {
        "proj": 2 * tok * wl.d_model * wtot,
        "attn": 2 * wl.n_qgroups * (wl.head_dim + wl.latent_dim) * causal_pairs(seqlens),
        "decoder": 2 * tok * wl.n_heads * wl.latent_dim * wl.head_dim,
        "out": 2 * tok * wl.n_heads * wl.head_dim * wl.d_model if with_wo else 0,
    }
    f["total"] = sum(f.values())
    return f


def elem_bytes(dtype: str) -> int:
    return 2 if dtype == "bf16" else 4


def decode_cache_bytes(wl, ctx_lens: Iterable[int]) -> int:
    """Bytes of grouped-key and latent-value cache one decode step must stream: every cached row
    (incl. the row appended by the step) of every sequence, once."""
    row = gta_cache_elems_per_token(wl.n_kgroups, wl.n_cgroups, wl.head_dim, wl.latent_dim)
    return sum(int(n) for n in ctx_lens) * row * elem_bytes(wl.dtype)


def decode_flops(wl, ctx_lens: Iterable[int]) -> int:
    """2 n_q (d_h + d_l) flops per cached row (the appendix's printed 2 n_h d_h N is the GQA line
    repeated; the prefill count n_q (d_h + d_l) per pair is the one consistent with Table 3)."""
    return 2 * wl.n_qgroups * (wl.head_dim + wl.latent_dim) * sum(int(n) for n in ctx_lens)
