"""Seeded synthetic inputs for the GTA attention pass: workload table and array generators.

This module holds NO arithmetic of the method: it only names shapes and draws random arrays, so
that the tests can hand the SAME arrays to the CPU oracle and to the HIP library.  The paper times
GTA-1B / GQA-1B checkpoints that are not available; since the cost of the pass does not depend on
the values, i.i.d. Gaussian tensors of the benchmark shapes stand in for them:

  hidden states ~ N(0, 1); every weight matrix ~ N(0, 0.02^2); decode cache contents ~ N(0, 1);
  no biases.  One numpy Generator (PCG64) per workload, seed = 1000 + index in WORKLOADS, drawn in
  this fixed order: sequence lengths (ragged workloads only), wq, wk, wc, wg, wp, [wo], hidden
  states, key cache, latent cache.  Draws are float32; for a bf16 workload every array is rounded
  once (round-to-nearest-even) to bf16 and the rounded values are what both sides consume.

The full-size decode caches (0.5-1 G elements) are drawn on the GPU with a seeded torch generator
instead (make_decode_cache_device); tests copy back the sequences they check on the host.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Dict, List, Optional, Tuple

import numpy as np


@dataclass(frozen=True)
class Workload:
    name: str
    kind: str                 # "prefill" | "decode"
    batch: int
    seqlen: int               # prefill: tokens per sequence (max for ragged); decode: cached ctx
    d_model: int
    n_heads: int
    n_qgroups: int
    n_kgroups: int
    n_cgroups: int
    head_dim: int
    latent_dim: int
    dtype: str                # "f32" | "bf16"
    rope: bool
    rope_base: float = 10000.0
    seed: int = 0
    min_seqlen: Optional[int] = None   # set => ragged lengths uniform in [min_seqlen, seqlen]

    @property
    def kv_width(self) -> Tuple[int, int]:
        return self.n_kgroups * self.head_dim, self.n_cgroups * self.latent_dim


# The five benchmark workloads.  "One shared key per group" is read as n_k = n_q and the stated
# latent dimension as one latent group (n_c = 1) of that width.
WORKLOADS: List[Workload] = [
    Workload("tiny_prefill_f32", "prefill", 1, 128, 256, 8, 2, 2, 1, 32, 64, "f32", False, seed=1000),
    Workload("prefill_1b_bf16", "prefill", 4, 4096, 2048, 16, 4, 4, 1, 128, 512, "bf16", True, seed=1001),
    Workload("decode_b64_8k_bf16", "decode", 64, 8192, 2048, 16, 4, 4, 1, 128, 512, "bf16", True, seed=1002),
    Workload("decode_b8_32k_bf16", "decode", 8, 32768, 2048, 16, 4, 4, 1, 128, 512, "bf16", True, seed=1003),
    Workload("varlen_prefill_bf16", "prefill", 16, 16384, 4096, 32, 8, 8, 1, 128, 1024, "bf16", True,
             seed=1004, min_seqlen=512),
]


# One attention layer of the paper's 1B-class models (Appendix, model hyper-parameter table): hidden
# size 1280, 20 heads of 64, GTA-1B with 5 map groups, one shared key and one 128-wide latent value;
# batch sizes and lengths from the paper's efficiency runs (prefill 32 x up to 2048 tokens, decode at
# batch 64).  Seeds continue after the benchmark table.
PAPER_WORKLOADS: List[Workload] = [
    Workload("gta1b_prefill_b32_t2048", "prefill", 32, 2048, 1280, 20, 5, 1, 1, 64, 128, "bf16", True, seed=1100),
    Workload("gta1b_decode_b64_t2048", "decode", 64, 2048, 1280, 20, 5, 1, 1, 64, 128, "bf16", True, seed=1101),
]


def by_name(name: str) -> Workload:
    for w in WORKLOADS + PAPER_WORKLOADS:
        if w.name == name:
            return w
    raise KeyError(name)


def scaled(w: Workload, **kw) -> Workload:
    """A copy of a workload with some fields replaced (smaller batch / length for tests)."""
    return replace(w, **kw)


# ---------------------------------------------------------------------------------- bf16 helpers
def bf16_bits(a: np.ndarray) -> np.ndarray:
    """float32 -> bf16 bit patterns (uint16), round-to-nearest-even (finite inputs)."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    r = ((u >> 16) & 1) + np.uint32(0x7FFF)
    return ((u + r) >> 16).astype(np.uint16)


def bf16_to_f32(bits: np.ndarray) -> np.ndarray:
    return (bits.astype(np.uint32) << 16).view(np.float32)


def round_to_dtype(a: np.ndarray, dtype: str) -> np.ndarray:
    """float32 array whose values are exactly representable in `dtype`."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    return bf16_to_f32(bf16_bits(a)).reshape(a.shape) if dtype == "bf16" else a


# ---------------------------------------------------------------------------------- generators
def make_rng(w: Workload) -> np.random.Generator:
    return np.random.default_rng(w.seed)


def draw_seqlens(w: Workload, rng: np.random.Generator) -> np.ndarray:
    """Per-sequence token counts; consumes random numbers only for ragged workloads."""
    if w.min_seqlen is None:
        return np.full(w.batch, w.seqlen, dtype=np.int32)
    return rng.integers(w.min_seqlen, w.seqlen + 1, size=w.batch).astype(np.int32)


def draw_weights(w: Workload, rng: np.random.Generator, with_wo: bool = False,
                 std: float = 0.02) -> Dict[str, np.ndarray]:
    H, dh, dl = w.d_model, w.head_dim, w.latent_dim
    shapes = [("wq", (H, w.n_qgroups * dh)), ("wk", (H, w.n_kgroups * dh)),
              ("wc", (H, w.n_cgroups * dl)), ("wg", (H, w.n_heads * dh)),
              ("wp", (w.n_heads, dl, dh))]
    if with_wo:
        shapes.append(("wo", (w.n_heads * dh, H)))
    out = {}
    for name, shp in shapes:
        out[name] = round_to_dtype(rng.standard_normal(shp, dtype=np.float32) * np.float32(std), w.dtype)
    return out


def draw_hidden(w: Workload, rng: np.random.Generator, n_tokens: int) -> np.ndarray:
    return round_to_dtype(rng.standard_normal((n_tokens, w.d_model), dtype=np.float32), w.dtype)


def draw_cache(w: Workload, rng: np.random.Generator, n_slots: int, max_seq: int):
    """Key cache [n_slots, max_seq, n_k*d_h] and latent cache [n_slots, max_seq, n_c*d_l]."""
    kw, cw = w.kv_width
    k = round_to_dtype(rng.standard_normal((n_slots, max_seq, kw), dtype=np.float32), w.dtype)
    c = round_to_dtype(rng.standard_normal((n_slots, max_seq, cw), dtype=np.float32), w.dtype)
    return k, c


def prefill_inputs(w: Workload, with_wo: bool = False):
    """(seqlens, cu_seqlens, weights, hidden) of a prefill workload in the documented draw order."""
    rng = make_rng(w)
    lens = draw_seqlens(w, rng)
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    weights = draw_weights(w, rng, with_wo)
    x = draw_hidden(w, rng, int(cu[-1]))
    return lens, cu, weights, x


def decode_inputs(w: Workload, with_wo: bool = False, with_cache: bool = True, max_seq: Optional[int] = None):
    """(weights, x_new, kcache, ccache) of a decode workload; the caches hold w.seqlen valid rows
    in max_seq (default seqlen + 1) allocated rows per slot, all drawn (rows past the valid
    length are noise the kernels must never read)."""
    rng = make_rng(w)
    weights = draw_weights(w, rng, with_wo)
    x = draw_hidden(w, rng, w.batch)
    if not with_cache:
        return weights, x, None, None
    ms = max_seq or (w.seqlen + 1)
    k, c = draw_cache(w, rng, w.batch, ms)
    return weights, x, k, c


def make_decode_cache_device(w: Workload, max_seq: int, device: str = "cuda", salt: int = 0):
    """Full-size decode caches drawn directly in GPU memory (seeded torch generator), returned as
    torch tensors of the workload's dtype.  Used where the host generator would need minutes."""
    import torch
    g = torch.Generator(device=device)
    g.manual_seed(w.seed * 7919 + salt)
    dt = torch.bfloat16 if w.dtype == "bf16" else torch.float32
    kw, cw = w.kv_width
    k = torch.empty((w.batch, max_seq, kw), dtype=dt, device=device)
    c = torch.empty((w.batch, max_seq, cw), dtype=dt, device=device)
    k.normal_(0.0, 1.0, generator=g)
    c.normal_(0.0, 1.0, generator=g)
    return k, c
