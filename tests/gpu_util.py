"""Helpers of the GPU parity tests: upload seeded inputs, call the C ABI, compare with the oracle."""
from __future__ import annotations

import numpy as np
import torch

from oracle import gta_oracle as orc
from paper_2506_17286_amd import binding as B

# Tolerances of the parity gate.  fp32: max-abs 1e-5.  bf16 inputs with fp32 accumulation:
# max-abs 2e-2 and relative RMS 5e-3 (bf16 rounding of Q, K, C, the softmax weights, the group
# output and the result each contribute ~2^-9/sqrt(3) relative error).
TOL = {"f32": dict(max_abs=1e-5, rel_rms=1e-5), "bf16": dict(max_abs=2e-2, rel_rms=5e-3)}


def oracle_config(wl, gate=True) -> orc.OracleConfig:
    return orc.OracleConfig(d_model=wl.d_model, n_heads=wl.n_heads, n_qgroups=wl.n_qgroups,
                            n_kgroups=wl.n_kgroups, n_cgroups=wl.n_cgroups, head_dim=wl.head_dim,
                            latent_dim=wl.latent_dim, rope=wl.rope, rope_base=wl.rope_base, gate=gate)


def oracle_weights(w) -> orc.OracleWeights:
    return orc.OracleWeights(w["wq"], w["wk"], w["wc"], w["wg"], w["wp"], w.get("wo")).f64()


def upload_weights(w, dtype):
    return {k: B.to_device(v, dtype) for k, v in w.items()}


def f64(t: torch.Tensor) -> np.ndarray:
    return t.detach().to(torch.float64).cpu().numpy()


def errors(got: np.ndarray, ref: np.ndarray):
    d = got.astype(np.float64) - ref
    return float(np.abs(d).max()), float(np.linalg.norm(d) / max(np.linalg.norm(ref), 1e-300))


def assert_close(got, ref, dtype, what="", abs_scale=1.0):
    """abs_scale widens the max-abs bound only (never the relative one): used where the reference values
    are a known factor larger than the Sigmoid-gated outputs the bound was stated for."""
    assert np.all(np.isfinite(got)), f"{what}: non-finite values"
    ma, rr = errors(got, ref)
    tol = dict(TOL[dtype])
    tol["max_abs"] *= abs_scale
    assert ma <= tol["max_abs"] and rr <= tol["rel_rms"], \
        f"{what}: max_abs {ma:.3e} (tol {tol['max_abs']:.0e}), rel_rms {rr:.3e} (tol {tol['rel_rms']:.0e})"
    return ma, rr


class DeviceCache:
    """Caller-owned cache tensors plus the gta_cache struct that points at them."""

    def __init__(self, wl, n_slots, max_seq, k=None, c=None, seq_lens=None, fill=None):
        dt = torch.bfloat16 if wl.dtype == "bf16" else torch.float32
        kw, cw = wl.kv_width
        if k is None:
            k = torch.zeros((n_slots, max_seq, kw), dtype=dt, device="cuda")
            c = torch.zeros((n_slots, max_seq, cw), dtype=dt, device="cuda")
            if fill is not None:   # canary pattern in every row
                k.fill_(fill); c.fill_(fill)
        self.k, self.c = k, c
        self.seq_lens = torch.zeros(n_slots, dtype=torch.int32, device="cuda") if seq_lens is None else seq_lens
        self.status = torch.zeros(n_slots, dtype=torch.int32, device="cuda")
        self.struct = B.make_cache(self.k, self.c, self.seq_lens, self.status)
        self.max_seq = self.k.shape[1]


class PagedDeviceCache:
    """Block-table caches: pools of pages, a table that deals every slot `pages_per_slot` distinct pages
    in a seeded random order (`missing`: (slot, page index) entries left without a page), and spare pages
    nobody owns.  `logical()` gathers the pools back into [slots, max_seq, width] arrays."""

    def __init__(self, wl, n_slots, page_size, pages_per_slot, spare_pages=3, seed=0, fill=None, missing=()):
        dt = torch.bfloat16 if wl.dtype == "bf16" else torch.float32
        kw, cw = wl.kv_width
        self.page_size, self.pages_per_slot = page_size, pages_per_slot
        self.max_seq = page_size * pages_per_slot
        self.num_pages = n_slots * pages_per_slot + spare_pages
        perm = np.random.default_rng(seed).permutation(self.num_pages)
        self.table_np = perm[:n_slots * pages_per_slot].reshape(n_slots, pages_per_slot).astype(np.int32)
        for (s, i) in missing:
            self.table_np[s, i] = -1
        self.k = torch.zeros((self.num_pages, page_size, kw), dtype=dt, device="cuda")
        self.c = torch.zeros((self.num_pages, page_size, cw), dtype=dt, device="cuda")
        if fill is not None:
            self.k.fill_(fill); self.c.fill_(fill)
        self.table = torch.from_numpy(self.table_np).cuda()
        self.seq_lens = torch.zeros(n_slots, dtype=torch.int32, device="cuda")
        self.status = torch.zeros(n_slots, dtype=torch.int32, device="cuda")
        self.struct = B.make_paged_cache(self.k, self.c, self.seq_lens, self.status, self.table)

    def _index(self):
        idx = torch.from_numpy(np.maximum(self.table_np, 0).astype(np.int64)).cuda()
        return idx

    def store(self, k_logical: torch.Tensor, c_logical: torch.Tensor):
        """Scatter [slots, max_seq, width] tensors into the pages (entries without a page are skipped)."""
        n_slots = self.table_np.shape[0]
        kl = k_logical.reshape(n_slots, self.pages_per_slot, self.page_size, -1)
        cl = c_logical.reshape(n_slots, self.pages_per_slot, self.page_size, -1)
        for s in range(n_slots):
            for i in range(self.pages_per_slot):
                pg = int(self.table_np[s, i])
                if pg >= 0:
                    self.k[pg] = kl[s, i]; self.c[pg] = cl[s, i]

    def logical(self):
        """(k, c) as [slots, max_seq, width] tensors gathered through the table (missing pages read page 0)."""
        idx = self._index()
        n_slots = self.table_np.shape[0]
        k = self.k[idx].reshape(n_slots, self.max_seq, -1)
        c = self.c[idx].reshape(n_slots, self.max_seq, -1)
        return k, c

    def spare_untouched(self, fill) -> bool:
        """True if the pages no slot owns still hold the fill value."""
        owned = set(int(p) for p in self.table_np.ravel() if p >= 0)
        spare = [p for p in range(self.num_pages) if p not in owned]
        idx = torch.tensor(spare, dtype=torch.int64, device="cuda")
        return bool((self.k[idx] == fill).all() and (self.c[idx] == fill).all())


def run_prefill(wl, wdev, x_np, cu_np=None, batch=None, max_seqlen=None, cache: DeviceCache = None,
                slots=None, gate=True, workspace=None):
    """gta_prefill through the C ABI on numpy hidden states; returns the output tensor."""
    cfg = B.config_of(wl)
    cfg.gate = B.GATE_CODES[gate]
    total = x_np.shape[0]
    x = B.to_device(x_np, wl.dtype)
    if cu_np is not None:
        cu = torch.from_numpy(np.asarray(cu_np, dtype=np.int32)).cuda()
        batch = len(cu_np) - 1
        lens = np.diff(cu_np)
        max_seqlen = int(lens.max()) if max_seqlen is None else max_seqlen
    else:
        cu = None
        batch = batch or 1
        max_seqlen = total // batch if max_seqlen is None else max_seqlen
    width = wl.d_model if wdev.get("wo") is not None else wl.n_heads * wl.head_dim
    out = torch.full((total, width), float("nan"), dtype=x.dtype, device="cuda")
    nbytes = B.gta_workspace_bytes(cfg, B.GTA_MODE_PREFILL, batch, total, max_seqlen)
    ws = workspace if workspace is not None else B.alloc_workspace(nbytes)
    sl = None if slots is None else torch.from_numpy(np.asarray(slots, dtype=np.int32)).cuda()
    B.gta_prefill(cfg, B.make_weights(wdev), x, cu, batch, total, max_seqlen,
                  None if cache is None else cache.struct, sl, out, ws)
    torch.cuda.synchronize()
    return out


def run_decode(wl, wdev, x_np, cache: DeviceCache, slots=None, num_splits=0, gate=True):
    cfg = B.config_of(wl)
    cfg.gate = B.GATE_CODES[gate]
    batch = x_np.shape[0]
    x = B.to_device(x_np, wl.dtype)
    width = wl.d_model if wdev.get("wo") is not None else wl.n_heads * wl.head_dim
    out = torch.full((batch, width), float("nan"), dtype=x.dtype, device="cuda")
    nbytes = B.gta_workspace_bytes(cfg, B.GTA_MODE_DECODE, batch, 0, cache.max_seq, num_splits)
    ws = B.alloc_workspace(nbytes)
    sl = None if slots is None else torch.from_numpy(np.asarray(slots, dtype=np.int32)).cuda()
    B.gta_decode(cfg, B.make_weights(wdev), x, batch, cache.struct, sl, out, num_splits, ws)
    torch.cuda.synchronize()
    return out


def run_prefill_chunk(wl, wdev, x_np, cu_np, cache: DeviceCache, slots=None, gate=True):
    """gta_prefill_chunk through the C ABI: the chunks follow whatever the slots already hold."""
    cfg = B.config_of(wl)
    cfg.gate = B.GATE_CODES[gate]
    total = x_np.shape[0]
    x = B.to_device(x_np, wl.dtype)
    cu = torch.from_numpy(np.asarray(cu_np, dtype=np.int32)).cuda()
    batch = len(cu_np) - 1
    max_chunk = int(np.diff(cu_np).max())
    width = wl.d_model if wdev.get("wo") is not None else wl.n_heads * wl.head_dim
    out = torch.full((total, width), float("nan"), dtype=x.dtype, device="cuda")
    ws = B.alloc_workspace(B.gta_workspace_bytes(cfg, B.GTA_MODE_PREFILL_CHUNK, batch, total, max_chunk))
    sl = None if slots is None else torch.from_numpy(np.asarray(slots, dtype=np.int32)).cuda()
    B.gta_prefill_chunk(cfg, B.make_weights(wdev), x, cu, batch, total, max_chunk, cache.struct, sl, out, ws)
    torch.cuda.synchronize()
    return out
