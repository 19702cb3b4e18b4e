"""ctypes binding of libgta.so: same names as the C ABI (include/gta.h), argument marshalling only.

Every step of the attention pass runs in the library's HIP kernels; PyTorch tensors are used as
device memory and `torch.cuda.current_stream()` as the stream.  There is no fallback: if the
library is not built, loading raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Dict, Optional

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libgta.so")

GTA_F32, GTA_BF16 = 0, 1
GTA_GATE_SIGMOID, GTA_GATE_OFF, GTA_GATE_SILU, GTA_GATE_RELU2 = 0, 1, 2, 3
GATE_CODES = {True: GTA_GATE_SIGMOID, "sigmoid": GTA_GATE_SIGMOID, False: GTA_GATE_OFF, "off": GTA_GATE_OFF,
              "silu": GTA_GATE_SILU, "relu2": GTA_GATE_RELU2}
GTA_MODE_PREFILL, GTA_MODE_DECODE, GTA_MODE_PREFILL_CHUNK = 0, 1, 2
GTA_OK = 0
GTA_ERR_NULL, GTA_ERR_SHAPE, GTA_ERR_ALIGN, GTA_ERR_DTYPE = -1, -2, -3, -4
GTA_ERR_UNSUPPORTED, GTA_ERR_WORKSPACE, GTA_ERR_HIP, GTA_ERR_CACHE_FULL = -5, -6, -7, -8

GTA_STATIC_SCRATCH_BYTES = 32 << 20
EXPORTS = ["gta_workspace_bytes", "gta_prefill", "gta_prefill_chunk", "gta_decode", "gta_decode_static", "gta_cache_append", "gta_strerror",
           "gta_uses_tuned_kernels", "gta_prefill_projection", "gta_prefill_decoder", "gta_output_projection", "gta_prefill_attention", "gta_decode_attention", "gta_decode_combine", "gta_calibration_copy",
           "gta_calibration_read", "gta_calibration_mfma"]


class gta_config(ctypes.Structure):
    _fields_ = [("d_model", ctypes.c_int32), ("n_heads", ctypes.c_int32), ("n_qgroups", ctypes.c_int32),
                ("n_kgroups", ctypes.c_int32), ("n_cgroups", ctypes.c_int32), ("head_dim", ctypes.c_int32),
                ("latent_dim", ctypes.c_int32), ("dtype", ctypes.c_int32), ("rope", ctypes.c_int32),
                ("rope_base", ctypes.c_float), ("gate", ctypes.c_int32), ("softmax_scale", ctypes.c_float)]


class gta_weights(ctypes.Structure):
    _fields_ = [(n, ctypes.c_void_p) for n in ("wq", "wk", "wc", "wg", "wp", "wo")]


class gta_cache(ctypes.Structure):
    _fields_ = [("k", ctypes.c_void_p), ("c", ctypes.c_void_p), ("seq_lens", ctypes.c_void_p),
                ("status", ctypes.c_void_p), ("max_batch", ctypes.c_int32), ("max_seq", ctypes.c_int32),
                ("block_table", ctypes.c_void_p), ("page_size", ctypes.c_int32),
                ("pages_per_slot", ctypes.c_int32), ("num_pages", ctypes.c_int32)]


class GtaError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {strerror(code)} ({code})")


_lib = None


def load(path: Optional[str] = None) -> ctypes.CDLL:
    """Loads libgta.so (once).  Raises if it has not been built: there is no other code path."""
    global _lib
    if _lib is not None and path is None:
        return _lib
    # PyTorch ships its own HIP runtime: import it first so libgta.so binds to the SAME runtime
    # (and thus the same device context and streams) instead of pulling in a second copy.
    import torch  # noqa: F401
    p = path or LIB_PATH
    if not os.path.exists(p):
        raise FileNotFoundError(
            f"{p} not found: build it with `python -m paper_2506_17286_amd.build` (hipcc, gfx950)")
    lib = ctypes.CDLL(p)
    vp, i32, i64, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_size_t
    cfgp, wp, cp = ctypes.POINTER(gta_config), ctypes.POINTER(gta_weights), ctypes.POINTER(gta_cache)
    lib.gta_workspace_bytes.restype = sz
    lib.gta_workspace_bytes.argtypes = [cfgp, ctypes.c_int, i32, i64, i32, i32]
    lib.gta_prefill.restype = ctypes.c_int
    lib.gta_prefill.argtypes = [cfgp, wp, vp, vp, i32, i64, i32, cp, vp, vp, vp, sz, vp]
    lib.gta_prefill_chunk.restype = ctypes.c_int
    lib.gta_prefill_chunk.argtypes = [cfgp, wp, vp, vp, i32, i64, i32, cp, vp, vp, vp, sz, vp]
    lib.gta_decode.restype = ctypes.c_int
    lib.gta_decode.argtypes = [cfgp, wp, vp, i32, cp, vp, vp, i32, vp, sz, vp]
    lib.gta_decode_static.restype = ctypes.c_int
    lib.gta_decode_static.argtypes = [cfgp, wp, vp, i32, cp, vp, vp, i32, vp]
    lib.gta_cache_append.restype = ctypes.c_int
    lib.gta_cache_append.argtypes = [cfgp, cp, vp, vp, vp, vp, i32, i32, vp]
    lib.gta_prefill_projection.restype = ctypes.c_int
    lib.gta_prefill_projection.argtypes = [cfgp, wp, vp, vp, i32, i64, i32, vp, vp, vp, vp, vp, sz, vp]
    lib.gta_prefill_decoder.restype = ctypes.c_int
    lib.gta_prefill_decoder.argtypes = [cfgp, wp, vp, vp, i64, vp, vp]
    lib.gta_output_projection.restype = ctypes.c_int
    lib.gta_output_projection.argtypes = [cfgp, wp, vp, i64, vp, vp]
    lib.gta_prefill_attention.restype = ctypes.c_int
    lib.gta_prefill_attention.argtypes = [cfgp, vp, vp, vp, vp, i32, i64, i32, vp, vp]
    lib.gta_decode_attention.restype = ctypes.c_int
    lib.gta_decode_attention.argtypes = [cfgp, vp, cp, vp, i32, i32, vp, sz, vp]
    lib.gta_decode_combine.restype = ctypes.c_int
    lib.gta_decode_combine.argtypes = [cfgp, cp, vp, i32, i32, vp, sz, vp, vp]
    lib.gta_calibration_copy.restype = ctypes.c_int
    lib.gta_calibration_copy.argtypes = [vp, vp, i64, vp]
    lib.gta_calibration_read.restype = ctypes.c_int
    lib.gta_calibration_read.argtypes = [vp, i64, ctypes.c_int32, vp, vp]
    lib.gta_calibration_mfma.restype = ctypes.c_int
    lib.gta_calibration_mfma.argtypes = [ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, vp, vp]
    lib.gta_strerror.restype = ctypes.c_char_p
    lib.gta_strerror.argtypes = [ctypes.c_int]
    lib.gta_uses_tuned_kernels.restype = ctypes.c_int
    lib.gta_uses_tuned_kernels.argtypes = [cfgp, ctypes.c_int]
    if path is None:
        _lib = lib
    return lib


def strerror(code: int) -> str:
    return load().gta_strerror(code).decode()


# ------------------------------------------------------------------------------ marshalling
def make_config(*, d_model, n_heads, n_qgroups, n_kgroups, n_cgroups, head_dim, latent_dim, dtype,
                rope=False, rope_base=10000.0, gate=True, softmax_scale=0.0) -> gta_config:
    dt = {"f32": GTA_F32, "bf16": GTA_BF16}.get(dtype, dtype)
    return gta_config(d_model, n_heads, n_qgroups, n_kgroups, n_cgroups, head_dim, latent_dim, dt,
                      int(bool(rope)), float(rope_base), GATE_CODES[gate],
                      float(softmax_scale))


def config_of(wl) -> gta_config:
    """gta_config of a workloads.Workload."""
    return make_config(d_model=wl.d_model, n_heads=wl.n_heads, n_qgroups=wl.n_qgroups, n_kgroups=wl.n_kgroups,
                       n_cgroups=wl.n_cgroups, head_dim=wl.head_dim, latent_dim=wl.latent_dim, dtype=wl.dtype,
                       rope=wl.rope, rope_base=wl.rope_base)


def _ptr(t) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        stream = torch.cuda.current_stream()
    h = stream if isinstance(stream, int) else stream.cuda_stream
    return h or None


def make_weights(w: Dict[str, "object"]) -> gta_weights:
    return gta_weights(_ptr(w["wq"]), _ptr(w["wk"]), _ptr(w["wc"]), _ptr(w["wg"]), _ptr(w["wp"]), _ptr(w.get("wo")))


def make_cache(k, c, seq_lens, status) -> gta_cache:
    """k [slots, max_seq, n_k*d_h], c [slots, max_seq, n_c*d_l], seq_lens/status int32 [slots] (device)."""
    return gta_cache(_ptr(k), _ptr(c), _ptr(seq_lens), _ptr(status), k.shape[0], k.shape[1])


def make_paged_cache(k_pool, c_pool, seq_lens, status, block_table) -> gta_cache:
    """k_pool [num_pages, page_size, n_k*d_h], c_pool [num_pages, page_size, n_c*d_l], block_table int32
    [slots, pages_per_slot] (device): row p of slot s is row p % page_size of page block_table[s, p // page_size]."""
    slots, pps = block_table.shape
    return gta_cache(_ptr(k_pool), _ptr(c_pool), _ptr(seq_lens), _ptr(status), slots, pps * k_pool.shape[1],
                     _ptr(block_table), k_pool.shape[1], pps, k_pool.shape[0])


def _check(rc: int, where: str) -> None:
    if rc != GTA_OK:
        raise GtaError(rc, where)


# ------------------------------------------------------------------------------ entry points
def gta_workspace_bytes(cfg: gta_config, mode: int, batch: int, total_tokens: int, max_len: int,
                        num_splits: int = 0) -> int:
    return int(load().gta_workspace_bytes(ctypes.byref(cfg), mode, batch, total_tokens, max_len, num_splits))


def gta_uses_tuned_kernels(cfg: gta_config, mode: int) -> int:
    return int(load().gta_uses_tuned_kernels(ctypes.byref(cfg), mode))


def gta_prefill(cfg: gta_config, weights: gta_weights, x, cu_seqlens, batch: int, total_tokens: int,
                max_seqlen: int, cache: Optional[gta_cache], slots, out, workspace, stream=None,
                check: bool = True) -> int:
    rc = load().gta_prefill(ctypes.byref(cfg), ctypes.byref(weights), _ptr(x), _ptr(cu_seqlens), batch,
                            total_tokens, max_seqlen, ctypes.byref(cache) if cache is not None else None,
                            _ptr(slots), _ptr(out), _ptr(workspace),
                            0 if workspace is None else workspace.numel() * workspace.element_size(),
                            _stream(stream))
    if check:
        _check(rc, "gta_prefill")
    return rc


def gta_prefill_chunk(cfg: gta_config, weights: gta_weights, x, cu_seqlens, batch: int, total_tokens: int,
                      max_chunk: int, cache: gta_cache, slots, out, workspace, stream=None, check: bool = True) -> int:
    rc = load().gta_prefill_chunk(ctypes.byref(cfg), ctypes.byref(weights), _ptr(x), _ptr(cu_seqlens), batch,
                                  total_tokens, max_chunk, ctypes.byref(cache) if cache is not None else None,
                                  _ptr(slots), _ptr(out), _ptr(workspace),
                                  0 if workspace is None else workspace.numel() * workspace.element_size(),
                                  _stream(stream))
    if check:
        _check(rc, "gta_prefill_chunk")
    return rc


def gta_decode(cfg: gta_config, weights: gta_weights, x_new, batch: int, cache: gta_cache, slots, out,
               num_splits: int, workspace, stream=None, check: bool = True) -> int:
    rc = load().gta_decode(ctypes.byref(cfg), ctypes.byref(weights), _ptr(x_new), batch,
                           ctypes.byref(cache) if cache is not None else None, _ptr(slots), _ptr(out),
                           num_splits, _ptr(workspace),
                           0 if workspace is None else workspace.numel() * workspace.element_size(),
                           _stream(stream))
    if check:
        _check(rc, "gta_decode")
    return rc


def gta_decode_static(cfg: gta_config, weights: gta_weights, x_new, batch: int, cache: gta_cache, slots, out,
                      num_splits: int, stream=None, check: bool = True) -> int:
    rc = load().gta_decode_static(ctypes.byref(cfg), ctypes.byref(weights), _ptr(x_new), batch,
                                  ctypes.byref(cache) if cache is not None else None, _ptr(slots), _ptr(out),
                                  num_splits, _stream(stream))
    if check:
        _check(rc, "gta_decode_static")
    return rc


def gta_cache_append(cfg: gta_config, cache: gta_cache, slots, k_new, c_new, cu_new, batch: int,
                     max_new: int, stream=None, check: bool = True) -> int:
    rc = load().gta_cache_append(ctypes.byref(cfg), ctypes.byref(cache) if cache is not None else None,
                                 _ptr(slots), _ptr(k_new), _ptr(c_new), _ptr(cu_new), batch, max_new,
                                 _stream(stream))
    if check:
        _check(rc, "gta_cache_append")
    return rc


def gta_prefill_projection(cfg: gta_config, weights: gta_weights, x, cu_seqlens, batch: int, total_tokens: int,
                           max_seqlen: int, q_out, k_out, c_out, g_out, workspace, stream=None, check: bool = True) -> int:
    rc = load().gta_prefill_projection(ctypes.byref(cfg), ctypes.byref(weights), _ptr(x), _ptr(cu_seqlens), batch,
                                       total_tokens, max_seqlen, _ptr(q_out), _ptr(k_out), _ptr(c_out), _ptr(g_out),
                                       _ptr(workspace), 0 if workspace is None else workspace.numel() * workspace.element_size(),
                                       _stream(stream))
    if check:
        _check(rc, "gta_prefill_projection")
    return rc


def gta_prefill_decoder(cfg: gta_config, weights: gta_weights, l, g, total_tokens: int, out, stream=None,
                        check: bool = True) -> int:
    rc = load().gta_prefill_decoder(ctypes.byref(cfg), ctypes.byref(weights), _ptr(l), _ptr(g), total_tokens, _ptr(out),
                                    _stream(stream))
    if check:
        _check(rc, "gta_prefill_decoder")
    return rc


def gta_output_projection(cfg: gta_config, weights: gta_weights, heads, total_tokens: int, out, stream=None,
                          check: bool = True) -> int:
    rc = load().gta_output_projection(ctypes.byref(cfg), ctypes.byref(weights), _ptr(heads), total_tokens, _ptr(out),
                                      _stream(stream))
    if check:
        _check(rc, "gta_output_projection")
    return rc


def gta_prefill_attention(cfg: gta_config, q, k, c, cu_seqlens, batch: int, total_tokens: int, max_seqlen: int,
                          l_out, stream=None, check: bool = True) -> int:
    rc = load().gta_prefill_attention(ctypes.byref(cfg), _ptr(q), _ptr(k), _ptr(c), _ptr(cu_seqlens), batch,
                                      total_tokens, max_seqlen, _ptr(l_out), _stream(stream))
    if check:
        _check(rc, "gta_prefill_attention")
    return rc


def gta_decode_attention(cfg: gta_config, q, cache: gta_cache, slots, batch: int, num_splits: int, workspace,
                         stream=None, check: bool = True) -> int:
    rc = load().gta_decode_attention(ctypes.byref(cfg), _ptr(q), ctypes.byref(cache), _ptr(slots), batch, num_splits,
                                     _ptr(workspace), workspace.numel() * workspace.element_size(), _stream(stream))
    if check:
        _check(rc, "gta_decode_attention")
    return rc


def gta_decode_combine(cfg: gta_config, cache: gta_cache, slots, batch: int, num_splits: int, workspace, l_out,
                       stream=None, check: bool = True) -> int:
    rc = load().gta_decode_combine(ctypes.byref(cfg), ctypes.byref(cache), _ptr(slots), batch, num_splits,
                                   _ptr(workspace), workspace.numel() * workspace.element_size(), _ptr(l_out),
                                   _stream(stream))
    if check:
        _check(rc, "gta_decode_combine")
    return rc


def gta_calibration_copy(src, dst, nbytes: int, stream=None) -> int:
    rc = load().gta_calibration_copy(_ptr(src), _ptr(dst), nbytes, _stream(stream))
    _check(rc, "gta_calibration_copy")
    return rc


def gta_calibration_read(src, nbytes: int, workgroups: int, sink, stream=None) -> int:
    rc = load().gta_calibration_read(_ptr(src), nbytes, workgroups, _ptr(sink), _stream(stream))
    _check(rc, "gta_calibration_read")
    return rc


def gta_calibration_mfma(workgroups: int, iters: int, random_operands: bool, sink, stream=None) -> int:
    rc = load().gta_calibration_mfma(workgroups, iters, int(bool(random_operands)), _ptr(sink), _stream(stream))
    _check(rc, "gta_calibration_mfma")
    return rc


# ------------------------------------------------------------------------------ memory helpers
def to_device(a, dtype: str, device: str = "cuda"):
    """numpy float32 array (values representable in `dtype`) -> torch tensor of that dtype."""
    import torch
    t = torch.from_numpy(a)
    return t.to(device=device, dtype=torch.bfloat16 if dtype == "bf16" else torch.float32).contiguous()


def alloc_workspace(nbytes: int, device: str = "cuda"):
    import torch
    return torch.empty(max(nbytes, 256), dtype=torch.uint8, device=device)
