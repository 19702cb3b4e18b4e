"""Host-side checks of the C ABI that need no GPU: the library loads, exports every function
include/gta.h declares, sizes workspaces, and rejects bad arguments before touching the device."""
import ctypes
import os
import re

import pytest

from paper_2506_17286_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    src = open(os.path.join(ROOT, "include", "gta.h")).read()
    return sorted(set(re.findall(r"GTA_API\s+[\w\s\*]+?\b(gta_\w+)\s*\(", src)))


def test_library_exports_every_declared_function():
    lib = B.load()
    names = _declared_functions()
    assert set(names) == set(B.EXPORTS) and len(names) >= 6
    for n in names:
        assert getattr(lib, n) is not None


def test_struct_layouts_match_header():
    assert ctypes.sizeof(B.gta_config) == 12 * 4
    assert ctypes.sizeof(B.gta_weights) == 6 * 8
    assert ctypes.sizeof(B.gta_cache) == 4 * 8 + 8 + 8 + 3 * 4 + 4   # ... block_table, three ints, tail padding
    assert B.gta_cache.block_table.offset == 40 and B.gta_cache.page_size.offset == 48


def _cfg(**kw):
    base = dict(d_model=256, n_heads=8, n_qgroups=2, n_kgroups=2, n_cgroups=1, head_dim=32, latent_dim=64, dtype="f32")
    base.update(kw)
    return B.make_config(**base)


def test_strerror_and_status_codes():
    assert B.strerror(0) == "ok"
    for code in range(-8, 0):
        assert B.strerror(code) != "unknown gta_status"
    assert B.strerror(-99) == "unknown gta_status"


def test_workspace_bytes():
    cfg = _cfg()
    a = B.gta_workspace_bytes(cfg, B.GTA_MODE_PREFILL, 1, 128, 128)
    b = B.gta_workspace_bytes(cfg, B.GTA_MODE_PREFILL, 1, 256, 256)
    assert 0 < a < b
    d1 = B.gta_workspace_bytes(cfg, B.GTA_MODE_DECODE, 4, 0, 4096, 1)
    d8 = B.gta_workspace_bytes(cfg, B.GTA_MODE_DECODE, 4, 0, 4096, 8)
    assert 0 < d1 < d8
    assert B.gta_workspace_bytes(_cfg(n_qgroups=3), B.GTA_MODE_PREFILL, 1, 128, 128) == 0   # invalid config


@pytest.mark.parametrize("kw,code", [
    (dict(n_qgroups=3), B.GTA_ERR_SHAPE),            # n_h % n_q
    (dict(n_kgroups=4), B.GTA_ERR_SHAPE),            # n_q % n_k
    (dict(latent_dim=16), B.GTA_ERR_SHAPE),          # d_l < d_h
    (dict(dtype=7), B.GTA_ERR_DTYPE),
    (dict(head_dim=31, latent_dim=64, rope=True), B.GTA_ERR_SHAPE),
])
def test_invalid_configs_are_rejected(kw, code):
    assert B.gta_uses_tuned_kernels(_cfg(**kw), B.GTA_MODE_PREFILL) == code


def test_null_and_misaligned_arguments_are_rejected_on_the_host():
    lib = B.load()
    cfg = _cfg()
    w = B.gta_weights(16, 16, 16, 16, 16, None)
    fake = 4096  # never dereferenced: every call below fails validation first
    rc = lib.gta_prefill(ctypes.byref(cfg), ctypes.byref(w), None, None, 1, 128, 128, None, None, fake, fake, 1 << 30, None)
    assert rc == B.GTA_ERR_NULL
    rc = lib.gta_prefill(ctypes.byref(cfg), ctypes.byref(w), fake + 4, None, 1, 128, 128, None, None, fake, fake, 1 << 30, None)
    assert rc == B.GTA_ERR_ALIGN
    rc = lib.gta_prefill(ctypes.byref(cfg), ctypes.byref(w), fake, None, 0, 128, 128, None, None, fake, fake, 1 << 30, None)
    assert rc == B.GTA_ERR_SHAPE
    rc = lib.gta_prefill(ctypes.byref(cfg), ctypes.byref(w), fake, None, 3, 128, 128, None, None, fake, fake, 1 << 30, None)
    assert rc == B.GTA_ERR_SHAPE                       # 128 tokens do not split into 3 equal sequences
    rc = lib.gta_prefill(ctypes.byref(cfg), ctypes.byref(w), fake, None, 1, 128, 128, None, None, fake, fake, 16, None)
    assert rc == B.GTA_ERR_WORKSPACE
    rc = lib.gta_prefill(ctypes.byref(cfg), ctypes.byref(w), fake, None, 1, 128, 128, None, None, fake, None, 0, None)
    assert rc == B.GTA_ERR_WORKSPACE
    wnull = B.gta_weights(16, None, 16, 16, 16, None)
    rc = lib.gta_prefill(ctypes.byref(cfg), ctypes.byref(wnull), fake, None, 1, 128, 128, None, None, fake, fake, 1 << 30, None)
    assert rc == B.GTA_ERR_NULL
    cache = B.gta_cache(fake, fake, fake, fake, 2, 64)
    rc = lib.gta_prefill(ctypes.byref(cfg), ctypes.byref(w), fake, None, 1, 128, 128, ctypes.byref(cache), None, fake, fake, 1 << 30, None)
    assert rc == B.GTA_ERR_SHAPE                       # sequence longer than the cache rows
    rc = lib.gta_prefill_chunk(ctypes.byref(cfg), ctypes.byref(w), fake, None, 1, 16, 16, None, None, fake, fake, 1 << 30, None)
    assert rc == B.GTA_ERR_NULL                        # chunked prefill needs a cache
    rc = lib.gta_prefill_chunk(ctypes.byref(cfg), ctypes.byref(w), fake, None, 1, 128, 128, ctypes.byref(cache), None, fake, fake, 1 << 30, None)
    assert rc == B.GTA_ERR_SHAPE                       # chunk longer than the cache rows
    rc = lib.gta_prefill_chunk(ctypes.byref(cfg), ctypes.byref(w), fake, None, 1, 16, 16, ctypes.byref(cache), None, fake, fake, 16, None)
    assert rc == B.GTA_ERR_WORKSPACE
    rc = lib.gta_prefill_chunk(ctypes.byref(cfg), ctypes.byref(w), fake, None, 3, 16, 16, ctypes.byref(cache), None, fake, fake, 1 << 30, None)
    assert rc == B.GTA_ERR_SHAPE                       # 16 tokens do not split into 3 equal chunks
    rc = lib.gta_decode(ctypes.byref(cfg), ctypes.byref(w), fake, 1, None, None, fake, 0, fake, 1 << 30, None)
    assert rc == B.GTA_ERR_NULL
    paged = B.gta_cache(fake, fake, fake, fake, 2, 64, fake, 16, 3, 8)   # 16 * 3 != 64
    rc = lib.gta_decode(ctypes.byref(cfg), ctypes.byref(w), fake, 1, ctypes.byref(paged), None, fake, 0, fake, 1 << 30, None)
    assert rc == B.GTA_ERR_SHAPE
    paged = B.gta_cache(fake, fake, fake, fake, 2, 64, fake, 16, 4, 0)   # no pages in the pool
    rc = lib.gta_decode(ctypes.byref(cfg), ctypes.byref(w), fake, 1, ctypes.byref(paged), None, fake, 0, fake, 1 << 30, None)
    assert rc == B.GTA_ERR_SHAPE
    paged = B.gta_cache(fake, fake, fake, fake, 2, 64, fake + 2, 16, 4, 8)
    rc = lib.gta_decode(ctypes.byref(cfg), ctypes.byref(w), fake, 1, ctypes.byref(paged), None, fake, 0, fake, 1 << 30, None)
    assert rc == B.GTA_ERR_ALIGN
    rc = lib.gta_decode(ctypes.byref(cfg), ctypes.byref(w), fake, 3, ctypes.byref(cache), None, fake, 0, fake, 1 << 30, None)
    assert rc == B.GTA_ERR_SHAPE                       # batch exceeds the cache's slots
    rc = lib.gta_cache_append(ctypes.byref(cfg), ctypes.byref(cache), None, fake, None, fake, 1, 1, None)
    assert rc == B.GTA_ERR_NULL
    with pytest.raises(B.GtaError):
        B._check(rc, "gta_cache_append")
