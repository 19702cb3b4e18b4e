"""GPU parity of the block-table ("paged") cache layout.  The layout changes where a cache row lives, not
what is computed: every call must give bit-for-bit what the same call gives on contiguous caches holding
the same rows (same kernels, same order of arithmetic), which in turn is checked against the oracle; the
rows the call stores must land in the pages the table names and nowhere else."""
import numpy as np
import pytest
import torch

from oracle import gta_oracle as orc
from paper_2506_17286_amd import binding as B
from paper_2506_17286_amd import workloads as W

import gpu_util as U

pytestmark = pytest.mark.gpu

FILL = -3.0


def _base(shape, kind):
    i = 0 if kind == "prefill" else 1
    if shape == "1b":
        return W.WORKLOADS[1] if kind == "prefill" else W.WORKLOADS[2]
    if shape == "wide":
        return W.WORKLOADS[4] if kind == "prefill" else W.scaled(W.WORKLOADS[4], kind="decode", min_seqlen=None)
    if shape == "paper":
        return W.PAPER_WORKLOADS[i]
    if shape == "paper_nc2":
        return W.scaled(W.PAPER_WORKLOADS[i], n_qgroups=10, n_cgroups=2)
    if shape == "fp32_small":
        return W.scaled(W.WORKLOADS[0], kind=kind, rope=True)
    raise KeyError(shape)


def _same_bits(a: torch.Tensor, b: torch.Tensor) -> bool:
    return bool(torch.equal(a.contiguous().view(torch.uint8), b.contiguous().view(torch.uint8)))


@pytest.mark.parametrize("shape,page_size", [("1b", 16), ("1b", 256), ("wide", 64), ("paper", 16), ("paper", 128),
                                             ("paper_nc2", 32), ("fp32_small", 16), ("paper", 24), ("1b", 8)])
def test_decode_on_paged_caches(shape, page_size):
    """Decode steps over ragged contexts (incl. 0, page borders and a slot with one row left) on paged
    caches against the same steps on contiguous caches, bit for bit, and against the oracle.  Page sizes
    that are not a power of two >= 16 take the shape-generic kernels; all others the streaming ones."""
    ctx = [0, 1, page_size - 1, page_size, page_size + 1, 3 * page_size, 333, 700, 1023]
    pps = (1024 + page_size - 1) // page_size
    max_seq = pps * page_size
    ctx[-1] = max_seq - 1
    wl = W.scaled(_base(shape, "decode"), batch=len(ctx), seqlen=max(ctx))
    cfg = B.config_of(wl)
    rng = W.make_rng(wl)
    w = W.draw_weights(wl, rng, with_wo=(page_size == 128))
    x = W.draw_hidden(wl, rng, wl.batch)
    k_np, c_np = W.draw_cache(wl, rng, wl.batch, max_seq)
    wdev = U.upload_weights(w, wl.dtype)
    kd, cd = B.to_device(k_np, wl.dtype), B.to_device(c_np, wl.dtype)
    seq = torch.tensor(ctx, dtype=torch.int32).cuda()
    flat = U.DeviceCache(wl, wl.batch, max_seq, k=kd.clone(), c=cd.clone(), seq_lens=seq.clone())
    paged = U.PagedDeviceCache(wl, wl.batch, page_size, pps, seed=page_size, fill=FILL)
    paged.store(kd, cd)
    paged.seq_lens.copy_(seq)
    streaming_pages = page_size >= 16 and page_size & (page_size - 1) == 0
    tuned = B.gta_uses_tuned_kernels(cfg, B.GTA_MODE_DECODE) == 1
    same_kernels = streaming_pages or not tuned   # else: contiguous runs the streaming kernels, paged the generic ones
    for splits in (0, 3):
        flat.seq_lens.copy_(seq); paged.seq_lens.copy_(seq)
        out_flat = U.run_decode(wl, wdev, x, flat, num_splits=splits)
        out_paged = U.run_decode(wl, wdev, x, paged, num_splits=splits)
        kl, cl = paged.logical()
        if same_kernels:
            assert _same_bits(out_flat, out_paged), f"{shape} page {page_size} splits {splits}: outputs differ"
            assert _same_bits(kl, flat.k) and _same_bits(cl, flat.c), "appended rows differ or landed elsewhere"
        else:
            U.assert_close(U.f64(kl), U.f64(flat.k), wl.dtype, "K rows")
            U.assert_close(U.f64(cl), U.f64(flat.c), wl.dtype, "C rows")
        assert paged.seq_lens.cpu().tolist() == [n + 1 for n in ctx]
        assert paged.spare_untouched(FILL)
    sl = np.array(ctx, dtype=np.int32); st = np.zeros(len(ctx), dtype=np.int32)
    ref = orc.decode(U.oracle_config(wl), U.oracle_weights(w), x, k_np.astype(np.float64), c_np.astype(np.float64),
                     sl, st, list(range(len(ctx))))
    U.assert_close(U.f64(out_paged), ref, wl.dtype, f"paged decode {shape} page {page_size}")
    assert np.all(paged.status.cpu().numpy() == 0)


@pytest.mark.parametrize("shape", ["1b", "paper", "fp32_small"])
def test_decode_into_a_row_without_a_page_treats_the_slot_as_full(shape):
    """Sequence 1's next row falls on a table entry without a page: nothing is stored, its output row is
    zero, its length stays, its status is flagged; the other sequences are as on contiguous caches."""
    ps, pps = 16, 4
    ctx = [5, 32, 40]            # sequence 1 would append row 32 = first row of its page index 2
    wl = W.scaled(_base(shape, "decode"), batch=3, seqlen=max(ctx))
    rng = W.make_rng(wl)
    w = W.draw_weights(wl, rng)
    x = W.draw_hidden(wl, rng, 3)
    k_np, c_np = W.draw_cache(wl, rng, 3, ps * pps)
    wdev = U.upload_weights(w, wl.dtype)
    kd, cd = B.to_device(k_np, wl.dtype), B.to_device(c_np, wl.dtype)
    seq = torch.tensor(ctx, dtype=torch.int32).cuda()
    flat = U.DeviceCache(wl, 3, ps * pps, k=kd.clone(), c=cd.clone(), seq_lens=seq.clone())
    paged = U.PagedDeviceCache(wl, 3, ps, pps, seed=5, fill=FILL, missing=[(1, 2), (1, 3)])
    paged.store(kd, cd)
    paged.seq_lens.copy_(seq)
    before_k, before_c = paged.k.clone(), paged.c.clone()
    out_flat = U.run_decode(wl, wdev, x, flat)
    out = U.run_decode(wl, wdev, x, paged)
    assert _same_bits(out[0], out_flat[0]) and _same_bits(out[2], out_flat[2])
    assert bool((out[1] == 0).all())
    assert paged.seq_lens.cpu().tolist() == [6, 32, 41]
    assert paged.status.cpu().tolist() == [0, B.GTA_ERR_CACHE_FULL, 0]
    # only the two rows appended for sequences 0 and 2 changed in the pools
    changed_k = (paged.k != before_k).any(dim=2).sum().item()
    changed_c = (paged.c != before_c).any(dim=2).sum().item()
    assert changed_k == 2 and changed_c == 2
    assert paged.spare_untouched(FILL)


@pytest.mark.parametrize("shape,page_size", [("1b", 64), ("paper", 16), ("fp32_small", 8), ("paper", 40)])
def test_prefill_writes_paged_caches(shape, page_size):
    """A packed ragged prefill into paged caches: outputs and gathered cache rows bit for bit as on
    contiguous caches, rows past the lengths and spare pages untouched, oracle parity of the rows."""
    lens = [1, 37, 256, 300, 129, 64]
    slots = [5, 0, 3, 1, 6, 2]
    if shape == "fp32_small":
        lens = [1, 37, 56, 60, 29, 64]
    pps = (320 + page_size - 1) // page_size
    max_seq = pps * page_size
    wl = W.scaled(_base(shape, "prefill"), batch=len(lens), seqlen=max(lens), min_seqlen=None)
    rng = W.make_rng(wl)
    w = W.draw_weights(wl, rng)
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    x = W.draw_hidden(wl, rng, int(cu[-1]))
    wdev = U.upload_weights(w, wl.dtype)
    flat = U.DeviceCache(wl, 7, max_seq, fill=FILL)
    paged = U.PagedDeviceCache(wl, 7, page_size, pps, seed=11, fill=FILL)
    out_flat = U.run_prefill(wl, wdev, x, cu, cache=flat, slots=slots)
    out = U.run_prefill(wl, wdev, x, cu, cache=paged, slots=slots)
    assert _same_bits(out, out_flat)
    kl, cl = paged.logical()
    assert _same_bits(kl, flat.k) and _same_bits(cl, flat.c)
    assert paged.seq_lens.cpu().tolist() == flat.seq_lens.cpu().tolist()
    assert paged.spare_untouched(FILL) and np.all(paged.status.cpu().numpy() == 0)
    ref, Kref, Cref = orc.prefill(U.oracle_config(wl), U.oracle_weights(w), x, cu)
    U.assert_close(U.f64(out), ref, wl.dtype, f"prefill with paged caches {shape}")
    kc, cc = U.f64(kl), U.f64(cl)
    for b, s in enumerate(slots):
        U.assert_close(kc[s, :lens[b]], Kref[cu[b]:cu[b + 1]], wl.dtype, "K cache")
        U.assert_close(cc[s, :lens[b]], Cref[cu[b]:cu[b + 1]], wl.dtype, "C cache")


def test_prefill_into_missing_pages_flags_the_slot():
    """A sequence whose rows reach a table entry without a page keeps its old length and is flagged; its
    output rows do not depend on the cache and are still right; the other sequence is stored."""
    ps, pps = 16, 4
    lens = [40, 20]
    wl = W.scaled(W.PAPER_WORKLOADS[0], batch=2, seqlen=40, min_seqlen=None)
    rng = W.make_rng(wl)
    w = W.draw_weights(wl, rng)
    cu = np.array([0, 40, 60], dtype=np.int32)
    x = W.draw_hidden(wl, rng, 60)
    wdev = U.upload_weights(w, wl.dtype)
    paged = U.PagedDeviceCache(wl, 2, ps, pps, seed=3, fill=FILL, missing=[(0, 2)])   # rows 32..47 of slot 0
    out = U.run_prefill(wl, wdev, x, cu, cache=paged)
    ref, Kref, Cref = orc.prefill(U.oracle_config(wl), U.oracle_weights(w), x, cu)
    U.assert_close(U.f64(out), ref, wl.dtype, "prefill, one slot short of pages")
    assert paged.seq_lens.cpu().tolist() == [0, 20]
    assert paged.status.cpu().tolist() == [B.GTA_ERR_CACHE_FULL, 0]
    kl, _ = paged.logical()
    U.assert_close(U.f64(kl)[1, :20], Kref[40:], wl.dtype, "K cache of the stored sequence")
    assert paged.spare_untouched(FILL)


@pytest.mark.parametrize("shape,ps", [("paper", 16), ("fp32_small", 16), ("paper", 32), ("1b", 64), ("wide", 32)])
def test_chunked_prefill_and_append_on_paged_caches(shape, ps):
    """Prefix by gta_cache_append (rows copied bit-exactly into the pages), then a chunk by
    gta_prefill_chunk: chunk outputs and gathered rows against one oracle pass.  Pages of 32 rows or
    more (a power of two) keep the MFMA attention kernel, smaller ones take the shape-generic kernels."""
    pps = 384 // ps
    lens = [70, 33, 96, 380]
    pre = [30, 0, 64, 100]
    nb = len(lens)
    wl = W.scaled(_base(shape, "prefill"), batch=nb, seqlen=max(lens), min_seqlen=None)
    cfg = B.config_of(wl)
    rng = W.make_rng(wl)
    w = W.draw_weights(wl, rng)
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    x = W.draw_hidden(wl, rng, int(cu[-1]))
    wdev = U.upload_weights(w, wl.dtype)
    ref, Kref, Cref = orc.prefill(U.oracle_config(wl), U.oracle_weights(w), x, cu)
    paged = U.PagedDeviceCache(wl, nb, ps, pps, seed=8, fill=FILL)
    # the prefixes' rows as the element type would hold them
    k_new = B.to_device(np.concatenate([Kref[cu[b]:cu[b] + pre[b]] for b in range(nb)]), wl.dtype)
    c_new = B.to_device(np.concatenate([Cref[cu[b]:cu[b] + pre[b]] for b in range(nb)]), wl.dtype)
    cu_new = torch.from_numpy(np.concatenate([[0], np.cumsum(pre)]).astype(np.int32)).cuda()
    B.gta_cache_append(cfg, paged.struct, None, k_new, c_new, cu_new, nb, max(pre))
    torch.cuda.synchronize()
    assert paged.seq_lens.cpu().tolist() == pre
    kl, cl = paged.logical()
    off = 0
    for b in range(nb):
        assert _same_bits(kl[b, :pre[b]], k_new[off:off + pre[b]]) and _same_bits(cl[b, :pre[b]], c_new[off:off + pre[b]])
        off += pre[b]
    xc = np.concatenate([x[cu[b] + pre[b]:cu[b + 1]] for b in range(nb)])
    cuc = np.concatenate([[0], np.cumsum([lens[b] - pre[b] for b in range(nb)])]).astype(np.int32)
    out = U.run_prefill_chunk(wl, wdev, xc, cuc, paged)
    ref_rows = np.concatenate([ref[cu[b] + pre[b]:cu[b + 1]] for b in range(nb)])
    U.assert_close(U.f64(out), ref_rows, wl.dtype, f"chunked prefill on paged caches {shape}")
    assert paged.seq_lens.cpu().tolist() == lens
    kl, cl = paged.logical()
    for b in range(nb):
        U.assert_close(U.f64(kl)[b, :lens[b]], Kref[cu[b]:cu[b + 1]], wl.dtype, "K cache")
        U.assert_close(U.f64(cl)[b, :lens[b]], Cref[cu[b]:cu[b + 1]], wl.dtype, "C cache")
    assert paged.spare_untouched(FILL) and np.all(paged.status.cpu().numpy() == 0)
