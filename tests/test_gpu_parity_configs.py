"""GPU parity at the full sizes of the five benchmark workloads, in the launch configuration
bench.py times.  Configs 1-4 compare every output element of every sequence with the fp64 oracle.
Config 5 (135k packed tokens at d_model 4096) compares every row of its two shortest sequences and,
on each of the 16 sequences, the rows around every 256-query tile boundary plus at least 256 random
rows; the sample is stated in the test."""
import numpy as np
import pytest
import torch

from oracle import gta_oracle as orc
from paper_2506_17286_amd import binding as B
from paper_2506_17286_amd import workloads as W

import gpu_util as U

pytestmark = pytest.mark.gpu


def _sample_rows(T, rng, n_random=48, tile=None):
    """First / last rows, the rows around small block edges, around T/2 and (with `tile`) around every
    multiple of the query tile, plus n_random distinct random rows."""
    rows = {0, 1, T - 1, T - 2}
    edges = [31, 32, 63, 64, 127, 128, 255, 256, 1023, 1024, T // 2]
    if tile:
        edges += list(range(tile, T, tile))
    for edge in edges:
        for r in (edge - 1, edge, edge + 1):
            if 0 <= r < T:
                rows.add(r)
    fixed = len(rows)
    rows.update(int(r) for r in rng.choice(T, size=min(n_random, T), replace=False))
    while len(rows) < min(T, fixed + n_random):   # random draws that hit a fixed row are replaced
        rows.add(int(rng.integers(0, T)))
    return sorted(rows)


def _check_prefill_workload(wl, full_seqs, sampled_seqs, n_random=48, tile=None):
    lens, cu, w, x = W.prefill_inputs(wl)
    wdev = U.upload_weights(w, wl.dtype)
    max_seq = int(lens.max())
    cache = U.DeviceCache(wl, wl.batch, max_seq)
    out = U.run_prefill(wl, wdev, x, cu if wl.min_seqlen is not None else None, batch=wl.batch, cache=cache,
                        max_seqlen=max_seq)
    cfg, wo = U.oracle_config(wl), U.oracle_weights(w)
    rng = np.random.default_rng(wl.seed + 99)
    assert np.array_equal(cache.seq_lens.cpu().numpy(), lens)
    for b in sorted(set(full_seqs) | set(sampled_seqs)):
        T = int(lens[b])
        rows = None if b in full_seqs else _sample_rows(T, rng, n_random, tile)
        ref, Kref, Cref = orc.prefill_sequence(cfg, wo, x[cu[b]:cu[b + 1]], rows=rows)
        got = U.f64(out[cu[b]:cu[b + 1]])
        got = got if rows is None else got[rows]
        ma, rr = U.assert_close(got, ref, wl.dtype, f"{wl.name} seq {b} ({'all' if rows is None else len(rows)} rows)")
        U.assert_close(U.f64(cache.k[b, :T]), Kref, wl.dtype, f"{wl.name} K cache seq {b}")
        U.assert_close(U.f64(cache.c[b, :T]), Cref, wl.dtype, f"{wl.name} C cache seq {b}")
        print(f"{wl.name} seq {b} T={T}: max_abs {ma:.3e} rel_rms {rr:.3e}", flush=True)
    assert torch.isfinite(out.float()).all()


def test_config2_prefill_1b_bf16():
    """B=4, T=4096, d_model 2048, 16 heads of 128, 4 maps, d_l 512, RoPE.  Oracle: every row of all
    four sequences and every cached key / latent row."""
    _check_prefill_workload(W.WORKLOADS[1], full_seqs=[0, 1, 2, 3], sampled_seqs=[])


def _check_decode_workload(wl, check_seqs):
    rng = W.make_rng(wl)
    w = W.draw_weights(wl, rng)
    x = W.draw_hidden(wl, rng, wl.batch)
    wdev = U.upload_weights(w, wl.dtype)
    max_seq = wl.seqlen + 1
    k, c = W.make_decode_cache_device(wl, max_seq)
    k0_last = k[:, wl.seqlen].clone()                 # noise in the row the step will overwrite
    seq = torch.full((wl.batch,), wl.seqlen, dtype=torch.int32, device="cuda")
    cache = U.DeviceCache(wl, wl.batch, max_seq, k=k, c=c, seq_lens=seq)
    assert B.gta_uses_tuned_kernels(B.config_of(wl), B.GTA_MODE_DECODE) == 1
    out = U.run_decode(wl, wdev, x, cache)
    assert (cache.seq_lens == wl.seqlen + 1).all() and (cache.status == 0).all()
    assert not torch.equal(k[:, wl.seqlen], k0_last)
    cfg, wo = U.oracle_config(wl), U.oracle_weights(w)
    got = U.f64(out)
    for b in check_seqs:
        kc = U.f64(k[b:b + 1]); cc = U.f64(c[b:b + 1])
        kc[0, wl.seqlen] = np.nan; cc[0, wl.seqlen] = np.nan       # the oracle must write this row itself
        sl = np.array([wl.seqlen], dtype=np.int32); st = np.zeros(1, dtype=np.int32)
        ref = orc.decode(cfg, wo, x[b:b + 1], kc, cc, sl, st, [0])
        ma, rr = U.assert_close(got[b:b + 1], ref, wl.dtype, f"{wl.name} seq {b}")
        U.assert_close(U.f64(k[b, wl.seqlen]), kc[0, wl.seqlen], wl.dtype, "appended key row")
        U.assert_close(U.f64(c[b, wl.seqlen]), cc[0, wl.seqlen], wl.dtype, "appended latent row")
        print(f"{wl.name} seq {b}: max_abs {ma:.3e} rel_rms {rr:.3e}", flush=True)


def test_config3_decode_b64_ctx8k_bf16():
    """B=64, 8192 cached tokens each, 1 new token.  Oracle on all 64 sequences."""
    _check_decode_workload(W.WORKLOADS[2], check_seqs=list(range(64)))


def test_config4_decode_b8_ctx32k_bf16():
    """B=8, 32768 cached tokens each, split-K.  Oracle on all 8 sequences."""
    _check_decode_workload(W.WORKLOADS[3], check_seqs=list(range(8)))


def test_config5_varlen_prefill_bf16():
    """16 ragged sequences (lengths uniform in [512, 16384]), d_model 4096, 32 heads, 8 maps,
    d_l 1024.  Oracle: every row of the two shortest sequences; on each of the other 14 the first and
    last rows, the rows around every multiple of the 256-query tile and around the small block edges,
    and 256 further random rows (320 to 450 rows per sequence); every cached key / latent row of all 16."""
    wl = W.WORKLOADS[4]
    lens = W.draw_seqlens(wl, W.make_rng(wl))
    order = [int(i) for i in np.argsort(lens)]
    _check_prefill_workload(wl, full_seqs=order[:2], sampled_seqs=order[2:], n_random=256, tile=256)


def test_paper_layer_prefill_b32_t2048_bf16():
    """One attention layer of the paper's GTA-1B model at the batch of its efficiency runs: B=32, T=2048,
    d_model 1280, 20 heads of 64 in 5 groups, one shared key, one latent of 128 (packed projection,
    attention with the fused value decoder).  Oracle: every row of sequences 0 and 31, sampled rows of
    sequences 7 and 16; caches of those four."""
    _check_prefill_workload(W.PAPER_WORKLOADS[0], full_seqs=[0, 31], sampled_seqs=[7, 16])


def test_paper_layer_decode_b64_t2048_bf16():
    """The same layer, decode at batch 64 with 2048 cached tokens (narrow-row kernel).  Oracle on all 64."""
    _check_decode_workload(W.PAPER_WORKLOADS[1], check_seqs=list(range(64)))


WIDE_ROW_GROUPINGS = {   # other head groupings the wide-row decode kernel is compiled for (heads of 128, d_l 512)
    "q8k4": dict(n_heads=16, n_qgroups=8, n_kgroups=4, n_cgroups=1),      # two maps share a key
    "c2": dict(n_heads=16, n_qgroups=4, n_kgroups=4, n_cgroups=2),        # two latents
    "q8k4c2": dict(n_heads=16, n_qgroups=8, n_kgroups=4, n_cgroups=2),
    "c4": dict(n_heads=8, n_qgroups=4, n_kgroups=4, n_cgroups=4),         # every map its own latent
}


@pytest.mark.parametrize("shape", ["1b", "wide", "paper", "paper_nq3", "paper_nq6", "paper_nc2", "paper_nc2_nq6",
                                   "q8k4", "c2", "q8k4c2", "c4"])
def test_tuned_decode_ragged_contexts(shape):
    """The streaming decode kernels (wide rows, and the narrow-row kernel of the paper's own layer
    shapes) on ragged context lengths incl. 0, 1, block tails and empty splits, every output element
    against the oracle."""
    if shape == "paper":
        base = W.PAPER_WORKLOADS[1]
    elif shape == "paper_nq3":   # the 160M-class layer: 12 heads of 64 in 3 groups
        base = W.scaled(W.PAPER_WORKLOADS[1], d_model=768, n_heads=12, n_qgroups=3)
    elif shape == "paper_nq6":   # its sibling with 6 groups (two heads per group)
        base = W.scaled(W.PAPER_WORKLOADS[1], d_model=768, n_heads=12, n_qgroups=6)
    elif shape == "paper_nc2":   # 10 maps sharing one key and two latents (two-latent variant of the kernel)
        base = W.scaled(W.PAPER_WORKLOADS[1], n_qgroups=10, n_cgroups=2)
    elif shape == "paper_nc2_nq6":
        base = W.scaled(W.PAPER_WORKLOADS[1], d_model=768, n_heads=12, n_qgroups=6, n_cgroups=2)
    elif shape in WIDE_ROW_GROUPINGS:
        base = W.scaled(W.WORKLOADS[2], **WIDE_ROW_GROUPINGS[shape])
    else:
        base = W.WORKLOADS[2] if shape == "1b" else W.scaled(W.WORKLOADS[4], kind="decode", min_seqlen=None)
    ctx = [0, 1, 7, 8, 31, 32, 33, 255, 777, 1500]
    wl = W.scaled(base, batch=len(ctx), seqlen=max(ctx))
    assert B.gta_uses_tuned_kernels(B.config_of(wl), B.GTA_MODE_DECODE) == 1
    for splits in (0, 1, 5, 64):
        rng = W.make_rng(wl)
        w = W.draw_weights(wl, rng, with_wo=(splits == 5))
        x = W.draw_hidden(wl, rng, wl.batch)
        max_seq = max(ctx) + 1
        k_np, c_np = W.draw_cache(wl, rng, wl.batch, max_seq)
        wdev = U.upload_weights(w, wl.dtype)
        cache = U.DeviceCache(wl, wl.batch, max_seq, k=B.to_device(k_np, wl.dtype), c=B.to_device(c_np, wl.dtype),
                              seq_lens=torch.tensor(ctx, dtype=torch.int32).cuda())
        out = U.run_decode(wl, wdev, x, cache, num_splits=splits)
        kc, cc = k_np.astype(np.float64), c_np.astype(np.float64)
        sl = np.array(ctx, dtype=np.int32); st = np.zeros(len(ctx), dtype=np.int32)
        ref = orc.decode(U.oracle_config(wl), U.oracle_weights(w), x, kc, cc, sl, st, list(range(len(ctx))))
        U.assert_close(U.f64(out), ref, wl.dtype, f"tuned decode {shape} splits={splits}")
        assert np.array_equal(cache.seq_lens.cpu().numpy(), sl)


@pytest.mark.parametrize("shape,batch", [("1b", 70), ("1b", 37), ("paper", 131), ("paper_nc2", 33), ("wide", 131),
                                         ("wide", 200)])
def test_tuned_decode_batches_that_do_not_fill_the_last_workgroup(shape, batch):
    """Batch sizes that are not multiples of the sequences a tail workgroup takes (8, 4, 2): short ragged
    contexts, every output element against the oracle.  The wide shape (8 keys of 128, latent of 1024) at
    128..255 sequences is the tail launch whose eight rows need more than 64 KiB of LDS."""
    if shape == "wide":
        base = W.scaled(W.WORKLOADS[4], kind="decode", min_seqlen=None)
    else:
        base = W.WORKLOADS[2] if shape == "1b" else W.PAPER_WORKLOADS[1]
    if shape == "paper_nc2":
        base = W.scaled(base, n_qgroups=10, n_cgroups=2)
    ctx = [(13 * b + 3) % 97 for b in range(batch)]
    wl = W.scaled(base, batch=batch, seqlen=max(ctx))
    rng = W.make_rng(wl)
    w = W.draw_weights(wl, rng)
    x = W.draw_hidden(wl, rng, batch)
    max_seq = max(ctx) + 1
    k_np, c_np = W.draw_cache(wl, rng, batch, max_seq)
    wdev = U.upload_weights(w, wl.dtype)
    cache = U.DeviceCache(wl, batch, max_seq, k=B.to_device(k_np, wl.dtype), c=B.to_device(c_np, wl.dtype),
                          seq_lens=torch.tensor(ctx, dtype=torch.int32).cuda())
    out = U.run_decode(wl, wdev, x, cache)
    sl = np.array(ctx, dtype=np.int32); st = np.zeros(batch, dtype=np.int32)
    ref = orc.decode(U.oracle_config(wl), U.oracle_weights(w), x, k_np.astype(np.float64), c_np.astype(np.float64),
                     sl, st, list(range(batch)))
    U.assert_close(U.f64(out), ref, wl.dtype, f"decode {shape} batch {batch}")
    assert np.array_equal(cache.seq_lens.cpu().numpy(), sl)


@pytest.mark.parametrize("shape,batch,with_wo", [("1b", 300, False), ("1b", 257, True), ("paper", 300, False),
                                                 ("paper", 1100, True), ("wide", 256, False)])
def test_tuned_decode_large_batches(shape, batch, with_wo):
    """From 256 sequences on the decode tail runs as a GEMM on bf16 operands (beyond 1024 on the 256-row
    tiles): short ragged contexts incl. empty ones and a full slot, every output element against the oracle."""
    if shape == "1b":
        base = W.WORKLOADS[2]
    elif shape == "paper":
        base = W.PAPER_WORKLOADS[1]
    else:
        base = W.scaled(W.WORKLOADS[4], kind="decode", min_seqlen=None)
    ctx = [(7 * b + 3) % 41 for b in range(batch)]
    max_seq = 41
    ctx[5] = max_seq          # a full slot: zero output row, status flagged, length unchanged
    wl = W.scaled(base, batch=batch, seqlen=max_seq)
    rng = W.make_rng(wl)
    w = W.draw_weights(wl, rng, with_wo=with_wo)
    x = W.draw_hidden(wl, rng, batch)
    k_np, c_np = W.draw_cache(wl, rng, batch, max_seq)
    wdev = U.upload_weights(w, wl.dtype)
    cache = U.DeviceCache(wl, batch, max_seq, k=B.to_device(k_np, wl.dtype), c=B.to_device(c_np, wl.dtype),
                          seq_lens=torch.tensor(ctx, dtype=torch.int32).cuda())
    out = U.f64(U.run_decode(wl, wdev, x, cache))
    sl = np.array(ctx, dtype=np.int32); st = np.zeros(batch, dtype=np.int32)
    ref = orc.decode(U.oracle_config(wl), U.oracle_weights(w), x, k_np.astype(np.float64), c_np.astype(np.float64),
                     sl, st, list(range(batch)))
    U.assert_close(out, ref, wl.dtype, f"decode {shape} batch {batch}")
    assert np.all(out[5] == 0.0) and np.all(ref[5] == 0.0)
    want = [n + 1 for n in ctx]; want[5] = max_seq
    assert cache.seq_lens.cpu().tolist() == want
    stt = cache.status.cpu().tolist()
    assert stt[5] == B.GTA_ERR_CACHE_FULL and sum(1 for v in stt if v) == 1


@pytest.mark.parametrize("shape,with_wo", [("1b", False), ("1b", True), ("wide", False), ("paper", False),
                                           ("paper", True), ("packed128", False), ("slim", False),
                                           ("paper_nq3", True), ("paper_nq6", False), ("paper_nc2", False),
                                           ("packed128_pad", False), ("mid384", True), ("q8k4c2", False),
                                           ("c4", True)])
@pytest.mark.parametrize("tokens", ["few", "many"])
def test_tuned_prefill_ragged_small(shape, with_wo, tokens):
    """The MFMA prefill path (1B and wide shapes, the paper's own layer shape with heads of 64 and one
    shared key, and a shape with heads of 128 whose tiles straddle the Q | K | C | gate boundaries) on
    short ragged sequences spanning several tiles and tails, every output element and every cached row
    against the oracle.  The last three are the paper's smaller layer shapes, whose summed projection
    width is not a multiple of the 256-column tile (zero-padded packed weights), one of them with two
    latent groups."""
    if shape == "paper":
        base = W.PAPER_WORKLOADS[0]
    elif shape == "paper_nq3":   # 12 heads of 64 in 3 groups: width 192 + 64 + 128 + 768
        base = W.scaled(W.PAPER_WORKLOADS[0], d_model=768, n_heads=12, n_qgroups=3)
    elif shape == "paper_nq6":   # two heads per group
        base = W.scaled(W.PAPER_WORKLOADS[0], d_model=768, n_heads=12, n_qgroups=6)
    elif shape == "paper_nc2":   # 10 groups sharing one key and two latents: width 640 + 64 + 256 + 1280
        base = W.scaled(W.PAPER_WORKLOADS[0], n_qgroups=10, n_cgroups=2)
    elif shape == "packed128":
        base = W.scaled(W.WORKLOADS[1], d_model=512, n_heads=4, n_qgroups=2, n_kgroups=1, n_cgroups=1, latent_dim=128)
    elif shape == "packed128_pad":   # heads of 128, summed width 768 + 128 + 256 + 768 = 7.5 tiles of 256
        base = W.scaled(W.WORKLOADS[1], d_model=512, n_heads=6, n_qgroups=6, n_kgroups=1, n_cgroups=1, latent_dim=256)
    elif shape == "mid384":   # heads of 128 with a latent of 384: the 128-column attention tile, three per group
        base = W.scaled(W.WORKLOADS[1], d_model=512, n_heads=4, n_qgroups=2, n_kgroups=2, n_cgroups=1, latent_dim=384)
    elif shape == "slim":   # GQA-like: one map per head, latent as wide as a head, several key / latent groups
        base = W.scaled(W.PAPER_WORKLOADS[0], d_model=512, n_heads=8, n_qgroups=8, n_kgroups=2, n_cgroups=2, latent_dim=64)
    elif shape in WIDE_ROW_GROUPINGS:   # several maps per key / several latents at heads of 128
        base = W.scaled(W.WORKLOADS[1], **WIDE_ROW_GROUPINGS[shape])
    else:
        base = W.WORKLOADS[1] if shape == "1b" else W.WORKLOADS[4]
    # calls of few tokens take the short-prefill kernels (split-K projection on 64-row tiles; the limit
    # depends on the shape and is at most 4096 tokens), longer ones the 256-row tiles: both on a ragged mix
    lens = [1, 37, 256, 300, 129, 64]
    slots = [5, 0, 3, 1, 6, 2]
    if tokens == "many":
        lens += [320, 700, 800, 900, 701]          # 4204 tokens in all
        slots += [10, 7, 11, 8, 9]
    wl = W.scaled(base, batch=len(lens), seqlen=max(lens), min_seqlen=None)
    assert B.gta_uses_tuned_kernels(B.config_of(wl), B.GTA_MODE_PREFILL) == 1
    rng = W.make_rng(wl)
    w = W.draw_weights(wl, rng, with_wo=with_wo)
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    x = W.draw_hidden(wl, rng, int(cu[-1]))
    wdev = U.upload_weights(w, wl.dtype)
    cache = U.DeviceCache(wl, 12, 904, fill=-3.0)
    out = U.run_prefill(wl, wdev, x, cu, cache=cache, slots=slots)
    ref, Kref, Cref = orc.prefill(U.oracle_config(wl), U.oracle_weights(w), x, cu)
    U.assert_close(U.f64(out), ref, wl.dtype, f"tuned prefill {shape}")
    kc, cc = U.f64(cache.k), U.f64(cache.c)
    for b, s in enumerate(slots):
        U.assert_close(kc[s, :lens[b]], Kref[cu[b]:cu[b + 1]], wl.dtype, "K cache")
        U.assert_close(cc[s, :lens[b]], Cref[cu[b]:cu[b + 1]], wl.dtype, "C cache")
        assert np.all(kc[s, lens[b]:] == -3.0) and np.all(cc[s, lens[b]:] == -3.0)
        assert int(cache.seq_lens[s]) == lens[b]
    assert np.all(kc[4] == -3.0) and int(cache.seq_lens[4]) == 0
