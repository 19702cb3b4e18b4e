"""GPU parity of chunked prefill (a chunk of new tokens behind the rows a slot already holds):
splitting sequences into a prefix and a chunk, or into several chunks, must give the rows of ONE causal
pass over the whole sequences, which is what the oracle computes."""
import numpy as np
import pytest
import torch

from oracle import gta_oracle as orc
from paper_2506_17286_amd import binding as B
from paper_2506_17286_amd import workloads as W

import gpu_util as U

pytestmark = pytest.mark.gpu


def _base(shape):
    if shape == "paper":
        return W.PAPER_WORKLOADS[0]
    return W.WORKLOADS[1] if shape == "1b" else W.WORKLOADS[4]


def _inputs(wl, lens, with_wo=False):
    rng = W.make_rng(wl)
    w = W.draw_weights(wl, rng, with_wo=with_wo)
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    x = W.draw_hidden(wl, rng, int(cu[-1]))
    return w, cu, x


@pytest.mark.parametrize("shape,with_wo", [("1b", False), ("paper", False), ("paper", True), ("wide", False)])
def test_prefix_then_chunk_equals_one_pass(shape, with_wo):
    """Sequences cut into (prefix, chunk) at points inside and on tile borders, one of them with an empty
    prefix: prefill the prefixes, then the chunks; outputs of the chunk rows, every cached row and the
    lengths against one oracle pass over the whole sequences."""
    lens = [300, 129, 64, 37, 513]
    pre = [37, 0, 63, 36, 256]
    slots = [4, 0, 5, 2, 1]
    wl = W.scaled(_base(shape), batch=len(lens), seqlen=max(lens), min_seqlen=None)
    w, cu, x = _inputs(wl, lens, with_wo)
    wdev = U.upload_weights(w, wl.dtype)
    cache = U.DeviceCache(wl, 6, 520, fill=-3.0)
    # prefixes of the sequences that have one
    has = [b for b in range(len(lens)) if pre[b] > 0]
    xp = np.concatenate([x[cu[b]:cu[b] + pre[b]] for b in has])
    cup = np.concatenate([[0], np.cumsum([pre[b] for b in has])]).astype(np.int32)
    U.run_prefill(wl, wdev, xp, cup, cache=cache, slots=[slots[b] for b in has])
    # the chunks of all sequences
    xc = np.concatenate([x[cu[b] + pre[b]:cu[b + 1]] for b in range(len(lens))])
    cuc = np.concatenate([[0], np.cumsum([lens[b] - pre[b] for b in range(len(lens))])]).astype(np.int32)
    out = U.run_prefill_chunk(wl, wdev, xc, cuc, cache, slots=slots)
    ref, Kref, Cref = orc.prefill(U.oracle_config(wl), U.oracle_weights(w), x, cu)
    ref_rows = np.concatenate([ref[cu[b] + pre[b]:cu[b + 1]] for b in range(len(lens))])
    U.assert_close(U.f64(out), ref_rows, wl.dtype, f"chunked prefill {shape}")
    kc, cc = U.f64(cache.k), U.f64(cache.c)
    for b, s in enumerate(slots):
        U.assert_close(kc[s, :lens[b]], Kref[cu[b]:cu[b + 1]], wl.dtype, "K cache")
        U.assert_close(cc[s, :lens[b]], Cref[cu[b]:cu[b + 1]], wl.dtype, "C cache")
        assert np.all(kc[s, lens[b]:] == -3.0) and np.all(cc[s, lens[b]:] == -3.0)
        assert int(cache.seq_lens[s]) == lens[b]
    assert np.all(kc[3] == -3.0) and int(cache.seq_lens[3]) == 0
    assert np.all(cache.status.cpu().numpy() == 0)


@pytest.mark.parametrize("shape", ["1b", "paper"])
def test_chunk_beyond_the_short_prefill_limit(shape):
    """A chunk call with more tokens than the short-prefill kernels take (1536 at the 1B shape, 4096 at the
    paper's): 256-row projection tiles with per-token RoPE rows.  A long and a short chunk behind 100 and
    650 cached rows."""
    long_len = 1900 if shape == "1b" else 4500
    lens, pre = [long_len, 700], [100, 650]
    wl = W.scaled(_base(shape), batch=2, seqlen=long_len, min_seqlen=None)
    w, cu, x = _inputs(wl, lens)
    wdev = U.upload_weights(w, wl.dtype)
    cache = U.DeviceCache(wl, 2, long_len + 12, fill=-3.0)
    xp = np.concatenate([x[cu[b]:cu[b] + pre[b]] for b in range(2)])
    U.run_prefill(wl, wdev, xp, np.array([0, 100, 750], dtype=np.int32), cache=cache)
    xc = np.concatenate([x[cu[b] + pre[b]:cu[b + 1]] for b in range(2)])
    cuc = np.array([0, long_len - 100, long_len - 100 + 50], dtype=np.int32)
    out = U.run_prefill_chunk(wl, wdev, xc, cuc, cache)
    ref, Kref, Cref = orc.prefill(U.oracle_config(wl), U.oracle_weights(w), x, cu)
    ref_rows = np.concatenate([ref[cu[b] + pre[b]:cu[b + 1]] for b in range(2)])
    U.assert_close(U.f64(out), ref_rows, wl.dtype, f"long chunk {shape}")
    kc, cc = U.f64(cache.k), U.f64(cache.c)
    for b in range(2):
        U.assert_close(kc[b, :lens[b]], Kref[cu[b]:cu[b + 1]], wl.dtype, "K cache")
        U.assert_close(cc[b, :lens[b]], Cref[cu[b]:cu[b + 1]], wl.dtype, "C cache")
        assert np.all(kc[b, lens[b]:] == -3.0) and np.all(cc[b, lens[b]:] == -3.0)
    assert cache.seq_lens.cpu().tolist() == lens


@pytest.mark.parametrize("shape", ["1b", "paper"])
def test_several_chunks_in_a_row(shape):
    """One sequence of 700 tokens fed as chunks of 100, 344 and 256 next to a short one fed as 1, 1, 30."""
    lens = [700, 32]
    parts = [[100, 344, 256], [1, 1, 30]]
    wl = W.scaled(_base(shape), batch=2, seqlen=700, min_seqlen=None)
    w, cu, x = _inputs(wl, lens)
    wdev = U.upload_weights(w, wl.dtype)
    cache = U.DeviceCache(wl, 2, 704)
    ref, Kref, Cref = orc.prefill(U.oracle_config(wl), U.oracle_weights(w), x, cu)
    done = [0, 0]
    for step in range(3):
        n = [parts[b][step] for b in range(2)]
        xc = np.concatenate([x[cu[b] + done[b]:cu[b] + done[b] + n[b]] for b in range(2)])
        cuc = np.concatenate([[0], np.cumsum(n)]).astype(np.int32)
        out = U.run_prefill_chunk(wl, wdev, xc, cuc, cache)
        ref_rows = np.concatenate([ref[cu[b] + done[b]:cu[b] + done[b] + n[b]] for b in range(2)])
        U.assert_close(U.f64(out), ref_rows, wl.dtype, f"chunk {step}")
        done = [done[b] + n[b] for b in range(2)]
        assert cache.seq_lens.cpu().tolist() == done
    U.assert_close(U.f64(cache.k)[0, :700], Kref[:700], wl.dtype, "K cache")
    U.assert_close(U.f64(cache.c)[1, :32], Cref[700:], wl.dtype, "C cache")


@pytest.mark.parametrize("shape", ["1b", "paper"])
def test_empty_sequences_in_a_packed_batch(shape):
    """Sequences without tokens inside a packed batch (equal consecutive offsets): a fresh prefill sets their
    length to 0, a chunked prefill leaves their slot as it is; the other sequences are unaffected."""
    lens = [40, 0, 70, 0]
    wl = W.scaled(_base(shape), batch=4, seqlen=70, min_seqlen=None)
    w, cu, x = _inputs(wl, lens)
    wdev = U.upload_weights(w, wl.dtype)
    cache = U.DeviceCache(wl, 4, 128, fill=-3.0)
    cache.seq_lens[1] = 9
    ref, Kref, Cref = orc.prefill(U.oracle_config(wl), U.oracle_weights(w), x, np.array([0, 40, 110], dtype=np.int32))
    out = U.run_prefill(wl, wdev, x, cu, cache=cache)
    U.assert_close(U.f64(out), ref, wl.dtype, "prefill with empty sequences")
    assert cache.seq_lens.cpu().tolist() == [40, 0, 70, 0]
    # now a chunk for sequences 0 and 3 only; 1 and 2 get nothing
    lens2 = [5, 0, 0, 3]
    w2, cu2, x2 = w, np.concatenate([[0], np.cumsum(lens2)]).astype(np.int32), W.draw_hidden(wl, W.make_rng(W.scaled(wl, seed=77)), 8)
    out2 = U.run_prefill_chunk(wl, wdev, x2, cu2, cache)
    full0 = np.concatenate([x[:40], x2[:5]])
    r0, _, _ = orc.prefill_sequence(U.oracle_config(wl), U.oracle_weights(w), full0)
    r3, _, _ = orc.prefill_sequence(U.oracle_config(wl), U.oracle_weights(w), x2[5:])
    U.assert_close(U.f64(out2)[:5], r0[40:], wl.dtype, "chunk behind 40 rows")
    U.assert_close(U.f64(out2)[5:], r3, wl.dtype, "chunk on an empty slot")
    assert cache.seq_lens.cpu().tolist() == [45, 0, 70, 3]
    assert np.all(cache.status.cpu().numpy() == 0)


def test_chunk_that_does_not_fit_is_skipped():
    """A chunk that would overflow its slot stores nothing, returns zero rows and flags the slot; the
    other sequence of the call is unaffected."""
    lens = [60, 40]
    wl = W.scaled(W.PAPER_WORKLOADS[0], batch=2, seqlen=60, min_seqlen=None)
    w, cu, x = _inputs(wl, lens)
    wdev = U.upload_weights(w, wl.dtype)
    cache = U.DeviceCache(wl, 2, 64, fill=-3.0)
    cache.seq_lens[0] = 10          # 10 + 60 > 64: does not fit (the 10 rows are never read)
    out = U.run_prefill_chunk(wl, wdev, x, cu, cache)
    ref, Kref, Cref = orc.prefill(U.oracle_config(wl), U.oracle_weights(w), x[60:], np.array([0, 40], dtype=np.int32))
    got = U.f64(out)
    assert np.all(got[:60] == 0.0)
    U.assert_close(got[60:], ref, wl.dtype, "sequence that fits")
    assert cache.seq_lens.cpu().tolist() == [10, 40]
    assert cache.status.cpu().tolist() == [B.GTA_ERR_CACHE_FULL, 0]
    assert np.all(U.f64(cache.k)[0] == -3.0) and np.all(U.f64(cache.c)[0] == -3.0)


@pytest.mark.parametrize("shape", ["fp32_small", "bf16_odd"])
def test_chunked_prefill_on_the_shape_generic_kernels(shape):
    """Configurations the MFMA kernels do not cover (fp32 elements; bf16 with dimensions off the tile
    grid) take the shape-generic kernels: prefix then chunk, against one oracle pass, plus a chunk that
    does not fit."""
    if shape == "fp32_small":
        base = W.WORKLOADS[0]
    else:
        base = W.scaled(W.WORKLOADS[1], d_model=200, n_heads=6, head_dim=24, n_qgroups=3, n_kgroups=3, n_cgroups=1,
                        latent_dim=40)
    lens = [45, 17, 33, 20]
    pre = [13, 0, 32, 5]
    slots = [2, 0, 3, 1]
    wl = W.scaled(base, batch=len(lens), seqlen=max(lens), min_seqlen=None)
    cfg = B.config_of(wl)
    assert B.gta_uses_tuned_kernels(cfg, B.GTA_MODE_PREFILL_CHUNK) == 0
    w, cu, x = _inputs(wl, lens, with_wo=(shape == "bf16_odd"))
    wdev = U.upload_weights(w, wl.dtype)
    cache = U.DeviceCache(wl, 4, 48, fill=-3.0)
    has = [b for b in range(len(lens)) if pre[b] > 0]
    xp = np.concatenate([x[cu[b]:cu[b] + pre[b]] for b in has])
    cup = np.concatenate([[0], np.cumsum([pre[b] for b in has])]).astype(np.int32)
    U.run_prefill(wl, wdev, xp, cup, cache=cache, slots=[slots[b] for b in has])
    cache.seq_lens[1] = 40   # 40 + 15 > 48: the chunk of sequence 3 does not fit
    xc = np.concatenate([x[cu[b] + pre[b]:cu[b + 1]] for b in range(len(lens))])
    cuc = np.concatenate([[0], np.cumsum([lens[b] - pre[b] for b in range(len(lens))])]).astype(np.int32)
    out = U.f64(U.run_prefill_chunk(wl, wdev, xc, cuc, cache, slots=slots))
    ref, Kref, Cref = orc.prefill(U.oracle_config(wl), U.oracle_weights(w), x, cu)
    kc, cc = U.f64(cache.k), U.f64(cache.c)
    for b, s_ in enumerate(slots):
        rows = slice(int(cuc[b]), int(cuc[b + 1]))
        if b == 3:
            assert np.all(out[rows] == 0.0)
            continue
        U.assert_close(out[rows], ref[cu[b] + pre[b]:cu[b + 1]], wl.dtype, f"generic chunked prefill {shape} seq {b}")
        U.assert_close(kc[s_, :lens[b]], Kref[cu[b]:cu[b + 1]], wl.dtype, "K cache")
        U.assert_close(cc[s_, :lens[b]], Cref[cu[b]:cu[b + 1]], wl.dtype, "C cache")
        assert np.all(kc[s_, lens[b]:] == -3.0) and np.all(cc[s_, lens[b]:] == -3.0)
    assert cache.seq_lens.cpu().tolist() == [17, 40, 45, 33]
    assert cache.status.cpu().tolist() == [0, B.GTA_ERR_CACHE_FULL, 0, 0]
