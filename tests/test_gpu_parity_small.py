"""GPU parity: the HIP library through the C ABI against the fp64 oracle, element by element,
at sizes the oracle finishes in seconds (several tiles plus ragged tails), and the edge cases."""
import numpy as np
import pytest
import torch

from oracle import gta_oracle as orc
from paper_2506_17286_amd import binding as B
from paper_2506_17286_amd import workloads as W

import gpu_util as U

pytestmark = pytest.mark.gpu


def _wl(name, **kw):
    base = dict(name=name, kind="prefill", batch=1, seqlen=64, d_model=64, n_heads=4, n_qgroups=2, n_kgroups=2,
                n_cgroups=1, head_dim=16, latent_dim=32, dtype="f32", rope=False, seed=7)
    base.update(kw)
    return W.Workload(**base)


def _check_prefill(wl, lens, with_wo=False, gate=True, with_cache=True, slots=None):
    rng = W.make_rng(wl)
    w = W.draw_weights(wl, rng, with_wo=with_wo, std=0.02 if wl.d_model >= 256 else 0.15)
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    x = W.draw_hidden(wl, rng, int(cu[-1]))
    wdev = U.upload_weights(w, wl.dtype)
    n_slots = len(lens) + 2
    max_seq = int(max(lens)) + 3
    cache = U.DeviceCache(wl, n_slots, max_seq, fill=-7.0) if with_cache else None
    out = U.run_prefill(wl, wdev, x, cu, cache=cache, slots=slots, gate=gate)
    ref, Kref, Cref = orc.prefill(U.oracle_config(wl, gate), U.oracle_weights(w), x, cu)
    U.assert_close(U.f64(out), ref, wl.dtype, f"{wl.name} out")
    if with_cache:
        sl = list(range(len(lens))) if slots is None else list(slots)
        seq = cache.seq_lens.cpu().numpy()
        kc, cc = U.f64(cache.k), U.f64(cache.c)
        for b, s in enumerate(sl):
            assert seq[s] == lens[b]                                        # integer bookkeeping: exact
            U.assert_close(kc[s, :lens[b]], Kref[cu[b]:cu[b + 1]], wl.dtype, f"{wl.name} K cache")
            U.assert_close(cc[s, :lens[b]], Cref[cu[b]:cu[b + 1]], wl.dtype, f"{wl.name} C cache")
            assert np.all(kc[s, lens[b]:] == -7.0) and np.all(cc[s, lens[b]:] == -7.0)   # rows past T untouched
        for s in set(range(n_slots)) - set(sl):
            assert seq[s] == 0 and np.all(kc[s] == -7.0) and np.all(cc[s] == -7.0)
        assert np.all(cache.status.cpu().numpy() == 0)


def test_config1_tiny_prefill_fp32():
    """BASELINE config 1 as stated: B=1, T=128, d_model=256, 8 heads of 32 in 2 groups, d_l=64."""
    wl = W.WORKLOADS[0]
    lens, cu, w, x = W.prefill_inputs(wl)
    wdev = U.upload_weights(w, wl.dtype)
    cache = U.DeviceCache(wl, 1, 128)
    out = U.run_prefill(wl, wdev, x, None, batch=1, cache=cache)
    ref, Kref, Cref = orc.prefill_sequence(U.oracle_config(wl), U.oracle_weights(w), x)
    ma, rr = U.assert_close(U.f64(out), ref, "f32", "config 1")
    U.assert_close(U.f64(cache.k)[0], Kref, "f32", "config 1 K cache")
    U.assert_close(U.f64(cache.c)[0], Cref, "f32", "config 1 C cache")
    assert int(cache.seq_lens[0]) == 128
    assert B.gta_uses_tuned_kernels(B.config_of(wl), B.GTA_MODE_PREFILL) == 0


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("case", [
    dict(lens=[70], rope=True),
    dict(lens=[1], rope=True),
    dict(lens=[5, 1, 129, 64], rope=True, slots=[3, 0, 5, 1]),
    dict(lens=[33, 95], rope=False, with_wo=True),
    dict(lens=[77], n_heads=6, n_qgroups=3, n_kgroups=1, n_cgroups=1, head_dim=8, latent_dim=24, rope=True),
    dict(lens=[40, 41], n_heads=4, n_qgroups=4, n_kgroups=2, n_cgroups=4, head_dim=16, latent_dim=16, rope=True, gate=False),
    dict(lens=[50], d_model=40, n_heads=2, n_qgroups=1, n_kgroups=1, n_cgroups=1, head_dim=6, latent_dim=10, rope=True, with_wo=True),
])
def test_prefill_small_shapes(dtype, case):
    case = dict(case)
    lens = case.pop("lens"); with_wo = case.pop("with_wo", False); gate = case.pop("gate", True)
    slots = case.pop("slots", None)
    wl = _wl("small", dtype=dtype, **case)
    _check_prefill(wl, lens, with_wo=with_wo, gate=gate, slots=slots)


def test_prefill_without_cache_and_paper_shape():
    """The paper's own layer shape (GTA-1B: H=1280, 20 heads of 64, 5 maps, 1 key, 1 latent of 128)."""
    wl = _wl("gta1b_layer", d_model=1280, n_heads=20, n_qgroups=5, n_kgroups=1, n_cgroups=1, head_dim=64,
             latent_dim=128, dtype="bf16", rope=True)
    _check_prefill(wl, [150, 31], with_cache=False)


def _decode_case(wl, ctx_lens, max_seq, with_wo=False, num_splits=0, slots=None):
    rng = W.make_rng(wl)
    w = W.draw_weights(wl, rng, with_wo=with_wo, std=0.02 if wl.d_model >= 256 else 0.15)
    Bn = len(ctx_lens)
    x = W.draw_hidden(wl, rng, Bn)
    n_slots = Bn + 1
    k_np, c_np = W.draw_cache(wl, rng, n_slots, max_seq)
    wdev = U.upload_weights(w, wl.dtype)
    sl = list(range(Bn)) if slots is None else list(slots)
    seq = np.zeros(n_slots, dtype=np.int32)
    for b, s in enumerate(sl):
        seq[s] = ctx_lens[b]
    cache = U.DeviceCache(wl, n_slots, max_seq, k=B.to_device(k_np, wl.dtype), c=B.to_device(c_np, wl.dtype),
                          seq_lens=torch.from_numpy(seq.copy()).cuda())
    out = U.run_decode(wl, wdev, x, cache, slots=slots, num_splits=num_splits)
    kc, cc = k_np.astype(np.float64), c_np.astype(np.float64)
    seq_ref = seq.copy(); status_ref = np.zeros(n_slots, dtype=np.int32)
    ref = orc.decode(U.oracle_config(wl), U.oracle_weights(w), x, kc, cc, seq_ref, status_ref, sl)
    return out, ref, cache, (kc, cc, seq_ref, status_ref), (k_np, c_np)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("splits", [0, 1, 3, 7])
def test_decode_small(dtype, splits):
    wl = _wl("dec", kind="decode", dtype=dtype, rope=True, n_heads=4, n_qgroups=2, n_kgroups=1)
    ctx = [0, 1, 63, 64, 200]
    out, ref, cache, (kc, cc, seq_ref, status_ref), (k0, c0) = _decode_case(wl, ctx, 256, num_splits=splits,
                                                                            slots=[4, 2, 0, 1, 3])
    U.assert_close(U.f64(out), ref, dtype, "decode out")
    np.testing.assert_array_equal(cache.seq_lens.cpu().numpy(), seq_ref)
    np.testing.assert_array_equal(cache.status.cpu().numpy(), status_ref)
    gk, gc = U.f64(cache.k), U.f64(cache.c)
    for s in range(6):
        n = seq_ref[s]
        if n > 0 and s != 5:
            U.assert_close(gk[s, n - 1], kc[s, n - 1], dtype, "appended key row")
            U.assert_close(gc[s, n - 1], cc[s, n - 1], dtype, "appended latent row")
            gk[s, n - 1] = k0[s, n - 1]; gc[s, n - 1] = c0[s, n - 1]
    np.testing.assert_array_equal(gk, k0.astype(np.float64))        # every other row bit-identical
    np.testing.assert_array_equal(gc, c0.astype(np.float64))


def test_decode_full_slot_is_flagged_and_zeroed():
    wl = _wl("dec_full", kind="decode", dtype="bf16", rope=True)
    out, ref, cache, (kc, cc, seq_ref, status_ref), (k0, c0) = _decode_case(wl, [16, 5], 16, with_wo=True)
    assert status_ref.tolist()[0] == orc.CACHE_FULL == B.GTA_ERR_CACHE_FULL
    np.testing.assert_array_equal(cache.status.cpu().numpy(), status_ref)
    np.testing.assert_array_equal(cache.seq_lens.cpu().numpy(), seq_ref)
    got = U.f64(out)
    assert np.all(got[0] == 0.0)
    U.assert_close(got[1:], ref[1:], "bf16", "decode beside a full slot")
    np.testing.assert_array_equal(U.f64(cache.k)[0], k0[0].astype(np.float64))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_decode_equals_last_row_of_prefill(dtype):
    """Prefill T-1 tokens into the cache, decode token T: equals row T of a full prefill."""
    wl = _wl("consistency", dtype=dtype, rope=True, d_model=96, n_heads=6, n_qgroups=3, n_kgroups=3,
             n_cgroups=1, head_dim=16, latent_dim=48)
    rng = W.make_rng(wl)
    w = W.draw_weights(wl, rng, std=0.1)
    T = 83
    x = W.draw_hidden(wl, rng, T)
    wdev = U.upload_weights(w, dtype)
    full = U.f64(U.run_prefill(wl, wdev, x, [0, T]))
    cache = U.DeviceCache(wl, 1, 128)
    U.run_prefill(wl, wdev, x[:T - 1], [0, T - 1], cache=cache)
    step = U.f64(U.run_decode(wl, wdev, x[T - 1:], cache, num_splits=4))
    assert int(cache.seq_lens[0]) == T
    tol = 2e-6 if dtype == "f32" else 2e-2
    assert np.abs(step[0] - full[T - 1]).max() <= tol
    ref, _, _ = orc.prefill_sequence(U.oracle_config(wl), U.oracle_weights(w), x, rows=[T - 1])
    U.assert_close(step, ref, dtype, "decode after prefill")


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_cache_append_bit_exact(dtype):
    wl = _wl("append", dtype=dtype, n_kgroups=1, head_dim=16, latent_dim=40)     # 16- and 40-wide rows
    rng = W.make_rng(wl)
    n_slots, max_seq = 5, 12
    k_np, c_np = W.draw_cache(wl, rng, n_slots, max_seq)
    new_counts = [3, 0, 4, 1]          # sequences -> slots [4, 1, 2, 0]; slot 2 overflows (10 + 4 > 12)
    slots = [4, 1, 2, 0]
    seq0 = np.array([11, 6, 10, 0, 2], dtype=np.int32)
    cu_new = np.concatenate([[0], np.cumsum(new_counts)]).astype(np.int32)
    kw, cw = wl.kv_width
    k_new = W.round_to_dtype(rng.standard_normal((cu_new[-1], kw), dtype=np.float32), dtype)
    c_new = W.round_to_dtype(rng.standard_normal((cu_new[-1], cw), dtype=np.float32), dtype)
    cache = U.DeviceCache(wl, n_slots, max_seq, k=B.to_device(k_np, dtype), c=B.to_device(c_np, dtype),
                          seq_lens=torch.from_numpy(seq0.copy()).cuda())
    B.gta_cache_append(B.config_of(wl), cache.struct, torch.tensor(slots, dtype=torch.int32).cuda(),
                       B.to_device(k_new, dtype), B.to_device(c_new, dtype),
                       torch.from_numpy(cu_new).cuda(), len(slots), max(new_counts))
    torch.cuda.synchronize()
    kr, cr = k_np.copy(), c_np.copy()
    seq_ref = seq0.copy(); st_ref = np.zeros(n_slots, dtype=np.int32)
    orc.cache_append(kr, cr, seq_ref, st_ref, slots, k_new, c_new, cu_new)
    bits = (lambda t: t.view(torch.int16).cpu().numpy()) if dtype == "bf16" else (lambda t: t.view(torch.int32).cpu().numpy())
    ref_bits = (lambda a: W.bf16_bits(a).view(np.int16).reshape(a.shape)) if dtype == "bf16" else (lambda a: a.view(np.int32))
    np.testing.assert_array_equal(bits(cache.k), ref_bits(kr))
    np.testing.assert_array_equal(bits(cache.c), ref_bits(cr))
    np.testing.assert_array_equal(cache.seq_lens.cpu().numpy(), seq_ref)
    np.testing.assert_array_equal(cache.status.cpu().numpy(), st_ref)
    assert st_ref[2] == B.GTA_ERR_CACHE_FULL
