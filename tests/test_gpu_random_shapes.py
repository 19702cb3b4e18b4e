"""GPU parity on seeded random configurations: dimensions off every tile grid, random group structure,
both element types, RoPE on or off, with or without W_O, contiguous or block-table caches.  Each case runs
a whole life of a batch through the C ABI — ragged prefill, a chunk behind it, two decode steps — and
compares every stage with ONE oracle pass over the full sequences (causality makes its rows the expected
rows of every stage), plus the cache rows and the lengths."""
import numpy as np
import pytest
import torch

from oracle import gta_oracle as orc
from paper_2506_17286_amd import binding as B
from paper_2506_17286_amd import workloads as W

import gpu_util as U

pytestmark = pytest.mark.gpu


def _draw_config(seed):
    r = np.random.default_rng(9000 + seed)
    d_h = int(r.choice([8, 16, 24, 32, 48, 64]))
    n_q = int(r.choice([1, 2, 3, 4, 6]))
    hpq = int(r.choice([1, 2, 3, 4]))
    divs = [d for d in range(1, n_q + 1) if n_q % d == 0]
    n_k, n_c = int(r.choice(divs)), int(r.choice(divs))
    d_l = d_h + 8 * int(r.integers(0, 3 * d_h // 8 + 1))
    H = int(r.choice([40, 64, 96, 200, 256]))
    dtype = "f32" if seed % 2 == 0 else "bf16"
    wl = W.Workload(name=f"random_{seed}", kind="prefill", batch=int(r.integers(1, 5)), seqlen=96, d_model=H,
                    n_heads=n_q * hpq, n_qgroups=n_q, n_kgroups=n_k, n_cgroups=n_c, head_dim=d_h, latent_dim=d_l,
                    dtype=dtype, rope=bool(r.integers(0, 2)), seed=9100 + seed)
    page = int(r.choice([0, 0, 4, 8, 16, 32]))          # 0: contiguous caches
    return wl, page, bool(r.integers(0, 2)), r


def _life(wl, page, with_wo, pre, chunk, steps, slots, max_seq, seed):
    """Prefill `pre` tokens per sequence, then `chunk` more, then `steps` decode steps; every stage, the
    cache rows and the lengths against one oracle pass over the full sequences."""
    nb = len(pre)
    full = [pre[b] + chunk[b] + steps for b in range(nb)]
    rng = W.make_rng(wl)
    # projections of unit-variance hidden states come out with standard deviation about 1, the scale the
    # stated absolute tolerances are meant for
    w = W.draw_weights(wl, rng, with_wo=with_wo, std=1.0 / np.sqrt(wl.d_model))
    cu = np.concatenate([[0], np.cumsum(full)]).astype(np.int32)
    x = W.draw_hidden(wl, rng, int(cu[-1]))
    wdev = U.upload_weights(w, wl.dtype)
    ref, Kref, Cref = orc.prefill(U.oracle_config(wl), U.oracle_weights(w), x, cu)
    n_slots = max(slots) + 1
    if page:
        cache = U.PagedDeviceCache(wl, n_slots, page, max_seq // page, seed=seed, fill=-5.0)
    else:
        cache = U.DeviceCache(wl, n_slots, max_seq, fill=-5.0)
    what = f"seed {seed}: {wl} page {page} wo {with_wo}"

    def check(out, rs, stage):
        # rounding errors are relative: where the reference reaches beyond 1 the max-abs bound, stated
        # for unit-scale outputs, scales with its largest magnitude; the relative-RMS bound does not
        U.assert_close(U.f64(out), rs, wl.dtype, what + stage, abs_scale=max(1.0, float(np.abs(rs).max())))

    def rows(lo, hi):   # rows [lo[b], hi[b]) of every sequence, packed
        xs = np.concatenate([x[cu[b] + lo[b]:cu[b] + hi[b]] for b in range(nb)])
        rs = np.concatenate([ref[cu[b] + lo[b]:cu[b] + hi[b]] for b in range(nb)])
        cs = np.concatenate([[0], np.cumsum([hi[b] - lo[b] for b in range(nb)])]).astype(np.int32)
        return xs, rs, cs

    xs, rs, cs = rows([0] * nb, pre)
    check(U.run_prefill(wl, wdev, xs, cs, cache=cache, slots=slots), rs, " prefill")
    done = list(pre)
    if sum(chunk) > 0:
        hi = [done[b] + chunk[b] for b in range(nb)]
        xs, rs, cs = rows(done, hi)
        check(U.run_prefill_chunk(wl, wdev, xs, cs, cache, slots=slots), rs, " chunk")
        done = hi
    for _ in range(steps):
        hi = [d + 1 for d in done]
        xs, rs, cs = rows(done, hi)
        check(U.run_decode(wl, wdev, xs, cache, slots=slots), rs, " decode")
        done = hi
    seq = cache.seq_lens.cpu().tolist()
    kl, cl = cache.logical() if page else (cache.k, cache.c)
    kc, cc = U.f64(kl), U.f64(cl)
    for b, s_ in enumerate(slots):
        assert seq[s_] == full[b]
        U.assert_close(kc[s_, :full[b]], Kref[cu[b]:cu[b + 1]], wl.dtype, what + " K cache",
                       abs_scale=max(1.0, float(np.abs(Kref).max())))
        U.assert_close(cc[s_, :full[b]], Cref[cu[b]:cu[b + 1]], wl.dtype, what + " C cache",
                       abs_scale=max(1.0, float(np.abs(Cref).max())))
        assert np.all(kc[s_, full[b]:] == -5.0) and np.all(cc[s_, full[b]:] == -5.0)
    for s_ in set(range(n_slots)) - set(slots):
        assert seq[s_] == 0 and np.all(kc[s_] == -5.0)
    assert np.all(cache.status.cpu().numpy() == 0)


@pytest.mark.parametrize("seed", range(24))
def test_random_configuration_through_prefill_chunk_and_decode(seed):
    wl, page, with_wo, r = _draw_config(seed)
    nb = wl.batch
    pre = [int(v) for v in r.integers(1, 60, nb)]
    chunk = [int(v) for v in r.integers(0, 25, nb)]
    slots = [int(v) for v in r.permutation(nb + 1)[:nb]]
    _life(wl, page, with_wo, pre, chunk, 2, slots, 96, seed)


# the shape families of the MFMA / streaming kernels (at a small hidden size, so the oracle stays quick)
_TUNED = {
    "1b": dict(n_heads=16, n_qgroups=4, n_kgroups=4, n_cgroups=1, head_dim=128, latent_dim=512),
    "wide": dict(n_heads=32, n_qgroups=8, n_kgroups=8, n_cgroups=1, head_dim=128, latent_dim=1024),
    "paper": dict(n_heads=20, n_qgroups=5, n_kgroups=1, n_cgroups=1, head_dim=64, latent_dim=128),
    "paper_nq3": dict(n_heads=12, n_qgroups=3, n_kgroups=1, n_cgroups=1, head_dim=64, latent_dim=128),
    "paper_nq6": dict(n_heads=12, n_qgroups=6, n_kgroups=1, n_cgroups=1, head_dim=64, latent_dim=128),
    "paper_nc2": dict(n_heads=20, n_qgroups=10, n_kgroups=1, n_cgroups=2, head_dim=64, latent_dim=128),
}


@pytest.mark.parametrize("family,page,with_wo", [("1b", 0, False), ("1b", 64, True), ("wide", 32, False),
                                                 ("paper", 0, True), ("paper", 32, False), ("paper_nq3", 64, False),
                                                 ("paper_nq6", 16, False), ("paper_nc2", 128, False)])
def test_tuned_shape_families_through_prefill_chunk_and_decode(family, page, with_wo):
    """The same life of a batch on the shapes the MFMA and streaming kernels are compiled for, lengths
    that span several 256-row query tiles and 32-row key tiles with ragged tails, contiguous and
    block-table caches (pages of 16 rows keep the streaming decode kernels but not the MFMA attention
    kernel in cache mode, which then hands over to the shape-generic one)."""
    wl = W.Workload(name=f"life_{family}", kind="prefill", batch=4, seqlen=640, d_model=512, dtype="bf16", rope=True,
                    seed=9300 + len(family) + page, **_TUNED[family])
    cfg = B.config_of(wl)
    assert B.gta_uses_tuned_kernels(cfg, B.GTA_MODE_PREFILL) == 1 and B.gta_uses_tuned_kernels(cfg, B.GTA_MODE_DECODE) == 1
    _life(wl, page, with_wo, pre=[300, 1, 257, 64], chunk=[290, 33, 0, 256], steps=2, slots=[2, 0, 4, 1],
          max_seq=640, seed=page)
