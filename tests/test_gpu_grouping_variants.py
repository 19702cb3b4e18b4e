"""The two predecessors the paper derives GTA from (Sec. 3.1), run as parameter settings of the same
kernels and checked against the oracle in the same setting (tests/test_oracle_pins.py pins those
settings to plain shared-map attention):

  GVA  "Grouping Values to Share Attention Matrix": one map per group of heads, every head its own
       values.  n_q = n_k = n_c = groups, d_l = heads-per-group * d_h (the group's values side by
       side), W_{P,i} selects head i's slice, gate off.
  GHA  "Grouping Heads to Compress Attention": the heads of a group share query, key and one value
       source.  n_q = n_k = n_c = groups, d_l = width of the source, dense W_{P,i}, gate off.

Also the other head groupings the wide-row decode kernel is compiled for (several maps per key,
several latents)."""
import numpy as np
import pytest
import torch

from oracle import gta_oracle as orc
from paper_2506_17286_amd import binding as B
from paper_2506_17286_amd import workloads as W

import gpu_util as U

pytestmark = pytest.mark.gpu


def _setting(kind):
    if kind == "gva":      # 4 heads of 128 in 2 groups; latent = the two heads' values side by side
        return W.scaled(W.WORKLOADS[1], name="gva", d_model=512, n_heads=4, n_qgroups=2, n_kgroups=2, n_cgroups=2,
                        latent_dim=256)
    if kind == "gva_wide":  # 16 heads in 4 groups, latent 4 * 128 = 512: cache rows of the streaming decode kernel
        return W.scaled(W.WORKLOADS[1], name="gva_wide", d_model=1024, n_heads=16, n_qgroups=4, n_kgroups=4,
                        n_cgroups=4, latent_dim=512)
    if kind == "gha":      # 4 heads of 128 in 2 groups; shared value source as wide as a head
        return W.scaled(W.WORKLOADS[1], name="gha", d_model=512, n_heads=4, n_qgroups=2, n_kgroups=2, n_cgroups=2,
                        latent_dim=128)
    raise KeyError(kind)


@pytest.mark.parametrize("kind", ["gva", "gva_wide", "gha"])
def test_gva_and_gha_settings_prefill_then_decode(kind):
    base = _setting(kind)
    lens = [1, 37, 300, 129, 700]
    wl = W.scaled(base, batch=len(lens), seqlen=max(lens), min_seqlen=None)
    rng = W.make_rng(wl)
    w = W.draw_weights(wl, rng)
    if kind.startswith("gva"):   # W_{P,i}: head i's slice of its group's latent, exactly
        hpq, dh = wl.n_heads // wl.n_qgroups, wl.head_dim
        w["wp"] = np.zeros((wl.n_heads, wl.latent_dim, dh), dtype=np.float32)
        for i in range(wl.n_heads):
            w["wp"][i, (i % hpq) * dh:(i % hpq + 1) * dh, :] = np.eye(dh, dtype=np.float32)
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    x = W.draw_hidden(wl, rng, int(cu[-1]) + len(lens))
    xp, xd = x[:cu[-1]], x[cu[-1]:]
    wdev = U.upload_weights(w, wl.dtype)
    cache = U.DeviceCache(wl, len(lens), max(lens) + 1)
    assert B.gta_uses_tuned_kernels(B.config_of(wl), B.GTA_MODE_PREFILL) == 1
    out = U.run_prefill(wl, wdev, xp, cu, cache=cache, gate=False)
    cfg, wo = U.oracle_config(wl, gate=False), U.oracle_weights(w)
    ref, Kref, Cref = orc.prefill(cfg, wo, xp, cu)
    U.assert_close(U.f64(out), ref, wl.dtype, f"{kind} prefill")
    # one decode step behind it: the new token of every sequence against one more oracle row
    step = U.run_decode(wl, wdev, xd, cache, gate=False)
    for b, T in enumerate(lens):
        full, _, _ = orc.prefill_sequence(cfg, wo, np.concatenate([xp[cu[b]:cu[b + 1]], xd[b:b + 1]]), rows=[T])
        U.assert_close(U.f64(step[b:b + 1]), full, wl.dtype, f"{kind} decode seq {b}")
    assert cache.seq_lens.cpu().tolist() == [T + 1 for T in lens]
    if kind == "gva_wide":
        assert B.gta_uses_tuned_kernels(B.config_of(wl), B.GTA_MODE_DECODE) == 1
