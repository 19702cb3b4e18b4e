"""Stage-wise parity of the tuned prefill: the projection GEMM (with RoPE), the value-decoder GEMM (with
the gate) and the output projection each alone against the oracle's function for that stage, on inputs
that were rounded to bf16 once, so that a stage's own rounding is all that separates the two sides."""
import numpy as np
import pytest
import torch

from oracle import gta_oracle as orc
from paper_2506_17286_amd import binding as B
from paper_2506_17286_amd import workloads as W

import gpu_util as U

pytestmark = pytest.mark.gpu

SHAPES = {
    "1b": W.WORKLOADS[1],
    "wide": W.WORKLOADS[4],
    "paper": W.PAPER_WORKLOADS[0],
}


@pytest.mark.parametrize("shape", list(SHAPES))
@pytest.mark.parametrize("tokens", ["few", "many"])
def test_projection_decoder_and_output_projection_stages(shape, tokens):
    lens = [1, 37, 256, 300, 129, 64] + ([320, 700, 800, 900, 701] if tokens == "many" else [])
    wl = W.scaled(SHAPES[shape], batch=len(lens), seqlen=max(lens), min_seqlen=None)
    cfg = B.config_of(wl)
    assert B.gta_uses_tuned_kernels(cfg, B.GTA_MODE_PREFILL) == 1
    rng = W.make_rng(wl)
    w = W.draw_weights(wl, rng, with_wo=True)
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    total = int(cu[-1])
    x = W.draw_hidden(wl, rng, total)
    wdev = U.upload_weights(w, wl.dtype)
    gw = B.make_weights(wdev)
    ocfg, ow = U.oracle_config(wl), U.oracle_weights(w)
    dh, dl = wl.head_dim, wl.latent_dim
    mk = lambda n: torch.full((total, n), float("nan"), dtype=torch.bfloat16, device="cuda")
    # ---- projection stage against the oracle's projections + RoPE, sequence by sequence
    q, k, c, g = mk(wl.n_qgroups * dh), mk(wl.n_kgroups * dh), mk(wl.n_cgroups * dl), mk(wl.n_heads * dh)
    ws = B.alloc_workspace(B.gta_workspace_bytes(cfg, B.GTA_MODE_PREFILL, len(lens), total, max(lens)))
    B.gta_prefill_projection(cfg, gw, B.to_device(x, wl.dtype), torch.from_numpy(cu).cuda(), len(lens), total, max(lens),
                             q, k, c, g, ws)
    torch.cuda.synchronize()
    for b, T in enumerate(lens):
        Q, K, C, G = orc.project_tokens(ocfg, ow, x[cu[b]:cu[b + 1]], np.arange(T))
        sl = slice(cu[b], cu[b + 1])
        for name, got, ref in (("q", q, Q), ("k", k, K), ("c", c, C), ("gate", g, G)):
            U.assert_close(U.f64(got[sl]), ref.reshape(T, -1), wl.dtype, f"{shape} projection {name} seq {b}")
    # ---- decoder stage: group outputs and gate pre-activations drawn here, rounded to bf16 once
    L = W.round_to_dtype(rng.standard_normal((total, wl.n_qgroups * dl), dtype=np.float32) * 0.5, wl.dtype)
    Gp = W.round_to_dtype(rng.standard_normal((total, wl.n_heads * dh), dtype=np.float32), wl.dtype)
    heads = mk(wl.n_heads * dh)
    B.gta_prefill_decoder(cfg, gw, B.to_device(L, wl.dtype), B.to_device(Gp, wl.dtype), total, heads)
    torch.cuda.synchronize()
    no_wo = orc.OracleWeights(ow.wq, ow.wk, ow.wc, ow.wg, ow.wp, None)
    ref = orc.decode_heads(ocfg, no_wo, L.astype(np.float64).reshape(total, wl.n_qgroups, dl),
                           Gp.astype(np.float64).reshape(total, wl.n_heads, dh))
    U.assert_close(U.f64(heads), ref, wl.dtype, f"{shape} decoder stage")
    # ---- output projection on the heads the decoder stage produced (as stored: bf16)
    out = mk(wl.d_model)
    B.gta_output_projection(cfg, gw, heads, total, out)
    torch.cuda.synchronize()
    U.assert_close(U.f64(out), U.f64(heads) @ ow.wo, wl.dtype, f"{shape} output projection")


def test_stage_entry_points_refuse_the_generic_path():
    wl = W.WORKLOADS[0]   # fp32: shape-generic kernels
    cfg = B.config_of(wl)
    rng = W.make_rng(wl)
    w = W.draw_weights(wl, rng, with_wo=True)
    gw = B.make_weights(U.upload_weights(w, wl.dtype))
    t = torch.zeros((128, 1024), dtype=torch.float32, device="cuda")
    ws = B.alloc_workspace(1 << 20)
    assert B.gta_prefill_projection(cfg, gw, t, None, 1, 128, 128, t, t, t, t, ws, check=False) == B.GTA_ERR_UNSUPPORTED
    assert B.gta_prefill_decoder(cfg, gw, t, t, 128, t, check=False) == B.GTA_ERR_UNSUPPORTED
    assert B.gta_output_projection(cfg, gw, t, 128, t, check=False) == B.GTA_ERR_UNSUPPORTED


@pytest.mark.parametrize("shape", ["1b", "paper"])
@pytest.mark.parametrize("trend", ["rising", "falling", "jumps"])
def test_attention_stage_when_scores_run_away_from_the_first_maximum(shape, trend):
    """The attention kernel keeps the running maximum where it is for as long as the probabilities stay
    far from overflow and falls back to the full online-softmax step when a block's row sum explodes.
    Scores that climb by hundreds of nats along the keys (rising), that start at their maximum (falling)
    and that jump up in a few places force that fall-back again and again; the stage is compared with
    the oracle's materialised softmax."""
    wl = W.scaled(SHAPES[shape], batch=2, seqlen=1100, min_seqlen=None)
    cfg = B.config_of(wl)
    T, dh, dl, nq = wl.seqlen, wl.head_dim, wl.latent_dim, wl.n_qgroups
    rng = np.random.default_rng(7)
    lens = [T, 700]
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    total = int(cu[-1])
    kw, cw = wl.kv_width
    pos = np.concatenate([np.arange(n) for n in lens]).astype(np.float32)
    u = rng.standard_normal(dh).astype(np.float32)
    u /= np.linalg.norm(u)
    if trend == "rising":
        amp = pos * 0.9                       # raw score q.k grows by ~0.9 * sqrt(d_h) per key
    elif trend == "falling":
        amp = (1200.0 - pos) * 0.9
    else:
        amp = np.where((pos.astype(np.int64) % 257) == 200, 400.0 + pos * 0.5, 0.0).astype(np.float32)
    q = np.tile(u * np.sqrt(dh), (total, nq)) + rng.standard_normal((total, nq * dh)).astype(np.float32) * 0.1
    k = np.tile(u, (total, kw // dh)) * amp[:, None] + rng.standard_normal((total, kw)).astype(np.float32) * 0.1
    c = rng.standard_normal((total, cw)).astype(np.float32)
    q, k, c = (W.round_to_dtype(v.astype(np.float32), wl.dtype) for v in (q, k, c))
    out = torch.full((total, nq * dl), float("nan"), dtype=torch.bfloat16, device="cuda")
    B.gta_prefill_attention(cfg, B.to_device(q, wl.dtype), B.to_device(k, wl.dtype), B.to_device(c, wl.dtype),
                            torch.from_numpy(cu).cuda(), len(lens), total, max(lens), out)
    torch.cuda.synchronize()
    ocfg = U.oracle_config(wl)
    got = U.f64(out)
    for b, n in enumerate(lens):
        sl = slice(cu[b], cu[b + 1])
        Q = q[sl].astype(np.float64).reshape(n, nq, dh); K = k[sl].astype(np.float64).reshape(n, -1, dh)
        C = c[sl].astype(np.float64).reshape(n, -1, dl)
        for g in range(nq):
            A = orc.attention_map_rows(ocfg, Q[:, g], np.arange(n), K[:, ocfg.k_of_group(g)])
            ref = A @ C[:, ocfg.c_of_group(g)]
            U.assert_close(got[sl, g * dl:(g + 1) * dl], ref, wl.dtype, f"{shape} {trend} seq {b} group {g}", abs_scale=2.5)
