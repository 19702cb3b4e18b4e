"""GPU parity of the gate nonlinearities other than Sigmoid (Silu, ReLU^2: the ablation on the choice of
nonlinearity) and of the gate switched off, on every kernel that applies the gate: the shape-generic
path, the MFMA value-decoder kernels (pairs of heads, several heads per tile, one head per tile), the
decoder fused into the attention kernel, and both decode tails."""
import numpy as np
import pytest
import torch

from oracle import gta_oracle as orc
from paper_2506_17286_amd import binding as B
from paper_2506_17286_amd import workloads as W

import gpu_util as U

pytestmark = pytest.mark.gpu

SHAPES = {
    "generic_f32": W.Workload("g", "prefill", 1, 64, 64, 4, 2, 2, 1, 16, 32, "f32", True, seed=21),
    "1b": W.WORKLOADS[1],                       # decoder_pair_kernel, decode_tail1_kernel
    "paper": W.PAPER_WORKLOADS[0],              # decoder fused into the attention kernel, decode_tail_kernel
    "paper_nq6": W.scaled(W.PAPER_WORKLOADS[0], d_model=768, n_heads=12, n_qgroups=6),   # decoder_gemm_kernel, 64-wide tile
    "multi": W.scaled(W.WORKLOADS[1], d_model=512, n_heads=4, n_qgroups=2, n_kgroups=1, n_cgroups=1, latent_dim=128),
}


@pytest.mark.parametrize("gate", ["silu", "relu2", False])
@pytest.mark.parametrize("shape", list(SHAPES))
def test_prefill_gate_variants(shape, gate):
    lens = [70, 33] if shape == "generic_f32" else [300, 129, 1]
    wl = W.scaled(SHAPES[shape], batch=len(lens), seqlen=max(lens), min_seqlen=None)
    rng = W.make_rng(wl)
    # the benchmark recipe's weights: gate pre-activations of order 1, so the nonlinearities differ visibly
    # (ReLU^2 is zero for half of them)
    w = W.draw_weights(wl, rng, std=0.15 if wl.d_model < 256 else 0.02)
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    x = W.draw_hidden(wl, rng, int(cu[-1]))
    wdev = U.upload_weights(w, wl.dtype)
    out = U.run_prefill(wl, wdev, x, cu, gate=gate)
    ref, _, _ = orc.prefill(U.oracle_config(wl, gate), U.oracle_weights(w), x, cu)
    sig, _, _ = orc.prefill(U.oracle_config(wl, True), U.oracle_weights(w), x, cu)
    # Silu and ReLU^2 are unbounded, so the largest outputs (and their bf16 rounding steps) exceed those
    # of the Sigmoid-gated pass the max-abs bound was stated for: that bound is scaled by the ratio of
    # the largest reference magnitudes; the relative-RMS bound stays as it is
    scale = max(1.0, float(np.abs(ref).max() / np.abs(sig).max()))
    U.assert_close(U.f64(out), ref, wl.dtype, f"{shape} gate={gate}", abs_scale=scale)
    assert np.abs(ref - sig).max() > 1e-3      # the case does tell the nonlinearities apart


@pytest.mark.parametrize("gate", ["silu", "relu2"])
@pytest.mark.parametrize("shape,batch", [("1b", 3), ("1b", 40), ("paper", 3), ("generic_f32", 2)])
def test_decode_gate_variants(shape, batch, gate):
    base = SHAPES[shape]
    ctx = [(17 * b + 5) % 90 for b in range(batch)]
    wl = W.scaled(base, kind="decode", batch=batch, seqlen=max(ctx), min_seqlen=None)
    rng = W.make_rng(wl)
    w = W.draw_weights(wl, rng, std=0.15 if wl.d_model < 256 else 0.02)
    x = W.draw_hidden(wl, rng, batch)
    max_seq = max(ctx) + 1
    k_np, c_np = W.draw_cache(wl, rng, batch, max_seq)
    wdev = U.upload_weights(w, wl.dtype)
    cache = U.DeviceCache(wl, batch, max_seq, k=B.to_device(k_np, wl.dtype), c=B.to_device(c_np, wl.dtype),
                          seq_lens=torch.tensor(ctx, dtype=torch.int32).cuda())
    out = U.run_decode(wl, wdev, x, cache, gate=gate)
    sl = np.array(ctx, dtype=np.int32); st = np.zeros(batch, dtype=np.int32)
    kc, cc = k_np.astype(np.float64), c_np.astype(np.float64)
    ref = orc.decode(U.oracle_config(wl, gate), U.oracle_weights(w), x, kc.copy(), cc.copy(), sl.copy(), st.copy(),
                     list(range(batch)))
    sig = orc.decode(U.oracle_config(wl, True), U.oracle_weights(w), x, kc, cc, sl, st, list(range(batch)))
    scale = max(1.0, float(np.abs(ref).max() / np.abs(sig).max()))   # see the prefill test
    U.assert_close(U.f64(out), ref, wl.dtype, f"decode {shape} gate={gate}", abs_scale=scale)
