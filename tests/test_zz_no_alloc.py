"""gta_decode_static: the decode step for callers that cannot allocate (its scratch memory is a fixed
array inside the library) against gta_decode on the same inputs and against the fp64 oracle: two calls
in a row, the second with a smaller input, so that the second runs on scratch the first left dirty."""
import numpy as np
import pytest
import torch

from oracle import gta_oracle as orc
from paper_2506_17286_amd import binding as B
from paper_2506_17286_amd import workloads as W

import gpu_util as U

pytestmark = pytest.mark.gpu


def _one_step(wl, ctx, with_wo, splits):
    """Runs the same decode step through gta_decode and gta_decode_static on two copies of one cache."""
    batch = len(ctx)
    rng = W.make_rng(wl)
    w = W.draw_weights(wl, rng, with_wo=with_wo)
    x_np = W.draw_hidden(wl, rng, batch)
    max_seq = max(ctx) + 1
    k_np, c_np = W.draw_cache(wl, rng, batch, max_seq)
    wdev = U.upload_weights(w, wl.dtype)
    cfg = B.config_of(wl)
    x = B.to_device(x_np, wl.dtype)
    width = wl.d_model if with_wo else wl.n_heads * wl.head_dim
    outs, caches = [], []
    for static in (False, True):
        cache = U.DeviceCache(wl, batch, max_seq, k=B.to_device(k_np, wl.dtype), c=B.to_device(c_np, wl.dtype),
                              seq_lens=torch.tensor(ctx, dtype=torch.int32).cuda())
        out = torch.full((batch, width), float("nan"), dtype=x.dtype, device="cuda")
        if static:
            B.gta_decode_static(cfg, B.make_weights(wdev), x, batch, cache.struct, None, out, splits)
        else:
            ws = B.alloc_workspace(B.gta_workspace_bytes(cfg, B.GTA_MODE_DECODE, batch, 0, max_seq, splits))
            B.gta_decode(cfg, B.make_weights(wdev), x, batch, cache.struct, None, out, splits, ws)
        torch.cuda.synchronize()
        outs.append(out); caches.append(cache)
    sl = np.array(ctx, dtype=np.int32); st = np.zeros(batch, dtype=np.int32)
    kc, cc = k_np.astype(np.float64), c_np.astype(np.float64)
    ref = orc.decode(U.oracle_config(wl), U.oracle_weights(w), x_np, kc, cc, sl, st, list(range(batch)))
    what = f"{wl.name} batch {batch}"
    U.assert_close(U.f64(outs[1]), ref, wl.dtype, f"gta_decode_static vs oracle, {what}")
    U.assert_close(U.f64(outs[0]), ref, wl.dtype, f"gta_decode vs oracle, {what}")
    # same kernels, same launch configuration, fixed summation order: the two entry points agree bit for bit
    assert torch.equal(outs[0], outs[1]), f"gta_decode_static differs from gta_decode, {what}"
    assert torch.equal(caches[0].k, caches[1].k) and torch.equal(caches[0].c, caches[1].c)
    assert torch.equal(caches[0].seq_lens, caches[1].seq_lens)
    assert np.array_equal(caches[1].seq_lens.cpu().numpy(), sl)
    assert int(caches[1].status.abs().sum()) == 0
    for b in range(batch):   # the appended rows against the oracle's
        U.assert_close(U.f64(caches[1].k[b, ctx[b]]), kc[b, ctx[b]], wl.dtype, "appended key row")
        U.assert_close(U.f64(caches[1].c[b, ctx[b]]), cc[b, ctx[b]], wl.dtype, "appended latent row")


@pytest.mark.parametrize("shape", ["1b", "paper", "generic_f32"])
def test_decode_static_matches_decode_on_two_calls_in_a_row(shape):
    if shape == "1b":
        base, with_wo = W.WORKLOADS[2], False
    elif shape == "paper":
        base, with_wo = W.PAPER_WORKLOADS[1], True
    else:   # the shape-generic kernels, fp32
        base, with_wo = W.scaled(W.WORKLOADS[0], kind="decode"), False
    big = [0, 1, 7, 33, 255, 777, 1500, 1023, 64, 300, 1499, 5]
    small = [40, 3, 130]
    _one_step(W.scaled(base, batch=len(big), seqlen=max(big)), big, with_wo, 0)
    _one_step(W.scaled(base, batch=len(small), seqlen=max(small)), small, with_wo, 0)   # smaller, on dirty scratch
    _one_step(W.scaled(base, batch=len(small), seqlen=max(small)), small, with_wo, 3)


def test_decode_static_refuses_what_does_not_fit():
    """A call that needs more than the fixed array is refused with GTA_ERR_WORKSPACE and touches nothing."""
    wl = W.scaled(W.WORKLOADS[2], batch=2048, seqlen=8)
    cfg = B.config_of(wl)
    assert B.gta_workspace_bytes(cfg, B.GTA_MODE_DECODE, wl.batch, 0, 9, 0) > B.GTA_STATIC_SCRATCH_BYTES
    rng = W.make_rng(wl)
    w = W.draw_weights(wl, rng)
    wdev = U.upload_weights(w, wl.dtype)
    x = B.to_device(W.draw_hidden(wl, rng, wl.batch), wl.dtype)
    cache = U.DeviceCache(wl, wl.batch, 9, fill=-3.0)
    out = torch.full((wl.batch, wl.n_heads * wl.head_dim), float("nan"), dtype=x.dtype, device="cuda")
    rc = B.gta_decode_static(cfg, B.make_weights(wdev), x, wl.batch, cache.struct, None, out, 0, check=False)
    torch.cuda.synchronize()
    assert rc == B.GTA_ERR_WORKSPACE
    assert torch.isnan(out.float()).all() and int(cache.seq_lens.sum()) == 0
    assert bool((cache.k == -3.0).all()) and bool((cache.c == -3.0).all())
