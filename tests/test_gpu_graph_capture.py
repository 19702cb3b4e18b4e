"""A decode step recorded into a HIP graph: the library allocates nothing, never synchronises and
keeps all per-step state (cached lengths, new rows) in device memory, so a captured gta_decode can be
replayed step after step.  Every replay is checked against the same step run eagerly on a copy of
the caches, with ordinary eager work and synchronisations between the replays."""
import numpy as np
import pytest
import torch

from paper_2506_17286_amd import binding as B
from paper_2506_17286_amd import workloads as W

import gpu_util as U

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("shape,page", [("1b", 0), ("paper", 0), ("1b", 64), ("paper", 16)])
def test_decode_step_replays_from_a_graph(shape, page):
    """page > 0: the graphed caches are block-table caches (pages in random order), the eager ones contiguous."""
    base = W.WORKLOADS[2] if shape == "1b" else W.PAPER_WORKLOADS[1]
    ctx = [40, 3, 300, 129]
    wl = W.scaled(base, batch=len(ctx), seqlen=max(ctx))
    rng = W.make_rng(wl)
    w = W.draw_weights(wl, rng)
    wdev = U.upload_weights(w, wl.dtype)
    gw = B.make_weights(wdev)
    cfg = B.config_of(wl)
    max_seq = 320
    k_np, c_np = W.draw_cache(wl, rng, wl.batch, max_seq)

    def fresh_cache():
        return U.DeviceCache(wl, wl.batch, max_seq, k=B.to_device(k_np, wl.dtype), c=B.to_device(c_np, wl.dtype),
                             seq_lens=torch.tensor(ctx, dtype=torch.int32).cuda())

    eager, graphed = fresh_cache(), fresh_cache()
    if page:
        flat = graphed
        graphed = U.PagedDeviceCache(wl, wl.batch, page, max_seq // page, seed=page)
        graphed.store(flat.k, flat.c)
        graphed.seq_lens.copy_(flat.seq_lens)
    xs = [B.to_device(W.draw_hidden(wl, rng, wl.batch), wl.dtype) for _ in range(4)]
    x_in = torch.empty_like(xs[0])          # the graph reads its input from this fixed buffer
    out_g = torch.zeros((wl.batch, wl.n_heads * wl.head_dim), dtype=x_in.dtype, device="cuda")
    out_e = torch.zeros_like(out_g)
    ws_g = B.alloc_workspace(B.gta_workspace_bytes(cfg, B.GTA_MODE_DECODE, wl.batch, 0, max_seq, 0))
    ws_e = B.alloc_workspace(B.gta_workspace_bytes(cfg, B.GTA_MODE_DECODE, wl.batch, 0, max_seq, 0))
    # one eager step first (on a third copy): kernel attributes are set outside the capture
    warm = fresh_cache()
    B.gta_decode(cfg, gw, xs[0], wl.batch, warm.struct, None, out_e, 0, ws_e)
    torch.cuda.synchronize()

    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        x_in.copy_(xs[0])
        torch.cuda.synchronize()
        with torch.cuda.graph(graph, stream=side):
            B.gta_decode(cfg, gw, x_in, wl.batch, graphed.struct, None, out_g, 0, ws_g, stream=side)
    torch.cuda.synchronize()
    assert graphed.seq_lens.cpu().tolist() == ctx      # capturing ran nothing

    for step in range(4):
        x_in.copy_(xs[step])
        graph.replay()
        B.gta_decode(cfg, gw, xs[step], wl.batch, eager.struct, None, out_e, 0, ws_e)
        torch.cuda.synchronize()
        assert torch.equal(out_g, out_e), f"replay {step} differs from the eager step"
        assert graphed.seq_lens.cpu().tolist() == [n + step + 1 for n in ctx]
        gk, gc = graphed.logical() if page else (graphed.k, graphed.c)
        assert torch.equal(gk, eager.k) and torch.equal(gc, eager.c)
        # unrelated eager work between the replays
        _ = (out_e.float() @ out_e.float().T).sum().item()
