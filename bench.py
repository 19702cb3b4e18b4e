#!/usr/bin/env python3
"""Benchmark of the GTA attention pass on ONE MI355X: prints one JSON line.

The headline metric names two things, so both are measured in every run:
  * decode at 32K context (B=8, 32768 cached tokens, split-K): cache bytes streamed per second
    over the WHOLE gta_decode step and microseconds per generated token -- the line's `value`;
  * causal prefill of the 1B-class workload (B=4, T=4096, bf16): TFLOP/s of the whole
    gta_prefill call and fraction of the bf16 MFMA peak -- under the key "prefill".
The batched decode workload (B=64, 8192 cached tokens) is reported under "decode_b64_8k" and the
ragged packed prefill (16 sequences of 512..16384 tokens, H=4096, d_l=1024) under "varlen_prefill".
"chunked_prefill" is gta_prefill_chunk on the prefill workload's shape: 2048 new tokens per sequence behind
2048 cached ones.  "paper_layer_gta1b" holds one attention layer of the paper's own GTA-1B model (H=1280, 20 heads of 64
in 5 groups, one shared key, one latent of 128) at the batch sizes of its efficiency runs: prefill of
32 x 2048 tokens and a decode step at batch 64 with 2048 cached tokens.

A "step" is one library call (gta_decode or gta_prefill) on inputs already resident in HBM.
`roofline` objects are for the dominant kernel of each path, timed live with HIP events around
the stage entry point that launches exactly that kernel in the same configuration.
`cpu_baseline` is the fp64 oracle timed on the host cores of this machine on a stated sample.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA
PEAK_HBM_GBPS = 8000.0        # MI355X HBM3E

# HBM bytes per launch of a kernel, read from the committed rocprofv3 summaries (profiles/bench_*.txt:
# `--pmc FETCH_SIZE` and `--pmc WRITE_SIZE` runs of this file, each scaled by the reading for
# calibration_copy_kernel on a copy of known size; the summaries hold the commands and the raw
# readings).  Counters cannot be read from inside this process, so `traffic` is the recorded value of
# the profile that was last regenerated, never a live one: (summary file, kernel-name substring).
TRAFFIC_SOURCE = {
    ("decode_b8_32k_bf16", "decode_attn_kernel"): ("bench_decode32k.txt", "decode_attn_kernel"),
    ("decode_b64_8k_bf16", "decode_attn_kernel"): ("bench_decode8k.txt", "decode_attn_kernel"),
    ("decode_b512_2k_bf16", "decode_attn_kernel"): ("bench_decode512.txt", "decode_attn_kernel"),
    ("prefill_1b_bf16", "attn_prefill_kernel"): ("bench_prefill.txt", "attn_prefill_kernel"),
    ("prefill_1b_bf16", "projection"): ("bench_prefill.txt", "proj_gemm_kernel"),
    ("prefill_1b_bf16", "decoder"): ("bench_prefill.txt", "decoder_pair_kernel"),
    ("prefill_1b_bf16", "output_projection"): ("bench_prefill.txt", "plain_gemm_kernel"),
    ("varlen_prefill_bf16", "attn_prefill_kernel"): ("bench_varlen.txt", "attn_prefill_kernel"),
    ("varlen_prefill_bf16", "projection"): ("bench_varlen.txt", "proj_gemm_kernel"),
    ("varlen_prefill_bf16", "decoder"): ("bench_varlen.txt", "decoder_pair_kernel"),
    ("gta1b_prefill_b32_t2048", "attn_prefill_kernel"): ("bench_paper.txt", "AttnTile<64, 128>"),
    ("gta1b_decode_b64_t2048", "decode_attn_kernel"): ("bench_paper.txt", "decode_narrow_kernel"),
}


def recorded_traffic(workload, kernel):
    """fetch + write bytes per launch from the `fetch_MB_scaled write_MB_scaled` table of the summary, or None."""
    src = TRAFFIC_SOURCE.get((workload, kernel))
    if src is None:
        return None
    path = os.path.join(ROOT, "profiles", src[0])
    try:
        lines = open(path).read().splitlines()
    except OSError:
        return None
    in_table = False
    for ln in lines:
        if "fetch_MB_scaled" in ln and "write_MB_scaled" in ln:
            in_table = True
            continue
        if in_table:
            if not ln.strip():
                break
            if src[1] in ln:
                try:
                    f, w = (float(v) for v in ln.split()[-2:])
                except ValueError:
                    continue
                return (f + w) * 1e6
    return None


def _sync():
    import torch
    torch.cuda.synchronize()


def _time_steps(fn, steps, warmup):
    for i in range(warmup):
        fn(i)
    _sync()
    t0 = time.perf_counter()
    for i in range(steps):
        fn(warmup + i)
    _sync()
    return (time.perf_counter() - t0) / steps


def _event_time(fn, reps):
    """Average duration in seconds of one fn() launch: `reps` launches queued back to back between two
    HIP events on the current stream (the launches overlap their own submission latency, so the
    quotient is the kernel's duration plus the dispatch gap between consecutive kernels)."""
    import torch
    fn()
    _sync()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(reps):
        fn()
    b.record()
    _sync()
    return a.elapsed_time(b) / reps * 1e-3


def _event_median(fn, reps):
    """Median duration in seconds of one fn() launch, each launch between its own pair of HIP events."""
    import torch
    fn()
    _sync()
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
    for a, b in ev:
        a.record()
        fn()
        b.record()
    _sync()
    t = sorted(a.elapsed_time(b) for a, b in ev)
    return t[len(t) // 2] * 1e-3


def bench_decode(wl, steps, warmup, want_cpu_baseline):
    import numpy as np
    import torch
    from paper_2506_17286_amd import binding as B, workloads as W, costmodel as cm

    cfg = B.config_of(wl)
    rng = W.make_rng(wl)
    w = W.draw_weights(wl, rng)
    x_np = W.draw_hidden(wl, rng, wl.batch)
    wdev = {k: B.to_device(v, wl.dtype) for k, v in w.items()}
    gw = B.make_weights(wdev)
    x = B.to_device(x_np, wl.dtype)
    max_seq = wl.seqlen + steps + warmup + 8
    # two distinct cache allocations, alternated, so no step can be served from the Infinity Cache
    caches = []
    for salt in range(2):
        k, c = W.make_decode_cache_device(wl, max_seq, salt=salt)
        seq = torch.full((wl.batch,), wl.seqlen, dtype=torch.int32, device="cuda")
        st = torch.zeros(wl.batch, dtype=torch.int32, device="cuda")
        caches.append((k, c, seq, st, B.make_cache(k, c, seq, st)))
    out = torch.empty((wl.batch, wl.n_heads * wl.head_dim), dtype=x.dtype, device="cuda")
    ws = B.alloc_workspace(max(B.gta_workspace_bytes(cfg, B.GTA_MODE_DECODE, wl.batch, 0, m, 0)
                               for m in (max_seq, -(-max_seq // 64) * 64)))

    def step(i):
        B.gta_decode(cfg, gw, x, wl.batch, caches[i % 2][4], None, out, 0, ws)

    sec = _time_steps(step, steps, warmup)
    assert all(int(c[3].abs().sum()) == 0 for c in caches), "a cache slot overflowed"
    # context actually streamed in the timed steps: both caches advanced one row per call on them
    ctx = wl.seqlen + (warmup + steps) // 2
    cache_bytes = cm.decode_cache_bytes(wl, [ctx] * wl.batch)
    res = {
        "workload": wl.name, "batch": wl.batch, "context": wl.seqlen,
        "us_per_step": sec * 1e6, "us_per_token": sec * 1e6 / wl.batch,
        "tokens_per_s": wl.batch / sec, "cache_GBps": cache_bytes / sec / 1e9,
        "frac_hbm_peak_whole_step": cache_bytes / sec / 1e9 / PEAK_HBM_GBPS,
    }
    # dominant kernel: the split-K streaming attention kernel alone (stage entry point)
    q32 = torch.randn((wl.batch, wl.n_qgroups * wl.head_dim), device="cuda", dtype=torch.float32) * 0.9
    flip = [0]

    def attn_only():
        flip[0] ^= 1
        B.gta_decode_attention(cfg, q32, caches[flip[0]][4], None, wl.batch, 0, ws)

    ksec = _event_time(attn_only, max(steps, 10))
    kbytes = cm.decode_cache_bytes(wl, [int(caches[0][2][0])] * wl.batch)
    res["roofline"] = {"kernel": "decode_attn_kernel", "bound": "hbm", "achieved": kbytes / ksec / 1e9,
                       "peak": PEAK_HBM_GBPS, "unit": "GB/s", "frac": kbytes / ksec / 1e9 / PEAK_HBM_GBPS,
                       "traffic": recorded_traffic(wl.name, "decode_attn_kernel"),
                       "us_per_launch": ksec * 1e6, "us_per_launch_median": _event_median(attn_only, max(steps, 10)) * 1e6,
                       "algorithmic_bytes_per_launch": kbytes}
    if want_cpu_baseline:
        res["cpu_baseline"] = cpu_baseline_decode(wl, w, x_np, caches[0])
    # the same steps on block-table caches: pages of 64 rows dealt in random order over the pools
    ps = 64
    pps = -(-max_seq // ps)
    del caches
    paged = []
    for salt in range(2):
        k, c = W.make_decode_cache_device(wl, pps * ps, salt=salt)
        seq = torch.full((wl.batch,), wl.seqlen, dtype=torch.int32, device="cuda")
        st = torch.zeros(wl.batch, dtype=torch.int32, device="cuda")
        table = torch.from_numpy(np.random.default_rng(wl.seed + salt).permutation(wl.batch * pps)
                                 .astype(np.int32).reshape(wl.batch, pps)).cuda()
        kp, cp = k.view(wl.batch * pps, ps, -1), c.view(wl.batch * pps, ps, -1)
        paged.append((kp, cp, seq, st, table, B.make_paged_cache(kp, cp, seq, st, table)))

    def paged_step(i):
        B.gta_decode(cfg, gw, x, wl.batch, paged[i % 2][5], None, out, 0, ws)

    psec = _time_steps(paged_step, steps, warmup)
    assert all(int(c[3].abs().sum()) == 0 for c in paged), "a paged cache slot overflowed"
    res["paged"] = {"page_size": ps, "us_per_step": psec * 1e6, "cache_GBps": cache_bytes / psec / 1e9,
                    "vs_contiguous": sec / psec}
    return res


def bench_prefill(wl, steps, warmup, want_cpu_baseline, zero_operand_run=False):
    import numpy as np
    import torch
    from paper_2506_17286_amd import binding as B, workloads as W, costmodel as cm

    cfg = B.config_of(wl)
    lens, cu, w, x_np = W.prefill_inputs(wl)
    total = int(cu[-1])
    wdev = {k: B.to_device(v, wl.dtype) for k, v in w.items()}
    gw = B.make_weights(wdev)
    x = B.to_device(x_np, wl.dtype)
    max_seq = int(lens.max())
    kw, cw = wl.kv_width
    k = torch.zeros((wl.batch, max_seq, kw), dtype=x.dtype, device="cuda")
    c = torch.zeros((wl.batch, max_seq, cw), dtype=x.dtype, device="cuda")
    seq = torch.zeros(wl.batch, dtype=torch.int32, device="cuda")
    st = torch.zeros(wl.batch, dtype=torch.int32, device="cuda")
    cache = B.make_cache(k, c, seq, st)
    cud = torch.from_numpy(cu).cuda() if wl.min_seqlen is not None else None
    out = torch.empty((total, wl.n_heads * wl.head_dim), dtype=x.dtype, device="cuda")
    ws = B.alloc_workspace(B.gta_workspace_bytes(cfg, B.GTA_MODE_PREFILL, wl.batch, total, max_seq))

    def step(i):
        B.gta_prefill(cfg, gw, x, cud, wl.batch, total, max_seq, cache, None, out, ws)

    sec = _time_steps(step, steps, warmup)
    fl = cm.prefill_flops(wl, lens)
    res = {
        "workload": wl.name, "ms_per_step": sec * 1e3, "tokens_per_s": total / sec,
        "tflops": fl["total"] / sec / 1e12, "frac_mfma_peak_whole_call": fl["total"] / sec / 1e12 / PEAK_BF16_TFLOPS,
        "algorithmic_flops": fl,
    }
    # dominant kernel: the causal attention kernel alone (stage entry point), q/k/c of the
    # shapes and scale the projection produces
    qd = (torch.randn((total, wl.n_qgroups * wl.head_dim), device="cuda") * 0.9).to(x.dtype)
    kd = (torch.randn((total, kw), device="cuda") * 0.9).to(x.dtype)
    cd = (torch.randn((total, cw), device="cuda") * 0.9).to(x.dtype)
    ld = torch.empty((total, wl.n_qgroups * wl.latent_dim), dtype=x.dtype, device="cuda")

    def attn_only():
        B.gta_prefill_attention(cfg, qd, kd, cd, cud, wl.batch, total, max_seq, ld)

    reps = max(steps, 10)
    ksec = _event_time(attn_only, reps)
    res["roofline"] = {"kernel": "attn_prefill_kernel", "bound": "mfma", "achieved": fl["attn"] / ksec / 1e12,
                       "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": fl["attn"] / ksec / 1e12 / PEAK_BF16_TFLOPS,
                       "traffic": recorded_traffic(wl.name, "attn_prefill_kernel"),
                       "us_per_launch": ksec * 1e6, "us_per_launch_median": _event_median(attn_only, reps) * 1e6,
                       "algorithmic_flops_per_launch": fl["attn"]}
    # the same launch on all-zero operands: identical instruction stream and addresses, no operand bits
    # toggling -- how much of the kernel's time is the chip's power limit rather than its schedule
    # (left out of profiling runs, whose per-kernel averages must not mix the two)
    if zero_operand_run:
        zq, zk, zc = torch.zeros_like(qd), torch.zeros_like(kd), torch.zeros_like(cd)
        zsec = _event_time(lambda: B.gta_prefill_attention(cfg, zq, zk, zc, cud, wl.batch, total, max_seq, ld), reps)
        res["roofline"]["us_per_launch_on_zero_operands"] = zsec * 1e6
        del zq, zk, zc
    # the other kernels of the call, each alone through its stage entry point (same launch configuration
    # as inside gta_prefill): projection GEMM with RoPE, value-decoder GEMM with the gate, and the optional
    # output projection (not part of the timed gta_prefill call above, which runs without W_O)
    if B.gta_uses_tuned_kernels(cfg, B.GTA_MODE_PREFILL) == 1:
        gd = torch.empty((total, wl.n_heads * wl.head_dim), dtype=x.dtype, device="cuda")
        wo = (torch.randn((wl.n_heads * wl.head_dim, wl.d_model), device="cuda") * 0.02).to(x.dtype)
        gwo = B.make_weights(dict(wdev, wo=wo))
        uo = torch.empty((total, wl.d_model), dtype=x.dtype, device="cuda")
        fused = wl.head_dim == 64 and wl.latent_dim == 128 and wl.n_heads // wl.n_qgroups == 4   # decoder inside the attention kernel
        stages = {
            "projection": (lambda: B.gta_prefill_projection(cfg, gw, x, cud, wl.batch, total, max_seq, qd, kd, cd, gd, ws), fl["proj"]),
            **({} if fused else {"decoder": (lambda: B.gta_prefill_decoder(cfg, gw, ld, gd, total, out), fl["decoder"])}),
            "output_projection": (lambda: B.gta_output_projection(cfg, gwo, out, total, uo),
                                  2 * total * wl.n_heads * wl.head_dim * wl.d_model),
        }
        ker = {}
        for name, (fn, flops) in stages.items():
            sec_k = _event_time(fn, reps)
            ker[name] = {"bound": "mfma", "achieved": flops / sec_k / 1e12, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                         "frac": flops / sec_k / 1e12 / PEAK_BF16_TFLOPS, "us_per_launch": sec_k * 1e6,
                         "us_per_launch_median": _event_median(fn, reps) * 1e6, "algorithmic_flops_per_launch": flops,
                         "traffic": recorded_traffic(wl.name, name)}
        res["kernels"] = ker
    if want_cpu_baseline:
        res["cpu_baseline"] = cpu_baseline_prefill(wl, w, x_np, lens, cu)
    return res


def bench_prefill_chunk(wl, prefix, steps, warmup):
    """Chunked prefill: every slot already holds `prefix` tokens, one call adds the remaining seqlen - prefix
    tokens of every sequence (gta_prefill_chunk).  Flops: projections and decoder of the chunk's tokens, the
    causal pairs the chunk's rows have with the whole sequence."""
    import numpy as np
    import torch
    from paper_2506_17286_amd import binding as B, workloads as W, costmodel as cm
    cfg = B.config_of(wl)
    lens, cu, w, x_np = W.prefill_inputs(wl)
    wdev = {k: B.to_device(v, wl.dtype) for k, v in w.items()}
    gw = B.make_weights(wdev)
    T, n = wl.seqlen, wl.seqlen - prefix
    x = B.to_device(x_np, wl.dtype).view(wl.batch, T, wl.d_model)
    xp, xc = x[:, :prefix].reshape(-1, wl.d_model).contiguous(), x[:, prefix:].reshape(-1, wl.d_model).contiguous()
    kw, cw = wl.kv_width
    k = torch.zeros((wl.batch, T, kw), dtype=x.dtype, device="cuda")
    c = torch.zeros((wl.batch, T, cw), dtype=x.dtype, device="cuda")
    seq = torch.zeros(wl.batch, dtype=torch.int32, device="cuda")
    st = torch.zeros(wl.batch, dtype=torch.int32, device="cuda")
    cache = B.make_cache(k, c, seq, st)
    outp = torch.empty((wl.batch * prefix, wl.n_heads * wl.head_dim), dtype=x.dtype, device="cuda")
    outc = torch.empty((wl.batch * n, wl.n_heads * wl.head_dim), dtype=x.dtype, device="cuda")
    ws = B.alloc_workspace(max(B.gta_workspace_bytes(cfg, B.GTA_MODE_PREFILL, wl.batch, wl.batch * prefix, prefix),
                               B.gta_workspace_bytes(cfg, B.GTA_MODE_PREFILL_CHUNK, wl.batch, wl.batch * n, n)))
    B.gta_prefill(cfg, gw, xp, None, wl.batch, wl.batch * prefix, prefix, cache, None, outp, ws)

    def step(i):
        seq.fill_(prefix)          # every timed call starts from the same prefix (a tiny fill kernel)
        B.gta_prefill_chunk(cfg, gw, xc, None, wl.batch, wl.batch * n, n, cache, None, outc, ws)

    sec = _time_steps(step, steps, warmup)
    assert int(st.abs().sum()) == 0 and int(seq[0]) == T
    pairs = wl.batch * (n * prefix + n * (n + 1) // 2)
    tok = wl.batch * n
    wtot = (wl.n_qgroups + wl.n_kgroups) * wl.head_dim + wl.n_cgroups * wl.latent_dim + wl.n_heads * wl.head_dim
    fl = 2 * tok * wl.d_model * wtot + 2 * wl.n_qgroups * (wl.head_dim + wl.latent_dim) * pairs \
        + 2 * tok * wl.n_heads * wl.latent_dim * wl.head_dim
    return {"workload": f"{wl.name}: {prefix} cached + {n} new tokens per sequence", "ms_per_step": sec * 1e3,
            "tokens_per_s": tok / sec, "tflops": fl / sec / 1e12, "algorithmic_flops": fl}


def bench_attention_comparator(steps):
    """Causal attention stage alone (gta_prefill_attention) at 32 x 2048 tokens for the paper's GTA-1B layer
    and for the GQA-1B layer written as the degenerate GTA setting (one map per head, 5 key and 5 value
    groups, latent width = head width): the measured counterpart of the paper's attention-compute ratio."""
    import torch
    from paper_2506_17286_amd import binding as B, workloads as W, costmodel as cm
    gta = W.by_name("gta1b_prefill_b32_t2048")
    gqa = W.scaled(gta, name="gqa1b_as_degenerate_gta", n_qgroups=20, n_kgroups=5, n_cgroups=5, latent_dim=64)
    res = {}
    for wl in (gta, gqa):
        cfg = B.config_of(wl)
        total = wl.batch * wl.seqlen
        kw, cw = wl.kv_width
        mk = lambda n: (torch.randn((total, n), device="cuda") * 0.9).to(torch.bfloat16)
        q, k, c = mk(wl.n_qgroups * wl.head_dim), mk(kw), mk(cw)
        out = torch.empty((total, wl.n_qgroups * wl.latent_dim), dtype=torch.bfloat16, device="cuda")
        sec = _event_time(lambda: B.gta_prefill_attention(cfg, q, k, c, None, wl.batch, total, wl.seqlen, out), max(steps, 10))
        fl = cm.prefill_flops(wl, [wl.seqlen] * wl.batch)["attn"]
        res[wl.name] = {"us": sec * 1e6, "algorithmic_flops": fl, "tflops": fl / sec / 1e12,
                        "cache_bytes_per_token": (kw + cw) * 2}
    a, b = res[gta.name], res[gqa.name]
    res["gta_over_gqa"] = {"time": a["us"] / b["us"], "attention_flops": a["algorithmic_flops"] / b["algorithmic_flops"],
                           "cache_bytes": a["cache_bytes_per_token"] / b["cache_bytes_per_token"]}
    return res


def bench_paper_grid(steps, warmup):
    """The batch / length grid of the paper's efficiency runs on one attention layer of its 1B models
    (Sec. 5.3, App. C.2: prefill of 32 sequences of 128 / 512 / 1024 / 2048 tokens; 128 tokens generated at
    batch 64), whole calls WITH the output projection: GTA-1B (20 heads of 64, 5 maps, one key, one latent
    of 128) next to GQA-1B written as the degenerate setting (20 maps, 5 key and 5 value groups, latent
    as wide as a head, gate off).  The GQA decode step has no tuned kernel here (shape-generic path)."""
    import numpy as np
    import torch
    from paper_2506_17286_amd import binding as B, workloads as W
    gta = W.by_name("gta1b_prefill_b32_t2048")
    gqa = W.scaled(gta, name="gqa1b_as_degenerate_gta", n_qgroups=20, n_kgroups=5, n_cgroups=5, latent_dim=64)
    res = {}
    for wl, gate in ((gta, True), (gqa, False)):
        cfg = B.config_of(wl)
        cfg.gate = B.GATE_CODES[gate]
        rng = W.make_rng(wl)
        w = W.draw_weights(wl, rng, with_wo=True)
        wdev = {k: B.to_device(v, wl.dtype) for k, v in w.items()}
        gw = B.make_weights(wdev)
        kw, cw = wl.kv_width
        entry = {"cache_bytes_per_token": (kw + cw) * 2, "prefill_b32": {}}
        for T in (128, 512, 1024, 2048):
            total = 32 * T
            x = torch.randn((total, wl.d_model), device="cuda").to(torch.bfloat16)
            k = torch.zeros((32, T, kw), dtype=torch.bfloat16, device="cuda")
            c = torch.zeros((32, T, cw), dtype=torch.bfloat16, device="cuda")
            seq = torch.zeros(32, dtype=torch.int32, device="cuda"); st = torch.zeros(32, dtype=torch.int32, device="cuda")
            cache = B.make_cache(k, c, seq, st)
            out = torch.empty((total, wl.d_model), dtype=torch.bfloat16, device="cuda")
            ws = B.alloc_workspace(B.gta_workspace_bytes(cfg, B.GTA_MODE_PREFILL, 32, total, T))
            sec = _time_steps(lambda i: B.gta_prefill(cfg, gw, x, None, 32, total, T, cache, None, out, ws), steps, warmup)
            entry["prefill_b32"][str(T)] = {"ms": sec * 1e3, "tokens_per_s": total / sec}
        # 128 consecutive decode steps at batch 64 behind 2048 cached tokens
        dw = W.scaled(wl, kind="decode", batch=64, seqlen=2048)
        n_gen = 128
        k, c = W.make_decode_cache_device(dw, 2048 + n_gen + 8)
        seq = torch.full((64,), 2048, dtype=torch.int32, device="cuda"); st = torch.zeros(64, dtype=torch.int32, device="cuda")
        cache = B.make_cache(k, c, seq, st)
        x = torch.randn((64, wl.d_model), device="cuda").to(torch.bfloat16)
        out = torch.empty((64, wl.d_model), dtype=torch.bfloat16, device="cuda")
        ws = B.alloc_workspace(B.gta_workspace_bytes(cfg, B.GTA_MODE_DECODE, 64, 0, 2048 + n_gen + 8, 0))
        for _ in range(3):
            B.gta_decode(cfg, gw, x, 64, cache, None, out, 0, ws)
        seq.fill_(2048)
        _sync()
        t0 = time.perf_counter()
        for _ in range(n_gen):
            B.gta_decode(cfg, gw, x, 64, cache, None, out, 0, ws)
        _sync()
        sec = time.perf_counter() - t0
        assert int(st.abs().sum()) == 0 and int(seq[0]) == 2048 + n_gen
        entry["decode_b64_128_tokens"] = {"ms_total": sec * 1e3, "us_per_step": sec / n_gen * 1e6,
                                          "tokens_per_s": 64 * n_gen / sec,
                                          "tuned_kernels": B.gta_uses_tuned_kernels(cfg, B.GTA_MODE_DECODE) == 1}
        res[wl.name] = entry
    a, b = res[gta.name], res[gqa.name]
    res["gta_over_gqa_time"] = {**{f"prefill_b32_{T}": a["prefill_b32"][T]["ms"] / b["prefill_b32"][T]["ms"] for T in a["prefill_b32"]},
                                "decode_b64_128_tokens": a["decode_b64_128_tokens"]["ms_total"] / b["decode_b64_128_tokens"]["ms_total"],
                                "cache_bytes": a["cache_bytes_per_token"] / b["cache_bytes_per_token"]}
    return res


def _blas_threads():
    try:
        from threadpoolctl import threadpool_info
        n = [p.get("num_threads", 1) for p in threadpool_info() if p.get("user_api") == "blas"]
        return max(n) if n else 1
    except Exception:
        return 1


def cpu_baseline_decode(wl, w, x_np, cache0, budget_s=12.0):
    """The oracle's decode step on the same workload (every sequence), host cores of this machine; the
    step is repeated until about `budget_s` seconds of oracle time have been spent."""
    import numpy as np
    import torch
    from oracle import gta_oracle as orc
    from paper_2506_17286_amd import costmodel as cm
    cfg = orc.OracleConfig(wl.d_model, wl.n_heads, wl.n_qgroups, wl.n_kgroups, wl.n_cgroups, wl.head_dim,
                           wl.latent_dim, rope=wl.rope, rope_base=wl.rope_base)
    ow = orc.OracleWeights(w["wq"], w["wk"], w["wc"], w["wg"], w["wp"]).f64()
    k, c, seq = cache0[0], cache0[1], cache0[2]
    seqs = []
    for b in range(wl.batch):   # fp64 host copies, made once, outside the timed region
        n = int(seq[b])
        seqs.append((n, k[b:b + 1, :n + 1].to(torch.float64).cpu().numpy(), c[b:b + 1, :n + 1].to(torch.float64).cpu().numpy()))
    t = 0.0
    rows = 0
    reps = 0
    while t < budget_s and reps < 400:
        for b, (n, kc, cc) in enumerate(seqs):
            sl = np.array([n], dtype=np.int32); stt = np.zeros(1, dtype=np.int32)
            t0 = time.perf_counter()
            orc.decode(cfg, ow, x_np[b:b + 1], kc, cc, sl, stt, [0])
            t += time.perf_counter() - t0
            rows += n + 1
        reps += 1
    by = cm.decode_cache_bytes(wl, [rows])
    return {"value": by / t / 1e9, "unit": "GB/s", "cores": _blas_threads(), "kind": "oracle",
            "sample": f"oracle decode step of all {wl.batch} sequences, repeated {reps} times ({rows} cached rows in "
                      f"all, fp64 copies of the same cache made outside the timed region; bytes counted at the "
                      f"bf16 cache size), {t:.2f} s of oracle time"}


def cpu_baseline_prefill(wl, w, x_np, lens, cu, budget_s=12.0):
    """The oracle's prefill of whole sequences of the same workload until about `budget_s` seconds."""
    import numpy as np
    from oracle import gta_oracle as orc
    from paper_2506_17286_amd import costmodel as cm
    cfg = orc.OracleConfig(wl.d_model, wl.n_heads, wl.n_qgroups, wl.n_kgroups, wl.n_cgroups, wl.head_dim,
                           wl.latent_dim, rope=wl.rope, rope_base=wl.rope_base)
    ow = orc.OracleWeights(w["wq"], w["wk"], w["wc"], w["wg"], w["wp"]).f64()
    t = 0.0
    done = []
    i = 0
    while t < budget_s and i < 4 * wl.batch:
        b = i % wl.batch
        t0 = time.perf_counter()
        orc.prefill_sequence(cfg, ow, x_np[cu[b]:cu[b + 1]])
        t += time.perf_counter() - t0
        done.append(int(lens[b]))
        i += 1
    fl = cm.prefill_flops(wl, done)["total"]
    return {"value": fl / t / 1e12, "unit": "TFLOP/s", "cores": _blas_threads(), "kind": "oracle",
            "sample": f"oracle prefill of {len(done)} whole sequences (the {wl.batch} of the workload, cycled; "
                      f"T={done[0]}, every row; algorithmic flops of those sequences / wall time), {t:.2f} s"}


def measured_ceilings():
    """What this GPU sustains on kernels that do nothing but the bounding operation: a streaming read of
    512 MiB and back-to-back bf16 MFMAs.  Context for the roofline fractions, which stay relative to
    the published peaks."""
    import torch
    from paper_2506_17286_amd import binding as B
    sink = torch.zeros(1024, dtype=torch.uint8, device="cuda")
    nbytes = 512 << 20
    bufs = [torch.ones(nbytes, dtype=torch.uint8, device="cuda") for _ in range(2)]
    flip = [0]

    def rd():
        flip[0] ^= 1
        B.gta_calibration_read(bufs[flip[0]], nbytes, 512, sink)

    t_rd = _event_time(rd, 20)
    del bufs
    wgs, iters = 1024, 2000
    fl = wgs * 4 * iters * 16 * 32768.0
    t_mm = _event_time(lambda: B.gta_calibration_mfma(wgs, iters, False, sink), 5)
    t_mr = _event_time(lambda: B.gta_calibration_mfma(wgs, iters, True, sink), 5)
    return {"hbm_read_GBps": nbytes / t_rd / 1e9, "hbm_read_frac_of_peak": nbytes / t_rd / 1e9 / PEAK_HBM_GBPS,
            "mfma_bf16_TFLOPs": fl / t_mr / 1e12, "mfma_bf16_frac_of_peak": fl / t_mr / 1e12 / PEAK_BF16_TFLOPS,
            "mfma_bf16_constant_operands_TFLOPs": fl / t_mm / 1e12,
            "what": "gta_calibration_read (512 MiB, 512 workgroups, non-temporal loads) and gta_calibration_mfma "
                    "(1024 workgroups x 4 waves x 32000 v_mfma_f32_32x32x16_bf16, nothing else; operands spread like "
                    "activations and weights and rotating, which is what mfma_bf16_TFLOPs is, and one constant pair), timed here"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--only", choices=["decode32k", "decode8k", "decode512", "prefill", "chunk", "varlen", "paper"], default=None,
                    help="measure one workload only (profiling runs)")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run calibration_copy_kernel once on 512 MiB (reads 512 MiB, writes 512 MiB): "
                         "the reference the FETCH_SIZE / WRITE_SIZE counters of a --pmc run are scaled by")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no collectives, no sharding): use --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2506_17286_amd import binding as B, workloads as W
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    B.load()   # fails loudly if the HIP library is not built
    torch.cuda.set_device(0)
    cpu = not args.no_cpu_baseline
    if args.calibration_copy:
        src = torch.ones(512 << 20, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        B.gta_calibration_copy(src, dst, 512 << 20)
        torch.cuda.synchronize()
        del src, dst
    dec = pre = dec8 = var = pap = None
    if args.only in (None, "decode32k"):
        dec = bench_decode(W.by_name("decode_b8_32k_bf16"), args.steps, args.warmup, cpu)
    if args.only in (None, "prefill"):
        pre = bench_prefill(W.by_name("prefill_1b_bf16"), args.steps, args.warmup, cpu, zero_operand_run=args.only is None)
    if args.only in (None, "decode8k"):
        dec8 = bench_decode(W.by_name("decode_b64_8k_bf16"), args.steps, args.warmup, False)
    dec512 = None
    if args.only in (None, "decode512"):   # a serving-size batch: 512 sequences with 2048 cached tokens each
        dec512 = bench_decode(W.scaled(W.by_name("decode_b64_8k_bf16"), batch=512, seqlen=2048, name="decode_b512_2k_bf16"),
                              args.steps, args.warmup, False)
    chk = None
    if args.only in (None, "chunk"):    # second half of every sequence of the prefill workload behind the first
        chk = bench_prefill_chunk(W.by_name("prefill_1b_bf16"), 2048, args.steps, args.warmup)
    short = None
    if args.only in (None, "chunk"):    # latency of short prompts: one sequence of 128 / 512 / 1024 tokens, 1B shape
        short = {}
        for T in (128, 512, 1024):
            r = bench_prefill(W.scaled(W.by_name("prefill_1b_bf16"), batch=1, seqlen=T, name=f"prefill_1b_1x{T}"),
                              args.steps, args.warmup, False)
            short[f"1x{T}"] = {"us_per_call": r["ms_per_step"] * 1e3, "tflops": r["tflops"]}
    if args.only in (None, "varlen"):   # ragged packed batch, 16 sequences of 512..16384 tokens, wider model
        var = bench_prefill(W.by_name("varlen_prefill_bf16"), min(args.steps, 10), min(args.warmup, 3), False,
                            zero_operand_run=args.only is None)
    if args.only in (None, "paper"):    # one attention layer of the paper's GTA-1B model (heads of 64, d_l = 128)
        pap = {"prefill": bench_prefill(W.by_name("gta1b_prefill_b32_t2048"), args.steps, args.warmup, False),
               "decode": bench_decode(W.by_name("gta1b_decode_b64_t2048"), args.steps, args.warmup, False)}
        pap["prefill"]["roofline"]["kernel"] = "attn_prefill_kernel (heads of 64, latent 128)"
        pap["decode"]["roofline"]["kernel"] = "decode_narrow_kernel"
        pap["attention_vs_gqa"] = bench_attention_comparator(args.steps)
        pap["efficiency_grid"] = bench_paper_grid(min(args.steps, 10), min(args.warmup, 3))
    main_res = dec or pre or dec8 or dec512 or var or (pap["prefill"] if pap else None)
    if main_res is None:   # --only chunk: the chunked figure alone
        print(json.dumps({"chunked_prefill": chk, "short_prefill_1b": short}))
        return
    line = {
        "metric": "GTA decode HBM GB/s & us/token @32K ctx; prefill bf16 TFLOP/s (% of peak)",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
    }
    if main_res is dec or main_res is dec8 or main_res is dec512:
        line.update({"value": main_res["cache_GBps"], "unit": "GB/s", "ms_per_step": main_res["us_per_step"] / 1e3,
                     "us_per_token": main_res["us_per_token"],
                     "config": {"workload": main_res["workload"], "batch": main_res["batch"],
                                "context": main_res["context"], "value_is": "cache bytes / whole gta_decode step"}})
    else:
        line.update({"value": main_res["tflops"], "unit": "TFLOP/s", "ms_per_step": main_res["ms_per_step"],
                     "config": {"workload": main_res["workload"], "value_is": "algorithmic flops / whole gta_prefill call"}})
    line["roofline"] = main_res["roofline"]
    if "paged" in main_res:
        line["paged_caches"] = main_res["paged"]
    line["measured_ceilings"] = mc = measured_ceilings()
    # the same fractions against what this GPU sustained in this run (clock under load), next to the published peaks
    for r in [line["roofline"]] + [v["roofline"] for v in (pre, dec8, dec512, var) if v is not None and v is not main_res]:
        ceil = mc["mfma_bf16_TFLOPs"] if r["bound"] == "mfma" else mc["hbm_read_GBps"]
        r["frac_of_measured_ceiling"] = r["achieved"] / ceil
    if "cpu_baseline" in main_res:
        line["cpu_baseline"] = main_res.pop("cpu_baseline")
    if pre is not None and main_res is not pre:
        line["prefill"] = pre
    if dec8 is not None and main_res is not dec8:
        line["decode_b64_8k"] = dec8
    if dec512 is not None and main_res is not dec512:
        line["decode_b512_2k"] = dec512
    if var is not None and main_res is not var:
        line["varlen_prefill"] = var
    if chk is not None:
        line["chunked_prefill"] = chk
    if short is not None:
        line["short_prefill_1b"] = short
    if pap is not None:
        line["paper_layer_gta1b"] = pap if main_res is not pap["prefill"] else {k: v for k, v in pap.items() if k != "prefill"}
    print(json.dumps(line))


if __name__ == "__main__":
    main()
