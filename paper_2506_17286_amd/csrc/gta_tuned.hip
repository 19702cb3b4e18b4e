// Orchestration of the tuned bf16 prefill: which kernels run, in which order, on which buffers.
#include "gta_tuned.h"

namespace gta {

bool tuned_prefill_supported(const Dims &d) { return gemm_shapes_supported(d); }

int tuned_prefill(const Dims &d, const gta_weights &w, const void *x, const int32_t *cu, int batch, int64_t total,
                  int max_len, const gta_cache *cache, const int32_t *slots, void *out, const PrefillWs &ws,
                  hipStream_t st) {
  const int M = (int)total;
  launch_prefill_setup(d, cu, batch, total, max_len, ws.seq_id, ws.pos, ws.rope, cache, slots, st);
  // Sec. 3.2 projections + App. B.1.1 RoPE + cache write, one MFMA GEMM
  launch_proj_gemm(d, w, x, M, ws, cache, slots, max_len, st);
  void *heads = w.wo ? ws.o : out;   // gated heads [M, n_h*d_h]
  if (attn_decoder_fusable(d, max_len)) {
    // Sec. 3.3 with the Sec. 3.2 value decoder and gate in the attention kernel's epilogue
    launch_attn_decoder_bf16(d, ws.q, ws.k, ws.c, cu, batch, total, max_len, w.wp, ws.g, heads, st);
  } else {
    // Sec. 3.3: one causal softmax map per group applied to the latent values
    if (attn_prefill_supported(d, max_len)) launch_attn_prefill_bf16(d, ws.q, ws.k, ws.c, cu, batch, total, max_len, ws.l, st);
    else launch_attn_prefill_rowwise(d, ws.q, ws.k, ws.c, cu, batch, total, max_len, ws.l, st);
    // Sec. 3.2 value decoder with the gate in the epilogue
    launch_decoder_gemm(d, ws.l, w.wp, ws.g, heads, M, st);
  }
  if (w.wo) launch_plain_gemm(ws.o, d.wg_w, M, d.H, d.wg_w, w.wo, out, st);   // Sec. 3.3 output projection
  return check_launch();
}

bool tuned_prefill_chunk_supported(const Dims &d, int max_seq) {
  return tuned_prefill_supported(d) && attn_prefill_supported(d, max_seq);
}

// a 32-row key tile of the attention kernel must not straddle pages
bool tuned_chunk_layout_ok(const gta_cache &cache) {
  if (!cache.block_table) return true;
  const int ps = cache.page_size;
  return ps >= 32 && (ps & (ps - 1)) == 0;
}

// Chunked prefill: App. B.1.3 for several new tokens per sequence.  The projection stores the chunk's
// key / latent rows behind the cached ones; attention then reads keys and latents from the caches.
int tuned_prefill_chunk(const Dims &d, const gta_weights &w, const void *x, const int32_t *cu, int batch,
                        int64_t total, int max_chunk, const gta_cache &cache, const int32_t *slots, void *out,
                        const PrefillWs &ws, hipStream_t st) {
  const int M = (int)total;
  launch_prefill_chunk_setup(d, cu, batch, total, ws.seq_id, ws.pos, ws.rope, ws.prefix, cache, slots, st);
  launch_proj_gemm(d, w, x, M, ws, &cache, slots, max_chunk, st, true);
  void *heads = w.wo ? ws.o : out;
  const bool fuse = attn_decoder_fusable(d, cache.max_seq);
  launch_attn_chunk_bf16(d, ws.q, cache, slots, ws.prefix, cu, batch, total, max_chunk, ws.l, w.wp, ws.g, heads, fuse, st);
  if (!fuse) launch_decoder_gemm(d, ws.l, w.wp, ws.g, heads, M, st);
  if (w.wo) launch_plain_gemm(ws.o, d.wg_w, M, d.H, d.wg_w, w.wo, out, st);
  launch_prefill_chunk_commit(cache, slots, cu, batch, total, ws.prefix, st);
  return check_launch();
}

}  // namespace gta
