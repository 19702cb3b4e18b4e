// Tuned bf16 path for gfx950: MFMA GEMMs, MFMA prefill attention, streaming split-K decode.
#pragma once
#include "gta_internal.h"

namespace gta {

bool tuned_prefill_supported(const Dims &d);
bool tuned_decode_supported(const Dims &d);
int tuned_decode_target_workgroups(const Dims &d);      // split-K launch size the kernel of this shape wants
int tuned_decode_max_splits(const Dims &d, int batch);   // most splits the cheapest tail kernel of this call takes
bool tuned_decode_layout_ok(const gta_cache &cache);   // block-table layouts the streaming decode kernels take
bool tuned_chunk_layout_ok(const gta_cache &cache);    // ... and the MFMA attention kernel in cache mode

int tuned_prefill(const Dims &d, const gta_weights &w, const void *x, const int32_t *cu, int batch,
                  int64_t total, int max_len, const gta_cache *cache, const int32_t *slots, void *out,
                  const PrefillWs &ws, hipStream_t st);
// chunked prefill: the chunk's tokens follow the rows the slots already hold (needs the MFMA attention kernel)
bool tuned_prefill_chunk_supported(const Dims &d, int max_seq);
int tuned_prefill_chunk(const Dims &d, const gta_weights &w, const void *x, const int32_t *cu, int batch,
                        int64_t total, int max_chunk, const gta_cache &cache, const int32_t *slots, void *out,
                        const PrefillWs &ws, hipStream_t st);
int tuned_decode(const Dims &d, const gta_weights &w, const void *x_new, int batch, const gta_cache &cache,
                 const int32_t *slots, void *out, const DecodeWs &ws, hipStream_t st);

void tuned_decode_attention(const Dims &d, const float *q, const int32_t *oldlen_in, int32_t *oldlen_out,
                            const gta_cache &cache, const int32_t *slots, int batch, int splits, float *part,
                            hipStream_t st);
void tuned_decode_combine(const Dims &d, const float *part, const int32_t *oldlen, int splits, int batch, float *L,
                          hipStream_t st);

// bf16 MFMA GEMMs (gta_gemm_bf16.hip)
bool gemm_shapes_supported(const Dims &d);
size_t proj_packed_bytes(const Dims &d);   // workspace for the packed [H, Wtot] weights, 0 if not used
int proj_small_ksplit(const Dims &d, int64_t M);   // > 0: M tokens take the short-prefill projection with this split
size_t proj_small_rows_bound(const Dims &d);       // rows of [.., W_tot] fp32 partials that path needs at most
void launch_proj_gemm(const Dims &d, const gta_weights &w, const void *x, int M, const PrefillWs &ws,
                      const gta_cache *cache, const int32_t *slots, int max_len, hipStream_t st,
                      bool rope_by_token = false);
void launch_decoder_gemm(const Dims &d, const void *L, const void *wp, const void *g, void *out, int M,
                         hipStream_t st);
int skinny_ksplit(const Dims &d, int M);
void launch_skinny_proj(const Dims &d, const gta_weights &w, const void *x, int M, float *part, int ksplit,
                        hipStream_t st);
void launch_plain_gemm(const void *A, int64_t lda, int M, int N, int K, const void *B, void *C, hipStream_t st);

// bf16 MFMA causal prefill attention (gta_prefill_bf16.hip)
bool attn_prefill_supported(const Dims &d, int max_len);
void launch_attn_prefill_bf16(const Dims &d, const void *q, const void *k, const void *c, const int32_t *cu,
                              int batch, int64_t total, int max_len, void *L, hipStream_t st);
// attention with the value decoder and gate fused into its epilogue (narrow shapes): writes the heads
bool attn_decoder_fusable(const Dims &d, int max_len);
void launch_attn_decoder_bf16(const Dims &d, const void *q, const void *k, const void *c, const int32_t *cu,
                              int batch, int64_t total, int max_len, const void *wp, const void *gate, void *out,
                              hipStream_t st);
// The same two against the caches: sequence b's keys / latents are rows 0 .. prefix[b] + T_b - 1 of its
// slot, its queries sit at positions prefix[b] .. (prefix[b] < 0: zero rows).  L may be NULL when fused.
void launch_attn_chunk_bf16(const Dims &d, const void *q, const gta_cache &cache, const int32_t *slots,
                            const int32_t *prefix, const int32_t *cu, int batch, int64_t total, int max_chunk,
                            void *L, const void *wp, const void *gate, void *out, bool fuse, hipStream_t st);

}  // namespace gta
