/*
 * libgta -- Grouped-head latenT Attention (GTA, arXiv 2506.17286) attention forward pass for
 * AMD MI355X (gfx950).  C ABI: plain structs, plain pointers, sizes; no C++ or framework types.
 *
 * Notation follows the paper (Sec. 3.2): H = d_model, n_h heads, n_q attention-map (query)
 * groups, n_k key groups, n_c latent-value groups, d_h head dim, d_l latent dim (d_l >= d_h).
 * Row-vector convention: projections are x . W with W stored row-major [in, out].
 *
 * Group maps (the paper leaves q(i), k(i), c(i) open; contiguous blocks are used):
 *   q(i) = i / (n_h / n_q),   k(g) = g / (n_q / n_k),   c(g) = g / (n_q / n_c),
 * so n_k | n_q | n_h and n_c | n_q are required.
 *
 * Conventions for every entry point
 *   - Pointers marked "device" are HIP device memory owned by the caller, 16-byte aligned,
 *     dense row-major.  Config/weight/cache structs are host memory, read only during the call.
 *   - The library allocates, frees and retains nothing.  Scratch memory comes in through
 *     `workspace` (device), sized by gta_workspace_bytes(); gta_decode_static uses a fixed array
 *     inside the library instead.
 *   - All work is enqueued on `hip_stream` (a hipStream_t passed as void*; NULL = the null
 *     stream).  No call synchronises with the host.
 *   - Return value: GTA_OK or a negative gta_status.  On a host-detected error nothing has been
 *     enqueued or written.  A sequence whose new rows would not fit its cache slot is detected on
 *     the device and cache->status[slot] is set to GTA_ERR_CACHE_FULL.  gta_decode,
 *     gta_prefill_chunk and gta_cache_append then leave the slot as it was (no row stored, length
 *     unchanged) and the first two zero-fill the sequence's output rows.  (gta_prefill refuses
 *     max_seqlen > cache->max_seq on the host; a slot whose block table lacks a page for some row
 *     is flagged, its length is still set, rows without a page are not stored and the output rows
 *     are computed as usual.)
 *   - Re-entrant.  Two calls that touch the same cache slot, output or workspace must be ordered
 *     by the caller (same stream or events).  The only process state is a table of "this kernel may
 *     use more than 64 KiB of LDS on this device" attributes, set idempotently on the first launch of
 *     such a kernel per device (and the scratch address of gta_decode_static): make the first call of
 *     each entry point and shape on a device OUTSIDE stream capture; later calls may be captured.
 */
#ifndef GTA_H_
#define GTA_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define GTA_API __attribute__((visibility("default")))

typedef enum {
  GTA_OK = 0,
  GTA_ERR_NULL = -1,        /* a required pointer is NULL */
  GTA_ERR_SHAPE = -2,       /* divisibility / range violation (n_q % n_k, d_l < d_h, batch <= 0 ...) */
  GTA_ERR_ALIGN = -3,       /* a device pointer is not 16-byte aligned */
  GTA_ERR_DTYPE = -4,       /* unknown dtype / gate / rope code */
  GTA_ERR_UNSUPPORTED = -5, /* dimensions outside what the kernels handle */
  GTA_ERR_WORKSPACE = -6,   /* workspace NULL or smaller than gta_workspace_bytes() */
  GTA_ERR_HIP = -7,         /* a kernel launch failed (hipGetLastError) */
  GTA_ERR_CACHE_FULL = -8   /* device-side: written to cache->status[slot] */
} gta_status;

enum { GTA_F32 = 0, GTA_BF16 = 1 };            /* gta_config.dtype */
enum { GTA_GATE_SIGMOID = 0, GTA_GATE_OFF = 1, GTA_GATE_SILU = 2, GTA_GATE_RELU2 = 3 }; /* gta_config.gate  */
enum { GTA_MODE_PREFILL = 0, GTA_MODE_DECODE = 1, GTA_MODE_PREFILL_CHUNK = 2 };

/* Hyper-parameters of one GTA layer (Sec. 3.2).  Host memory. */
typedef struct {
  int32_t d_model;       /* H */
  int32_t n_heads;       /* n_h */
  int32_t n_qgroups;     /* n_q: attention maps per token */
  int32_t n_kgroups;     /* n_k */
  int32_t n_cgroups;     /* n_c */
  int32_t head_dim;      /* d_h */
  int32_t latent_dim;    /* d_l per latent group */
  int32_t dtype;         /* GTA_F32 | GTA_BF16: element type of x, weights, caches and out.
                            Accumulation, softmax statistics and the gate are always fp32. */
  int32_t rope;          /* 0 = none; 1 = rotate-half RoPE on q and k (App. B.1.1): pair
                            (j, j + d_h/2) turns by pos * rope_base^(-2j/d_h); the latent value is
                            never rotated.  Positions count from 0 within each sequence. */
  float   rope_base;     /* e.g. 10000 */
  int32_t gate;          /* GTA_GATE_SIGMOID (Sec. 3.2) | GTA_GATE_SILU, GTA_GATE_RELU2 (the other two
                            nonlinearities of the ablation: z*Sigmoid(z), max(z,0)^2) | GTA_GATE_OFF
                            (factor 1; for tests) */
  float   softmax_scale; /* 0 => 1/sqrt(d_h) (Sec. 3.3) */
} gta_config;

/* Layer weights (Sec. 3.2, 3.3).  Struct in host memory, pointers device, element type = dtype. */
typedef struct {
  const void *wq;  /* [H, n_q*d_h] */
  const void *wk;  /* [H, n_k*d_h] */
  const void *wc;  /* [H, n_c*d_l] */
  const void *wg;  /* [H, n_h*d_h]   W_{G,i} = columns [i*d_h, (i+1)*d_h) */
  const void *wp;  /* [n_h, d_l, d_h] W_{P,i} */
  const void *wo;  /* [n_h*d_h, H], or NULL: the output is the concatenated gated heads */
} gta_weights;

/* Grouped-key / latent-value caches (Sec. 3.3, App. B.1.3).  Struct host, arrays device.  Slot s
 * holds seq_lens[s] valid tokens in rows 0..seq_lens[s]-1; row p is position p.
 * Two layouts:
 *   contiguous (block_table NULL): k and c are [max_batch, max_seq, width]; the last three fields are
 *     ignored.
 *   block table ("paged"): k and c are pools [num_pages, page_size, width]; row p of slot s is row
 *     p % page_size of page block_table[s * pages_per_slot + p / page_size], and max_seq must equal
 *     page_size * pages_per_slot.  An entry outside [0, num_pages) means "no page": rows there are
 *     never written, and a call that would append into them treats the slot as full
 *     (GTA_ERR_CACHE_FULL in status, length unchanged, zero output rows where the call defines them
 *     for a full slot).  Rows below seq_lens are expected to have pages; a missing one is read from
 *     page 0 (never from outside the pools).  Pages must not be shared between slots that a call
 *     writes.  The streaming decode kernels need a power-of-two page_size >= 16; other sizes run on
 *     the shape-generic kernels. */
typedef struct {
  void    *k;         /* keys after RoPE, width n_k*d_h */
  void    *c;         /* latent values (no RoPE), width n_c*d_l */
  int32_t *seq_lens;  /* [max_batch] */
  int32_t *status;    /* [max_batch]; kernels write it only to flag a slot (GTA_ERR_CACHE_FULL,
                         GTA_ERR_SHAPE), never to clear it */
  int32_t  max_batch;
  int32_t  max_seq;
  const int32_t *block_table; /* [max_batch, pages_per_slot] device, or NULL */
  int32_t  page_size;
  int32_t  pages_per_slot;
  int32_t  num_pages;
} gta_cache;

/* Bytes of device workspace the call described by the arguments needs.
 *   mode PREFILL: batch sequences, total_tokens packed tokens, longest sequence <= max_len.
 *   mode DECODE : batch sequences, max_len = cache->max_seq, num_splits as passed to gta_decode
 *                 (0 = library's choice).
 *   mode PREFILL_CHUNK: as PREFILL, for gta_prefill_chunk (max_len = max_chunk).
 * Returns 0 if cfg is NULL or invalid. */
GTA_API size_t gta_workspace_bytes(const gta_config *cfg, int mode, int32_t batch, int64_t total_tokens,
                           int32_t max_len, int32_t num_splits);

/* Causal prefill (Sec. 3.2-3.3; per-token form App. B.1.1-B.1.2) of `batch` packed sequences.
 *   x           device [total_tokens, H]
 *   cu_seqlens  device [batch+1] token offsets (cu[0] = 0, cu[batch] = total_tokens), or NULL:
 *               batch equal sequences of total_tokens / batch tokens
 *   max_seqlen  host upper bound of the longest sequence (sizes the launch)
 *   cache       NULL, or the caches to fill: rows 0..T_b-1 of slot slots[b] receive the keys
 *               (after RoPE) and latent values of sequence b and seq_lens[slot] is SET to T_b
 *               (a fresh prefill; requires max_seqlen <= cache->max_seq)
 *   slots       device [batch] slot of each sequence, or NULL for slot b = b
 *   out         device [total_tokens, n_h*d_h]; [total_tokens, H] when weights->wo is set */
GTA_API int gta_prefill(const gta_config *cfg, const gta_weights *weights, const void *x,
                const int32_t *cu_seqlens, int32_t batch, int64_t total_tokens,
                int32_t max_seqlen, const gta_cache *cache, const int32_t *slots, void *out,
                void *workspace, size_t workspace_bytes, void *hip_stream);

/* Chunked / prefix prefill: App. B.1.3 (append, then attend over everything cached) for a chunk of
 * new tokens per sequence instead of one.  Token i of sequence b takes position seq_lens[slot] + i:
 * q and k are rotated there, k and c are stored as row seq_lens[slot] + i, the token attends over
 * rows 0 .. seq_lens[slot] + i, and seq_lens[slot] grows by the chunk length.  On an empty slot this
 * equals gta_prefill; splitting a sequence into chunks of any sizes gives the rows of one prefill.
 *   x, cu_seqlens, slots, out   as for gta_prefill (lengths are chunk lengths)
 *   max_chunk   host upper bound of the longest chunk (sizes the launch), <= cache->max_seq
 *   cache       required.  A sequence whose chunk does not fit (seq_lens + T_b > max_seq) or whose slot
 *               is out of range stores nothing, gets zero output rows and status GTA_ERR_CACHE_FULL.
 * Runs on the MFMA kernels where gta_uses_tuned_kernels(cfg, GTA_MODE_PREFILL_CHUNK) is 1 (and a
 * slot's key / latent rows stay below 2 GiB), on the shape-generic kernels otherwise.  Workspace:
 * mode PREFILL_CHUNK. */
GTA_API int gta_prefill_chunk(const gta_config *cfg, const gta_weights *weights, const void *x,
                      const int32_t *cu_seqlens, int32_t batch, int64_t total_tokens,
                      int32_t max_chunk, const gta_cache *cache, const int32_t *slots, void *out,
                      void *workspace, size_t workspace_bytes, void *hip_stream);

/* One decode step (App. B.1.3) for `batch` sequences: project x_new, rotate q and k at position
 * seq_lens[slot], append k and c as row seq_lens[slot], increment seq_lens[slot], then attend
 * over all rows of the slot including the new one; gate and decoder use the new token.
 *   x_new       device [batch, H]
 *   slots       device [batch] distinct slots, or NULL for slot b = b
 *   out         device [batch, n_h*d_h] (or [batch, H] with wo)
 *   num_splits  context splits per sequence (split-K); 0 = library's choice */
GTA_API int gta_decode(const gta_config *cfg, const gta_weights *weights, const void *x_new,
               int32_t batch, const gta_cache *cache, const int32_t *slots, void *out,
               int32_t num_splits, void *workspace, size_t workspace_bytes, void *hip_stream);

/* gta_decode for callers that cannot hand over a workspace they allocated: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, semantics and kernels
 * as gta_decode, minus `workspace`: the scratch memory is a fixed array of GTA_STATIC_SCRATCH_BYTES that
 * lives in the library's device image (one copy per GPU the library runs on, held until the process
 * ends).  The call allocates and frees nothing.
 *   - A call whose gta_workspace_bytes(cfg, GTA_MODE_DECODE, batch, 0, cache->max_seq, num_splits)
 *     exceeds GTA_STATIC_SCRATCH_BYTES returns GTA_ERR_WORKSPACE and does nothing (32 MiB covers, e.g.,
 *     64 sequences at the 1B layer shape with any context length; use gta_decode beyond that).
 *   - All calls on one GPU share that GPU's array: calls that may overlap in time (different streams,
 *     different host threads) race; order them.  The array keeps the last call's contents and nothing
 *     in it needs clearing between calls.
 *   - The first call on a device looks the array's address up (a runtime query, no allocation); make
 *     it outside stream capture, like the first call of any entry point. */
#define GTA_STATIC_SCRATCH_BYTES (32u << 20)
GTA_API int gta_decode_static(const gta_config *cfg, const gta_weights *weights, const void *x_new,
                      int32_t batch, const gta_cache *cache, const int32_t *slots, void *out,
                      int32_t num_splits, void *hip_stream);

/* Append already projected (and rotated) rows to the caches (App. B.1.3): pure data movement,
 * bit-exact.  Rows [cu_new[b], cu_new[b+1]) of k_new / c_new go to slot slots[b] at positions
 * seq_lens[slot].., then seq_lens[slot] += their count.
 *   k_new   device [total_new, n_k*d_h];  c_new  device [total_new, n_c*d_l]
 *   cu_new  device [batch+1];  slots device [batch] distinct slots or NULL
 *   max_new host upper bound of rows per sequence (sizes the launch); a sequence with more rows
 *           is skipped and its slot's status is set to GTA_ERR_SHAPE */
GTA_API int gta_cache_append(const gta_config *cfg, const gta_cache *cache, const int32_t *slots,
                     const void *k_new, const void *c_new, const int32_t *cu_new, int32_t batch,
                     int32_t max_new, void *hip_stream);

/* ---- stage entry points: one stage of the pass on already projected inputs, in the launch
 * configuration gta_prefill / gta_decode use (for stage-wise tests and per-kernel timing). ---- */

/* Projection stage of the prefill (Sec. 3.2 input projections and gate matrix; App. B.1.1 RoPE on q and
 * k at positions counted from 0 within each sequence): [q | k | c | g] = x . [W_Q | W_K | W_C | W_G].
 *   x, cu_seqlens, batch, total_tokens, max_seqlen  as for gta_prefill
 *   q_out [total, n_q*d_h], k_out [total, n_k*d_h] (both rotated), c_out [total, n_c*d_l],
 *   g_out [total, n_h*d_h] gate pre-activations; device, element type = cfg->dtype
 *   workspace  mode PREFILL.  No cache is written.
 * Tuned (bf16 MFMA) path only: GTA_ERR_UNSUPPORTED where gta_uses_tuned_kernels(cfg, PREFILL) is 0. */
GTA_API int gta_prefill_projection(const gta_config *cfg, const gta_weights *weights, const void *x,
                                   const int32_t *cu_seqlens, int32_t batch, int64_t total_tokens,
                                   int32_t max_seqlen, void *q_out, void *k_out, void *c_out, void *g_out,
                                   void *workspace, size_t workspace_bytes, void *hip_stream);

/* Value-decoder stage (Sec. 3.2 decoder equation applied after the map, as in the reformulated form
 * of Sec. 3.3): out[t, i*d_h : (i+1)*d_h] = (l[t, q(i)*d_l : (q(i)+1)*d_l] . W_{P,i}) * gate(g[t, i*d_h : ..]).
 *   l [total, n_q*d_l] normalised group outputs, g [total, n_h*d_h] gate pre-activations,
 *   out [total, n_h*d_h]; device, element type = cfg->dtype.  Tuned path only (as above). */
GTA_API int gta_prefill_decoder(const gta_config *cfg, const gta_weights *weights, const void *l, const void *g,
                                int64_t total_tokens, void *out, void *hip_stream);

/* Output projection (Sec. 3.3): out [total, H] = heads [total, n_h*d_h] . W_O; weights->wo required.
 * Tuned path only (as above). */
GTA_API int gta_output_projection(const gta_config *cfg, const gta_weights *weights, const void *heads,
                                  int64_t total_tokens, void *out, void *hip_stream);

/* Attention stage of the prefill (Sec. 3.3, reformulated form): for every map group g and token t,
 * l_out[t, g*d_l : (g+1)*d_l] = sum_{j<=t} Softmax_j(q_g[t].k_{k(g)}[j] / sqrt(d_h)) c_{c(g)}[j].
 *   q [total, n_q*d_h], k [total, n_k*d_h] (both already rotated), c [total, n_c*d_l],
 *   l_out [total, n_q*d_l]; all device, element type = cfg->dtype; cu_seqlens as in gta_prefill. */
GTA_API int gta_prefill_attention(const gta_config *cfg, const void *q, const void *k, const void *c,
                                  const int32_t *cu_seqlens, int32_t batch, int64_t total_tokens,
                                  int32_t max_seqlen, void *l_out, void *hip_stream);

/* Split-K attention stage of the decode step (App. B.1.3) over the seq_lens[slot] rows ALREADY in
 * the caches (nothing is appended): leaves one un-normalised partial (accumulator, running max,
 * running sum) per (sequence, split, group) in `workspace`.
 *   q  device fp32 [batch, n_q*d_h], already rotated; workspace sized by gta_workspace_bytes(DECODE) */
GTA_API int gta_decode_attention(const gta_config *cfg, const float *q, const gta_cache *cache,
                                 const int32_t *slots, int32_t batch, int32_t num_splits, void *workspace,
                                 size_t workspace_bytes, void *hip_stream);

/* Merges the partials gta_decode_attention left in `workspace` (same batch / num_splits) by their
 * log-sum-exp weights:  l_out fp32 [batch, n_q*d_l] = the normalised group outputs L_g. */
GTA_API int gta_decode_combine(const gta_config *cfg, const gta_cache *cache, const int32_t *slots,
                               int32_t batch, int32_t num_splits, void *workspace, size_t workspace_bytes,
                               float *l_out, void *hip_stream);

/* Plain device-to-device copy of `bytes` (a multiple of 16) by one kernel that reads every byte of
 * src once and writes every byte of dst once: the known-traffic reference that per-dispatch
 * hardware counters of HBM bytes are calibrated against when profiling the kernels above. */
GTA_API int gta_calibration_copy(const void *src, void *dst, int64_t bytes, void *hip_stream);

/* Roofline calibration, not part of the attention pass: one kernel that only reads `bytes` of device
 * memory at `src` once with non-temporal 16-byte loads, `workgroups` workgroups of 256 threads, each a
 * contiguous slice (bytes must be a multiple of workgroups * 32768).  Timed by the caller, it gives
 * the streaming-read rate the machine reaches next to the published HBM peak.  `sink` is device
 * memory of at least 1 KiB that is (practically never) written.  GTA_ERR_SHAPE / _NULL / _ALIGN on
 * misuse, nothing launched then. */
GTA_API int gta_calibration_read(const void *src, int64_t bytes, int32_t workgroups, void *sink, void *hip_stream);

/* Roofline calibration: `workgroups` workgroups of four waves, each wave issuing iters * 16
 * v_mfma_f32_32x32x16_bf16 (32768 flop each) on 16 independent accumulators and nothing else.  Timed
 * by the caller it gives the bf16 MFMA rate the chip sustains at the clock it holds under matrix load,
 * next to the published 2.5 PFLOP/s.  random_operands 0: one pair of small constant operands;
 * 1: eight operand pairs per lane with values spread like activations and weights, used in rotation
 * (the rate is power-limited and depends on how many operand bits change between instructions).
 * `sink`: device memory of at least 1 KiB. */
GTA_API int gta_calibration_mfma(int32_t workgroups, int32_t iters, int32_t random_operands, void *sink,
                                 void *hip_stream);

/* Static string for a gta_status value. */
GTA_API const char *gta_strerror(int code);

/* 1 if the configuration runs on the tuned bf16 MFMA/streaming kernels, 0 if it runs on the
 * shape-generic kernels (still HIP, any dimensions, but 10-100x slower), negative gta_status if
 * invalid.  Tuned: bf16, d_h 64 or 128, every projection width a multiple of 64 (of 128 for heads of
 * 128), H a multiple of 128; decode in addition needs cache rows of a compiled shape: heads of 128
 * with (n_k, n_q, n_c, d_l) in {(4,4,1,512), (8,8,1,1024), (4,8,1,512), (4,4,2,512), (4,8,2,512),
 * (4,4,4,512)}, or one key of 64 with latents of 128: n_c = 1 with n_q in {3,5,6}, n_c = 2 with n_q in
 * {6,10}.  With GTA_DEBUG set in the environment a bf16 call that takes the generic kernels says so
 * on stderr. */
GTA_API int gta_uses_tuned_kernels(const gta_config *cfg, int mode);

#ifdef __cplusplus
}
#endif
#endif /* GTA_H_ */
