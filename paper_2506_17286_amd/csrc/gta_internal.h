// Internal declarations shared by the translation units of libgta (not part of the C ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

#include <mutex>

#include "gta.h"

namespace gta {

// A kernel that takes more than 64 KiB of dynamic LDS needs the limit raised once per device it runs
// on (the attribute belongs to the kernel's image on the current device).  Fixed table, no allocation.
inline void allow_dynamic_lds(const void *fn, int bytes) {
  struct Entry { const void *fn; int dev; };
  static Entry seen[256];
  static int n = 0;
  static std::mutex mu;
  int dev = 0;
  (void)hipGetDevice(&dev);
  std::lock_guard<std::mutex> lock(mu);
  for (int i = 0; i < n; ++i)
    if (seen[i].fn == fn && seen[i].dev == dev) return;
  (void)hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
  if (n < 256) seen[n++] = Entry{fn, dev};   // table full: the attribute is simply set again next time
}

// Validated, derived view of a gta_config.
struct Dims {
  int H, nh, nq, nk, nc, dh, dl;
  int hpq;          // heads per map group        n_h / n_q
  int qpk;          // map groups per key group   n_q / n_k
  int qpc;          // map groups per latent group n_q / n_c
  int wq_w, wk_w, wc_w, wg_w;  // widths of Q, K, C and gate pre-activation rows
  int wtot;         // wq_w + wk_w + wc_w + wg_w
  int dtype;        // GTA_F32 | GTA_BF16
  int rope;         // 0 | 1
  int gate;         // kGateOff | kGateSigmoid | kGateSilu | kGateRelu2
  float scale;      // softmax scale
  double rope_base;
  int esize() const { return dtype == GTA_BF16 ? 2 : 4; }
};

enum { kGateOff = 0, kGateSigmoid = 1, kGateSilu = 2, kGateRelu2 = 3 };

// Factor the decoded value is multiplied by, from the gate pre-activation z: Sigmoid(z) (Sec. 3.2), or
// one of the ablation's other nonlinearities, z * Sigmoid(z) and max(z, 0)^2.  kind != kGateOff.
__device__ __forceinline__ float gate_factor(int kind, float z) {
  const float s = __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-1.4426950408889634f * z));
  const float r = fmaxf(z, 0.f);
  return kind == kGateSigmoid ? s : (kind == kGateSilu ? z * s : r * r);
}

static inline size_t align_up(size_t v, size_t a = 256) { return (v + a - 1) / a * a; }

// ---- cache row addressing ---------------------------------------------------------------------
// Contiguous layout (table == NULL): row r of slot s is pool row s * max_seq + r.  Block-table layout:
// it is row r % page_size of page table[s * pages_per_slot + r / page_size]; an entry outside
// [0, num_pages) means "no page": such a row is never written and counts as missing capacity.
struct PageMap {
  const int32_t *table;
  int page_size, pages_per_slot, num_pages;
};

inline PageMap page_map_of(const gta_cache &c) {
  return PageMap{c.block_table, c.page_size, c.pages_per_slot, c.num_pages};
}

// Pool row of (slot, row), or -1 where the row has no page.  slot and row are in range.
__device__ __forceinline__ int64_t cache_row(const PageMap &pm, int max_seq, int slot, int row) {
  if (!pm.table) return (int64_t)slot * max_seq + row;
  const int pg = pm.table[(int64_t)slot * pm.pages_per_slot + row / pm.page_size];
  if (pg < 0 || pg >= pm.num_pages) return -1;
  return (int64_t)pg * pm.page_size + row % pm.page_size;
}

// The same for reads: a missing page reads page 0 (never outside the pools; the result is then the
// caller's problem, rows below seq_lens are expected to have pages).
__device__ __forceinline__ int64_t cache_row_clamped(const PageMap &pm, int max_seq, int slot, int row) {
  if (!pm.table) return (int64_t)slot * max_seq + row;
  int pg = pm.table[(int64_t)slot * pm.pages_per_slot + row / pm.page_size];
  pg = pg < 0 || pg >= pm.num_pages ? 0 : pg;
  return (int64_t)pg * pm.page_size + row % pm.page_size;
}

// Do rows [r0, r1) of a slot all have pages?  (One thread walks the slot's table entries.)
__device__ __forceinline__ bool rows_backed(const PageMap &pm, int slot, int r0, int r1) {
  if (!pm.table || r1 <= r0) return true;
  const int32_t *t = pm.table + (int64_t)slot * pm.pages_per_slot;
  for (int i = r0 / pm.page_size; i <= (r1 - 1) / pm.page_size; ++i)
    if (t[i] < 0 || t[i] >= pm.num_pages) return false;
  return true;
}

// ---- workspace carve-up (one function per mode so sizing and use cannot disagree) ----------
struct PrefillWs {
  int32_t *seq_id, *pos;   // [total] sequence index and position of each packed token
  float2 *rope;            // [max_len, d_h/2] (cos, sin)
  float *praw;             // generic path: raw fp32 projections [total, wtot]
  void *q, *k, *c;         // [total, wq_w], [total, wk_w], [total, wc_w]   element type = dtype
  void *g;                 // gate pre-activation [total, wg_w]; fp32 (generic) or dtype (tuned)
  void *l;                 // normalised group outputs [total, n_q*d_l]; fp32 (generic) or dtype
  void *o;                 // gated heads [total, wg_w] (dtype), only with W_O
  void *wpack;             // tuned path, some shapes: [W_Q | W_K | W_C | W_G] side by side, [H, wtot]
  int32_t *prefix;         // chunked prefill: [batch] rows cached before the chunk, or -1 (sequence skipped)
  size_t bytes;
};
PrefillWs carve_prefill(const Dims &d, bool tuned, bool with_wo, int batch, int64_t total,
                        int max_len, void *base, bool chunk = false);

struct DecodeWs {
  float *praw;             // [ksplit, batch, wtot] raw fp32 projections of the new tokens (split-K partials)
  float *q;                // [batch, wq_w] rotated queries
  float *g;                // [batch, wg_w] gate pre-activations
  float *part;             // [batch, splits, n_q, d_l + 2]  (acc[d_l], m, l)
  float *l;                // [batch, n_q*d_l]
  float *o;                // [batch, wg_w] gated heads, only with W_O
  int32_t *oldlen;         // [batch] tokens cached before the step, or -1 if the slot is full
  size_t bytes;
  int splits;
};
int choose_splits(const Dims &d, int batch, int max_seq, int requested);
DecodeWs carve_decode(const Dims &d, bool with_wo, int batch, int splits, void *base);

// ---- shape-generic path (any dims, fp32 or bf16 elements), gta_generic.hip ------------------
int generic_prefill(const Dims &d, const gta_weights &w, const void *x, const int32_t *cu,
                    int batch, int64_t total, int max_len, const gta_cache *cache,
                    const int32_t *slots, void *out, const PrefillWs &ws, hipStream_t st);
int generic_prefill_chunk(const Dims &d, const gta_weights &w, const void *x, const int32_t *cu, int batch,
                          int64_t total, int max_chunk, const gta_cache &cache, const int32_t *slots, void *out,
                          const PrefillWs &ws, hipStream_t st);
int generic_decode(const Dims &d, const gta_weights &w, const void *x_new, int batch,
                   const gta_cache &cache, const int32_t *slots, void *out, const DecodeWs &ws,
                   hipStream_t st);
int generic_cache_append(const Dims &d, const gta_cache &cache, const int32_t *slots,
                         const void *k_new, const void *c_new, const int32_t *cu_new, int batch,
                         int max_new, hipStream_t st);

// Pieces of the generic path reused by the tuned path.
void generic_decode_project(const Dims &d, const gta_weights &w, const void *x_new, int batch,
                            const gta_cache &cache, const int32_t *slots, const DecodeWs &ws, hipStream_t st);
void launch_decode_commit(const gta_cache &cache, const int32_t *slots, const int32_t *oldlen, int batch,
                          hipStream_t st);
void generic_out_proj_f32in(const Dims &d, const gta_weights &w, const float *O, int M, void *out, hipStream_t st);

void launch_attn_prefill_rowwise(const Dims &d, const void *q, const void *k, const void *c, const int32_t *cu,
                                 int batch, int64_t total, int max_len, void *L, hipStream_t st);
void launch_finalize_decode_bf16(const Dims &d, const float *part, int nsum, int batch, const gta_cache &cache,
                                 const int32_t *slots, const DecodeWs &ws, hipStream_t st);
void launch_cached_len(const gta_cache &cache, const int32_t *slots, int batch, int32_t *oldlen, hipStream_t st);
void generic_decode_attention(const Dims &d, const float *q, const int32_t *oldlen, const gta_cache &cache,
                              const int32_t *slots, int batch, int splits, float *part, hipStream_t st);
void generic_decode_combine(const Dims &d, const float *part, const int32_t *oldlen, int splits, int batch, float *L,
                            hipStream_t st);
int launch_calibration_copy(const void *src, void *dst, int64_t bytes, hipStream_t st);
int launch_calibration_read(const void *src, int64_t bytes, int workgroups, void *sink, hipStream_t st);
int launch_calibration_mfma(int workgroups, int iters, bool random_operands, void *sink, hipStream_t st);
void launch_rowmap(const int32_t *cu, int batch, int64_t total, int32_t *seq_id, int32_t *pos,
                   hipStream_t st);
void launch_rope_table(float2 *tab, int max_pos, int dh, double base, hipStream_t st);
void launch_prefill_commit(const gta_cache &cache, const int32_t *slots, const int32_t *cu,
                           int batch, int64_t total, hipStream_t st);
// chunked prefill: row map with positions behind the cached rows, per-token RoPE rows, prefix[]; commit
void launch_prefill_chunk_setup(const Dims &d, const int32_t *cu, int batch, int64_t total, int32_t *seq_id,
                                int32_t *pos, float2 *tab, int32_t *prefix, const gta_cache &cache,
                                const int32_t *slots, hipStream_t st);
void launch_prefill_chunk_commit(const gta_cache &cache, const int32_t *slots, const int32_t *cu, int batch,
                                 int64_t total, const int32_t *prefix, hipStream_t st);
// row map, RoPE table (if d.rope) and cached lengths (if cache) of one prefill call in one launch
void launch_prefill_setup(const Dims &d, const int32_t *cu, int batch, int64_t total, int max_len,
                          int32_t *seq_id, int32_t *pos, float2 *tab, const gta_cache *cache,
                          const int32_t *slots, hipStream_t st);

// hipGetLastError after the launches of a call; with GTA_DEBUG set in the environment the HIP error
// string goes to stderr (the only thing the library ever prints).
static inline int check_launch() {
  hipError_t e = hipGetLastError();
  if (e == hipSuccess) return GTA_OK;
  if (getenv("GTA_DEBUG")) fprintf(stderr, "libgta: HIP error %d: %s\n", (int)e, hipGetErrorString(e));
  return GTA_ERR_HIP;
}

}  // namespace gta
