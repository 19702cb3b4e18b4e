// C-ABI entry points of libgta: argument validation, workspace carve-up and dispatch to the
// tuned bf16 kernels or the shape-generic kernels.  No kernels in this file; the only device object
// is the fixed scratch array of gta_decode_static.
#include <math.h>

#include <algorithm>
#include "gta_internal.h"
#include "gta_tuned.h"

namespace gta {

static int make_dims(const gta_config *c, Dims *out) {
  if (!c) return GTA_ERR_NULL;
  if (c->dtype != GTA_F32 && c->dtype != GTA_BF16) return GTA_ERR_DTYPE;
  if (c->gate != GTA_GATE_SIGMOID && c->gate != GTA_GATE_OFF && c->gate != GTA_GATE_SILU && c->gate != GTA_GATE_RELU2)
    return GTA_ERR_DTYPE;
  if (c->rope != 0 && c->rope != 1) return GTA_ERR_DTYPE;
  if (c->d_model <= 0 || c->n_heads <= 0 || c->n_qgroups <= 0 || c->n_kgroups <= 0 || c->n_cgroups <= 0 ||
      c->head_dim <= 0 || c->latent_dim <= 0)
    return GTA_ERR_SHAPE;
  // every dimension is bounded before anything is multiplied or added (no overflow on hostile values)
  const int32_t kMaxDim = 1 << 24;
  if (c->d_model > kMaxDim || c->n_heads > kMaxDim || c->n_qgroups > kMaxDim || c->n_kgroups > kMaxDim ||
      c->n_cgroups > kMaxDim || c->head_dim > kMaxDim || c->latent_dim > kMaxDim)
    return GTA_ERR_UNSUPPORTED;
  if (c->n_heads % c->n_qgroups || c->n_qgroups % c->n_kgroups || c->n_qgroups % c->n_cgroups) return GTA_ERR_SHAPE;
  if (c->latent_dim < c->head_dim) return GTA_ERR_SHAPE;  // Sec. 3.2: d_l >= d_h
  if (c->rope && (c->head_dim % 2 || !(c->rope_base > 0.f))) return GTA_ERR_SHAPE;
  if (!(c->softmax_scale >= 0.f)) return GTA_ERR_SHAPE;
  const int64_t wtot = ((int64_t)c->n_qgroups + c->n_kgroups + c->n_heads) * c->head_dim +
                       (int64_t)c->n_cgroups * c->latent_dim;
  if (wtot > (1 << 24) || c->d_model > (1 << 24) || (int64_t)c->n_qgroups * c->latent_dim > (1 << 24))
    return GTA_ERR_UNSUPPORTED;
  Dims d{};
  d.H = c->d_model; d.nh = c->n_heads; d.nq = c->n_qgroups; d.nk = c->n_kgroups; d.nc = c->n_cgroups;
  d.dh = c->head_dim; d.dl = c->latent_dim;
  d.hpq = d.nh / d.nq; d.qpk = d.nq / d.nk; d.qpc = d.nq / d.nc;
  d.wq_w = d.nq * d.dh; d.wk_w = d.nk * d.dh; d.wc_w = d.nc * d.dl; d.wg_w = d.nh * d.dh;
  d.wtot = (int)wtot;
  d.dtype = c->dtype; d.rope = c->rope; d.gate = c->gate == GTA_GATE_SIGMOID ? kGateSigmoid : c->gate == GTA_GATE_SILU ? kGateSilu :
           c->gate == GTA_GATE_RELU2 ? kGateRelu2 : kGateOff;
  d.scale = c->softmax_scale > 0.f ? c->softmax_scale : (float)(1.0 / sqrt((double)c->head_dim));
  d.rope_base = (double)c->rope_base;
  *out = d;
  return GTA_OK;
}

static inline bool misaligned(const void *p) { return ((uintptr_t)p & 15u) != 0; }

// ---------------------------------------------------------------------------- workspace layout
namespace {
struct Carver {
  char *base; size_t off = 0;
  explicit Carver(void *b) : base((char *)b) {}
  template <typename T> T *take(size_t bytes) {
    T *p = base ? (T *)(base + off) : nullptr;
    off += align_up(bytes);
    return p;
  }
};
}  // namespace

PrefillWs carve_prefill(const Dims &d, bool tuned, bool with_wo, int batch, int64_t total, int max_len, void *base,
                        bool chunk) {
  Carver cv(base);
  PrefillWs w{};
  const size_t n = (size_t)total, es = (size_t)d.esize();
  w.seq_id = cv.take<int32_t>(n * 4);
  w.pos = cv.take<int32_t>(n * 4);
  // RoPE rows: one per position (fresh prefill) or one per packed token (chunked prefill)
  w.rope = cv.take<float2>(d.rope ? (size_t)(chunk ? total : max_len) * (d.dh / 2) * sizeof(float2) : 0);
  // generic path: raw projections of every token; tuned path: split-K partials of a short prefill (the
  // same amount whatever the token count, so that a workspace sized for many tokens also serves few)
  w.praw = cv.take<float>(tuned ? proj_small_rows_bound(d) * d.wtot * 4 : n * d.wtot * 4);
  w.q = cv.take<void>(n * d.wq_w * es);
  w.k = cv.take<void>(n * d.wk_w * es);
  w.c = cv.take<void>(n * d.wc_w * es);
  w.g = cv.take<void>(n * d.wg_w * (tuned ? es : 4));
  w.l = cv.take<void>(n * (size_t)d.nq * d.dl * (tuned ? es : 4));
  w.o = cv.take<void>(with_wo ? n * d.wg_w * (tuned ? es : 4) : 0);
  w.wpack = cv.take<void>(tuned ? proj_packed_bytes(d) : 0);
  w.prefix = cv.take<int32_t>(chunk ? (size_t)batch * 4 : 0);
  w.bytes = cv.off;
  return w;
}

// Relative time of one split-K launch of `batch` sequences in `s` splits on kernels that keep one workgroup
// per CU busy.  Measured at the 1B shape, 8K rows: one workgroup streams about 46 GB/s, so about 124 of them
// saturate the memory system and anything from 124 to 256 workgroups takes the same time give or take 6 %
// (the larger launches being the faster ones); past 256 the launch runs in rounds, and a last round of a few
// workgroups costs a whole slice at one workgroup's rate (batch 96: 288 workgroups 360 us, 192 workgroups
// 290 us; batch 72: 288 -> 280 us, 216 -> 227 us; batch 192: 384 -> 584 us, 192 -> 540 us).
static double split_launch_cost(int batch, int s, int max_seq) {
  const double kSaturating = 124.0;
  const int64_t w = (int64_t)batch * s;
  const int64_t full = w / 256, rem = w % 256;
  double rounds = full * (256.0 / kSaturating);
  if (rem) rounds += rem > kSaturating ? rem / kSaturating : 1.0;
  const double rows = (double)((max_seq + s - 1) / s);
  double cost = rows * rounds;
  if (w <= 256) cost *= 1.0 - 0.15 * (double)w / 256.0;
  return cost + 0.5 * s;   // partials to write and merge
}

int choose_splits(const Dims &d, int batch, int max_seq, int requested) {
  if (requested > 0) return requested > 1024 ? 1024 : requested;
  // enough (sequence, split) blocks to put one or two on every one of the 256 CUs (the kernel's choice), but
  // no split shorter than 256 cached rows.
  const int target = tuned_decode_target_workgroups(d);
  int want = (target + batch - 1) / batch;
  int cap = max_seq / 256;
  if (cap < 1) cap = 1;
  const bool tuned = tuned_decode_supported(d);
  if (tuned) cap = std::min(cap, tuned_decode_max_splits(d, batch));
  cap = std::min(cap, 256);
  if (tuned && target == 256) {
    // one workgroup per CU: the split count whose launch fills whole rounds of 256
    int best = 1;
    double best_cost = split_launch_cost(batch, 1, max_seq);
    for (int s = 2; s <= cap && (int64_t)batch * s <= 1024; ++s) {
      const double c = split_launch_cost(batch, s, max_seq);
      if (c < best_cost) { best_cost = c; best = s; }
    }
    return best;
  }
  // two workgroups per CU: a launch of just over 512 workgroups runs a second round for the few left over
  // (paper layer, 2K rows, whole step: batch 72 54 us with 8 splits, 42.5 us with 7; batch 96 57 -> 47;
  // batch 160 73 -> 60), so the count is rounded down to what fits
  if (tuned && batch <= target && (int64_t)batch * want > target) want = target / batch;
  int s = want < cap ? want : cap;
  if (s < 1) s = 1;
  return s;
}

DecodeWs carve_decode(const Dims &d, bool with_wo, int batch, int splits, void *base) {
  Carver cv(base);
  DecodeWs w{};
  const size_t b = (size_t)batch;
  w.splits = splits;
  w.praw = cv.take<float>(b * d.wtot * 4 * 16);   // up to 16 split-K partials
  w.q = cv.take<float>(b * d.wq_w * 4);
  w.g = cv.take<float>(b * d.wg_w * 4);
  w.part = cv.take<float>(b * splits * d.nq * (size_t)(d.dl + 2) * 4);
  w.l = cv.take<float>(b * d.nq * (size_t)d.dl * 4);
  w.o = cv.take<float>(with_wo ? b * d.wg_w * 4 : 0);
  w.oldlen = cv.take<int32_t>(b * 4);
  w.bytes = cv.off;
  return w;
}

static int check_weights(const gta_weights *w) {
  if (!w || !w->wq || !w->wk || !w->wc || !w->wg || !w->wp) return GTA_ERR_NULL;
  if (misaligned(w->wq) || misaligned(w->wk) || misaligned(w->wc) || misaligned(w->wg) || misaligned(w->wp) ||
      misaligned(w->wo))
    return GTA_ERR_ALIGN;
  return GTA_OK;
}

static int check_cache(const gta_cache *c) {
  if (!c->k || !c->c || !c->seq_lens || !c->status) return GTA_ERR_NULL;
  if (c->max_batch <= 0 || c->max_seq <= 0) return GTA_ERR_SHAPE;
  if (misaligned(c->k) || misaligned(c->c) || ((uintptr_t)c->seq_lens & 3u) || ((uintptr_t)c->status & 3u))
    return GTA_ERR_ALIGN;
  if (c->block_table) {
    if ((uintptr_t)c->block_table & 3u) return GTA_ERR_ALIGN;
    if (c->page_size <= 0 || c->pages_per_slot <= 0 || c->num_pages <= 0) return GTA_ERR_SHAPE;
    if ((int64_t)c->page_size * c->pages_per_slot != c->max_seq) return GTA_ERR_SHAPE;
  }
  return GTA_OK;
}

static const int kMaxBatch = 65535;  // grid.y / grid.z limit

// ---- fixed scratch of gta_decode_static ---------------------------------------------------------
// One copy per GPU the library runs on, held until the process ends.  `scratch` is only a host-side
// stand-in for the symbol: host code never passes it to a kernel, it asks the runtime once per device
// for that device's address of the array and uses the address from then on.
static __device__ __align__(256) unsigned char scratch[GTA_STATIC_SCRATCH_BYTES];

static const int kMaxDevices = 64;
static void *scratch_of_device[kMaxDevices];   // device address of `scratch`, NULL until resolved
static std::mutex scratch_mu;

// Address of the current device's copy of the scratch array (resolved on the first call on a device).
static int static_scratch(void **out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return GTA_ERR_HIP;
  std::lock_guard<std::mutex> lock(scratch_mu);
  if (!scratch_of_device[dev]) {
    void *p = nullptr;
    const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !p) {
      if (getenv("GTA_DEBUG")) fprintf(stderr, "libgta: hipGetSymbolAddress(scratch): %s\n", hipGetErrorString(e));
      return GTA_ERR_HIP;
    }
    scratch_of_device[dev] = p;
  }
  *out = scratch_of_device[dev];
  return GTA_OK;
}

static bool decode_is_tuned(const Dims &d, const gta_cache &c) {
  return tuned_decode_supported(d) && tuned_decode_layout_ok(c);
}

// With GTA_DEBUG set, a bf16 call that runs on the shape-generic kernels says so on stderr: those
// kernels are one to two orders of magnitude slower than the tuned ones, and which shapes are tuned is
// a closed list (gta_uses_tuned_kernels answers the same question without a call).
static void note_generic_path(const Dims &d, const char *entry) {
  if (d.dtype != GTA_BF16 || !getenv("GTA_DEBUG")) return;
  fprintf(stderr, "libgta: %s runs on the shape-generic kernels (H=%d n_h=%d n_q=%d n_k=%d n_c=%d d_h=%d d_l=%d)\n",
          entry, d.H, d.nh, d.nq, d.nk, d.nc, d.dh, d.dl);
}

}  // namespace gta

using namespace gta;

extern "C" {

const char *gta_strerror(int code) {
  switch (code) {
    case GTA_OK: return "ok";
    case GTA_ERR_NULL: return "a required pointer is NULL";
    case GTA_ERR_SHAPE: return "shape / divisibility / range violation";
    case GTA_ERR_ALIGN: return "device pointer not 16-byte aligned";
    case GTA_ERR_DTYPE: return "unknown dtype, gate or rope code";
    case GTA_ERR_UNSUPPORTED: return "dimensions not supported by the kernels";
    case GTA_ERR_WORKSPACE: return "workspace missing or too small";
    case GTA_ERR_HIP: return "HIP kernel launch failed";
    case GTA_ERR_CACHE_FULL: return "cache slot full";
    default: return "unknown gta_status";
  }
}

int gta_uses_tuned_kernels(const gta_config *cfg, int mode) {
  Dims d;
  int rc = make_dims(cfg, &d);
  if (rc != GTA_OK) return rc;
  if (mode == GTA_MODE_PREFILL) return tuned_prefill_supported(d) ? 1 : 0;
  if (mode == GTA_MODE_DECODE) return tuned_decode_supported(d) ? 1 : 0;
  if (mode == GTA_MODE_PREFILL_CHUNK) return tuned_prefill_chunk_supported(d, 1) ? 1 : 0;   // up to the cache-size limit
  return GTA_ERR_DTYPE;
}

size_t gta_workspace_bytes(const gta_config *cfg, int mode, int32_t batch, int64_t total_tokens, int32_t max_len,
                           int32_t num_splits) {
  Dims d;
  if (make_dims(cfg, &d) != GTA_OK || batch <= 0 || max_len < 0) return 0;
  if (mode == GTA_MODE_PREFILL_CHUNK) {
    // the call picks the kernels by the cache's capacity too: sized for either choice
    if (total_tokens < 0) return 0;
    size_t n = carve_prefill(d, false, true, batch, total_tokens, max_len, nullptr, true).bytes;
    if (tuned_prefill_supported(d)) n = std::max(n, carve_prefill(d, true, true, batch, total_tokens, max_len, nullptr, true).bytes);
    return n + 256;
  }
  if (mode == GTA_MODE_PREFILL) {
    if (total_tokens < 0) return 0;
    // sized for a call with W_O (a superset of the call without)
    return carve_prefill(d, tuned_prefill_supported(d), true, batch, total_tokens, max_len, nullptr).bytes + 256;
  }
  if (mode == GTA_MODE_DECODE) {
    int splits = choose_splits(d, batch, max_len, num_splits);
    return carve_decode(d, true, batch, splits, nullptr).bytes + 256;
  }
  return 0;
}

int gta_prefill(const gta_config *cfg, const gta_weights *weights, const void *x, const int32_t *cu_seqlens,
                int32_t batch, int64_t total_tokens, int32_t max_seqlen, const gta_cache *cache,
                const int32_t *slots, void *out, void *workspace, size_t workspace_bytes, void *hip_stream) {
  Dims d;
  int rc = make_dims(cfg, &d);
  if (rc != GTA_OK) return rc;
  if ((rc = check_weights(weights)) != GTA_OK) return rc;
  if (!x || !out) return GTA_ERR_NULL;
  if (batch <= 0 || batch > kMaxBatch || total_tokens < 0 || total_tokens > INT32_MAX || max_seqlen < 0)
    return GTA_ERR_SHAPE;
  if (!cu_seqlens && (total_tokens % batch != 0 || total_tokens / batch > max_seqlen)) return GTA_ERR_SHAPE;
  if ((int64_t)total_tokens * d.wtot > ((int64_t)1 << 40)) return GTA_ERR_UNSUPPORTED;
  if (misaligned(x) || misaligned(out) || ((uintptr_t)cu_seqlens & 3u) || ((uintptr_t)slots & 3u)) return GTA_ERR_ALIGN;
  if (cache) {
    if ((rc = check_cache(cache)) != GTA_OK) return rc;
    if (max_seqlen > cache->max_seq || (!slots && batch > cache->max_batch)) return GTA_ERR_SHAPE;
  }
  if (total_tokens == 0 || max_seqlen == 0) return GTA_OK;
  const bool tuned = tuned_prefill_supported(d);
  if (!workspace || misaligned(workspace)) return GTA_ERR_WORKSPACE;
  PrefillWs ws = carve_prefill(d, tuned, weights->wo != nullptr, batch, total_tokens, max_seqlen, workspace);
  if (ws.bytes > workspace_bytes) return GTA_ERR_WORKSPACE;
  hipStream_t st = (hipStream_t)hip_stream;
  if (tuned)
    return tuned_prefill(d, *weights, x, cu_seqlens, batch, total_tokens, max_seqlen, cache, slots, out, ws, st);
  note_generic_path(d, "gta_prefill");
  return generic_prefill(d, *weights, x, cu_seqlens, batch, total_tokens, max_seqlen, cache, slots, out, ws, st);
}

int gta_prefill_chunk(const gta_config *cfg, const gta_weights *weights, const void *x, const int32_t *cu_seqlens,
                      int32_t batch, int64_t total_tokens, int32_t max_chunk, const gta_cache *cache,
                      const int32_t *slots, void *out, void *workspace, size_t workspace_bytes, void *hip_stream) {
  Dims d;
  int rc = make_dims(cfg, &d);
  if (rc != GTA_OK) return rc;
  if ((rc = check_weights(weights)) != GTA_OK) return rc;
  if (!x || !out || !cache) return GTA_ERR_NULL;
  if (batch <= 0 || batch > kMaxBatch || total_tokens < 0 || total_tokens > INT32_MAX || max_chunk < 0)
    return GTA_ERR_SHAPE;
  if (!cu_seqlens && (total_tokens % batch != 0 || total_tokens / batch > max_chunk)) return GTA_ERR_SHAPE;
  if ((int64_t)total_tokens * d.wtot > ((int64_t)1 << 40)) return GTA_ERR_UNSUPPORTED;
  if (misaligned(x) || misaligned(out) || ((uintptr_t)cu_seqlens & 3u) || ((uintptr_t)slots & 3u)) return GTA_ERR_ALIGN;
  if ((rc = check_cache(cache)) != GTA_OK) return rc;
  if (max_chunk > cache->max_seq || (!slots && batch > cache->max_batch)) return GTA_ERR_SHAPE;
  if (total_tokens == 0 || max_chunk == 0) return GTA_OK;
  if (!workspace || misaligned(workspace)) return GTA_ERR_WORKSPACE;
  const bool tuned = tuned_prefill_chunk_supported(d, cache->max_seq) && tuned_chunk_layout_ok(*cache);
  PrefillWs ws = carve_prefill(d, tuned, weights->wo != nullptr, batch, total_tokens, max_chunk, workspace, true);
  if (ws.bytes > workspace_bytes) return GTA_ERR_WORKSPACE;
  if (tuned)
    return tuned_prefill_chunk(d, *weights, x, cu_seqlens, batch, total_tokens, max_chunk, *cache, slots, out, ws,
                               (hipStream_t)hip_stream);
  note_generic_path(d, "gta_prefill_chunk");
  return generic_prefill_chunk(d, *weights, x, cu_seqlens, batch, total_tokens, max_chunk, *cache, slots, out, ws,
                               (hipStream_t)hip_stream);
}

int gta_decode(const gta_config *cfg, const gta_weights *weights, const void *x_new, int32_t batch,
               const gta_cache *cache, const int32_t *slots, void *out, int32_t num_splits, void *workspace,
               size_t workspace_bytes, void *hip_stream) {
  Dims d;
  int rc = make_dims(cfg, &d);
  if (rc != GTA_OK) return rc;
  if ((rc = check_weights(weights)) != GTA_OK) return rc;
  if (!x_new || !out || !cache) return GTA_ERR_NULL;
  if ((rc = check_cache(cache)) != GTA_OK) return rc;
  if (batch <= 0 || batch > kMaxBatch || num_splits < 0 || (!slots && batch > cache->max_batch)) return GTA_ERR_SHAPE;
  if (misaligned(x_new) || misaligned(out) || ((uintptr_t)slots & 3u)) return GTA_ERR_ALIGN;
  if (!workspace || misaligned(workspace)) return GTA_ERR_WORKSPACE;
  const int splits = choose_splits(d, batch, cache->max_seq, num_splits);
  DecodeWs ws = carve_decode(d, weights->wo != nullptr, batch, splits, workspace);
  if (ws.bytes > workspace_bytes) return GTA_ERR_WORKSPACE;
  hipStream_t st = (hipStream_t)hip_stream;
  if (decode_is_tuned(d, *cache)) return tuned_decode(d, *weights, x_new, batch, *cache, slots, out, ws, st);
  note_generic_path(d, "gta_decode");
  return generic_decode(d, *weights, x_new, batch, *cache, slots, out, ws, st);
}

int gta_decode_static(const gta_config *cfg, const gta_weights *weights, const void *x_new, int32_t batch,
                      const gta_cache *cache, const int32_t *slots, void *out, int32_t num_splits, void *hip_stream) {
  // the size check comes first: an oversized call is refused before anything else is touched
  const size_t need = cache ? gta_workspace_bytes(cfg, GTA_MODE_DECODE, batch, 0, cache->max_seq, num_splits) : 0;
  if (need > (size_t)GTA_STATIC_SCRATCH_BYTES) return GTA_ERR_WORKSPACE;
  void *ws = nullptr;
  const int rc = static_scratch(&ws);
  if (rc != GTA_OK) return rc;
  // nothing in the decode workspace has to start at zero: every word a kernel reads was written by an
  // earlier kernel of the same call
  return gta_decode(cfg, weights, x_new, batch, cache, slots, out, num_splits, ws, (size_t)GTA_STATIC_SCRATCH_BYTES, hip_stream);
}

int gta_prefill_attention(const gta_config *cfg, const void *q, const void *k, const void *c,
                          const int32_t *cu_seqlens, int32_t batch, int64_t total_tokens, int32_t max_seqlen,
                          void *l_out, void *hip_stream) {
  Dims d;
  int rc = make_dims(cfg, &d);
  if (rc != GTA_OK) return rc;
  if (!q || !k || !c || !l_out) return GTA_ERR_NULL;
  if (batch <= 0 || batch > kMaxBatch || total_tokens < 0 || total_tokens > INT32_MAX || max_seqlen < 0)
    return GTA_ERR_SHAPE;
  if (!cu_seqlens && (total_tokens % batch != 0 || total_tokens / batch > max_seqlen)) return GTA_ERR_SHAPE;
  if (misaligned(q) || misaligned(k) || misaligned(c) || misaligned(l_out) || ((uintptr_t)cu_seqlens & 3u))
    return GTA_ERR_ALIGN;
  if (total_tokens == 0 || max_seqlen == 0) return GTA_OK;
  hipStream_t st = (hipStream_t)hip_stream;
  if (attn_prefill_supported(d, max_seqlen))
    launch_attn_prefill_bf16(d, q, k, c, cu_seqlens, batch, total_tokens, max_seqlen, l_out, st);
  else
    launch_attn_prefill_rowwise(d, q, k, c, cu_seqlens, batch, total_tokens, max_seqlen, l_out, st);
  return check_launch();
}

int gta_prefill_projection(const gta_config *cfg, const gta_weights *weights, const void *x, const int32_t *cu_seqlens,
                           int32_t batch, int64_t total_tokens, int32_t max_seqlen, void *q_out, void *k_out,
                           void *c_out, void *g_out, void *workspace, size_t workspace_bytes, void *hip_stream) {
  Dims d;
  int rc = make_dims(cfg, &d);
  if (rc != GTA_OK) return rc;
  if ((rc = check_weights(weights)) != GTA_OK) return rc;
  if (!x || !q_out || !k_out || !c_out || !g_out) return GTA_ERR_NULL;
  if (batch <= 0 || batch > kMaxBatch || total_tokens < 0 || total_tokens > INT32_MAX || max_seqlen < 0)
    return GTA_ERR_SHAPE;
  if (!cu_seqlens && (total_tokens % batch != 0 || total_tokens / batch > max_seqlen)) return GTA_ERR_SHAPE;
  if (misaligned(x) || misaligned(q_out) || misaligned(k_out) || misaligned(c_out) || misaligned(g_out) ||
      ((uintptr_t)cu_seqlens & 3u))
    return GTA_ERR_ALIGN;
  if (!tuned_prefill_supported(d)) return GTA_ERR_UNSUPPORTED;
  if (total_tokens == 0 || max_seqlen == 0) return GTA_OK;
  if (!workspace || misaligned(workspace)) return GTA_ERR_WORKSPACE;
  PrefillWs ws = carve_prefill(d, true, weights->wo != nullptr, batch, total_tokens, max_seqlen, workspace);
  if (ws.bytes > workspace_bytes) return GTA_ERR_WORKSPACE;
  ws.q = q_out; ws.k = k_out; ws.c = c_out; ws.g = g_out;
  hipStream_t st = (hipStream_t)hip_stream;
  launch_prefill_setup(d, cu_seqlens, batch, total_tokens, max_seqlen, ws.seq_id, ws.pos, ws.rope, nullptr, nullptr, st);
  launch_proj_gemm(d, *weights, x, (int)total_tokens, ws, nullptr, nullptr, max_seqlen, st);
  return check_launch();
}

int gta_prefill_decoder(const gta_config *cfg, const gta_weights *weights, const void *l, const void *g,
                        int64_t total_tokens, void *out, void *hip_stream) {
  Dims d;
  int rc = make_dims(cfg, &d);
  if (rc != GTA_OK) return rc;
  if ((rc = check_weights(weights)) != GTA_OK) return rc;
  if (!l || !g || !out) return GTA_ERR_NULL;
  if (total_tokens < 0 || total_tokens > INT32_MAX) return GTA_ERR_SHAPE;
  if (misaligned(l) || misaligned(g) || misaligned(out)) return GTA_ERR_ALIGN;
  if (!tuned_prefill_supported(d)) return GTA_ERR_UNSUPPORTED;
  if (total_tokens == 0) return GTA_OK;
  launch_decoder_gemm(d, l, weights->wp, g, out, (int)total_tokens, (hipStream_t)hip_stream);
  return check_launch();
}

int gta_output_projection(const gta_config *cfg, const gta_weights *weights, const void *heads, int64_t total_tokens,
                          void *out, void *hip_stream) {
  Dims d;
  int rc = make_dims(cfg, &d);
  if (rc != GTA_OK) return rc;
  if ((rc = check_weights(weights)) != GTA_OK) return rc;
  if (!weights->wo || !heads || !out) return GTA_ERR_NULL;
  if (total_tokens < 0 || total_tokens > INT32_MAX) return GTA_ERR_SHAPE;
  if (misaligned(heads) || misaligned(out)) return GTA_ERR_ALIGN;
  if (!tuned_prefill_supported(d)) return GTA_ERR_UNSUPPORTED;
  if (total_tokens == 0) return GTA_OK;
  launch_plain_gemm(heads, d.wg_w, (int)total_tokens, d.H, d.wg_w, weights->wo, out, (hipStream_t)hip_stream);
  return check_launch();
}

static int decode_stage_args(const gta_config *cfg, const gta_cache *cache, const int32_t *slots, int32_t batch,
                             int32_t num_splits, void *workspace, size_t workspace_bytes, Dims *d, DecodeWs *ws) {
  int rc = make_dims(cfg, d);
  if (rc != GTA_OK) return rc;
  if (!cache) return GTA_ERR_NULL;
  if ((rc = check_cache(cache)) != GTA_OK) return rc;
  if (batch <= 0 || batch > kMaxBatch || num_splits < 0 || (!slots && batch > cache->max_batch)) return GTA_ERR_SHAPE;
  if ((uintptr_t)slots & 3u) return GTA_ERR_ALIGN;
  if (!workspace || misaligned(workspace)) return GTA_ERR_WORKSPACE;
  *ws = carve_decode(*d, true, batch, choose_splits(*d, batch, cache->max_seq, num_splits), workspace);
  return ws->bytes > workspace_bytes ? GTA_ERR_WORKSPACE : GTA_OK;
}

int gta_decode_attention(const gta_config *cfg, const float *q, const gta_cache *cache, const int32_t *slots,
                         int32_t batch, int32_t num_splits, void *workspace, size_t workspace_bytes,
                         void *hip_stream) {
  Dims d;
  DecodeWs ws;
  int rc = decode_stage_args(cfg, cache, slots, batch, num_splits, workspace, workspace_bytes, &d, &ws);
  if (rc != GTA_OK) return rc;
  if (!q) return GTA_ERR_NULL;
  if (misaligned(q)) return GTA_ERR_ALIGN;
  hipStream_t st = (hipStream_t)hip_stream;
  if (decode_is_tuned(d, *cache)) {
    tuned_decode_attention(d, q, nullptr, ws.oldlen, *cache, slots, batch, ws.splits, ws.part, st);
  } else {
    launch_cached_len(*cache, slots, batch, ws.oldlen, st);
    generic_decode_attention(d, q, ws.oldlen, *cache, slots, batch, ws.splits, ws.part, st);
  }
  return check_launch();
}

int gta_decode_combine(const gta_config *cfg, const gta_cache *cache, const int32_t *slots, int32_t batch,
                       int32_t num_splits, void *workspace, size_t workspace_bytes, float *l_out,
                       void *hip_stream) {
  Dims d;
  DecodeWs ws;
  int rc = decode_stage_args(cfg, cache, slots, batch, num_splits, workspace, workspace_bytes, &d, &ws);
  if (rc != GTA_OK) return rc;
  if (!l_out) return GTA_ERR_NULL;
  if (misaligned(l_out)) return GTA_ERR_ALIGN;
  hipStream_t st = (hipStream_t)hip_stream;
  if (decode_is_tuned(d, *cache)) tuned_decode_combine(d, ws.part, ws.oldlen, ws.splits, batch, l_out, st);
  else generic_decode_combine(d, ws.part, ws.oldlen, ws.splits, batch, l_out, st);
  return check_launch();
}

int gta_calibration_copy(const void *src, void *dst, int64_t bytes, void *hip_stream) {
  if (!src || !dst) return GTA_ERR_NULL;
  if (bytes < 0 || bytes % 16) return GTA_ERR_SHAPE;
  if (misaligned(src) || misaligned(dst)) return GTA_ERR_ALIGN;
  if (bytes == 0) return GTA_OK;
  return launch_calibration_copy(src, dst, bytes, (hipStream_t)hip_stream);
}

int gta_calibration_read(const void *src, int64_t bytes, int32_t workgroups, void *sink, void *hip_stream) {
  if (!src || !sink) return GTA_ERR_NULL;
  if (workgroups <= 0 || workgroups > 65535 || bytes <= 0 || bytes % ((int64_t)workgroups * 256 * 8 * 16)) return GTA_ERR_SHAPE;
  if (misaligned(src) || misaligned(sink)) return GTA_ERR_ALIGN;
  return launch_calibration_read(src, bytes, workgroups, sink, (hipStream_t)hip_stream);
}

int gta_calibration_mfma(int32_t workgroups, int32_t iters, int32_t random_operands, void *sink, void *hip_stream) {
  if (!sink) return GTA_ERR_NULL;
  if (workgroups <= 0 || workgroups > 65535 || iters <= 0) return GTA_ERR_SHAPE;
  if (misaligned(sink)) return GTA_ERR_ALIGN;
  if (random_operands != 0 && random_operands != 1) return GTA_ERR_DTYPE;
  return launch_calibration_mfma(workgroups, iters, random_operands == 1, sink, (hipStream_t)hip_stream);
}

int gta_cache_append(const gta_config *cfg, const gta_cache *cache, const int32_t *slots, const void *k_new,
                     const void *c_new, const int32_t *cu_new, int32_t batch, int32_t max_new, void *hip_stream) {
  Dims d;
  int rc = make_dims(cfg, &d);
  if (rc != GTA_OK) return rc;
  if (!cache || !k_new || !c_new || !cu_new) return GTA_ERR_NULL;
  if ((rc = check_cache(cache)) != GTA_OK) return rc;
  if (batch <= 0 || batch > kMaxBatch || max_new < 0 || max_new > (1 << 30) || (!slots && batch > cache->max_batch))
    return GTA_ERR_SHAPE;
  if (misaligned(k_new) || misaligned(c_new) || ((uintptr_t)cu_new & 3u) || ((uintptr_t)slots & 3u)) return GTA_ERR_ALIGN;
  return generic_cache_append(d, *cache, slots, k_new, c_new, cu_new, batch, max_new, (hipStream_t)hip_stream);
}

}  // extern "C"
