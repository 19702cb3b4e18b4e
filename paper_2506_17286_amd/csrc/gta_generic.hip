// Shape-generic HIP kernels of the GTA attention pass: any dimensions, fp32 or bf16 elements,
// fp32 arithmetic throughout.  They are the path for the fp32 workloads and for shapes the tuned
// bf16 kernels do not cover; they favour being obviously right over speed.
//
// Pipeline (paper Sec. 3.2-3.3, per-token form App. B.1):
//   prefill: row map -> RoPE table -> 4 projection GEMMs (raw fp32) -> finalize (RoPE, split into
//            Q/K/C/gate, cache write) -> one wave per (query row, map group) online-softmax
//            attention over the latent values -> decoder GEMM with sigmoid-gate epilogue -> [W_O]
//   decode : projection GEMMs -> finalize (RoPE at pos = seq_len, append row) -> split-K attention
//            partials -> log-sum-exp combine -> decoder GEMM with gate epilogue -> [W_O] -> commit
#include <math.h>

#include "gta_internal.h"

namespace gta {
namespace {

typedef __bf16 bf16;

template <typename T> __device__ __forceinline__ float ldf(const T *p, int64_t i) { return (float)p[i]; }
template <typename T> __device__ __forceinline__ void stf(T *p, int64_t i, float v) { p[i] = (T)v; }

__device__ __forceinline__ float sigmoid_f32(float z) { return 1.0f / (1.0f + expf(-z)); }

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

// ------------------------------------------------------------------------------ small kernels
__device__ __forceinline__ void rowmap_row(const int32_t *cu, int batch, int per_seq, int64_t t, int32_t *seq_id,
                                           int32_t *pos) {
  if (!cu) {
    seq_id[t] = (int32_t)(t / per_seq);
    pos[t] = (int32_t)(t % per_seq);
    return;
  }
  int lo = 0, hi = batch;  // largest b with cu[b] <= t
  while (hi - lo > 1) {
    int mid = (lo + hi) >> 1;
    if (cu[mid] <= t) lo = mid; else hi = mid;
  }
  seq_id[t] = lo;
  pos[t] = (int32_t)(t - cu[lo]);
}

__global__ void rowmap_kernel(const int32_t *cu, int batch, int64_t total, int per_seq,
                              int32_t *seq_id, int32_t *pos) {
  int64_t t = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
  if (t < total) rowmap_row(cu, batch, per_seq, t, seq_id, pos);
}

// (cos, sin) of pos * base^(-2j/d_h), evaluated in fp64 and rounded once to fp32 (App. B.1.1).
__device__ __forceinline__ void rope_table_entry(float2 *tab, int half, int dh, double base, int64_t i) {
  int p = (int)(i / half), j = (int)(i % half);
  double ang = (double)p * pow(base, -2.0 * (double)j / (double)dh);
  double s, c;
  sincos(ang, &s, &c);
  tab[i] = make_float2((float)c, (float)s);
}

__global__ void rope_table_kernel(float2 *tab, int max_pos, int half, int dh, double base) {
  int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
  if (i < (int64_t)max_pos * half) rope_table_entry(tab, half, dh, base, i);
}

// ------------------------------------------------------------------------------ generic GEMM
struct EpiStoreF32 {
  float *out; int64_t ld; int col_off;
  __device__ void operator()(int row, int col, int, float v) const { out[(int64_t)row * ld + col_off + col] = v; }
};
template <typename T> struct EpiStoreT {
  T *out; int64_t ld;
  __device__ void operator()(int row, int col, int, float v) const { stf(out, (int64_t)row * ld + col, v); }
};
// Value-decoder epilogue (Sec. 3.2): head z, element col: v * Sigmoid(gate pre-activation).
template <typename TO> struct EpiGate {
  TO *out; int64_t ldo; const float *g; int64_t ldg; int dh; int gate;
  __device__ void operator()(int row, int col, int z, float v) const {
    int c = z * dh + col;
    if (gate == kGateSigmoid) v *= sigmoid_f32(g[(int64_t)row * ldg + c]);
    else if (gate) v *= gate_factor(gate, g[(int64_t)row * ldg + c]);
    stf(out, (int64_t)row * ldo + c, v);
  }
};

// out(z) = A(z / a_bdiv) [M,K] . B(z) [K,N], fp32 accumulation, 64x64x16 LDS tiles.
template <typename TA, typename TB, typename Epi>
__global__ __launch_bounds__(256) void gemm_generic_kernel(const TA *A, int64_t lda, int64_t a_bstride,
                                                           int a_bdiv, const TB *B, int64_t ldb,
                                                           int64_t b_bstride, int M, int N, int K, Epi epi) {
  __shared__ float As[16][65];
  __shared__ float Bs[16][65];
  const int z = blockIdx.z;
  A += (int64_t)(z / a_bdiv) * a_bstride;
  B += (int64_t)z * b_bstride;
  const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
  const int m0 = blockIdx.y * 64, n0 = blockIdx.x * 64;
  float acc[4][4] = {};
  for (int k0 = 0; k0 < K; k0 += 16) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      int idx = tid + i * 256;
      int am = idx >> 4, ak = idx & 15;
      As[ak][am] = (m0 + am < M && k0 + ak < K) ? ldf(A, (int64_t)(m0 + am) * lda + k0 + ak) : 0.f;
      int bk = idx >> 6, bn = idx & 63;
      Bs[bk][bn] = (k0 + bk < K && n0 + bn < N) ? ldf(B, (int64_t)(k0 + bk) * ldb + n0 + bn) : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < 16; ++kk) {
      float a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) { a[i] = As[kk][ty * 4 + i]; b[i] = Bs[kk][tx * 4 + i]; }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] += a[i] * b[j];
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      int row = m0 + ty * 4 + i, col = n0 + tx * 4 + j;
      if (row < M && col < N) epi(row, col, z, acc[i][j]);
    }
}

template <typename TA, typename TB, typename Epi>
void launch_gemm(const TA *A, int64_t lda, int64_t a_bstride, int a_bdiv, const TB *B, int64_t ldb,
                 int64_t b_bstride, int M, int N, int K, int nbatch, Epi epi, hipStream_t st) {
  if (M <= 0 || N <= 0) return;
  dim3 grid((N + 63) / 64, (M + 63) / 64, nbatch);
  gemm_generic_kernel<TA, TB, Epi><<<grid, 256, 0, st>>>(A, lda, a_bstride, a_bdiv, B, ldb, b_bstride, M, N, K, epi);
}

// ------------------------------------------------------------------------------ finalize
struct CacheView {
  void *k, *c;
  int32_t *seq_lens, *status;
  const int32_t *slots;
  int max_batch, max_seq;
  PageMap pm;
};

// Splits the raw projections into Q | K | C | gate, rotates q and k (App. B.1.1) and stores the
// key / latent rows into the caches at row = position.  rope_by_token: the RoPE table has one row per
// packed token (chunked prefill) instead of one per position; a position < 0 marks a skipped sequence.
template <typename T>
__global__ void finalize_prefill_kernel(Dims d, const float *praw, const int32_t *seq_id, const int32_t *pos,
                                        const float2 *rope, int max_len, int64_t total, T *Q, T *K, T *C,
                                        float *G, CacheView cv, int rope_by_token = 0) {
  int64_t idx = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
  if (idx >= total * d.wtot) return;
  int64_t t = idx / d.wtot;
  int col = (int)(idx % d.wtot);
  float v = praw[idx];
  const int p = pos[t];
  const int qk_w = d.wq_w + d.wk_w;
  if (col < qk_w && d.rope && (rope_by_token || p < max_len)) {
    int e = col % d.dh, half = d.dh / 2;
    float2 cs = rope[(rope_by_token ? t : (int64_t)p) * half + (e % half)];
    if (e < half) v = v * cs.x - praw[idx + half] * cs.y;
    else          v = v * cs.x + praw[idx - half] * cs.y;
  }
  int slot = -1;
  if (cv.k) {
    int b = seq_id[t];
    slot = cv.slots ? cv.slots[b] : b;
    if (slot < 0 || slot >= cv.max_batch || p >= cv.max_seq || p < 0) slot = -1;
  }
  if (col < d.wq_w) {
    stf(Q, t * d.wq_w + col, v);
  } else if (col < qk_w) {
    int c = col - d.wq_w;
    stf(K, t * d.wk_w + c, v);
    const int64_t cr = slot >= 0 ? cache_row(cv.pm, cv.max_seq, slot, p) : -1;
    if (cr >= 0) stf((T *)cv.k, cr * d.wk_w + c, v);
  } else if (col < qk_w + d.wc_w) {
    int c = col - qk_w;
    stf(C, t * d.wc_w + c, v);
    const int64_t cr = slot >= 0 ? cache_row(cv.pm, cv.max_seq, slot, p) : -1;
    if (cr >= 0) stf((T *)cv.c, cr * d.wc_w + c, v);
  } else {
    G[t * d.wg_w + (col - qk_w - d.wc_w)] = v;
  }
}

__device__ __forceinline__ void prefill_commit_seq(const CacheView &cv, const int32_t *cu, int per_seq, int b) {
  int n = cu ? cu[b + 1] - cu[b] : per_seq;
  int slot = cv.slots ? cv.slots[b] : b;
  if (slot < 0 || slot >= cv.max_batch) return;
  if (n <= cv.max_seq && rows_backed(cv.pm, slot, 0, n)) cv.seq_lens[slot] = n;
  else cv.status[slot] = GTA_ERR_CACHE_FULL;
}

__global__ void prefill_commit_kernel(CacheView cv, const int32_t *cu, int batch, int per_seq) {
  int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b < batch) prefill_commit_seq(cv, cu, per_seq, b);
}

// Everything a prefill call derives from the sequence offsets alone, in one launch: blocks
// [0, nb_row) fill the row -> (sequence, position) map, the next nb_rope blocks the RoPE table, the
// rest set the cached lengths (nothing below reads the lengths back during the call).
__global__ void prefill_setup_kernel(const int32_t *cu, int batch, int64_t total, int per_seq, int32_t *seq_id,
                                     int32_t *pos, int nb_row, float2 *tab, int max_pos, int half, int dh,
                                     double base, int nb_rope, CacheView cv) {
  int blk = blockIdx.x;
  if (blk < nb_row) {
    int64_t t = blk * (int64_t)blockDim.x + threadIdx.x;
    if (t < total) rowmap_row(cu, batch, per_seq, t, seq_id, pos);
    return;
  }
  blk -= nb_row;
  if (blk < nb_rope) {
    int64_t i = blk * (int64_t)blockDim.x + threadIdx.x;
    if (i < (int64_t)max_pos * half) rope_table_entry(tab, half, dh, base, i);
    return;
  }
  blk -= nb_rope;
  int b = blk * blockDim.x + threadIdx.x;
  if (b < batch) prefill_commit_seq(cv, cu, per_seq, b);
}

// Chunked prefill (a chunk of new tokens behind the rows a slot already holds, App. B.1.3 applied to
// several tokens at once).  prefix[b] = rows cached before the chunk, or -1 if the slot is invalid or
// the chunk does not fit (the sequence is then skipped: nothing stored, zero output, status flagged at
// commit).  Token t of sequence b gets position prefix[b] + (t - cu[b]); the RoPE table is per packed
// token here (row t), since positions of different sequences no longer coincide.  Blocks [0, nb_row):
// row map, then nb_rope blocks: RoPE rows, last blocks: prefix[].  Nothing in this launch writes the
// cached lengths, so every block may read them.
__device__ __forceinline__ int chunk_prefix(const CacheView &cv, const int32_t *cu, int per_seq, int b) {
  const int slot = cv.slots ? cv.slots[b] : b;
  if (slot < 0 || slot >= cv.max_batch) return -1;
  const int old = cv.seq_lens[slot], n = cu ? cu[b + 1] - cu[b] : per_seq;
  return (old >= 0 && old + n <= cv.max_seq && rows_backed(cv.pm, slot, old, old + n)) ? old : -1;
}

__global__ void prefill_chunk_setup_kernel(const int32_t *cu, int batch, int64_t total, int per_seq, int32_t *seq_id,
                                           int32_t *pos, int nb_row, float2 *tab, int half, int dh, double base,
                                           int nb_rope, CacheView cv, int32_t *prefix) {
  int blk = blockIdx.x;
  auto locate = [&](int64_t t, int &b, int &i) {
    if (!cu) { b = (int)(t / per_seq); i = (int)(t % per_seq); return; }
    int lo = 0, hi = batch;
    while (hi - lo > 1) {
      int mid = (lo + hi) >> 1;
      if (cu[mid] <= t) lo = mid; else hi = mid;
    }
    b = lo; i = (int)(t - cu[lo]);
  };
  if (blk < nb_row) {
    int64_t t = blk * (int64_t)blockDim.x + threadIdx.x;
    if (t >= total) return;
    int b, i;
    locate(t, b, i);
    const int pre = chunk_prefix(cv, cu, per_seq, b);
    seq_id[t] = b;
    pos[t] = pre < 0 ? -1 : pre + i;
    return;
  }
  blk -= nb_row;
  if (blk < nb_rope) {
    int64_t e = blk * (int64_t)blockDim.x + threadIdx.x;
    if (e >= total * half) return;
    int b, i;
    locate(e / half, b, i);
    const int pre = chunk_prefix(cv, cu, per_seq, b), j = (int)(e % half);
    double ang = (double)(pre < 0 ? 0 : pre + i) * pow(base, -2.0 * (double)j / (double)dh);
    double sn, cs;
    sincos(ang, &sn, &cs);
    tab[e] = make_float2((float)cs, (float)sn);
    return;
  }
  blk -= nb_rope;
  int b = blk * blockDim.x + threadIdx.x;
  if (b < batch) prefix[b] = chunk_prefix(cv, cu, per_seq, b);
}

__global__ void prefill_chunk_commit_kernel(CacheView cv, const int32_t *cu, int batch, int per_seq,
                                            const int32_t *prefix) {
  int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b >= batch) return;
  const int slot = cv.slots ? cv.slots[b] : b;
  if (slot < 0 || slot >= cv.max_batch) return;
  if (prefix[b] >= 0) cv.seq_lens[slot] = prefix[b] + (cu ? cu[b + 1] - cu[b] : per_seq);
  else cv.status[slot] = GTA_ERR_CACHE_FULL;
}

// Decode: position = tokens already cached; the new key / latent row is appended at that row.
template <typename T>
__global__ void finalize_decode_kernel(Dims d, const float *praw, int nsum, int batch, float *Qo, float *Go,
                                       int32_t *oldlen, CacheView cv) {
  int64_t idx = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
  if (idx >= (int64_t)batch * d.wtot) return;
  int b = (int)(idx / d.wtot);
  int col = (int)(idx % d.wtot);
  int slot = cv.slots ? cv.slots[b] : b;
  bool slot_ok = slot >= 0 && slot < cv.max_batch;
  int p = slot_ok ? cv.seq_lens[slot] : 0;
  bool ok = slot_ok && p >= 0 && p < cv.max_seq;
  const int64_t cr = ok ? cache_row(cv.pm, cv.max_seq, slot, p) : -1;   // a row without a page: slot full
  ok = cr >= 0;
  if (col == 0) oldlen[b] = ok ? p : -1;
  if (!ok) return;
  // the projection may arrive as `nsum` split-K partials of [batch, wtot]
  const int64_t pstride = (int64_t)batch * d.wtot;
  auto raw = [&](int64_t i) {
    float a = praw[i];
    for (int s = 1; s < nsum; ++s) a += praw[s * pstride + i];
    return a;
  };
  float v = raw(idx);
  const int qk_w = d.wq_w + d.wk_w;
  if (col < qk_w && d.rope) {
    int e = col % d.dh, half = d.dh / 2;
    double ang = (double)p * pow(d.rope_base, -2.0 * (double)(e % half) / (double)d.dh);
    double sn, cs;
    sincos(ang, &sn, &cs);
    if (e < half) v = v * (float)cs - raw(idx + half) * (float)sn;
    else          v = v * (float)cs + raw(idx - half) * (float)sn;
  }
  if (col < d.wq_w) {
    Qo[(int64_t)b * d.wq_w + col] = v;
  } else if (col < qk_w) {
    stf((T *)cv.k, cr * d.wk_w + (col - d.wq_w), v);
  } else if (col < qk_w + d.wc_w) {
    stf((T *)cv.c, cr * d.wc_w + (col - qk_w), v);
  } else {
    Go[(int64_t)b * d.wg_w + (col - qk_w - d.wc_w)] = v;
  }
}

// Stage entry support: attend over the rows already cached (no append): "old length" = seq_len - 1.
__global__ void cached_len_kernel(CacheView cv, int batch, int32_t *oldlen) {
  int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b >= batch) return;
  int slot = cv.slots ? cv.slots[b] : b;
  int n = (slot >= 0 && slot < cv.max_batch) ? cv.seq_lens[slot] : 0;
  oldlen[b] = (n > cv.max_seq ? cv.max_seq : n) - 1;
}

__global__ void decode_commit_kernel(CacheView cv, const int32_t *oldlen, int batch) {
  int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b >= batch) return;
  int slot = cv.slots ? cv.slots[b] : b;
  if (slot < 0 || slot >= cv.max_batch) return;
  if (oldlen[b] >= 0) cv.seq_lens[slot] = oldlen[b] + 1;
  else cv.status[slot] = GTA_ERR_CACHE_FULL;
}

// ------------------------------------------------------------------------------ attention
// One wave walks keys [j0, j1) of one (sequence, key group): scores of 64 keys at a time (one key
// per lane), running max / sum (Sec. 3.3 softmax, evaluated online), and the latent-value
// accumulation L += p_j C_j (reformulated form of Sec. 3.3) with lane-strided columns.
// row_of(j) = row of key / latent j in Kb / Cb (identity for a packed sequence, the page map for a cache).
template <typename T, int NACC, class RowOf>
__device__ void wave_attend(const float *qw, const T *Kb, int64_t kstride, const T *Cb, int64_t cstride,
                            int j0, int j1, int dh, int c0, int dl, int lane, float &m, float &l,
                            float (&acc)[NACC], RowOf row_of) {
  for (int jb = j0; jb < j1; jb += 64) {
    const int j = jb + lane;
    const bool valid = j < j1;
    float s = -INFINITY;
    if (valid) {
      const T *kr = Kb + row_of(j) * kstride;
      float a = 0.f;
      for (int e = 0; e < dh; ++e) a += qw[e] * ldf(kr, e);
      s = a;
    }
    const float m_new = fmaxf(m, wave_max(s));
    const float corr = expf(m - m_new);
    const float p = valid ? expf(s - m_new) : 0.f;
    l = l * corr + wave_sum(p);
#pragma unroll
    for (int i = 0; i < NACC; ++i) acc[i] *= corr;
    m = m_new;
    const int cnt = min(64, j1 - jb);
    for (int jj = 0; jj < cnt; ++jj) {
      const float pj = __shfl(p, jj, 64);
      const T *cr = Cb + row_of(jb + jj) * cstride + c0;
#pragma unroll
      for (int i = 0; i < NACC; ++i) {
        int col = lane + 64 * i;
        if (c0 + col < dl) acc[i] += pj * ldf(cr, col);
      }
    }
  }
}

constexpr int kNAcc = 16;  // 64 lanes x 16 = 1024 latent columns per pass

template <typename T, typename TL>
__global__ __launch_bounds__(256) void attn_prefill_generic_kernel(Dims d, const T *Q, const T *K, const T *C,
                                                                   const int32_t *cu, int per_seq, int max_len,
                                                                   TL *L) {
  extern __shared__ float qs[];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int b = blockIdx.z, g = blockIdx.y;
  const int64_t start = cu ? cu[b] : (int64_t)b * per_seq;
  const int Tb = min(cu ? cu[b + 1] - cu[b] : per_seq, max_len);
  const int t = blockIdx.x * 4 + wave;
  const bool active = t < Tb;
  float *qw = qs + wave * d.dh;
  if (active)
    for (int e = lane; e < d.dh; e += 64) qw[e] = ldf(Q, (start + t) * d.wq_w + g * d.dh + e) * d.scale;
  __syncthreads();
  if (!active) return;
  const T *Kb = K + start * d.wk_w + (g / d.qpk) * d.dh;
  const T *Cb = C + start * d.wc_w + (g / d.qpc) * d.dl;
  for (int c0 = 0; c0 < d.dl; c0 += 64 * kNAcc) {
    float m = -INFINITY, l = 0.f, acc[kNAcc] = {};
    wave_attend<T, kNAcc>(qw, Kb, d.wk_w, Cb, d.wc_w, 0, t + 1, d.dh, c0, d.dl, lane, m, l, acc,
                          [](int j) { return (int64_t)j; });
    const float inv = 1.0f / l;
    TL *Lr = L + (start + t) * (int64_t)(d.nq * d.dl) + g * d.dl + c0;
#pragma unroll
    for (int i = 0; i < kNAcc; ++i) {
      int col = lane + 64 * i;
      if (c0 + col < d.dl) stf(Lr, col, acc[i] * inv);
    }
  }
}

// Chunked prefill: token t of sequence b's chunk attends over cache rows 0 .. prefix[b] + t of its
// slot (the chunk's own rows are already stored there).  A skipped sequence (prefix < 0) gets zeros.
template <typename T, typename TL>
__global__ __launch_bounds__(256) void attn_chunk_generic_kernel(Dims d, const T *Q, CacheView cv, const int32_t *prefix,
                                                                 const int32_t *cu, int per_seq, TL *L) {
  extern __shared__ float qs[];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int b = blockIdx.z, g = blockIdx.y;
  const int64_t start = cu ? cu[b] : (int64_t)b * per_seq;
  const int Tb = cu ? cu[b + 1] - cu[b] : per_seq;
  const int t = blockIdx.x * 4 + wave;
  const bool active = t < Tb;
  const int P = prefix[b];
  float *qw = qs + wave * d.dh;
  if (active && P >= 0)
    for (int e = lane; e < d.dh; e += 64) qw[e] = ldf(Q, (start + t) * d.wq_w + g * d.dh + e) * d.scale;
  __syncthreads();
  if (!active) return;
  TL *Lrow = L + (start + t) * (int64_t)(d.nq * d.dl) + g * d.dl;
  if (P < 0) {
    for (int col = lane; col < d.dl; col += 64) stf(Lrow, col, 0.f);
    return;
  }
  const int slot = cv.slots ? cv.slots[b] : b;   // valid: prefix >= 0
  const T *Kb = (const T *)cv.k + (g / d.qpk) * d.dh;
  const T *Cb = (const T *)cv.c + (g / d.qpc) * d.dl;
  for (int c0 = 0; c0 < d.dl; c0 += 64 * kNAcc) {
    float m = -INFINITY, l = 0.f, acc[kNAcc] = {};
    wave_attend<T, kNAcc>(qw, Kb, d.wk_w, Cb, d.wc_w, 0, P + t + 1, d.dh, c0, d.dl, lane, m, l, acc,
                          [&](int j) { return cache_row_clamped(cv.pm, cv.max_seq, slot, j); });
    const float inv = 1.0f / l;
#pragma unroll
    for (int i = 0; i < kNAcc; ++i) {
      int col = lane + 64 * i;
      if (c0 + col < d.dl) stf(Lrow + c0, col, acc[i] * inv);
    }
  }
}

// Split-K decode: block (split, group, sequence) = one wave; un-normalised partial (acc, m, l).
template <typename T>
__global__ __launch_bounds__(64) void attn_decode_generic_kernel(Dims d, const float *Q, const int32_t *oldlen,
                                                                 CacheView cv, int splits, float *part) {
  extern __shared__ float qs[];
  const int lane = threadIdx.x;
  const int s = blockIdx.x, g = blockIdx.y, b = blockIdx.z;
  const int old = oldlen[b];
  float *pr = part + (((int64_t)b * splits + s) * d.nq + g) * (d.dl + 2);
  int j0 = 0, j1 = 0;
  const T *Kb = (const T *)cv.k + (g / d.qpk) * d.dh, *Cb = (const T *)cv.c + (g / d.qpc) * d.dl;
  int slot = 0;
  if (old >= 0) {
    const int n = old + 1;
    const int chunk = (n + splits - 1) / splits;
    j0 = min(n, s * chunk);
    j1 = min(n, j0 + chunk);
    slot = cv.slots ? cv.slots[b] : b;
    for (int e = lane; e < d.dh; e += 64) qs[e] = Q[(int64_t)b * d.wq_w + g * d.dh + e] * d.scale;
  }
  __syncthreads();
  for (int c0 = 0; c0 < d.dl; c0 += 64 * kNAcc) {
    float m = -INFINITY, l = 0.f, acc[kNAcc] = {};
    if (j1 > j0)
      wave_attend<T, kNAcc>(qs, Kb, d.wk_w, Cb, d.wc_w, j0, j1, d.dh, c0, d.dl, lane, m, l, acc,
                            [&](int j) { return cache_row_clamped(cv.pm, cv.max_seq, slot, j); });
#pragma unroll
    for (int i = 0; i < kNAcc; ++i) {
      int col = lane + 64 * i;
      if (c0 + col < d.dl) pr[c0 + col] = acc[i];
    }
    if (lane == 0) { pr[d.dl] = m; pr[d.dl + 1] = l; }
  }
}

// Merge the splits of one (sequence, group) by their log-sum-exp weights; L = sum acc / sum l.
__global__ void decode_combine_kernel(Dims d, const float *part, const int32_t *oldlen, int splits, float *L) {
  const int g = blockIdx.x, b = blockIdx.y;
  const float *pb = part + ((int64_t)b * splits * d.nq + g) * (d.dl + 2);
  const int64_t sstride = (int64_t)d.nq * (d.dl + 2);
  float *Lr = L + ((int64_t)b * d.nq + g) * d.dl;
  if (oldlen[b] < 0) {
    for (int c = threadIdx.x; c < d.dl; c += blockDim.x) Lr[c] = 0.f;
    return;
  }
  float mx = -INFINITY;
  for (int s = 0; s < splits; ++s) mx = fmaxf(mx, pb[s * sstride + d.dl]);
  float lsum = 0.f;
  for (int s = 0; s < splits; ++s) {
    float ms = pb[s * sstride + d.dl];
    if (ms > -INFINITY) lsum += expf(ms - mx) * pb[s * sstride + d.dl + 1];
  }
  const float inv = 1.0f / lsum;
  for (int c = threadIdx.x; c < d.dl; c += blockDim.x) {
    float a = 0.f;
    for (int s = 0; s < splits; ++s) {
      float ms = pb[s * sstride + d.dl];
      if (ms > -INFINITY) a += expf(ms - mx) * pb[s * sstride + c];
    }
    Lr[c] = a * inv;
  }
}

// ------------------------------------------------------------------------------ cache append
// Row copy in 16-, 4- or 2-byte words, whichever divides the row size (bit-exact by construction).
template <typename W>
__device__ void copy_row(const void *src, void *dst, int nbytes) {
  const W *s = (const W *)src;
  W *t = (W *)dst;
  for (int i = threadIdx.x; i < nbytes / (int)sizeof(W); i += blockDim.x) t[i] = s[i];
}
__device__ void copy_row_any(const void *src, void *dst, int nbytes) {
  if (nbytes % 16 == 0) copy_row<uint4>(src, dst, nbytes);
  else if (nbytes % 4 == 0) copy_row<uint32_t>(src, dst, nbytes);
  else copy_row<uint16_t>(src, dst, nbytes);
}

__global__ void append_copy_kernel(CacheView cv, const char *k_new, const char *c_new, const int32_t *cu_new,
                                   int krow_bytes, int crow_bytes, int max_new) {
  const int j = blockIdx.x, b = blockIdx.y;
  const int n = cu_new[b + 1] - cu_new[b];
  if (j >= n || n > max_new) return;
  const int slot = cv.slots ? cv.slots[b] : b;
  if (slot < 0 || slot >= cv.max_batch) return;
  const int p = cv.seq_lens[slot];
  if (p < 0 || (int64_t)p + n > cv.max_seq) return;
  if (!rows_backed(cv.pm, slot, p, p + n)) return;   // a row of the range has no page: nothing is stored, the commit kernel flags the slot
  const int64_t src = (int64_t)cu_new[b] + j, dst = cache_row(cv.pm, cv.max_seq, slot, p + j);
  if (dst < 0) return;
  copy_row_any(k_new + src * krow_bytes, (char *)cv.k + dst * krow_bytes, krow_bytes);
  copy_row_any(c_new + src * crow_bytes, (char *)cv.c + dst * crow_bytes, crow_bytes);
}

__global__ void append_commit_kernel(CacheView cv, const int32_t *cu_new, int batch, int max_new) {
  int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b >= batch) return;
  const int n = cu_new[b + 1] - cu_new[b];
  const int slot = cv.slots ? cv.slots[b] : b;
  if (slot < 0 || slot >= cv.max_batch || n <= 0) return;
  if (n > max_new) { cv.status[slot] = GTA_ERR_SHAPE; return; }  // caller's bound was wrong: nothing copied
  const int p = cv.seq_lens[slot];
  if (p < 0 || (int64_t)p + n > cv.max_seq || !rows_backed(cv.pm, slot, p, p + n)) cv.status[slot] = GTA_ERR_CACHE_FULL;
  else cv.seq_lens[slot] = p + n;
}

// Plain device-to-device copy in 16-byte words: the known-traffic reference that hardware
// counters (bytes fetched / written per dispatch) are calibrated against.
__global__ __launch_bounds__(256) void calibration_copy_kernel(const uint4 *__restrict__ src, uint4 *__restrict__ dst,
                                                               int64_t nwords) {
  for (int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; i < nwords; i += (int64_t)gridDim.x * blockDim.x)
    dst[i] = src[i];
}

// Streaming read of 16-byte words with non-temporal loads, one contiguous slice per workgroup: what
// the memory system delivers to a kernel that does nothing else.  The xor of everything read goes to
// `sink` only if it matches an arbitrary constant, so the loads cannot be dropped.
typedef unsigned int cal_u32x4 __attribute__((ext_vector_type(4)));
__global__ __launch_bounds__(256) void calibration_read_kernel(const cal_u32x4 *__restrict__ src, int64_t words_per_wg,
                                                               uint32_t *sink) {
  const cal_u32x4 *base = src + (int64_t)blockIdx.x * words_per_wg + threadIdx.x;
  cal_u32x4 acc = {0u, 0u, 0u, 0u};
  for (int64_t i = 0; i < words_per_wg; i += 256 * 8) {
    cal_u32x4 v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = __builtin_nontemporal_load(base + i + u * 256);
#pragma unroll
    for (int u = 0; u < 8; ++u) acc ^= v[u];
  }
  if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x9e3779b9u) sink[threadIdx.x] = acc.x;
}

// Nothing but v_mfma_f32_32x32x16_bf16 on 16 independent accumulators, four waves per CU (one per
// SIMD): the rate the matrix pipes sustain at the clock the chip holds under that load.
typedef __attribute__((ext_vector_type(8))) __bf16 cal_bf16x8;
typedef __attribute__((ext_vector_type(16))) float cal_f32x16;
// RANDOM: eight operand pairs per lane with values spread like the workloads' activations (about
// N(0,1)) and weights (about N(0,0.02)), used in rotation, so that the operand bits the matrix pipes
// see change from one instruction to the next as they do inside a GEMM; otherwise one pair of small
// constants.  What the chip sustains differs by a quarter between the two: it is power-limited.
__device__ __forceinline__ unsigned cal_hash(unsigned x) {
  x ^= x >> 16; x *= 0x7feb352du; x ^= x >> 15; x *= 0x846ca68bu; x ^= x >> 16;
  return x;
}
template <bool RANDOM>
__global__ __launch_bounds__(256) void calibration_mfma_kernel(int iters, float *sink) {
  constexpr int NS = RANDOM ? 8 : 1;
  cal_bf16x8 x[NS], y[NS];
#pragma unroll
  for (int s = 0; s < NS; ++s)
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      if (RANDOM) {
        const unsigned h1 = cal_hash(threadIdx.x * 977u + s * 131u + i * 7u + blockIdx.x * 7919u), h2 = cal_hash(h1 + 12345u);
        const float u = ((float)(h1 & 0xffff) + (float)(h1 >> 16) + (float)(h2 & 0xffff) + (float)(h2 >> 16)) / 65536.0f - 2.0f;
        x[s][i] = (__bf16)(u * 1.7f);
        y[s][i] = (__bf16)(-u * 0.034f + 0.001f * (float)i);
      } else {
        x[s][i] = (__bf16)(0.001f * (float)((threadIdx.x * 7 + i) % 13) - 0.006f);
        y[s][i] = (__bf16)(0.002f * (float)((threadIdx.x * 5 + i) % 11) - 0.01f);
      }
    }
  cal_f32x16 acc[16];
#pragma unroll
  for (int t = 0; t < 16; ++t)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[t][r] = 0.f;
  for (int it = 0; it < iters; ++it)
#pragma unroll
    for (int t = 0; t < 16; ++t)
      acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(x[t % NS], y[(t + t / NS) % NS], acc[t], 0, 0, 0);
  float v = 0.f;
#pragma unroll
  for (int t = 0; t < 16; ++t) v += acc[t][0] + acc[t][15];
  if (v == 123.456f) sink[threadIdx.x] = v;
}

CacheView view_of(const gta_cache *c, const int32_t *slots) {
  CacheView v{};
  if (c) {
    v.k = c->k; v.c = c->c; v.seq_lens = c->seq_lens; v.status = c->status;
    v.max_batch = c->max_batch; v.max_seq = c->max_seq;
    v.pm = page_map_of(*c);
  }
  v.slots = slots;
  return v;
}

inline dim3 grid1d(int64_t n, int block = 256) { return dim3((unsigned)((n + block - 1) / block)); }

// ------------------------------------------------------------------------------ drivers
template <typename T>
int prefill_impl(const Dims &d, const gta_weights &w, const T *x, const int32_t *cu, int batch, int64_t total,
                 int max_len, const gta_cache *cache, const int32_t *slots, T *out, const PrefillWs &ws,
                 hipStream_t st) {
  const int per_seq = (int)(total / batch);
  const int M = (int)total;
  launch_rowmap(cu, batch, total, ws.seq_id, ws.pos, st);
  if (d.rope) launch_rope_table(ws.rope, max_len, d.dh, d.rope_base, st);
  // Sec. 3.2 projections, raw fp32: [Q | K | C | gate pre-activation]
  const T *wmat[4] = {(const T *)w.wq, (const T *)w.wk, (const T *)w.wc, (const T *)w.wg};
  const int wn[4] = {d.wq_w, d.wk_w, d.wc_w, d.wg_w};
  int off = 0;
  for (int i = 0; i < 4; ++i) {
    launch_gemm(x, (int64_t)d.H, 0, 1, wmat[i], (int64_t)wn[i], 0, M, wn[i], d.H, 1,
                EpiStoreF32{ws.praw, d.wtot, off}, st);
    off += wn[i];
  }
  CacheView cv = view_of(cache, slots);
  finalize_prefill_kernel<T><<<grid1d(total * d.wtot), 256, 0, st>>>(
      d, ws.praw, ws.seq_id, ws.pos, ws.rope, max_len, total, (T *)ws.q, (T *)ws.k, (T *)ws.c, (float *)ws.g, cv);
  if (cache) launch_prefill_commit(*cache, slots, cu, batch, total, st);
  // shared attention map x latent values, one map per group (Sec. 3.3)
  dim3 agrid((max_len + 3) / 4, d.nq, batch);
  attn_prefill_generic_kernel<T, float><<<agrid, 256, 4 * d.dh * sizeof(float), st>>>(
      d, (const T *)ws.q, (const T *)ws.k, (const T *)ws.c, cu, per_seq, max_len, (float *)ws.l);
  // value decoder with gate epilogue (Sec. 3.2), then the optional output projection (Sec. 3.3)
  const float *L = (const float *)ws.l;
  if (w.wo) {
    float *O = (float *)ws.o;
    launch_gemm(L, (int64_t)d.nq * d.dl, (int64_t)d.dl, d.hpq, (const T *)w.wp, (int64_t)d.dh, (int64_t)d.dl * d.dh,
                M, d.dh, d.dl, d.nh, EpiGate<float>{O, d.wg_w, (const float *)ws.g, d.wg_w, d.dh, d.gate}, st);
    launch_gemm(O, (int64_t)d.wg_w, 0, 1, (const T *)w.wo, (int64_t)d.H, 0, M, d.H, d.wg_w, 1,
                EpiStoreT<T>{out, d.H}, st);
  } else {
    launch_gemm(L, (int64_t)d.nq * d.dl, (int64_t)d.dl, d.hpq, (const T *)w.wp, (int64_t)d.dh, (int64_t)d.dl * d.dh,
                M, d.dh, d.dl, d.nh, EpiGate<T>{out, d.wg_w, (const float *)ws.g, d.wg_w, d.dh, d.gate}, st);
  }
  return check_launch();
}

// Chunked prefill on the shape-generic kernels: same steps as prefill_impl with positions behind the
// cached rows, keys and latents read back from the caches.
template <typename T>
int prefill_chunk_impl(const Dims &d, const gta_weights &w, const T *x, const int32_t *cu, int batch, int64_t total,
                       int max_chunk, const gta_cache &cache, const int32_t *slots, T *out, const PrefillWs &ws,
                       hipStream_t st) {
  const int per_seq = (int)(total / batch);
  const int M = (int)total;
  launch_prefill_chunk_setup(d, cu, batch, total, ws.seq_id, ws.pos, ws.rope, ws.prefix, cache, slots, st);
  const T *wmat[4] = {(const T *)w.wq, (const T *)w.wk, (const T *)w.wc, (const T *)w.wg};
  const int wn[4] = {d.wq_w, d.wk_w, d.wc_w, d.wg_w};
  int off = 0;
  for (int i = 0; i < 4; ++i) {
    launch_gemm(x, (int64_t)d.H, 0, 1, wmat[i], (int64_t)wn[i], 0, M, wn[i], d.H, 1,
                EpiStoreF32{ws.praw, d.wtot, off}, st);
    off += wn[i];
  }
  CacheView cv = view_of(&cache, slots);
  finalize_prefill_kernel<T><<<grid1d(total * d.wtot), 256, 0, st>>>(
      d, ws.praw, ws.seq_id, ws.pos, ws.rope, max_chunk, total, (T *)ws.q, (T *)ws.k, (T *)ws.c, (float *)ws.g, cv, 1);
  dim3 agrid((max_chunk + 3) / 4, d.nq, batch);
  attn_chunk_generic_kernel<T, float><<<agrid, 256, 4 * d.dh * sizeof(float), st>>>(
      d, (const T *)ws.q, cv, ws.prefix, cu, per_seq, (float *)ws.l);
  const float *L = (const float *)ws.l;
  if (w.wo) {
    float *O = (float *)ws.o;
    launch_gemm(L, (int64_t)d.nq * d.dl, (int64_t)d.dl, d.hpq, (const T *)w.wp, (int64_t)d.dh, (int64_t)d.dl * d.dh,
                M, d.dh, d.dl, d.nh, EpiGate<float>{O, d.wg_w, (const float *)ws.g, d.wg_w, d.dh, d.gate}, st);
    launch_gemm(O, (int64_t)d.wg_w, 0, 1, (const T *)w.wo, (int64_t)d.H, 0, M, d.H, d.wg_w, 1,
                EpiStoreT<T>{out, d.H}, st);
  } else {
    launch_gemm(L, (int64_t)d.nq * d.dl, (int64_t)d.dl, d.hpq, (const T *)w.wp, (int64_t)d.dh, (int64_t)d.dl * d.dh,
                M, d.dh, d.dl, d.nh, EpiGate<T>{out, d.wg_w, (const float *)ws.g, d.wg_w, d.dh, d.gate}, st);
  }
  launch_prefill_chunk_commit(cache, slots, cu, batch, total, ws.prefix, st);
  return check_launch();
}

template <typename T>
void decode_project_impl(const Dims &d, const gta_weights &w, const T *x, int batch, const gta_cache &cache,
                         const int32_t *slots, const DecodeWs &ws, hipStream_t st) {
  const T *wmat[4] = {(const T *)w.wq, (const T *)w.wk, (const T *)w.wc, (const T *)w.wg};
  const int wn[4] = {d.wq_w, d.wk_w, d.wc_w, d.wg_w};
  int off = 0;
  for (int i = 0; i < 4; ++i) {
    launch_gemm(x, (int64_t)d.H, 0, 1, wmat[i], (int64_t)wn[i], 0, batch, wn[i], d.H, 1,
                EpiStoreF32{ws.praw, d.wtot, off}, st);
    off += wn[i];
  }
  finalize_decode_kernel<T><<<grid1d((int64_t)batch * d.wtot), 256, 0, st>>>(d, ws.praw, 1, batch, ws.q, ws.g,
                                                                            ws.oldlen, view_of(&cache, slots));
}

template <typename T>
int decode_impl(const Dims &d, const gta_weights &w, const T *x, int batch, const gta_cache &cache,
                const int32_t *slots, T *out, const DecodeWs &ws, hipStream_t st) {
  decode_project_impl<T>(d, w, x, batch, cache, slots, ws, st);
  CacheView cv = view_of(&cache, slots);
  dim3 agrid(ws.splits, d.nq, batch);
  attn_decode_generic_kernel<T><<<agrid, 64, d.dh * sizeof(float), st>>>(d, ws.q, ws.oldlen, cv, ws.splits, ws.part);
  decode_combine_kernel<<<dim3(d.nq, batch), 256, 0, st>>>(d, ws.part, ws.oldlen, ws.splits, ws.l);
  if (w.wo) {
    launch_gemm(ws.l, (int64_t)d.nq * d.dl, (int64_t)d.dl, d.hpq, (const T *)w.wp, (int64_t)d.dh,
                (int64_t)d.dl * d.dh, batch, d.dh, d.dl, d.nh,
                EpiGate<float>{ws.o, d.wg_w, ws.g, d.wg_w, d.dh, d.gate}, st);
    launch_gemm(ws.o, (int64_t)d.wg_w, 0, 1, (const T *)w.wo, (int64_t)d.H, 0, batch, d.H, d.wg_w, 1,
                EpiStoreT<T>{out, d.H}, st);
  } else {
    launch_gemm(ws.l, (int64_t)d.nq * d.dl, (int64_t)d.dl, d.hpq, (const T *)w.wp, (int64_t)d.dh,
                (int64_t)d.dl * d.dh, batch, d.dh, d.dl, d.nh,
                EpiGate<T>{out, d.wg_w, ws.g, d.wg_w, d.dh, d.gate}, st);
  }
  decode_commit_kernel<<<grid1d(batch), 256, 0, st>>>(cv, ws.oldlen, batch);
  return check_launch();
}

}  // namespace

// ------------------------------------------------------------------------------ exported helpers
void launch_rowmap(const int32_t *cu, int batch, int64_t total, int32_t *seq_id, int32_t *pos, hipStream_t st) {
  if (total <= 0) return;
  rowmap_kernel<<<grid1d(total), 256, 0, st>>>(cu, batch, total, (int)(total / batch), seq_id, pos);
}

void launch_rope_table(float2 *tab, int max_pos, int dh, double base, hipStream_t st) {
  const int half = dh / 2;
  if (max_pos <= 0 || half <= 0) return;
  rope_table_kernel<<<grid1d((int64_t)max_pos * half), 256, 0, st>>>(tab, max_pos, half, dh, base);
}

void launch_prefill_commit(const gta_cache &cache, const int32_t *slots, const int32_t *cu, int batch,
                           int64_t total, hipStream_t st) {
  prefill_commit_kernel<<<grid1d(batch), 256, 0, st>>>(view_of(&cache, slots), cu, batch, (int)(total / batch));
}

void launch_prefill_setup(const Dims &d, const int32_t *cu, int batch, int64_t total, int max_len, int32_t *seq_id,
                          int32_t *pos, float2 *tab, const gta_cache *cache, const int32_t *slots, hipStream_t st) {
  if (total <= 0) return;
  const int half = d.dh / 2;
  const int nb_row = (int)((total + 255) / 256);
  const int nb_rope = d.rope && max_len > 0 && half > 0 ? (int)(((int64_t)max_len * half + 255) / 256) : 0;
  const int nb_commit = cache ? (batch + 255) / 256 : 0;
  prefill_setup_kernel<<<nb_row + nb_rope + nb_commit, 256, 0, st>>>(
      cu, batch, total, (int)(total / batch), seq_id, pos, nb_row, tab, max_len, half, d.dh, d.rope_base, nb_rope,
      cache ? view_of(cache, slots) : CacheView{});
}

void launch_prefill_chunk_setup(const Dims &d, const int32_t *cu, int batch, int64_t total, int32_t *seq_id,
                                int32_t *pos, float2 *tab, int32_t *prefix, const gta_cache &cache,
                                const int32_t *slots, hipStream_t st) {
  if (total <= 0) return;
  const int half = d.dh / 2;
  const int nb_row = (int)((total + 255) / 256);
  const int nb_rope = d.rope && half > 0 ? (int)((total * half + 255) / 256) : 0;
  prefill_chunk_setup_kernel<<<nb_row + nb_rope + (batch + 255) / 256, 256, 0, st>>>(
      cu, batch, total, (int)(total / batch), seq_id, pos, nb_row, tab, half, d.dh, d.rope_base, nb_rope,
      view_of(&cache, slots), prefix);
}

void launch_prefill_chunk_commit(const gta_cache &cache, const int32_t *slots, const int32_t *cu, int batch,
                                 int64_t total, const int32_t *prefix, hipStream_t st) {
  prefill_chunk_commit_kernel<<<grid1d(batch), 256, 0, st>>>(view_of(&cache, slots), cu, batch, (int)(total / batch),
                                                             prefix);
}

int generic_prefill(const Dims &d, const gta_weights &w, const void *x, const int32_t *cu, int batch,
                    int64_t total, int max_len, const gta_cache *cache, const int32_t *slots, void *out,
                    const PrefillWs &ws, hipStream_t st) {
  if (d.dtype == GTA_BF16)
    return prefill_impl<bf16>(d, w, (const bf16 *)x, cu, batch, total, max_len, cache, slots, (bf16 *)out, ws, st);
  return prefill_impl<float>(d, w, (const float *)x, cu, batch, total, max_len, cache, slots, (float *)out, ws, st);
}

int generic_prefill_chunk(const Dims &d, const gta_weights &w, const void *x, const int32_t *cu, int batch,
                          int64_t total, int max_chunk, const gta_cache &cache, const int32_t *slots, void *out,
                          const PrefillWs &ws, hipStream_t st) {
  if (d.dtype == GTA_F32)
    return prefill_chunk_impl<float>(d, w, (const float *)x, cu, batch, total, max_chunk, cache, slots, (float *)out, ws, st);
  return prefill_chunk_impl<bf16>(d, w, (const bf16 *)x, cu, batch, total, max_chunk, cache, slots, (bf16 *)out, ws, st);
}

int generic_decode(const Dims &d, const gta_weights &w, const void *x_new, int batch, const gta_cache &cache,
                   const int32_t *slots, void *out, const DecodeWs &ws, hipStream_t st) {
  if (d.dtype == GTA_BF16)
    return decode_impl<bf16>(d, w, (const bf16 *)x_new, batch, cache, slots, (bf16 *)out, ws, st);
  return decode_impl<float>(d, w, (const float *)x_new, batch, cache, slots, (float *)out, ws, st);
}

void generic_decode_project(const Dims &d, const gta_weights &w, const void *x_new, int batch,
                            const gta_cache &cache, const int32_t *slots, const DecodeWs &ws, hipStream_t st) {
  if (d.dtype == GTA_BF16) decode_project_impl<bf16>(d, w, (const bf16 *)x_new, batch, cache, slots, ws, st);
  else decode_project_impl<float>(d, w, (const float *)x_new, batch, cache, slots, ws, st);
}

void launch_finalize_decode_bf16(const Dims &d, const float *part, int nsum, int batch, const gta_cache &cache,
                                 const int32_t *slots, const DecodeWs &ws, hipStream_t st) {
  finalize_decode_kernel<bf16><<<grid1d((int64_t)batch * d.wtot), 256, 0, st>>>(d, part, nsum, batch, ws.q, ws.g,
                                                                               ws.oldlen, view_of(&cache, slots));
}

void launch_cached_len(const gta_cache &cache, const int32_t *slots, int batch, int32_t *oldlen, hipStream_t st) {
  cached_len_kernel<<<grid1d(batch), 256, 0, st>>>(view_of(&cache, slots), batch, oldlen);
}

void generic_decode_attention(const Dims &d, const float *q, const int32_t *oldlen, const gta_cache &cache,
                              const int32_t *slots, int batch, int splits, float *part, hipStream_t st) {
  CacheView cv = view_of(&cache, slots);
  dim3 agrid(splits, d.nq, batch);
  if (d.dtype == GTA_BF16)
    attn_decode_generic_kernel<bf16><<<agrid, 64, d.dh * sizeof(float), st>>>(d, q, oldlen, cv, splits, part);
  else
    attn_decode_generic_kernel<float><<<agrid, 64, d.dh * sizeof(float), st>>>(d, q, oldlen, cv, splits, part);
}

void generic_decode_combine(const Dims &d, const float *part, const int32_t *oldlen, int splits, int batch, float *L,
                            hipStream_t st) {
  decode_combine_kernel<<<dim3(d.nq, batch), 256, 0, st>>>(d, part, oldlen, splits, L);
}

void launch_attn_prefill_rowwise(const Dims &d, const void *q, const void *k, const void *c, const int32_t *cu,
                                 int batch, int64_t total, int max_len, void *L, hipStream_t st) {
  dim3 agrid((max_len + 3) / 4, d.nq, batch);
  if (d.dtype == GTA_BF16)
    attn_prefill_generic_kernel<bf16, bf16><<<agrid, 256, 4 * d.dh * sizeof(float), st>>>(
        d, (const bf16 *)q, (const bf16 *)k, (const bf16 *)c, cu, (int)(total / batch), max_len, (bf16 *)L);
  else
    attn_prefill_generic_kernel<float, float><<<agrid, 256, 4 * d.dh * sizeof(float), st>>>(
        d, (const float *)q, (const float *)k, (const float *)c, cu, (int)(total / batch), max_len, (float *)L);
}

void launch_decode_commit(const gta_cache &cache, const int32_t *slots, const int32_t *oldlen, int batch,
                          hipStream_t st) {
  decode_commit_kernel<<<grid1d(batch), 256, 0, st>>>(view_of(&cache, slots), oldlen, batch);
}

void generic_out_proj_f32in(const Dims &d, const gta_weights &w, const float *O, int M, void *out, hipStream_t st) {
  if (d.dtype == GTA_BF16)
    launch_gemm(O, (int64_t)d.wg_w, 0, 1, (const bf16 *)w.wo, (int64_t)d.H, 0, M, d.H, d.wg_w, 1,
                EpiStoreT<bf16>{(bf16 *)out, d.H}, st);
  else
    launch_gemm(O, (int64_t)d.wg_w, 0, 1, (const float *)w.wo, (int64_t)d.H, 0, M, d.H, d.wg_w, 1,
                EpiStoreT<float>{(float *)out, d.H}, st);
}

int launch_calibration_read(const void *src, int64_t bytes, int workgroups, void *sink, hipStream_t st) {
  const int64_t words_per_wg = bytes / 16 / workgroups;
  calibration_read_kernel<<<workgroups, 256, 0, st>>>((const cal_u32x4 *)src, words_per_wg, (uint32_t *)sink);
  return check_launch();
}

int launch_calibration_mfma(int workgroups, int iters, bool random_operands, void *sink, hipStream_t st) {
  if (random_operands) calibration_mfma_kernel<true><<<workgroups, 256, 0, st>>>(iters, (float *)sink);
  else calibration_mfma_kernel<false><<<workgroups, 256, 0, st>>>(iters, (float *)sink);
  return check_launch();
}

int launch_calibration_copy(const void *src, void *dst, int64_t bytes, hipStream_t st) {
  calibration_copy_kernel<<<4096, 256, 0, st>>>((const uint4 *)src, (uint4 *)dst, bytes / 16);
  return check_launch();
}

int generic_cache_append(const Dims &d, const gta_cache &cache, const int32_t *slots, const void *k_new,
                         const void *c_new, const int32_t *cu_new, int batch, int max_new, hipStream_t st) {
  CacheView cv = view_of(&cache, slots);
  if (max_new > 0) {
    dim3 grid(max_new, batch);
    append_copy_kernel<<<grid, 128, 0, st>>>(cv, (const char *)k_new, (const char *)c_new, cu_new,
                                             d.wk_w * d.esize(), d.wc_w * d.esize(), max_new);
  }
  append_commit_kernel<<<grid1d(batch), 256, 0, st>>>(cv, cu_new, batch, max_new);
  return check_launch();
}

}  // namespace gta
