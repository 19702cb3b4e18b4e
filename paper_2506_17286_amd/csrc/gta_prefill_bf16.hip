// bf16 MFMA causal prefill attention of GTA for gfx950 (paper Sec. 3.3, reformulated form):
// for every map group g, L_g = Softmax(Q_g K_{k(g)}^T / sqrt(d_h)) C_{c(g)}, one shared map per
// group, output width d_l (normalised, bf16).  The value decoder runs afterwards as a GEMM.
//
// One workgroup = 256 queries of one (sequence, group) x 256 latent columns; each of its 8 waves
// (two per SIMD, so one wave's softmax overlaps the other's MFMAs) owns 32 queries and the whole
// column slice: the softmax statistics of a query live in one lane pair and nothing is exchanged
// between waves.  Wider latents are covered by several workgroups that each recompute the scores.  Both products are computed transposed:
//   S^T[key][query] = K . Q^T      (row operand: K tile from LDS, column operand: Q in registers)
//   L^T[col][query] += C^T . P^T   (row operand: latent tile through the LDS transpose read,
//                                   column operand: P straight from the S^T accumulator registers)
// so P never leaves registers and the per-query scale is a per-lane scalar.  Online softmax runs
// in the log2 domain with a lazy rescale: the running maximum is only raised when a new score
// exceeds it by more than 2^8, which keeps the 128 accumulator registers untouched in most tiles.
#include <math.h>

#include "gta_tuned.h"

namespace gta {
namespace {

typedef __bf16 bf16;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;

template <int DLW_, int BK_>
struct AttnTile {
  static constexpr int DH = 128, DLW = DLW_, BK = BK_, BQ = 256, NT = 512;
  static constexpr int NDLB = DLW / 32;            // 32-column accumulator blocks per wave
  static constexpr int NKB = BK / 32;              // 32-key score blocks per tile
  static constexpr int K_PITCH = DH * 2 + 16;      // 16 * odd: conflict-free 16-byte row reads
  static constexpr int C_PITCH = DLW * 2 + 64;     // == 64 mod 256: conflict-free transpose reads
  static constexpr int K_BYTES = BK * K_PITCH, C_BYTES = BK * C_PITCH, STAGE = K_BYTES + C_BYTES;
  static constexpr int SMEM = 2 * STAGE;
  static constexpr int K_PASSES = BK * (DH / 8) / NT, C_PASSES = BK * (DLW / 8) / NT;
  static_assert(BK % 32 == 0 && DLW % 32 == 0 && K_PASSES >= 1 && C_PASSES >= 1, "tile");
};

struct AttnArgs {
  const bf16 *q, *k, *c;     // packed [total, n_q*d_h], [total, n_k*d_h], [total, n_c*d_l]
  bf16 *L;                   // [total, n_q*d_l]
  const int32_t *cu; int per_seq;
  int nq, qpk, qpc, wq_w, wk_w, wc_w, dl, n_qtiles;
  float scale_log2e;
};

constexpr float kLazyThreshold = 8.0f;   // log2 units

template <class T>
__global__ __launch_bounds__(T::NT) void attn_prefill_kernel(AttnArgs a) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, h = lane >> 5;
  const int qt = a.n_qtiles - 1 - (int)blockIdx.x;      // longest (latest) query tiles first
  const int g = blockIdx.y % a.nq, dlc = blockIdx.y / a.nq, b = blockIdx.z;
  const int64_t start = a.cu ? a.cu[b] : (int64_t)b * a.per_seq;
  const int Tb = a.cu ? a.cu[b + 1] - a.cu[b] : a.per_seq;
  const int q0 = qt * T::BQ;
  if (q0 >= Tb) return;
  const int qw0 = q0 + wave * 32;                        // first query of this wave
  const int myq = qw0 + (lane & 31);                     // this lane's query position
  const bf16 *Kg = a.k + start * a.wk_w + (g / a.qpk) * T::DH;
  const bf16 *Cg = a.c + start * a.wc_w + (g / a.qpc) * a.dl + dlc * T::DLW;

  // Q^T column operand: lane holds d = ks*16 + h*8 .. +8 of its query, for the 8 k-steps
  bf16x8 qf[T::DH / 16];
  {
    const bf16 *qp = a.q + (start + min(myq, Tb - 1)) * a.wq_w + g * T::DH + h * 8;
#pragma unroll
    for (int ks = 0; ks < T::DH / 16; ++ks) qf[ks] = *reinterpret_cast<const bf16x8 *>(qp + ks * 16);
  }
  f32x16 acc[T::NDLB];
#pragma unroll
  for (int i = 0; i < T::NDLB; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;

  const int kend = min(q0 + T::BQ, Tb);                  // keys [0, kend) are visible to this tile
  const int ntiles = (kend + T::BK - 1) / T::BK;

  // cooperative tile staging: global -> registers -> LDS
  u32x4 rk[T::K_PASSES], rc[T::C_PASSES];
  auto gload = [&](int t) {
    const int j0 = t * T::BK;
#pragma unroll
    for (int i = 0; i < T::K_PASSES; ++i) {
      const int idx = tid + i * T::NT, row = idx / (T::DH / 8), ch = idx % (T::DH / 8);
      const int64_t j = min(j0 + row, Tb - 1);
      rk[i] = *reinterpret_cast<const u32x4 *>(Kg + j * a.wk_w + ch * 8);
    }
#pragma unroll
    for (int i = 0; i < T::C_PASSES; ++i) {
      const int idx = tid + i * T::NT, row = idx / (T::DLW / 8), ch = idx % (T::DLW / 8);
      const int64_t j = min(j0 + row, Tb - 1);
      rc[i] = *reinterpret_cast<const u32x4 *>(Cg + j * a.wc_w + ch * 8);
    }
  };
  auto sstore = [&](char *st) {
#pragma unroll
    for (int i = 0; i < T::K_PASSES; ++i) {
      const int idx = tid + i * T::NT, row = idx / (T::DH / 8), ch = idx % (T::DH / 8);
      *reinterpret_cast<u32x4 *>(st + row * T::K_PITCH + ch * 16) = rk[i];
    }
#pragma unroll
    for (int i = 0; i < T::C_PASSES; ++i) {
      const int idx = tid + i * T::NT, row = idx / (T::DLW / 8), ch = idx % (T::DLW / 8);
      *reinterpret_cast<u32x4 *>(st + T::K_BYTES + row * T::C_PITCH + ch * 16) = rc[i];
    }
  };
  const int koff = (lane & 31) * T::K_PITCH + h * 16;
  const int coff = T::K_BYTES + (4 * h + ((lane & 15) >> 2)) * T::C_PITCH + (((lane >> 4) & 1) * 16 + (lane & 3) * 4) * 2;

  auto compute = [&](const char *st, int t) {
    const int j0 = t * T::BK;
#pragma unroll
    for (int kb = 0; kb < T::NKB; ++kb) {
      const int jb = j0 + kb * 32;
      if (jb > qw0 + 31) continue;                       // block entirely above this wave's diagonal
      // scores S^T[key][query], fp32
      f32x16 s;
#pragma unroll
      for (int r = 0; r < 16; ++r) s[r] = 0.f;
#pragma unroll
      for (int ks = 0; ks < T::DH / 16; ++ks) {
        const bf16x8 kf = *reinterpret_cast<const bf16x8 *>(st + koff + kb * 32 * T::K_PITCH + ks * 32);
        s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[ks], s, 0, 0, 0);
      }
      // log2-domain scores, causal mask (key <= query), block maximum per query
      float bm = -INFINITY;
      const bool diag = jb + 31 > qw0;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        float x = s[r] * a.scale_log2e;
        if (diag) {
          const int key = jb + 8 * (r >> 2) + 4 * h + (r & 3);
          if (key > myq) x = -INFINITY;
        }
        s[r] = x;
        bm = fmaxf(bm, x);
      }
      bm = fmaxf(bm, __shfl_xor(bm, 32, 64));
      if (__any(bm > m_run + kLazyThreshold)) {          // raise the running maximum (rare)
        const float m_new = fmaxf(m_run, bm);
        const float corr = __builtin_amdgcn_exp2f(m_run - m_new);
        m_run = m_new;
        l_run *= corr;
#pragma unroll
        for (int i = 0; i < T::NDLB; ++i)
#pragma unroll
          for (int r = 0; r < 16; ++r) acc[i][r] *= corr;
      }
      float ps = 0.f;
#pragma unroll
      for (int r = 0; r < 16; ++r) { s[r] = __builtin_amdgcn_exp2f(s[r] - m_run); ps += s[r]; }
      l_run += ps;
      // P^T column operands: k-slot i of lane half h  <->  key 16*mm + 8*(i/4) + 4*h + i%4
      bf16x8 pf[2];
#pragma unroll
      for (int mm = 0; mm < 2; ++mm)
#pragma unroll
        for (int i = 0; i < 8; ++i) pf[mm][i] = (bf16)s[mm * 8 + i];
      // L^T += C^T . P^T, latent tile rows read through the transpose load with the same key order
#pragma unroll
      for (int dlb = 0; dlb < T::NDLB; ++dlb) {
#pragma unroll
        for (int mm = 0; mm < 2; ++mm) {
          const char *cp = st + coff + (kb * 32 + mm * 16) * T::C_PITCH + dlb * 64;
          s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(cp));
          s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(cp + 8 * T::C_PITCH));
          s16x8 c8 = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
          acc[dlb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, c8), pf[mm], acc[dlb], 0, 0, 0);
        }
      }
    }
  };

  gload(0);
  sstore(smem);
  __syncthreads();
  for (int t = 0; t < ntiles; ++t) {
    char *cur = smem + (t & 1) * T::STAGE;
    char *nxt = smem + ((t & 1) ^ 1) * T::STAGE;
    if (t + 1 < ntiles) gload(t + 1);
    compute(cur, t);
    if (t + 1 < ntiles) sstore(nxt);
    __syncthreads();
  }

  // normalise and store: lane owns query myq and 4 consecutive columns per (block, r/4)
  const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
  if (myq < Tb) {
    const float inv = 1.0f / l_tot;
    bf16 *Lr = a.L + (start + myq) * (int64_t)(a.nq * a.dl) + g * a.dl + dlc * T::DLW + 4 * h;
#pragma unroll
    for (int dlb = 0; dlb < T::NDLB; ++dlb)
#pragma unroll
      for (int rq = 0; rq < 4; ++rq) {
        bf16x4 v;
#pragma unroll
        for (int i = 0; i < 4; ++i) v[i] = (bf16)(acc[dlb][rq * 4 + i] * inv);
        *reinterpret_cast<bf16x4 *>(Lr + dlb * 32 + rq * 8) = v;
      }
  }
}

typedef AttnTile<256, 32> Attn256;

}  // namespace

bool attn_prefill_supported(const Dims &d) {
  return d.dtype == GTA_BF16 && d.dh == 128 && d.dl % 256 == 0 && d.wk_w % 8 == 0 && d.wc_w % 8 == 0;
}

void launch_attn_prefill_bf16(const Dims &d, const void *q, const void *k, const void *c, const int32_t *cu,
                              int batch, int64_t total, int max_len, void *L, hipStream_t st) {
  AttnArgs a{};
  a.q = (const bf16 *)q; a.k = (const bf16 *)k; a.c = (const bf16 *)c; a.L = (bf16 *)L;
  a.cu = cu; a.per_seq = (int)(total / batch);
  a.nq = d.nq; a.qpk = d.qpk; a.qpc = d.qpc; a.wq_w = d.wq_w; a.wk_w = d.wk_w; a.wc_w = d.wc_w; a.dl = d.dl;
  a.n_qtiles = (max_len + Attn256::BQ - 1) / Attn256::BQ;
  a.scale_log2e = d.scale * 1.4426950408889634f;
  static bool attr_set = false;
  if (!attr_set) {
    (void)hipFuncSetAttribute((const void *)attn_prefill_kernel<Attn256>, hipFuncAttributeMaxDynamicSharedMemorySize,
                              Attn256::SMEM);
    attr_set = true;
  }
  dim3 grid(a.n_qtiles, d.nq * (d.dl / Attn256::DLW), batch);
  attn_prefill_kernel<Attn256><<<grid, Attn256::NT, Attn256::SMEM, st>>>(a);
}

}  // namespace gta
