// bf16 MFMA causal prefill attention of GTA for gfx950 (paper Sec. 3.3, reformulated form):
// for every map group g, L_g = Softmax(Q_g K_{k(g)}^T / sqrt(d_h)) C_{c(g)}, one shared map per
// group, output width d_l (normalised, bf16).  The value decoder runs afterwards as a GEMM.
//
// One workgroup = 256 queries of one (sequence, group) x 256 latent columns; each of its 8 waves
// (two per SIMD, so one wave's softmax runs in the shadow of the other's MFMAs) owns 32 queries
// and the whole column slice (128 accumulator registers): the softmax statistics of a query live
// in one lane pair and nothing is exchanged between waves.  Wider latents are covered by several
// workgroups that each recompute the scores.  Both products are computed transposed:
//   S^T[key][query] = K . Q^T      (row operand: K tile from LDS, column operand: the wave's queries,
//                                   held in 32 registers for the whole kernel)
//   L^T[col][query] += C^T . P^T   (row operand: latent tile through the LDS transpose read,
//                                   column operand: P straight from the S^T accumulator registers)
// so P never leaves registers and the per-query scale is a per-lane scalar.
//
// Online softmax runs in the log2 domain.  Around the diagonal the running maximum of a query moves
// when a block exceeds it by more than 2^8, and the factor exp2(m_old - m_new) reaches the 128
// accumulator registers in a rarely taken branch.  In the main loop (blocks entirely below the
// diagonal) the block maximum is not formed at all: probabilities are taken relative to the maximum
// the query already has, whatever their size, and only a row sum beyond 2^32 sends the wave through
// the full step (bf16 probabilities and fp32 sums carry any scale; the final division cancels it).  The lane pair of a query is reduced with v_permlane32_swap, P is packed
// with v_cvt_pk_bf16_f32 and summed with v_dot2_f32_bf16 (so the row sum is the sum of the rounded
// values the MFMA sees).
//
// Key/latent tiles of 32 rows go global -> registers -> LDS through three stages: the loads of a
// tile are issued two tiles ahead and written to LDS one tile ahead of its use, one barrier per
// tile.  The finished tile is rounded to bf16, parked in LDS in output layout and
// written with 16-byte stores, 32 lanes per 512-byte row segment.
#include <math.h>

#include "gta_tuned.h"

namespace gta {
namespace {

typedef __bf16 bf16;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;

template <int DH_, int DLW_>
struct AttnTile {
  static constexpr int DH = DH_, DLW = DLW_, BK = 32, BQ = 256, NT = 512, NDLB = DLW / 32, NSTAGE = 3;
  static constexpr int K_PITCH = DH * 2 + 16;      // 16 * odd: conflict-free 16-byte row reads
  static constexpr int C_PITCH = DLW * 2 + 64 + (DLW % 128 ? 128 : 0);   // == 64 mod 256: conflict-free transpose reads
  static constexpr int K_BYTES = BK * K_PITCH, C_BYTES = BK * C_PITCH, STAGE = K_BYTES + C_BYTES;
  static constexpr int OUT_PITCH = DLW * 2 + 16;
  static constexpr int SMEM = BQ * OUT_PITCH > NSTAGE * STAGE ? BQ * OUT_PITCH : NSTAGE * STAGE;
  // 16-byte chunks per tile row, tile rows one pass of the 512 threads covers, passes per tile
  static constexpr int K_CPR = DH / 8, C_CPR = DLW / 8, K_CHUNKS = BK * K_CPR;
  static constexpr int C_RPP = NT / C_CPR < BK ? NT / C_CPR : BK, C_LOADS = BK / C_RPP, C_CHUNKS = C_RPP * C_CPR;
  // the hand-scheduled main loop deals 16 softmax slices over 2 * NDLB steps; others take the plain loop
  static constexpr bool PIPELINED = NDLB == 8 || NDLB == 4;
  static_assert(DH % 16 == 0 && DLW % 32 == 0 && K_CHUNKS <= NT && BK % C_RPP == 0 && C_LOADS >= 1, "tile");
  static_assert(SMEM <= 160 * 1024, "LDS budget");
};

struct AttnArgs {
  const bf16 *q, *k, *c;     // packed [total, n_q*d_h], [total, n_k*d_h], [total, n_c*d_l]
  bf16 *L;                   // [total, n_q*d_l]
  const int32_t *cu; int per_seq;
  int nq, qpk, qpc, wq_w, wk_w, wc_w, dl, n_qtiles, ndlc, batch;
  float scale_log2e;
  // fused value decoder (kernel template flag): O_i = (L_g W_{P,i}) * Sigmoid(gate) for the heads of g
  const bf16 *wp, *gate;     // [n_h, d_l, d_h]; gate pre-activations [total, n_h*d_h] or NULL (gate off)
  bf16 *out; int hpq, dh, nh;   // [total, n_h*d_h]
  int gate_kind;                // nonlinearity of the gate (kGateSigmoid, ..)
  // chunk mode (prefix != NULL): k, c are the caches [slot, max_seq, width]; the chunk's own rows are
  // already in them behind the prefix[b] rows cached before (prefix[b] < 0: sequence skipped, zero output)
  const int32_t *prefix, *slots; int max_seq;
  PageMap pm; int ps_shift;   // cache mode on a block-table layout: page_size = 1 << ps_shift, a multiple of BK
};

// LDS of the fused value decoder: the normalised 256 x DLW tile (row operand) and the DLW x 256
// decoder matrices of the group's heads side by side; afterwards the 256 x 256 gate / output tile.
template <class T>
struct FusedDecoder {
  static constexpr int N = 256;                         // heads per group x d_h
  static constexpr int W_PITCH = N * 2 + 64;            // == 64 mod 256 for the transpose reads
  static constexpr int W_OFF = T::BQ * T::OUT_PITCH;    // behind the L tile
  static constexpr int G_PITCH = N * 2 + 16;
  static constexpr int SMEM_LW = W_OFF + T::DLW * W_PITCH, SMEM_G = T::BQ * G_PITCH;
  static constexpr int SMEM = SMEM_LW > SMEM_G ? (SMEM_LW > T::SMEM ? SMEM_LW : T::SMEM) : (SMEM_G > T::SMEM ? SMEM_G : T::SMEM);
  static_assert(SMEM <= 160 * 1024, "LDS budget");
};

constexpr float kLazyThreshold = 8.0f;   // log2 units
constexpr float kRowSumLimit = 4294967296.0f;   // 2^32: a lane's sum of 16 probabilities that sends the wave to the full step

// maximum / sum over the lane pair (l, l + 32) that shares a query
__device__ __forceinline__ float pair_max(float v) {
  const u32x2 r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float pair_sum(float v) {
  const u32x2 r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

template <class T, bool FUSE>
__global__ __launch_bounds__(T::NT) void attn_prefill_kernel(AttnArgs a) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  const int tid = threadIdx.x, lane = tid & 63, h = lane >> 5, ln = lane & 31;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform: branches on it are scalar
  // Workgroups are dispatched in id order and a query tile costs (tile index + 1) key tiles, so the
  // tile index is the slowest digit of the id, longest first (list scheduling needs that to balance
  // the CUs); the sequence is the fastest digit, so the 8 XCDs (ids round-robin) each work on few
  // sequences and the workgroups of one XCD stream the same key range through its L2 in step.
  // Ids go to the XCDs round-robin whatever their cost, so with ragged lengths a fixed sequence digit
  // would tie each sequence to one XCD and the longest sequences would bound the launch: the
  // sequence digit is rotated by one per tile level, which spreads every sequence over all XCDs.
  const int per_qt = a.batch * a.nq * a.ndlc;
  const int lvl = (int)blockIdx.x / per_qt;
  const int qt = a.n_qtiles - 1 - lvl;
  const int rest = (int)blockIdx.x % per_qt;
  const int b = a.cu ? (rest % a.batch + lvl) % a.batch : rest % a.batch;
  const int g = (rest / a.batch) % a.nq, dlc = rest / (a.batch * a.nq);
  const int64_t start = a.cu ? a.cu[b] : (int64_t)b * a.per_seq;
  const int Tb = a.cu ? a.cu[b + 1] - a.cu[b] : a.per_seq;   // queries of this sequence
  const int q0 = qt * T::BQ;
  if (q0 >= Tb) return;
  const int P = a.prefix ? a.prefix[b] : 0;                  // keys cached before the first query
  if (P < 0) {   // skipped sequence: zero rows
    if constexpr (FUSE) {
      const int64_t ldo = (int64_t)a.nh * a.dh;
      bf16 *Ob = a.out + (start + q0) * ldo + g * a.hpq * a.dh;
      for (int i = tid; i < T::BQ * 32; i += T::NT)
        if (q0 + i / 32 < Tb) *reinterpret_cast<u32x4 *>(Ob + (int64_t)(i / 32) * ldo + (i % 32) * 8) = u32x4{0u, 0u, 0u, 0u};
    } else {
      bf16 *Lb = a.L + (start + q0) * (int64_t)(a.nq * a.dl) + g * a.dl + dlc * T::DLW;
      for (int i = tid; i < T::BQ * (T::DLW / 8); i += T::NT)
        if (q0 + i / (T::DLW / 8) < Tb)
          *reinterpret_cast<u32x4 *>(Lb + (int64_t)(i / (T::DLW / 8)) * (a.nq * a.dl) + (i % (T::DLW / 8)) * 8) = u32x4{0u, 0u, 0u, 0u};
    }
    return;
  }
  const int Tk = P + Tb;                                     // keys of this sequence
  const int qw0 = q0 + wave * 32;                            // first query of this wave
  const int qa0 = P + qw0;                                   // its position among the keys
  const int kend = P + min(q0 + T::BQ, Tb);                  // keys [0, kend) are visible to this tile
  const int ntiles = (kend + T::BK - 1) / T::BK;
  const int kend_w = qw0 < Tb ? P + min(qw0 + 32, Tb) : 0;   // keys [0, kend_w) are visible to this wave
  int64_t krow0 = start;                                     // first key / latent row of the sequence
  int slot = 0;
  if (a.prefix) {
    slot = a.slots ? a.slots[b] : b;
    krow0 = a.pm.table ? 0 : (int64_t)slot * a.max_seq;      // block table: Kb / Cb are the pools, rows per tile
  }
  const char *Kb = reinterpret_cast<const char *>(a.k + krow0 * a.wk_w + (g / a.qpk) * T::DH);
  const char *Cb = reinterpret_cast<const char *>(a.c + krow0 * a.wc_w + (g / a.qpc) * a.dl + dlc * T::DLW);
  const unsigned wk2 = a.wk_w * 2, wc2 = a.wc_w * 2;

  // The wave's queries stay in registers for the whole kernel: the Q^T column operand of k-step ks is
  // the 16-byte chunk d = ks*16 + h*8 .. +8 of the lane's query (rows past the sequence re-read its
  // last row; their output is never written).
  bf16x8 qf[T::DH / 16];
  {
    const bf16 *qg = a.q + (start + min(qw0 + ln, Tb - 1)) * a.wq_w + g * T::DH + h * 8;
#pragma unroll
    for (int ks = 0; ks < T::DH / 16; ++ks) qf[ks] = *reinterpret_cast<const bf16x8 *>(qg + ks * 16);
  }

  f32x16 acc[T::NDLB];
#pragma unroll
  for (int i = 0; i < T::NDLB; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;

  // cooperative tile staging: global -> registers -> LDS; rows past the sequence re-read its last row
  // (such keys are in the future of every valid query and are masked)
  u32x4 rk, rc[T::C_LOADS];
  const int k_row = tid / T::K_CPR, k_ch = tid % T::K_CPR, c_row = tid / T::C_CPR, c_ch = tid % T::C_CPR;
  // narrow tiles have fewer chunks than threads (no predicate at all where every thread loads)
  const bool k_loader = T::K_CHUNKS >= T::NT || tid < T::K_CHUNKS, c_loader = T::C_CHUNKS >= T::NT || tid < T::C_CHUNKS;
  auto gload = [&](int t) {
    const int j0 = t * T::BK;
    const char *Kt = Kb, *Ct = Cb;
    int sub = 0;
    if (a.pm.table) {   // the tile's 32 rows sit in one page: rows relative to the tile's first pool row
      const int jt = min(j0, (Tk - 1) & ~(T::BK - 1));   // tiles past the sequence re-read its last tile
      const int pi = __builtin_amdgcn_readfirstlane(jt >> a.ps_shift);
      int pg = a.pm.table[(int64_t)slot * a.pm.pages_per_slot + pi];
      pg = (unsigned)pg >= (unsigned)a.pm.num_pages ? 0 : pg;
      const int64_t prow = ((int64_t)pg << a.ps_shift) + (jt & (a.pm.page_size - 1));
      Kt = Kb + prow * wk2; Ct = Cb + prow * wc2;
      sub = jt;
    }
    if (k_loader) {
      const unsigned r = min(j0 + k_row, Tk - 1) - sub;
      rk = *reinterpret_cast<const u32x4 *>(Kt + (r * wk2 + k_ch * 16));
    }
    if (c_loader) {
#pragma unroll
      for (int i = 0; i < T::C_LOADS; ++i) {
        const unsigned r = min(j0 + c_row + i * T::C_RPP, Tk - 1) - sub;
        rc[i] = *reinterpret_cast<const u32x4 *>(Ct + (r * wc2 + c_ch * 16));
      }
    }
  };
  auto sstore = [&](char *st) {
    if (k_loader) *reinterpret_cast<u32x4 *>(st + k_row * T::K_PITCH + k_ch * 16) = rk;
    if (c_loader) {
#pragma unroll
      for (int i = 0; i < T::C_LOADS; ++i)
        *reinterpret_cast<u32x4 *>(st + T::K_BYTES + (c_row + i * T::C_RPP) * T::C_PITCH + c_ch * 16) = rc[i];
    }
  };
  const int koff = ln * T::K_PITCH + h * 16;
  const int coff = T::K_BYTES + (4 * h + ((lane & 15) >> 2)) * T::C_PITCH + (((lane >> 4) & 1) * 16 + (lane & 3) * 4) * 2;

  // scores S^T of one 32-key block (raw, unscaled); all key fragments are requested before the first
  // MFMA so that the chain of MFMAs pays one LDS round trip, not one per fragment
  auto scores = [&](const char *st, f32x16 &s) {
#pragma unroll
    for (int r = 0; r < 16; ++r) s[r] = 0.f;
    bf16x8 kf[T::DH / 16];
#pragma unroll
    for (int ks = 0; ks < T::DH / 16; ++ks) kf[ks] = *reinterpret_cast<const bf16x8 *>(st + koff + ks * 32);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int ks = 0; ks < T::DH / 16; ++ks) s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[ks], qf[ks], s, 0, 0, 0);
  };
  // keys after the lane's query are masked in a block that touches the diagonal
  auto mask = [&](f32x16 &s, int jb) {
    const int lim = qa0 + ln - jb;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int ko = 8 * (r >> 2) + 4 * h + (r & 3);
      s[r] = ko > lim ? -INFINITY : s[r];
    }
  };
  // softmax of one block: pn = exp2(scaled score - running maximum) as bf16 MFMA column operands
  // (k-slot i of lane half h  <->  key 16*mm + 8*(i/4) + 4*h + i%4); m_run / l_run are updated and
  // corr is the factor the accumulators still have to take before this block is added
  auto softmax = [&](const f32x16 &s, bf16x8 (&pn)[2], float &corr) {
    float bm = fmaxf(s[0], s[1]);
#pragma unroll
    for (int r = 2; r < 16; r += 2) bm = fmaxf(fmaxf(s[r], s[r + 1]), bm);   // v_max3
    const float m_cand = pair_max(bm) * a.scale_log2e;
    const float m_new = m_cand > m_run + kLazyThreshold ? fmaxf(m_run, m_cand) : m_run;
    corr = __builtin_amdgcn_exp2f(m_run - m_new);
    m_run = m_new;
    const bf16x2 ones = {(bf16)1.0f, (bf16)1.0f};
    float ps = 0.f;
#pragma unroll
    for (int mm = 0; mm < 2; ++mm)
#pragma unroll
      for (int i = 0; i < 8; i += 2) {
        const float p0 = __builtin_amdgcn_exp2f(fmaf(s[mm * 8 + i], a.scale_log2e, -m_new));
        const float p1 = __builtin_amdgcn_exp2f(fmaf(s[mm * 8 + i + 1], a.scale_log2e, -m_new));
        bf16x2 pk;
        pk[0] = (bf16)p0; pk[1] = (bf16)p1;
        pn[mm][i] = pk[0]; pn[mm][i + 1] = pk[1];
        ps = __builtin_amdgcn_fdot2_f32_bf16(pk, ones, ps, false);   // the row sum uses the rounded values
      }
    l_run = fmaf(l_run, corr, ps);
  };
  // L^T += C^T . P^T, latent tile rows read through the transpose load with the same key order
  auto pv = [&](const char *st, const bf16x8 (&pf)[2]) {
    // key half outermost: consecutive MFMAs go to different accumulators
#pragma unroll
    for (int mm = 0; mm < 2; ++mm) {
#pragma unroll
      for (int dlb = 0; dlb < T::NDLB; ++dlb) {
        const char *cp = st + coff + mm * 16 * T::C_PITCH + dlb * 64;
        s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(cp));
        s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(cp + 8 * T::C_PITCH));
        s16x8 c8 = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        acc[dlb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, c8), pf[mm], acc[dlb], 0, 0, 0);
      }
    }
  };

  // The waves of a workgroup meet at a barrier every tile and so run in phase: the overlap of softmax
  // arithmetic and MFMAs has to come from each wave's own instruction stream.  Iteration t issues the
  // score MFMAs of block t+1, then the map-times-latent MFMAs of block t with the softmax arithmetic
  // of block t+1 dealt out between them.
  // Stages: tile t+1 is read (scores) from `nxt`, tile t (latents) from `cur`, tile t+2 (loaded during
  // iteration t-1) is written to `fre`, tile t+3 is loaded.
  const int nb_w = (kend_w + 31) >> 5;   // blocks this wave needs: 0 .. nb_w-1
  bf16x8 pf[2];
  float corr = 1.f;
  gload(0);
  sstore(smem);
  gload(1);
  __syncthreads();
  if (nb_w > 0) {
    f32x16 s;
    scores(smem, s);
    if (31 > qa0) mask(s, 0);
    softmax(s, pf, corr);
    corr = 1.f;   // the accumulators are still zero
  }
  sstore(smem + T::STAGE);
  gload(2);
  __syncthreads();
  int cur = 0, nxt = T::STAGE, fre = 2 * T::STAGE;
  auto rotate = [&]() {
    const int tmp = cur;
    cur = nxt; nxt = fre; fre = tmp;
  };
  auto rescale = [&]() {
    if (__builtin_amdgcn_ballot_w64(corr != 1.f) != 0) {   // rare: the running maximum moved
#pragma unroll
      for (int i = 0; i < T::NDLB; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][r] *= corr;
    }
  };
  // main part: blocks t and t+1 both lie entirely below this wave's diagonal
  int t = 0;
  if constexpr (T::PIPELINED) {
  const int t_main = min(nb_w, qa0 >> 5) - 1;   // iterations 0 .. t_main-1
#pragma unroll 1
  for (; t < t_main; ++t) {
    // The fragment reads of the first score MFMAs and of the first two map-times-latent MFMAs go out
    // before anything else, so that the MFMAs below do not each wait for an LDS round trip; the second
    // half of the key fragments follows behind the first two score MFMAs.
    constexpr int KS = T::DH / 16, KS1 = KS / 2;
    const char *kst = smem + nxt + koff;
    bf16x8 kf[KS];
#pragma unroll
    for (int ks = 0; ks < KS1; ++ks) kf[ks] = *reinterpret_cast<const bf16x8 *>(kst + ks * 32);
    __builtin_amdgcn_sched_barrier(0);
    sstore(smem + fre);
    gload(t + 3);
    rescale();
    f32x16 s;
#pragma unroll
    for (int r = 0; r < 16; ++r) s[r] = 0.f;
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      if (ks == 1) {
#pragma unroll
        for (int k2 = KS1; k2 < KS; ++k2) kf[k2] = *reinterpret_cast<const bf16x8 *>(kst + k2 * 32);
      }
      s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[ks], qf[ks], s, 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
    // 2 * NDLB steps, each one MFMA of block t (latent fragment i, read two steps earlier), the
    // transpose reads of fragment i+2 and a slice of the softmax arithmetic of block t+1 (16 slices
    // dealt evenly over the steps); the scheduling barrier after every step pins this order, so each
    // MFMA is followed by arithmetic that runs in its shadow
    const char *st = smem + cur;
    constexpr int NS = 2 * T::NDLB, SPS = 16 / NS;   // steps, softmax slices per step
    auto cread = [&](int i) {
      const char *cp = st + coff + (i / T::NDLB) * 16 * T::C_PITCH + (i % T::NDLB) * 64;
      s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(cp));
      s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(cp + 8 * T::C_PITCH));
      s16x8 c8 = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
      return __builtin_bit_cast(bf16x8, c8);
    };
    constexpr int LA = 2;   // latent fragments in flight ahead of their MFMA (3 measured no better)
    bf16x8 cf[NS + LA], pn[2];
#pragma unroll
    for (int i = 0; i < LA; ++i) cf[i] = cread(i);
    // Below the diagonal the running maximum is left where it is and the block's own maximum is not
    // even formed: p = exp2(score - m_run) is taken as it comes and only its row sum is watched.  bf16
    // probabilities and fp32 sums carry any scale, so nothing is lost while p stays far from the top
    // of the fp32 range; a block whose row sum passes 2^32 (or is not finite) sends the whole wave
    // through the full online-softmax step once, which moves the maximum and redoes the block.
    float ps = 0.f;
    const float negm = -m_run;
    const bf16x2 ones = {(bf16)1.0f, (bf16)1.0f};
    auto soft_slice = [&](int k) {   // 16 slots; the 8 pairs of exponentials take the even ones
      if (k % 2 == 0) {
        const int e = k;   // elements e, e+1 -> k-slots e%8, e%8+1 of pn[e/8]
        const float p0 = __builtin_amdgcn_exp2f(fmaf(s[e], a.scale_log2e, negm));
        const float p1 = __builtin_amdgcn_exp2f(fmaf(s[e + 1], a.scale_log2e, negm));
        bf16x2 pk;
        pk[0] = (bf16)p0; pk[1] = (bf16)p1;
        pn[e >> 3][e & 7] = pk[0]; pn[e >> 3][(e & 7) + 1] = pk[1];
        ps = __builtin_amdgcn_fdot2_f32_bf16(pk, ones, ps, false);
      }
    };
#pragma unroll
    for (int i = 0; i < NS; ++i) {
      if (i + LA < NS) cf[i + LA] = cread(i + LA);
      acc[i % T::NDLB] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(cf[i], pf[i / T::NDLB], acc[i % T::NDLB], 0, 0, 0);
#pragma unroll
      for (int k = i * SPS; k < (i + 1) * SPS; ++k) soft_slice(k);
      __builtin_amdgcn_sched_barrier(0);
    }
    if (__builtin_amdgcn_ballot_w64(!(ps < kRowSumLimit)) != 0) {   // rare
      softmax(s, pn, corr);
    } else {
      l_run += ps;
      corr = 1.f;
    }
    pf[0] = pn[0]; pf[1] = pn[1];
    __syncthreads();
    rotate();
  }
  }
  // the blocks around the diagonal, then idle iterations that only keep staging for the other waves
#pragma unroll 1
  for (; t < ntiles; ++t) {
    sstore(smem + fre);
    gload(t + 3);
    if (t < nb_w) {
      rescale();
      f32x16 s;
      bf16x8 pn[2];
      if (t + 1 < nb_w) {
        scores(smem + nxt, s);
        if ((t + 1) * 32 + 31 > qa0) mask(s, (t + 1) * 32);
      } else {   // no further block: all-masked scores leave the statistics unchanged and give P = 0
#pragma unroll
        for (int r = 0; r < 16; ++r) s[r] = -INFINITY;
      }
      softmax(s, pn, corr);
      pv(smem + cur, pf);
      pf[0] = pn[0]; pf[1] = pn[1];
    }
    __syncthreads();
    rotate();
  }

  // ---- normalise, park the tile in LDS in output layout, write row-contiguous 16-byte chunks
  {
    const float inv = 1.0f / pair_sum(l_run);
    const int row = wave * 32 + ln;
#pragma unroll
    for (int dlb = 0; dlb < T::NDLB; ++dlb)
#pragma unroll
      for (int rq = 0; rq < 4; ++rq) {
        bf16x4 v;
#pragma unroll
        for (int i = 0; i < 4; ++i) v[i] = (bf16)(acc[dlb][rq * 4 + i] * inv);
        *reinterpret_cast<bf16x4 *>(smem + row * T::OUT_PITCH + (dlb * 32 + rq * 8 + 4 * h) * 2) = v;
      }
  }
  if constexpr (FUSE) {
    // ---- value decoder on the tile (Sec. 3.2): the workgroup holds the whole latent width of its
    // group, so the heads of the group are finished here and L never goes to memory
    typedef FusedDecoder<T> F;
    constexpr int WCH = T::DLW * (F::N / 8) / T::NT;     // 16-byte chunks of the decoder matrices per thread
    constexpr int GCH = T::BQ * (F::N / 8) / T::NT;      // chunks of the gate / output tile per thread
    const int head0 = g * a.hpq;
    const int64_t ldo = (int64_t)a.nh * a.dh;
    u32x4 wr[WCH];
#pragma unroll
    for (int i = 0; i < WCH; ++i) {
      const int c = tid + i * T::NT, k = c / (F::N / 8), col = (c % (F::N / 8)) * 8;
      wr[i] = *reinterpret_cast<const u32x4 *>(a.wp + ((int64_t)(head0 + col / a.dh) * a.dl + k) * a.dh + col % a.dh);
    }
#pragma unroll
    for (int i = 0; i < WCH; ++i) {
      const int c = tid + i * T::NT, k = c / (F::N / 8), col = (c % (F::N / 8)) * 8;
      *reinterpret_cast<u32x4 *>(smem + F::W_OFF + k * F::W_PITCH + col * 2) = wr[i];
    }
    // gate tile: requested now, parked in LDS once the operands are dead (rows past the sequence
    // re-read its last row; they are not stored)
    const int gr0 = tid / (F::N / 8), gch = tid % (F::N / 8);
    constexpr int GRPP = T::NT / (F::N / 8);
    u32x4 gt[GCH];
    if (a.gate) {
      const bf16 *gp = a.gate + head0 * a.dh + gch * 8;
#pragma unroll
      for (int i = 0; i < GCH; ++i)
        gt[i] = *reinterpret_cast<const u32x4 *>(gp + (start + min(q0 + i * GRPP + gr0, Tb - 1)) * ldo);
    }
    __syncthreads();
    f32x16 z[F::N / 32];
#pragma unroll
    for (int tn = 0; tn < F::N / 32; ++tn)
#pragma unroll
      for (int r = 0; r < 16; ++r) z[tn][r] = 0.f;
    const char *lrow = smem + (wave * 32 + ln) * T::OUT_PITCH + h * 16;
    const char *wfr = smem + F::W_OFF + (h * 8 + ((lane & 15) >> 2)) * F::W_PITCH + (((lane >> 4) & 1) * 16 + (lane & 3) * 4) * 2;
#pragma unroll
    for (int ks = 0; ks < T::DLW / 16; ++ks) {
      const bf16x8 xf = *reinterpret_cast<const bf16x8 *>(lrow + ks * 32);
#pragma unroll
      for (int tn = 0; tn < F::N / 32; ++tn) {
        const char *wp = wfr + ks * 16 * F::W_PITCH + tn * 64;
        s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(wp));
        s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(wp + 4 * F::W_PITCH));
        s16x8 w8 = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        z[tn] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, w8), xf, z[tn], 0, 0, 0);
      }
    }
    __syncthreads();   // operands dead: the same LDS now takes the gate tile in output layout
    if (a.gate) {
#pragma unroll
      for (int i = 0; i < GCH; ++i)
        *reinterpret_cast<u32x4 *>(smem + (i * GRPP + gr0) * F::G_PITCH + gch * 16) = gt[i];
      __syncthreads();
    }
    // lane: row wave*32 + ln, columns tn*32 + rq*8 + 4h .. +3
    char *orow = smem + (wave * 32 + ln) * F::G_PITCH + 4 * h * 2;
#pragma unroll
    for (int tn = 0; tn < F::N / 32; ++tn)
#pragma unroll
      for (int rq = 0; rq < 4; ++rq) {
        bf16x4 *slot = reinterpret_cast<bf16x4 *>(orow + (tn * 32 + rq * 8) * 2);
        float v[4] = {z[tn][rq * 4], z[tn][rq * 4 + 1], z[tn][rq * 4 + 2], z[tn][rq * 4 + 3]};
        if (a.gate) {
          const bf16x4 gz = *slot;
#pragma unroll
          for (int i = 0; i < 4; ++i) v[i] *= gate_factor(a.gate_kind, (float)gz[i]);
        }
        bf16x4 o;
#pragma unroll
        for (int i = 0; i < 4; ++i) o[i] = (bf16)v[i];
        *slot = o;
      }
    __syncthreads();
    bf16 *Ob = a.out + (start + q0) * ldo + head0 * a.dh + gch * 8;
#pragma unroll 4
    for (int i = 0; i < GCH; ++i) {
      const int r = i * GRPP + gr0;
      if (q0 + r < Tb)
        *reinterpret_cast<u32x4 *>(Ob + (int64_t)r * ldo) = *reinterpret_cast<const u32x4 *>(smem + r * F::G_PITCH + gch * 16);
    }
    return;
  }
  __syncthreads();
  bf16 *Lb = a.L + (start + q0) * (int64_t)(a.nq * a.dl) + g * a.dl + dlc * T::DLW;
  constexpr int CPR = T::DLW / 8, RPP = T::NT / CPR;   // 16-byte chunks per output row, rows per pass
  const int r0 = tid / CPR, ch = tid % CPR;
#pragma unroll 4
  for (int it = 0; it < T::BQ / RPP; ++it) {
    const int r = it * RPP + r0;
    if (q0 + r < Tb)
      *reinterpret_cast<u32x4 *>(Lb + (int64_t)r * (a.nq * a.dl) + ch * 8) =
          *reinterpret_cast<const u32x4 *>(smem + r * T::OUT_PITCH + ch * 16);
  }
}

typedef AttnTile<128, 256> AttnWide;     // d_h = 128, latent width a multiple of 256
typedef AttnTile<128, 128> AttnMid;      // d_h = 128, other latent widths that are multiples of 128
typedef AttnTile<64, 128> AttnNarrow;    // d_h = 64, latent width a multiple of 128
typedef AttnTile<64, 64> AttnSlim;       // d_h = 64, other latent widths that are multiples of 64 (e.g. the
                                         // GQA-degenerate setting d_l = d_h used as a comparator)

template <class T, bool FUSE>
void launch_attn(const AttnArgs &a0, const Dims &d, int batch, int max_len, hipStream_t st) {
  AttnArgs a = a0;
  a.n_qtiles = (max_len + T::BQ - 1) / T::BQ;
  a.ndlc = d.dl / T::DLW;
  int smem = T::SMEM;
  if constexpr (FUSE) smem = FusedDecoder<T>::SMEM;
  allow_dynamic_lds((const void *)attn_prefill_kernel<T, FUSE>, smem);
  attn_prefill_kernel<T, FUSE><<<a.n_qtiles * a.ndlc * d.nq * batch, T::NT, smem, st>>>(a);
}

}  // namespace

bool attn_prefill_supported(const Dims &d, int max_len) {
  // byte offsets inside one sequence's K / C rows are kept in 32 bits
  if ((int64_t)max_len * d.wc_w * 2 >= ((int64_t)1 << 31) || (int64_t)max_len * d.wk_w * 2 >= ((int64_t)1 << 31)) return false;
  if (d.dtype != GTA_BF16 || d.wq_w % 8 || d.wk_w % 8 || d.wc_w % 8) return false;
  return (d.dh == 128 && d.dl % 128 == 0) || (d.dh == 64 && d.dl % 64 == 0);
}

static AttnArgs attn_args(const Dims &d, const void *q, const void *k, const void *c, const int32_t *cu, int batch,
                          int64_t total) {
  AttnArgs a{};
  a.q = (const bf16 *)q; a.k = (const bf16 *)k; a.c = (const bf16 *)c;
  a.cu = cu; a.per_seq = (int)(total / batch);
  a.nq = d.nq; a.qpk = d.qpk; a.qpc = d.qpc; a.wq_w = d.wq_w; a.wk_w = d.wk_w; a.wc_w = d.wc_w; a.dl = d.dl;
  a.scale_log2e = d.scale * 1.4426950408889634f;
  a.batch = batch;
  return a;
}

void launch_attn_prefill_bf16(const Dims &d, const void *q, const void *k, const void *c, const int32_t *cu,
                              int batch, int64_t total, int max_len, void *L, hipStream_t st) {
  AttnArgs a = attn_args(d, q, k, c, cu, batch, total);
  a.L = (bf16 *)L;
  if (d.dh == 128 && d.dl % 256 == 0) launch_attn<AttnWide, false>(a, d, batch, max_len, st);
  else if (d.dh == 128) launch_attn<AttnMid, false>(a, d, batch, max_len, st);
  else if (d.dl % 128 == 0) launch_attn<AttnNarrow, false>(a, d, batch, max_len, st);
  else launch_attn<AttnSlim, false>(a, d, batch, max_len, st);
}

// One workgroup covers the whole latent width and the group's heads fill one 256-wide tile
bool attn_decoder_fusable(const Dims &d, int max_len) {
  return attn_prefill_supported(d, max_len) && d.dh == 64 && d.dl == AttnNarrow::DLW && d.hpq * d.dh == 256;
}

void launch_attn_decoder_bf16(const Dims &d, const void *q, const void *k, const void *c, const int32_t *cu,
                              int batch, int64_t total, int max_len, const void *wp, const void *gate, void *out,
                              hipStream_t st) {
  AttnArgs a = attn_args(d, q, k, c, cu, batch, total);
  a.wp = (const bf16 *)wp; a.gate = d.gate ? (const bf16 *)gate : nullptr; a.out = (bf16 *)out;
  a.hpq = d.hpq; a.dh = d.dh; a.nh = d.nh; a.gate_kind = d.gate;
  launch_attn<AttnNarrow, true>(a, d, batch, max_len, st);
}

void launch_attn_chunk_bf16(const Dims &d, const void *q, const gta_cache &cache, const int32_t *slots,
                            const int32_t *prefix, const int32_t *cu, int batch, int64_t total, int max_chunk,
                            void *L, const void *wp, const void *gate, void *out, bool fuse, hipStream_t st) {
  AttnArgs a = attn_args(d, q, cache.k, cache.c, cu, batch, total);
  a.prefix = prefix; a.slots = slots; a.max_seq = cache.max_seq;
  a.pm = page_map_of(cache);
  a.ps_shift = 0;
  while (a.pm.table && (1 << a.ps_shift) < a.pm.page_size) ++a.ps_shift;
  a.L = (bf16 *)L;
  if (fuse) {
    a.wp = (const bf16 *)wp; a.gate = d.gate ? (const bf16 *)gate : nullptr; a.out = (bf16 *)out;
    a.hpq = d.hpq; a.dh = d.dh; a.nh = d.nh; a.gate_kind = d.gate;
    launch_attn<AttnNarrow, true>(a, d, batch, max_chunk, st);
  } else if (d.dh == 128 && d.dl % 256 == 0) {
    launch_attn<AttnWide, false>(a, d, batch, max_chunk, st);
  } else if (d.dh == 128) {
    launch_attn<AttnMid, false>(a, d, batch, max_chunk, st);
  } else if (d.dl % 128 == 0) {
    launch_attn<AttnNarrow, false>(a, d, batch, max_chunk, st);
  } else {
    launch_attn<AttnSlim, false>(a, d, batch, max_chunk, st);
  }
}

}  // namespace gta
