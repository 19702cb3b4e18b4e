// Tuned bf16 decode for gfx950: split-K streaming attention over the grouped-key and latent-value
// caches (paper Sec. 3.3 reformulated form, decode cost App. B.1.3), then a log-sum-exp combine
// fused with the value decoder and sigmoid gate (Sec. 3.2).
//
// The step is HBM-bound (about 2.5 flop per cached byte), so the attention kernel is built around
// the stream: one workgroup per (sequence, context split) reads every key row and latent row of
// its slice exactly once, with one 16-byte load per lane covering a whole 1 KiB row per wave
// instruction, and serves ALL map groups from that single read.  Arithmetic is plain fp32 VALU:
// a per-lane partial dot product reduced inside the 8/16 lanes of a key group with DPP, online
// softmax in the log2 domain, and p * c accumulated with the weight broadcast from a scalar.
#include <math.h>

#include "gta_tuned.h"

namespace gta {
namespace {

typedef __bf16 bf16;
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;

template <int CTRL>
__device__ __forceinline__ float dpp_mov(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xF, 0xF, true));
}
// Sum over the LPG (8 or 16) consecutive lanes that hold one key group; every lane gets the sum.
template <int LPG>
__device__ __forceinline__ float group_sum(float v) {
  v += dpp_mov<0xB1>(v);    // quad_perm [1,0,3,2]
  v += dpp_mov<0x4E>(v);    // quad_perm [2,3,0,1]
  v += dpp_mov<0x141>(v);   // row_half_mirror: lane i <-> 7-i of each 8
  if (LPG == 16) v += dpp_mov<0x140>(v);  // row_mirror: lane i <-> 15-i of each 16
  return v;
}
__device__ __forceinline__ float lane_bcast(float v, int src_lane) {
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), src_lane));
}
__device__ __forceinline__ void unpack8(const u32x4 &w, float (&f)[8]) {
  f[0] = __uint_as_float(w.x << 16); f[1] = __uint_as_float(w.x & 0xffff0000u);
  f[2] = __uint_as_float(w.y << 16); f[3] = __uint_as_float(w.y & 0xffff0000u);
  f[4] = __uint_as_float(w.z << 16); f[5] = __uint_as_float(w.z & 0xffff0000u);
  f[6] = __uint_as_float(w.w << 16); f[7] = __uint_as_float(w.w & 0xffff0000u);
}
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Compile-time shape of one instantiation.  A key row is NK*DH elements = KCH chunks of 512
// (1 KiB, one 16-byte load per lane); a latent row is NC*DLC chunks of 512.
template <int DH_, int NK_, int QPK_, int NC_, int DLC_, int R_, int OCC_>
struct DecShape {
  static constexpr int DH = DH_, NK = NK_, QPK = QPK_, NC = NC_, DLC = DLC_, R = R_, OCC = OCC_;
  static constexpr int NQ = NK * QPK;
  static constexpr int QPC = NQ / NC;
  static constexpr int DL = DLC * 512;
  static constexpr int KCH = NK * DH / 512;
  static constexpr int CCH = NC * DLC;
  static constexpr int GPL = 512 / DH;   // key groups per chunk
  static constexpr int LPG = DH / 8;     // lanes per key group
  static_assert(NK * DH % 512 == 0 && NQ % NC == 0, "shape");
};

constexpr int kWaves = 4;
constexpr int kGemmTailBatch = 256;   // from this many sequences on the tail's decoder runs as a GEMM

// Where the queries, the context lengths and (for a full decode step) the new token's key/latent row
// come from:
//   stage call     q_direct given, oldlen_in NULL: attend over the seq_lens[slot] cached rows as they are;
//   pre-projected  q_direct and oldlen_in given:  the new row is already in the cache at oldlen_in[b];
//   fused step     praw given: every workgroup sums the split-K partials of the projection for its
//                  queries and rotates them at position seq_lens[slot] (App. B.1.1); the workgroup whose
//                  slice ends at the new token also builds that token's key and latent rows, appends them
//                  to the caches (App. B.1.3) and attends to them from LDS.
struct RopeFreq { double f[64]; };   // base^(-2j/d_h), j < d_h/2 <= 64, computed on the host

struct DecAttnArgs {
  const float *q_direct;        // [batch, n_q*d_h] fp32, rotated, or NULL
  const int32_t *oldlen_in;     // [batch] or NULL
  const float *praw; int nsum, wtot, batch, rope;   // split-K partials [nsum, batch, wtot]
  int32_t *oldlen_out;          // [batch] or NULL: index of the newest row that took part, or -1 (none / slot full)
  bf16 *kc, *cc; const int32_t *seq_lens, *slots; int max_batch, max_seq;
  PageMap pm; int ps_shift;     // block-table layout: page_size = 1 << ps_shift, a multiple of the rows of a step
  int splits; float scale_log2e;
  float *pacc, *pml;
};

// RoPE angle of position p and frequency f: reduced mod 2 pi in fp64, then fp32 sincos
__device__ __forceinline__ void rope_sincos(int p, double f, float &sn, float &cs) {
  const double ang = (double)p * f;
  const double k = rint(ang * 0.15915494309189535);
  double r = fma(-k, 6.283185307179586, ang);
  r = fma(-k, 2.4492935982947064e-16, r);
  sincosf((float)r, &sn, &cs);
}

template <class S>
__global__ __launch_bounds__(256, S::OCC) void decode_attn_kernel(DecAttnArgs a, RopeFreq rf) {
  constexpr int DH = S::DH, QPK = S::QPK, NQ = S::NQ, QPC = S::QPC, DL = S::DL, KCH = S::KCH, CCH = S::CCH;
  constexpr int GPL = S::GPL, LPG = S::LPG, R = S::R, DLC = S::DLC;
  constexpr int KROW = S::NK * DH / 8, CROW = S::NC * DL / 8;   // 16-byte words per cache row
  constexpr int WQ = NQ * DH, WK = S::NK * DH, WC = S::NC * DL;
  __shared__ float sm[kWaves][NQ], sl[kWaves][NQ];
  // merge area: one copy per wave where that fits beside a second workgroup (one barrier instead of
  // four rounds), else one copy that the waves add to in turn
  constexpr bool kOnePass = kWaves * NQ * DL * 4 <= 32 * 1024;
  __shared__ float lacc[(kOnePass ? kWaves : 1) * NQ * DL];
  __shared__ float qs[WQ];                                       // rotated queries * scale * log2(e)
  __shared__ __attribute__((aligned(16))) bf16 newrow[WK + WC];  // fused step: the new token's k | c row

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int s = blockIdx.x, b = blockIdx.y, splits = a.splits;
  float *pa = a.pacc + (int64_t)(b * splits + s) * NQ * DL;
  float *pm = a.pml + (int64_t)(b * splits + s) * NQ * 2;
  const int slot = a.slots ? a.slots[b] : b;
  const bool slot_ok = slot >= 0 && slot < a.max_batch;
  // old = index of the newest row that takes part, n = old + 1 rows in all
  int old;
  if (a.oldlen_in) old = a.oldlen_in[b];
  else if (a.praw) {   // a row without a page counts as a full slot
    const int p = slot_ok ? a.seq_lens[slot] : -1;
    old = (p >= 0 && p < a.max_seq && cache_row(a.pm, a.max_seq, slot, p) >= 0) ? p : -1;
  }
  else old = (slot_ok ? min(a.seq_lens[slot], a.max_seq) : 0) - 1;
  if (a.oldlen_out && s == 0 && tid == 0) a.oldlen_out[b] = old;
  if (old < 0 && (a.praw || a.oldlen_in)) {   // slot full: the tail kernel zero-fills this sequence
    if (tid < NQ) { pm[2 * tid] = -INFINITY; pm[2 * tid + 1] = 0.f; }
    return;
  }
  const int n = old + 1;
  // balanced slices in units of R rows (the waves of a workgroup take blocks of R rows round-robin)
  // In a fused step the last slice is made about 4 % shorter: its workgroup also builds the new row.
  const int64_t units = (n + R - 1) / R;
  const int64_t den = (int64_t)splits * 100 - (a.praw && splits > 1 ? 4 : 0);
  const int j0 = min(n, (int)(units * s * 100 / den) * R);
  int j1 = s + 1 == splits ? n : min(n, (int)(units * (s + 1) * 100 / den) * R);
  // fused step: the new row (index old) is not in the cache yet; the workgroup whose slice holds it
  // streams one row less and attends to the new row from LDS
  const bool has_new = a.praw != nullptr && j0 < j1 && j1 == n;
  if (has_new) j1 -= 1;
  const u32x4 *Kp = reinterpret_cast<const u32x4 *>(a.kc) + lane;
  const u32x4 *Cp = reinterpret_cast<const u32x4 *>(a.cc) + lane;
  // pool row of logical row jb, the first row of a step (a step never straddles a page)
  auto row0 = [&](int jb) -> int64_t {
    if (!a.pm.table) return (int64_t)slot * a.max_seq + jb;
    const int pi = __builtin_amdgcn_readfirstlane(jb >> a.ps_shift);   // wave-uniform: a scalar load
    int pg = a.pm.table[(int64_t)slot * a.pm.pages_per_slot + pi];
    pg = (unsigned)pg >= (unsigned)a.pm.num_pages ? 0 : pg;
    return ((int64_t)pg << a.ps_shift) + (jb & (a.pm.page_size - 1));
  };

  float m[KCH][QPK], l[KCH][QPK];
#pragma unroll
  for (int i = 0; i < KCH; ++i)
#pragma unroll
    for (int u = 0; u < QPK; ++u) { m[i][u] = -INFINITY; l[i][u] = 0.f; }
  float acc[CCH][QPC][8];
#pragma unroll
  for (int j = 0; j < CCH; ++j)
#pragma unroll
    for (int v = 0; v < QPC; ++v)
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[j][v][e] = 0.f;

  const int nblk = (j1 - j0 + R - 1) / R;   // j1 - j0 may be 0 (only the new row)
  u32x4 kA[R][KCH], cA[R][CCH], kB[R][KCH], cB[R][CCH];

  auto load = [&](u32x4 (&kb)[R][KCH], u32x4 (&cb)[R][CCH], int blk) {
    const int jb = j0 + blk * R;
    const int64_t rb = row0(jb);
#pragma unroll
    for (int r = 0; r < R; ++r) {
      const int64_t j = rb + min(r, j1 - 1 - jb);   // rows past the slice re-read its last row; weight 0
#pragma unroll
      for (int i = 0; i < KCH; ++i) kb[r][i] = __builtin_nontemporal_load(Kp + j * KROW + i * 64);
#pragma unroll
      for (int i = 0; i < CCH; ++i) cb[r][i] = __builtin_nontemporal_load(Cp + j * CROW + i * 64);
    }
  };

  // ---- queries (and the new row) into LDS.  Order of the requests: the partial sums of the queries
  // first, then the first two blocks of the cache stream (which do not depend on the queries), so
  // that the stream is already in flight while the queries are reduced and rotated.
  constexpr int half = DH / 2;
  constexpr int QPAIRS = WQ / 2 / 256;   // rotation pairs (e, e + d_h/2) of q per thread
  static_assert(WQ % 512 == 0 && WK % 512 == 0 && WC % 256 == 0, "prologue mapping");
  const int64_t pstride = (int64_t)a.batch * a.wtot;
  const float *pb = a.praw ? a.praw + (int64_t)b * a.wtot : nullptr;
  // sum over the split-K partials of column `c` (all loads independent, nsum <= 16)
  auto col_sum = [&](int c) {
    float pv[16];
#pragma unroll
    for (int k = 0; k < 16; ++k) pv[k] = k < a.nsum ? pb[k * pstride + c] : 0.f;
    float v = 0.f;
#pragma unroll
    for (int k = 0; k < 16; ++k) v += pv[k];
    return v;
  };
  auto rotate = [&](float &lo, float &hi, int j) {
    if (!a.rope) return;
    float sn, cs;
    rope_sincos(old, rf.f[j], sn, cs);
    const float l2 = lo * cs - hi * sn, h2 = hi * cs + lo * sn;
    lo = l2; hi = h2;
  };
  float q_lo[QPAIRS], q_hi[QPAIRS];
  if (a.praw) {
#pragma unroll
    for (int i = 0; i < QPAIRS; ++i) {
      const int pr = tid + i * 256, c0 = (pr / half) * DH + pr % half;
      q_lo[i] = col_sum(c0);
      q_hi[i] = col_sum(c0 + half);
    }
  } else {
#pragma unroll
    for (int i = 0; i < QPAIRS; ++i) {
      const int pr = tid + i * 256, c0 = (pr / half) * DH + pr % half;
      q_lo[i] = a.q_direct[(int64_t)b * WQ + c0];
      q_hi[i] = a.q_direct[(int64_t)b * WQ + c0 + half];
    }
  }
  __builtin_amdgcn_sched_barrier(0);   // keep the query loads ahead of the stream in the memory queue
  if (wave < nblk) load(kA, cA, wave);
  if (wave + kWaves < nblk) load(kB, cB, wave + kWaves);
  __builtin_amdgcn_sched_barrier(0);
#pragma unroll
  for (int i = 0; i < QPAIRS; ++i) {
    const int pr = tid + i * 256, c0 = (pr / half) * DH + pr % half;
    if (a.praw) rotate(q_lo[i], q_hi[i], pr % half);
    qs[c0] = q_lo[i] * a.scale_log2e;
    qs[c0 + half] = q_hi[i] * a.scale_log2e;
  }
  if (has_new) {   // the new token's key row (rotated) and latent row: LDS for this workgroup, cache for the rest
    const int64_t nr = cache_row(a.pm, a.max_seq, slot, old);   // >= 0: checked where old was set
    bf16 *krow = a.kc + nr * WK, *crow = a.cc + nr * WC;
    constexpr int KPAIRS = WK / 2 / 256, CCOLS = WC / 256;
    float k_lo[KPAIRS], k_hi[KPAIRS], cv[CCOLS];   // all partial loads of the row are requested together
#pragma unroll
    for (int i = 0; i < KPAIRS; ++i) {
      const int pr = tid + i * 256, c0 = (pr / half) * DH + pr % half;
      k_lo[i] = col_sum(WQ + c0);
      k_hi[i] = col_sum(WQ + c0 + half);
    }
#pragma unroll
    for (int i = 0; i < CCOLS; ++i) cv[i] = col_sum(WQ + WK + tid + i * 256);
#pragma unroll
    for (int i = 0; i < KPAIRS; ++i) {
      const int pr = tid + i * 256, c0 = (pr / half) * DH + pr % half;
      rotate(k_lo[i], k_hi[i], pr % half);
      const bf16 rl = (bf16)k_lo[i], rh = (bf16)k_hi[i];
      newrow[c0] = rl; newrow[c0 + half] = rh;
      krow[c0] = rl; krow[c0 + half] = rh;
    }
#pragma unroll
    for (int i = 0; i < CCOLS; ++i) {
      const bf16 r = (bf16)cv[i];
      newrow[WK + tid + i * 256] = r;
      crow[tid + i * 256] = r;
    }
  }
  __syncthreads();

  // this lane's slice of every query it scores against, as bf16 pairs: scores and the map-times-latent
  // update are bf16 dot products with fp32 sums (v_dot2_f32_bf16), the precision the prefill kernels
  // give the same products; two rows per instruction in the update
  typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
  static_assert(R % 2 == 0, "rows are taken in pairs");
  bf16x2 qh[KCH][QPK][4];
#pragma unroll
  for (int i = 0; i < KCH; ++i)
#pragma unroll
    for (int u = 0; u < QPK; ++u) {
      const int g = (i * GPL + lane / LPG) * QPK + u;
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        bf16x2 t;
        t[0] = (bf16)qs[g * DH + (lane % LPG) * 8 + 2 * w];
        t[1] = (bf16)qs[g * DH + (lane % LPG) * 8 + 2 * w + 1];
        qh[i][u][w] = t;
      }
    }
  const bf16x2 ones = {(bf16)1.0f, (bf16)1.0f};
  auto compute = [&](const u32x4 (&kb)[R][KCH], const u32x4 (&cb)[R][CCH], int nv) {
    float p[R][KCH][QPK];
    // scores of R keys against this lane's groups (log2 domain)
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
      for (int i = 0; i < KCH; ++i) {
        const unsigned kw[4] = {kb[r][i].x, kb[r][i].y, kb[r][i].z, kb[r][i].w};
#pragma unroll
        for (int u = 0; u < QPK; ++u) {
          float a = 0.f;
#pragma unroll
          for (int w = 0; w < 4; ++w) a = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, kw[w]), qh[i][u][w], a, false);
          a = group_sum<LPG>(a);
          p[r][i][u] = r < nv ? a : -INFINITY;
        }
      }
    // online softmax over the block; probabilities rounded to bf16 in row pairs, the row sum is the sum
    // of the rounded values
    float corr[KCH][QPK];
    int pk[R / 2][KCH][QPK];
    bool changed = false;
#pragma unroll
    for (int i = 0; i < KCH; ++i)
#pragma unroll
      for (int u = 0; u < QPK; ++u) {
        float bm = p[0][i][u];
#pragma unroll
        for (int r = 1; r < R; ++r) bm = fmaxf(bm, p[r][i][u]);
        const float mn = fmaxf(m[i][u], bm);
        const float ref = mn > -INFINITY ? mn : 0.f;   // nothing seen yet and nothing valid here
        corr[i][u] = fast_exp2(m[i][u] - ref);
        changed |= (mn != m[i][u]);
        float ps = l[i][u] * corr[i][u];
#pragma unroll
        for (int rp = 0; rp < R / 2; ++rp) {
          bf16x2 t;
          t[0] = (bf16)fast_exp2(p[2 * rp][i][u] - ref);
          t[1] = (bf16)fast_exp2(p[2 * rp + 1][i][u] - ref);
          pk[rp][i][u] = __builtin_bit_cast(int, t);
          ps = __builtin_amdgcn_fdot2_f32_bf16(t, ones, ps, false);
        }
        l[i][u] = ps;
        m[i][u] = mn;
      }
    if (__any(changed)) {
#pragma unroll
      for (int j = 0; j < CCH; ++j)
#pragma unroll
        for (int v = 0; v < QPC; ++v) {
          const int g = (j / DLC) * QPC + v, t = g / QPK;
          const float cg = lane_bcast(corr[t / GPL][g % QPK], (t % GPL) * LPG);
#pragma unroll
          for (int e = 0; e < 8; ++e) acc[j][v][e] *= cg;
        }
    }
    // L_g += p_g * c  for every map group fed by this latent chunk, two rows at a time: word e of cx is
    // (row A's element e, row B's element e)
#pragma unroll
    for (int rp = 0; rp < R / 2; ++rp)
#pragma unroll
      for (int j = 0; j < CCH; ++j) {
        const unsigned ca[4] = {cb[2 * rp][j].x, cb[2 * rp][j].y, cb[2 * rp][j].z, cb[2 * rp][j].w};
        const unsigned cbv[4] = {cb[2 * rp + 1][j].x, cb[2 * rp + 1][j].y, cb[2 * rp + 1][j].z, cb[2 * rp + 1][j].w};
        bf16x2 cx[8];
#pragma unroll
        for (int w = 0; w < 4; ++w) {
          cx[2 * w] = __builtin_bit_cast(bf16x2, __builtin_amdgcn_perm(cbv[w], ca[w], 0x05040100u));
          cx[2 * w + 1] = __builtin_bit_cast(bf16x2, __builtin_amdgcn_perm(cbv[w], ca[w], 0x07060302u));
        }
#pragma unroll
        for (int v = 0; v < QPC; ++v) {
          const int g = (j / DLC) * QPC + v, t = g / QPK;
          const bf16x2 pg = __builtin_bit_cast(bf16x2, __builtin_amdgcn_readlane(pk[rp][t / GPL][g % QPK], (t % GPL) * LPG));
#pragma unroll
          for (int e = 0; e < 8; ++e) acc[j][v][e] = __builtin_amdgcn_fdot2_f32_bf16(cx[e], pg, acc[j][v][e], false);
        }
      }
  };

  // waves interleave blocks of R keys; two register buffers keep the next block in flight
  auto nvalid = [&](int blk) { return min(R, j1 - (j0 + blk * R)); };
  int blk = wave;
  while (blk < nblk) {
    if (blk != wave && blk + kWaves < nblk) load(kB, cB, blk + kWaves);   // the first pair is already in flight
    compute(kA, cA, nvalid(blk));
    blk += kWaves;
    if (blk >= nblk) break;
    if (blk + kWaves < nblk) load(kA, cA, blk + kWaves);
    compute(kB, cB, nvalid(blk));
    blk += kWaves;
  }
  if (has_new && wave == 0) {   // the new token's own row, from LDS: one more block with a single valid row
    const u32x4 *nr = reinterpret_cast<const u32x4 *>(newrow) + lane;
#pragma unroll
    for (int r = 0; r < R; ++r) {
#pragma unroll
      for (int i = 0; i < KCH; ++i) kA[r][i] = nr[i * 64];
#pragma unroll
      for (int i = 0; i < CCH; ++i) cA[r][i] = nr[KROW + i * 64];
    }
    compute(kA, cA, 1);
  }

  // ---- merge the four waves (deterministic order), write the un-normalised partial
#pragma unroll
  for (int i = 0; i < KCH; ++i)
#pragma unroll
    for (int u = 0; u < QPK; ++u)
      if (lane % LPG == 0) {
        const int g = (i * GPL + lane / LPG) * QPK + u;
        sm[wave][g] = m[i][u];
        sl[wave][g] = l[i][u];
      }
  __syncthreads();
  float wscale[CCH][QPC];
#pragma unroll
  for (int j = 0; j < CCH; ++j)
#pragma unroll
    for (int v = 0; v < QPC; ++v) {
      const int g = (j / DLC) * QPC + v;
      float mx = sm[0][g];
#pragma unroll
      for (int w = 1; w < kWaves; ++w) mx = fmaxf(mx, sm[w][g]);
      wscale[j][v] = sm[wave][g] > -INFINITY ? fast_exp2(sm[wave][g] - mx) : 0.f;
    }
  if constexpr (kOnePass) {
#pragma unroll
    for (int j = 0; j < CCH; ++j)
#pragma unroll
      for (int v = 0; v < QPC; ++v) {
        const int g = (j / DLC) * QPC + v;
        float *dst = lacc + wave * NQ * DL + g * DL + (j % DLC) * 512 + lane * 8;
#pragma unroll
        for (int e = 0; e < 8; ++e) dst[e] = acc[j][v][e] * wscale[j][v];
      }
    __syncthreads();
    for (int i = tid; i < NQ * DL; i += 256) {
      float v = lacc[i];
#pragma unroll
      for (int w = 1; w < kWaves; ++w) v += lacc[w * NQ * DL + i];   // fixed order
      pa[i] = v;
    }
  } else {
    for (int w = 0; w < kWaves; ++w) {
      if (wave == w) {
#pragma unroll
        for (int j = 0; j < CCH; ++j)
#pragma unroll
          for (int v = 0; v < QPC; ++v) {
            const int g = (j / DLC) * QPC + v;
            float *dst = lacc + g * DL + (j % DLC) * 512 + lane * 8;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
              const float val = acc[j][v][e] * wscale[j][v];
              dst[e] = (w == 0) ? val : dst[e] + val;
            }
          }
      }
      __syncthreads();
    }
    for (int i = tid; i < NQ * DL; i += 256) pa[i] = lacc[i];
  }
  if (tid < NQ) {
    const int g = tid;
    float mx = sm[0][g];
    for (int w = 1; w < kWaves; ++w) mx = fmaxf(mx, sm[w][g]);
    float ls = 0.f;
    for (int w = 0; w < kWaves; ++w)
      if (sm[w][g] > -INFINITY) ls += sl[w][g] * fast_exp2(sm[w][g] - mx);
    pm[2 * g] = mx;
    pm[2 * g + 1] = ls;
  }
}

// ---- narrow rows: one shared key of 64 and one latent of 128 (the paper's own model shapes) --------
// A cache row is only 128 + 256 bytes, so one 1 KiB wave load covers 8 key rows (8 lanes each) or 4
// latent rows (16 lanes each).  A wave takes 8 rows per step: one key load and two latent loads.
// Scores are formed in the key layout (lane l: row l/8), the latent accumulators live in the latent
// layout (lane l: rows l/16 and 4 + l/16 of the step), so a wave runs four independent online-softmax
// streams (rows c and c+4 of every step, c = 0..3): the two key-layout lane groups of a stream are 32
// lanes apart and agree on its statistics with one exchange, and the latent-layout lanes of stream c
// fetch its two probabilities (one bf16 pair) and its rescale factor from lane 8c.  Scores and the
// probability-times-latent update are bf16 dot products with fp32 sums (v_dot2_f32_bf16, two rows per
// instruction), which is what keeps the kernel from being bound by VALU issue.  Streams, waves and
// splits are merged with the usual log-sum-exp weights.  Same three call modes as the kernel above.
// NC = 2 is the variant with two latents of 128 per row (a wave load covers 2 latent rows): two
// streams of four rows a step, each lane accumulating the maps of its own latent.
template <int NQ, int NC = 1>
__global__ __launch_bounds__(256) void decode_narrow_kernel(DecAttnArgs a, RopeFreq rf) {
  constexpr int DH = 64, DL = 128, WQ = NQ * DH, WK = DH, WC = NC * DL, half = DH / 2, R = 8;
  constexpr int KROW = WK / 8, CROW = WC / 8;   // 16-byte words per cache row
  constexpr int QPC = NQ / NC;                  // maps per latent
  constexpr int NCL = 2 * NC, RPL = R / NCL;    // latent loads per step, rows per latent load
  static_assert((NC == 1 || NC == 2) && NQ % NC == 0, "one or two latents");
  static_assert(WQ / 2 <= 512 && WC <= 256, "prologue mapping");
  __shared__ float sm[kWaves][NQ], sl[kWaves][NQ];
  __shared__ float lacc[kWaves * NQ * DL];   // one copy per wave: they merge in one pass
  __shared__ float qs[WQ];                                       // rotated queries * scale * log2(e)
  __shared__ __attribute__((aligned(16))) bf16 newrow[WK + WC];  // fused step: the new token's k | c row

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int s = blockIdx.x, b = blockIdx.y, splits = a.splits;
  float *pa = a.pacc + (int64_t)(b * splits + s) * NQ * DL;
  float *pm = a.pml + (int64_t)(b * splits + s) * NQ * 2;
  const int slot = a.slots ? a.slots[b] : b;
  const bool slot_ok = slot >= 0 && slot < a.max_batch;
  int old;   // index of the newest row that takes part
  if (a.oldlen_in) old = a.oldlen_in[b];
  else if (a.praw) {   // a row without a page counts as a full slot
    const int p = slot_ok ? a.seq_lens[slot] : -1;
    old = (p >= 0 && p < a.max_seq && cache_row(a.pm, a.max_seq, slot, p) >= 0) ? p : -1;
  }
  else old = (slot_ok ? min(a.seq_lens[slot], a.max_seq) : 0) - 1;
  if (a.oldlen_out && s == 0 && tid == 0) a.oldlen_out[b] = old;
  if (old < 0 && (a.praw || a.oldlen_in)) {   // slot full: the tail kernel zero-fills this sequence
    if (tid < NQ) { pm[2 * tid] = -INFINITY; pm[2 * tid + 1] = 0.f; }
    return;
  }
  const int n = old + 1;
  const int64_t units = (n + R - 1) / R;
  const int j0 = min(n, (int)(units * s / splits) * R);
  int j1 = s + 1 == splits ? n : min(n, (int)(units * (s + 1) / splits) * R);
  const bool has_new = a.praw != nullptr && j0 < j1 && j1 == n;
  if (has_new) j1 -= 1;
  const u32x4 *Kp = reinterpret_cast<const u32x4 *>(a.kc);
  const u32x4 *Cp = reinterpret_cast<const u32x4 *>(a.cc);
  // pool row of logical row jb, the first row of a step (a step never straddles a page)
  auto row0 = [&](int jb) -> int64_t {
    if (!a.pm.table) return (int64_t)slot * a.max_seq + jb;
    const int pi = __builtin_amdgcn_readfirstlane(jb >> a.ps_shift);   // wave-uniform: a scalar load
    int pg = a.pm.table[(int64_t)slot * a.pm.pages_per_slot + pi];
    pg = (unsigned)pg >= (unsigned)a.pm.num_pages ? 0 : pg;
    return ((int64_t)pg << a.ps_shift) + (jb & (a.pm.page_size - 1));
  };

  float m[NQ], l[NQ], acc[QPC][8];   // a latent-layout lane accumulates the maps of its own latent
#pragma unroll
  for (int g = 0; g < NQ; ++g) { m[g] = -INFINITY; l[g] = 0.f; }
#pragma unroll
  for (int v = 0; v < QPC; ++v)
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[v][e] = 0.f;
  const int nblk = (j1 - j0 + R - 1) / R;   // j1 - j0 may be 0 (only the new row)
  struct Blk { u32x4 k, c[NCL]; };
  Blk bA, bB, bC, bD;   // four steps (3 or 5 KiB each) in flight per wave
  auto load = [&](Blk &bk, int blk) {   // rows past the slice re-read its last row; weight 0
    const int jb = j0 + blk * R, last = j1 - 1 - jb;
    const int64_t rb = row0(jb);
    bk.k = __builtin_nontemporal_load(Kp + (rb + min(lane >> 3, last)) * KROW + (lane & 7));
#pragma unroll
    for (int i = 0; i < NCL; ++i)
      bk.c[i] = __builtin_nontemporal_load(Cp + (rb + min(i * RPL + lane / CROW, last)) * CROW + lane % CROW);
  };

  // ---- queries (and the new row) into LDS; the first cache blocks are requested right behind the
  // partial sums so that the stream is in flight while the queries are reduced and rotated
  const int64_t pstride = (int64_t)a.batch * a.wtot;
  const float *pb = a.praw ? a.praw + (int64_t)b * a.wtot : nullptr;
  auto col_sum = [&](int c) {
    float pv[16];
#pragma unroll
    for (int k = 0; k < 16; ++k) pv[k] = k < a.nsum ? pb[k * pstride + c] : 0.f;
    float v = 0.f;
#pragma unroll
    for (int k = 0; k < 16; ++k) v += pv[k];
    return v;
  };
  auto rotate = [&](float &lo, float &hi, int j) {
    if (!a.rope) return;
    float sn, cs;
    rope_sincos(old, rf.f[j], sn, cs);
    const float l2 = lo * cs - hi * sn, h2 = hi * cs + lo * sn;
    lo = l2; hi = h2;
  };
  constexpr int QPT = (WQ / 2 + 255) / 256;   // rotation pairs (qc0, qc0 + d_h/2) per thread
  float q_lo[QPT], q_hi[QPT];
#pragma unroll
  for (int i = 0; i < QPT; ++i) {
    const int pi = tid + i * 256, qc0 = (pi / half) * DH + pi % half;
    q_lo[i] = q_hi[i] = 0.f;
    if (pi < WQ / 2) {
      if (a.praw) { q_lo[i] = col_sum(qc0); q_hi[i] = col_sum(qc0 + half); }
      else { q_lo[i] = a.q_direct[(int64_t)b * WQ + qc0]; q_hi[i] = a.q_direct[(int64_t)b * WQ + qc0 + half]; }
    }
  }
  __builtin_amdgcn_sched_barrier(0);
  if (wave < nblk) load(bA, wave);
  if (wave + kWaves < nblk) load(bB, wave + kWaves);
  if (wave + 2 * kWaves < nblk) load(bC, wave + 2 * kWaves);
  if (wave + 3 * kWaves < nblk) load(bD, wave + 3 * kWaves);
  __builtin_amdgcn_sched_barrier(0);
#pragma unroll
  for (int i = 0; i < QPT; ++i) {
    const int pi = tid + i * 256, qc0 = (pi / half) * DH + pi % half;
    if (pi < WQ / 2) {
      if (a.praw) rotate(q_lo[i], q_hi[i], pi % half);
      qs[qc0] = q_lo[i] * a.scale_log2e;
      qs[qc0 + half] = q_hi[i] * a.scale_log2e;
    }
  }
  if (has_new) {   // the new token's key row (rotated) and latent row: LDS for this workgroup, cache for the rest
    const int64_t nr = cache_row(a.pm, a.max_seq, slot, old);   // >= 0: checked where old was set
    bf16 *krow = a.kc + nr * WK, *crow = a.cc + nr * WC;
    if (tid < half) {
      float k_lo = col_sum(WQ + tid), k_hi = col_sum(WQ + tid + half);
      rotate(k_lo, k_hi, tid);
      const bf16 rl = (bf16)k_lo, rh = (bf16)k_hi;
      newrow[tid] = rl; newrow[tid + half] = rh;
      krow[tid] = rl; krow[tid + half] = rh;
    }
    const int c = NC == 1 ? tid - 64 : tid;   // one latent: waves 1 and 2, beside the key row's wave
    if (c >= 0 && c < WC) {
      const bf16 r = (bf16)col_sum(WQ + WK + c);
      newrow[WK + c] = r;
      crow[c] = r;
    }
  }
  __syncthreads();

  // this lane's eighth of every query as bf16 pairs: the scores are bf16 dot products with fp32 sums
  // (v_dot2_f32_bf16), the precision the prefill kernels give the same product
  typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
  bf16x2 qh[NQ][4];
#pragma unroll
  for (int g = 0; g < NQ; ++g)
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      bf16x2 t;
      t[0] = (bf16)qs[g * DH + (lane & 7) * 8 + 2 * w];
      t[1] = (bf16)qs[g * DH + (lane & 7) * 8 + 2 * w + 1];
      qh[g][w] = t;
    }
  const bf16x2 ones = {(bf16)1.0f, (bf16)1.0f};
  // Key layout: lane l holds row l/8 of the step.  Latent layout: lane l holds rows i*RPL + l/CROW of
  // the step (i = 0 .. NCL-1), i.e. stream c = l/CROW takes rows c, c+RPL, ..., and the maps of latent
  // (l%CROW)/16.  One latent: 4 streams of 2 rows a step; two latents: 2 streams of 4 rows a step,
  // taken as two row pairs (c, c+2) and (c+4, c+6).  src = the key-layout lane on row c that hands
  // this lane its probabilities: with two latents, the odd lanes of a key row hold the second latent's maps.
  const int strm = lane / CROW, cgl = (lane % CROW) >> 4;
  const int src = strm * 8 + cgl;
  constexpr int PAIR_X = NC == 1 ? 32 : 16;   // lane distance to the other row of a pair (row ^ 4 or row ^ 2)
  auto compute = [&](const Blk &bk, int nv) {
    float corr[NQ];
    bf16x2 pk[NQ];   // (probability of this lane's row, of its pair's other row), rounded as the MFMA paths do
    const unsigned kw[4] = {bk.k.x, bk.k.y, bk.k.z, bk.k.w};
    const bool valid = (lane >> 3) < nv;
    bool changed = false;
#pragma unroll
    for (int g = 0; g < NQ; ++g) {
      float sc = 0.f;
#pragma unroll
      for (int w = 0; w < 4; ++w) sc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, kw[w]), qh[g][w], sc, false);
      sc = group_sum<8>(sc);
      sc = valid ? sc : -INFINITY;
      const float sc2 = __shfl_xor(sc, PAIR_X, 64);          // the pair's other row
      float mx = fmaxf(sc, sc2);
      if constexpr (NC == 2) mx = fmaxf(mx, __shfl_xor(mx, 32, 64));   // the stream's other pair
      const float mn = fmaxf(m[g], mx);
      const float ref = mn > -INFINITY ? mn : 0.f;            // a stream that has seen no row yet
      corr[g] = fast_exp2(m[g] - ref);
      changed |= mn != m[g];
      bf16x2 t;
      t[0] = (bf16)fast_exp2(sc - ref);
      t[1] = (bf16)fast_exp2(sc2 - ref);
      pk[g] = t;
      l[g] = __builtin_amdgcn_fdot2_f32_bf16(t, ones, l[g] * corr[g], false);   // the sum of the rounded values (of this pair)
      m[g] = mn;
    }
    // latent elements of a pair's two rows side by side: word e = (row A's element e, row B's element e)
    bf16x2 cx[NC][8];
#pragma unroll
    for (int pr = 0; pr < NC; ++pr) {
      const u32x4 &va = bk.c[2 * pr], &vb = bk.c[2 * pr + 1];
      const unsigned ca[4] = {va.x, va.y, va.z, va.w}, cb[4] = {vb.x, vb.y, vb.z, vb.w};
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        cx[pr][2 * w] = __builtin_bit_cast(bf16x2, __builtin_amdgcn_perm(cb[w], ca[w], 0x05040100u));
        cx[pr][2 * w + 1] = __builtin_bit_cast(bf16x2, __builtin_amdgcn_perm(cb[w], ca[w], 0x07060302u));
      }
    }
    const bool any_changed = __any(changed);
#pragma unroll
    for (int v = 0; v < QPC; ++v) {
      // what this key-layout lane hands out: the odd lanes of a row serve the second latent's maps
      int give = __builtin_bit_cast(int, pk[v]);
      float give_corr = corr[v];
      if constexpr (NC == 2) {
        if (lane & 1) { give = __builtin_bit_cast(int, pk[QPC + v]); give_corr = corr[QPC + v]; }
      }
      // lane src sits in the key layout on the first row of the stream's first pair: its pair is
      // (first latent load's probability, second's); the second pair's lane is four rows further
      bf16x2 pp[NC];
      pp[0] = __builtin_bit_cast(bf16x2, __shfl(give, src, 64));
      if constexpr (NC == 2) pp[1] = __builtin_bit_cast(bf16x2, __shfl(give, src + 32, 64));
      if (any_changed) {   // wave-uniform
        const float cr = __shfl(give_corr, src, 64);
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[v][e] *= cr;
      }
#pragma unroll
      for (int pr = 0; pr < NC; ++pr)
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[v][e] = __builtin_amdgcn_fdot2_f32_bf16(cx[pr][e], pp[pr], acc[v][e], false);
    }
  };
  int blk = wave;
  auto step = [&](Blk &bk) {   // consume a buffer, then refill it with the step four rounds ahead
    compute(bk, min(R, j1 - (j0 + blk * R)));
    if (blk + 4 * kWaves < nblk) load(bk, blk + 4 * kWaves);
    blk += kWaves;
  };
  while (blk < nblk) {
    step(bA);
    if (blk >= nblk) break;
    step(bB);
    if (blk >= nblk) break;
    step(bC);
    if (blk >= nblk) break;
    step(bD);
  }
  if (has_new && wave == 0) {   // the new token's own row, from LDS: one more step with a single valid row
    const u32x4 *nr = reinterpret_cast<const u32x4 *>(newrow);
    bA.k = nr[lane & 7];
#pragma unroll
    for (int i = 0; i < NCL; ++i) bA.c[i] = nr[KROW + lane % CROW];
    compute(bA, 1);
  }

  // ---- merge the streams of the wave, then the four waves (fixed order), write the partial.
  // One latent: streams 0..3 sit on key rows 0..3 (lanes l, l^8, l^16, l^24); each of a stream's two
  // key rows holds the stream's whole sum.  Two latents: streams 0 and 1 on rows 0 and 1 (lanes l,
  // l^8); key rows r and r^4 hold the sums of the stream's two pairs (lanes l, l^32).
  float mw[NQ], lw[NQ];
#pragma unroll
  for (int g = 0; g < NQ; ++g) {
    float mx = fmaxf(m[g], __shfl_xor(m[g], 8, 64));
    if constexpr (NC == 1) mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
    const float ref = mx > -INFINITY ? mx : 0.f;
    float lv = l[g] * fast_exp2(m[g] - ref);     // 0 for a stream without rows
    lv += __shfl_xor(lv, 8, 64);
    lv += __shfl_xor(lv, NC == 1 ? 16 : 32, 64);
    mw[g] = mx; lw[g] = lv;
  }
#pragma unroll
  for (int v = 0; v < QPC; ++v) {
    float give = m[v], mref = mw[v];             // mw is the same in every lane
    if constexpr (NC == 2) {
      if (lane & 1) give = m[QPC + v];
      if (cgl) mref = mw[QPC + v];
    }
    const float ms = __shfl(give, src, 64);      // this latent-layout lane's stream and map
    const float sc = fast_exp2(ms - (mref > -INFINITY ? mref : 0.f));
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      float val = acc[v][e] * sc;
      if constexpr (NC == 1) val += __shfl_xor(val, 16, 64);
      val += __shfl_xor(val, 32, 64);
      acc[v][e] = val;
    }
  }
  if (lane == 0) {
#pragma unroll
    for (int g = 0; g < NQ; ++g) { sm[wave][g] = mw[g]; sl[wave][g] = lw[g]; }
  }
  __syncthreads();
  if (lane < CROW) {   // lanes of stream 0 hold the wave's sums: latent cgl, elements (lane % 16) * 8 ..
#pragma unroll
    for (int v = 0; v < QPC; ++v) {
      const int g = cgl * QPC + v;
      float mx = sm[0][g];
#pragma unroll
      for (int x = 1; x < kWaves; ++x) mx = fmaxf(mx, sm[x][g]);
      const float mine = sm[wave][g];
      const float ws = mine > -INFINITY ? fast_exp2(mine - mx) : 0.f;
      float *dst = lacc + wave * NQ * DL + g * DL + (lane & 15) * 8;
#pragma unroll
      for (int e = 0; e < 8; ++e) dst[e] = acc[v][e] * ws;
    }
  }
  __syncthreads();
  for (int i = tid; i < NQ * DL; i += 256) {
    float v = lacc[i];
#pragma unroll
    for (int w = 1; w < kWaves; ++w) v += lacc[w * NQ * DL + i];   // fixed order
    pa[i] = v;
  }
  if (tid < NQ) {
    const int g = tid;
    float mx = sm[0][g];
    for (int w = 1; w < kWaves; ++w) mx = fmaxf(mx, sm[w][g]);
    float ls = 0.f;
    for (int w = 0; w < kWaves; ++w)
      if (sm[w][g] > -INFINITY) ls += sl[w][g] * fast_exp2(sm[w][g] - mx);
    pm[2 * g] = mx;
    pm[2 * g + 1] = ls;
  }
}

// Combine of the splits of one (sequence, map group): weights exp2(m_s - max) / sum_s exp2(m_s - max) l_s.
// grid (d_l / 256, n_q, batch); a full slot (oldlen < 0) gives a zero row.
__global__ __launch_bounds__(256) void decode_combine_kernel(Dims d, const float *__restrict__ pacc,
                                                             const float *__restrict__ pml,
                                                             const int32_t *__restrict__ oldlen, int splits,
                                                             float *__restrict__ L) {
  extern __shared__ float wt[];   // [splits]
  const int tid = threadIdx.x, lane = tid & 63;
  const int g = blockIdx.y, b = blockIdx.z;
  const int c = blockIdx.x * 256 + tid;
  float *Lr = L + ((int64_t)b * d.nq + g) * d.dl;
  if (oldlen[b] < 0) {
    if (c < d.dl) Lr[c] = 0.f;
    return;
  }
  const float *pm = pml + ((int64_t)b * splits * d.nq + g) * 2;
  const int64_t ms = (int64_t)d.nq * 2;
  if (tid < 64) {   // one wave computes the weights
    float mx = -INFINITY;
    for (int s = lane; s < splits; s += 64) mx = fmaxf(mx, pm[s * ms]);
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o, 64));
    float ls = 0.f;
    for (int s = lane; s < splits; s += 64) {
      const float m = pm[s * ms];
      if (m > -INFINITY) ls += exp2f(m - mx) * pm[s * ms + 1];
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) ls += __shfl_xor(ls, o, 64);
    const float inv = 1.0f / ls;
    for (int s = lane; s < splits; s += 64) {
      const float m = pm[s * ms];
      wt[s] = m > -INFINITY ? exp2f(m - mx) * inv : 0.f;
    }
  }
  __syncthreads();
  if (c >= d.dl) return;
  const float *pa = pacc + ((int64_t)b * splits * d.nq + g) * d.dl + c;
  const int64_t as = (int64_t)d.nq * d.dl;
  float a0 = 0.f, a1 = 0.f;
  int s = 0;
  for (; s + 1 < splits; s += 2) {
    a0 = fmaf(wt[s], pa[s * as], a0);
    a1 = fmaf(wt[s + 1], pa[(s + 1) * as], a1);
  }
  if (s < splits) a0 = fmaf(wt[s], pa[s * as], a0);
  Lr[c] = a0 + a1;
}

// Tail of the decode step in ONE launch, for one head and ROWS sequences per workgroup:
//   1. log-sum-exp weights of the context splits and the combined, normalised group output L_g,
//   2. value decoder and gate (Sec. 3.2): O_i = (L_g W_{P,i}) * Sigmoid(gate pre-activation of the
//      new token); 512 threads = d_h columns x (512 / d_h) slices of the latent dimension,
//   3. bookkeeping: seq_lens[slot] += 1, or the CACHE_FULL flag (head 0's workgroup only).
template <typename TO, int ROWS>
__global__ __launch_bounds__(512) void decode_tail_kernel(Dims d, const float *__restrict__ pacc,
                                                          const float *__restrict__ pml,
                                                          const int32_t *__restrict__ oldlen, int splits, int batch,
                                                          const float *__restrict__ G, int g_nsum, int64_t g_kstride, int g_ld,
                                                          const bf16 *__restrict__ wp,
                                                          TO *__restrict__ out, int32_t *seq_lens, int32_t *status,
                                                          const int32_t *__restrict__ slots, int max_batch) {
  extern __shared__ float smem[];
  float *Ls = smem;                          // [ROWS][dl]
  float *red = Ls + ROWS * d.dl;             // [8 waves][ROWS][dh] and, earlier, [4][128] float4
  float *wt = red + max(8 * ROWS * d.dh, 2048);   // [ROWS][splits]
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int head = blockIdx.x, g = head / d.hpq, b0 = blockIdx.y * ROWS;
  // gate pre-activations of this thread's outputs = sum of the projection's split-K partials (one term
  // if already summed); requested first, used last
  constexpr int kMaxOut = (ROWS * 128 + 511) / 512;
  float gz[kMaxOut];
#pragma unroll
  for (int o = 0; o < kMaxOut; ++o) {
    gz[o] = 0.f;
    const int i = tid + o * 512, r = i / d.dh, ee = i % d.dh;
    if (d.gate && i < ROWS * d.dh && b0 + r < batch)
      for (int k = 0; k < g_nsum; ++k) gz[o] += G[k * g_kstride + (int64_t)(b0 + r) * g_ld + head * d.dh + ee];
  }
  if (head == 0 && tid < ROWS && b0 + tid < batch) {
    const int b = b0 + tid, slot = slots ? slots[b] : b;
    if (slot >= 0 && slot < max_batch) {
      if (oldlen[b] >= 0) seq_lens[slot] = oldlen[b] + 1;
      else status[slot] = GTA_ERR_CACHE_FULL;
    }
  }
  for (int r = wave; r < ROWS; r += 8) {
    const int b = b0 + r;
    const bool live = b < batch && oldlen[b] >= 0;
    const float *pm = pml + ((int64_t)b * splits * d.nq + g) * 2;
    const int64_t ms = (int64_t)d.nq * 2;
    float mx = -INFINITY;
    if (live)
      for (int s = lane; s < splits; s += 64) mx = fmaxf(mx, pm[s * ms]);
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o, 64));
    float ls = 0.f;
    if (live)
      for (int s = lane; s < splits; s += 64) {
        const float m = pm[s * ms];
        if (m > -INFINITY) ls += exp2f(m - mx) * pm[s * ms + 1];
      }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) ls += __shfl_xor(ls, o, 64);
    const float inv = 1.0f / ls;
    for (int s = lane; s < splits; s += 64) {
      float w = 0.f;
      if (live) {
        const float m = pm[s * ms];
        if (m > -INFINITY) w = exp2f(m - mx) * inv;
      }
      wt[r * splits + s] = w;
    }
  }
  __syncthreads();
  // combined group output: the (row, 4-column group) items are dealt to the threads, with up to 4
  // threads per item that split the sum over the splits (summed through LDS); 8 independent 16-byte
  // loads in flight per thread, all rows of the workgroup in the same round trip
  const int64_t as4 = (int64_t)d.nq * d.dl / 4;
  const int nc4 = d.dl / 4, items = ROWS * nc4;
  const int P = items >= 512 ? 1 : (items >= 256 ? 2 : 4);   // phases
  const int per_pass = 512 / P;                               // items per pass
  float4 *red4 = reinterpret_cast<float4 *>(red);             // [P][per_pass], reused below
  for (int base = 0; base < items; base += per_pass) {
    const int idx = tid % per_pass, ph = tid / per_pass, it = base + idx;
    const int r = it / nc4, c4 = it % nc4, b = b0 + r;
    float4 a = make_float4(0.f, 0.f, 0.f, 0.f);
    if (it < items && b < batch && oldlen[b] >= 0) {
      const float4 *pa = reinterpret_cast<const float4 *>(pacc + ((int64_t)b * splits * d.nq + g) * d.dl) + c4;
      const float *w = wt + r * splits;
      for (int s0 = ph; s0 < splits; s0 += 8 * P) {
        float4 v[8];
        float ww[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          const int s = s0 + P * u;
          ww[u] = s < splits ? w[s] : 0.f;
          v[u] = ww[u] != 0.f ? pa[s * as4] : make_float4(0.f, 0.f, 0.f, 0.f);
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          a.x = fmaf(ww[u], v[u].x, a.x); a.y = fmaf(ww[u], v[u].y, a.y);
          a.z = fmaf(ww[u], v[u].z, a.z); a.w = fmaf(ww[u], v[u].w, a.w);
        }
      }
    }
    red4[ph * per_pass + idx] = a;
    __syncthreads();
    if (ph == 0 && it < items) {
      float4 o = red4[idx];
      for (int q = 1; q < P; ++q) {
        const float4 x = red4[q * per_pass + idx];
        o.x += x.x; o.y += x.y; o.z += x.z; o.w += x.w;
      }
      reinterpret_cast<float4 *>(Ls + r * d.dl)[c4] = o;
    }
    __syncthreads();
  }
  // decoder: thread = (8 output columns, one of 512*8/d_h latent phases); all its weight loads
  // (16 bytes each) are independent; phases are summed by shuffles and through LDS
  const int ncg = d.dh / 8, cg = tid % ncg, aph = tid / ncg, naph = 512 / ncg;
  float z[ROWS][8];
#pragma unroll
  for (int r = 0; r < ROWS; ++r)
#pragma unroll
    for (int e = 0; e < 8; ++e) z[r][e] = 0.f;
  const bf16 *wbase = wp + (int64_t)head * d.dl * d.dh + cg * 8;
#pragma unroll 16
  for (int a = aph; a < d.dl; a += naph) {
    const bf16x8 w8 = *reinterpret_cast<const bf16x8 *>(wbase + (int64_t)a * d.dh);
#pragma unroll
    for (int r = 0; r < ROWS; ++r) {
      const float lv = Ls[r * d.dl + a];
#pragma unroll
      for (int e = 0; e < 8; ++e) z[r][e] = fmaf(lv, (float)w8[e], z[r][e]);
    }
  }
  // lanes with equal cg inside a wave are ncg apart
#pragma unroll
  for (int r = 0; r < ROWS; ++r)
#pragma unroll
    for (int e = 0; e < 8; ++e)
      for (int o = ncg; o < 64; o <<= 1) z[r][e] += __shfl_xor(z[r][e], o, 64);
  if (lane < ncg) {
#pragma unroll
    for (int r = 0; r < ROWS; ++r)
#pragma unroll
      for (int e = 0; e < 8; ++e) red[(wave * ROWS + r) * d.dh + cg * 8 + e] = z[r][e];
  }
  __syncthreads();
#pragma unroll
  for (int o = 0; o < kMaxOut; ++o) {
    const int i = tid + o * 512;
    if (i >= ROWS * d.dh) break;
    const int r = i / d.dh, ee = i % d.dh, b = b0 + r;
    if (b >= batch) continue;
    float v = 0.f;
#pragma unroll
    for (int q = 0; q < 8; ++q) v += red[(q * ROWS + r) * d.dh + ee];
    const int col = head * d.dh + ee;
    if (d.gate == kGateSigmoid) v *= 1.0f / (1.0f + __expf(-gz[o]));
    else if (d.gate) v *= gate_factor(d.gate, gz[o]);
    out[(int64_t)b * d.wg_w + col] = (TO)v;
  }
}

// The same tail for ONE sequence per workgroup (small batches), d_l = 512, d_h = 128 and at most 64
// splits: every global load of the kernel -- split statistics, the 64 x 512 partial accumulators of
// the group, the head's 512 x 128 decoder matrix, the gate terms -- is requested up front, so the
// kernel costs one memory round trip instead of four dependent ones.
template <typename TO>
__global__ __launch_bounds__(512) void decode_tail1_kernel(Dims d, const float *__restrict__ pacc,
                                                           const float *__restrict__ pml,
                                                           const int32_t *__restrict__ oldlen, int splits,
                                                           const float *__restrict__ G, int g_nsum, int64_t g_kstride,
                                                           int g_ld, const bf16 *__restrict__ wp, TO *__restrict__ out,
                                                           int32_t *seq_lens, int32_t *status,
                                                           const int32_t *__restrict__ slots, int max_batch) {
  constexpr int DL = 512, DH = 128, MAXS = 64;
  __shared__ float wt[MAXS];
  __shared__ float4 red4[4][DL / 4];
  __shared__ float Ls[DL];
  __shared__ float redz[8][DH];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int head = blockIdx.x, g = head / d.hpq, b = blockIdx.y;
  const int old = oldlen[b];
  const bool live = old >= 0;
  // ---- all loads
  float gz = 0.f;
  if (d.gate && live && tid < DH)
    for (int k = 0; k < g_nsum; ++k) gz += G[k * g_kstride + (int64_t)b * g_ld + head * DH + tid];
  const int64_t ms = (int64_t)d.nq * 2;
  float m_s = -INFINITY, l_s = 0.f;
  if (live && tid < splits) {
    const float *pm = pml + ((int64_t)b * splits * d.nq + g) * 2 + tid * ms;
    m_s = pm[0]; l_s = pm[1];
  }
  const int c4 = tid & 127, ph = tid >> 7;
  float4 v[MAXS / 4];
  {
    const float4 *pa = reinterpret_cast<const float4 *>(pacc + ((int64_t)b * splits * d.nq + g) * DL) + c4;
    const int64_t as4 = (int64_t)d.nq * DL / 4;
#pragma unroll
    for (int u = 0; u < MAXS / 4; ++u) {
      const int sp = ph + 4 * u;
      v[u] = (live && sp < splits) ? pa[sp * as4] : make_float4(0.f, 0.f, 0.f, 0.f);
    }
  }
  const int cg = tid & 15, aph = tid >> 4;   // 8 output columns, one of 32 latent phases
  bf16x8 w8[DL / 32];
  {
    const bf16 *wb = wp + (int64_t)head * DL * DH + cg * 8;
#pragma unroll
    for (int i = 0; i < DL / 32; ++i) w8[i] = *reinterpret_cast<const bf16x8 *>(wb + (int64_t)(aph + 32 * i) * DH);
  }
  if (head == 0 && tid == 0) {
    const int slot = slots ? slots[b] : b;
    if (slot >= 0 && slot < max_batch) {
      if (live) seq_lens[slot] = old + 1;
      else status[slot] = GTA_ERR_CACHE_FULL;
    }
  }
  // ---- log-sum-exp weights of the splits (wave 0)
  if (wave == 0) {
    float mx = m_s;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o, 64));
    const float e = m_s > -INFINITY ? exp2f(m_s - mx) : 0.f;
    float ls = e * l_s;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) ls += __shfl_xor(ls, o, 64);
    wt[lane] = e / ls;
  }
  __syncthreads();
  // ---- combined, normalised group output
  {
    float4 acc4 = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
    for (int u = 0; u < MAXS / 4; ++u) {
      const int sp = ph + 4 * u;
      const float w = sp < splits ? wt[sp] : 0.f;
      if (w != 0.f) {   // a split without rows has weight 0 and an unwritten accumulator
        acc4.x = fmaf(w, v[u].x, acc4.x); acc4.y = fmaf(w, v[u].y, acc4.y);
        acc4.z = fmaf(w, v[u].z, acc4.z); acc4.w = fmaf(w, v[u].w, acc4.w);
      }
    }
    red4[ph][c4] = acc4;
  }
  __syncthreads();
  if (tid < DL / 4) {
    const float4 x0 = red4[0][tid], x1 = red4[1][tid], x2 = red4[2][tid], x3 = red4[3][tid];
    Ls[tid * 4 + 0] = (x0.x + x1.x) + (x2.x + x3.x);
    Ls[tid * 4 + 1] = (x0.y + x1.y) + (x2.y + x3.y);
    Ls[tid * 4 + 2] = (x0.z + x1.z) + (x2.z + x3.z);
    Ls[tid * 4 + 3] = (x0.w + x1.w) + (x2.w + x3.w);
  }
  __syncthreads();
  // ---- value decoder (Sec. 3.2) from the prefetched matrix, gate, store
  float z[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) z[e] = 0.f;
#pragma unroll
  for (int i = 0; i < DL / 32; ++i) {
    const float lv = Ls[aph + 32 * i];
#pragma unroll
    for (int e = 0; e < 8; ++e) z[e] = fmaf(lv, (float)w8[i][e], z[e]);
  }
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    z[e] += __shfl_xor(z[e], 16, 64);
    z[e] += __shfl_xor(z[e], 32, 64);
  }
  if (lane < 16) {
#pragma unroll
    for (int e = 0; e < 8; ++e) redz[wave][cg * 8 + e] = z[e];
  }
  __syncthreads();
  if (tid < DH) {
    float o = 0.f;
#pragma unroll
    for (int q = 0; q < 8; ++q) o += redz[q][tid];
    if (d.gate == kGateSigmoid) o *= 1.0f / (1.0f + __expf(-gz));
    else if (d.gate) o *= gate_factor(d.gate, gz);
    out[(int64_t)b * d.wg_w + head * DH + tid] = live ? (TO)o : (TO)0.f;
  }
}

// The tail for the narrow shapes (d_l = 128, d_h = 64, 1 / 2 / 4 heads per map group, at most 32 splits):
// one workgroup finishes the heads of ONE map group for two sequences, and, like the kernel above, asks
// for everything it reads -- split statistics, partial accumulators, the group's decoder matrices, the
// gate partials -- before it uses any of it.
template <typename TO, int HPQ>
__global__ __launch_bounds__(256) void decode_tail_narrow_kernel(Dims d, const float *__restrict__ pacc,
                                                                 const float *__restrict__ pml,
                                                                 const int32_t *__restrict__ oldlen, int splits,
                                                                 int batch, const float *__restrict__ G, int g_nsum,
                                                                 int64_t g_kstride, int g_ld,
                                                                 const bf16 *__restrict__ wp, TO *__restrict__ out,
                                                                 int32_t *seq_lens, int32_t *status,
                                                                 const int32_t *__restrict__ slots, int max_batch) {
  constexpr int DL = 128, DH = 64, MAXS = 32, ROWS = 2;
  constexpr int NPH = 256 / (HPQ * 8), APC = DL / NPH;      // latent phases per head, latent rows per phase
  constexpr int NOUT = ROWS * HPQ * DH / 256 > 0 ? ROWS * HPQ * DH / 256 : 1;   // outputs per thread
  __shared__ float wt[ROWS][MAXS];
  __shared__ float4 red4[4][ROWS * DL / 4];
  __shared__ float Ls[ROWS][DL];
  __shared__ float redz[NPH][ROWS][HPQ * DH];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int g = blockIdx.x, b0 = blockIdx.y * ROWS;
  auto live = [&](int r) { return b0 + r < batch && oldlen[b0 + r] >= 0; };
  // ---- all loads
  float gz[NOUT];
#pragma unroll
  for (int o = 0; o < NOUT; ++o) {
    gz[o] = 0.f;
    const int i = tid + o * 256, r = i / (HPQ * DH), c = i % (HPQ * DH);
    if (d.gate && i < ROWS * HPQ * DH && live(r))
      for (int k = 0; k < g_nsum; ++k) gz[o] += G[k * g_kstride + (int64_t)(b0 + r) * g_ld + g * HPQ * DH + c];
  }
  const int64_t ms = (int64_t)d.nq * 2;
  float m_s = -INFINITY, l_s = 0.f;
  if (wave == 0) {   // lane = (row, split)
    const int r = lane / MAXS, sp = lane % MAXS;
    if (live(r) && sp < splits) {
      const float *pm = pml + ((int64_t)(b0 + r) * splits * d.nq + g) * 2 + sp * ms;
      m_s = pm[0]; l_s = pm[1];
    }
  }
  const int item = tid % (ROWS * DL / 4), sph = tid / (ROWS * DL / 4);   // (row, 4 columns), one of 4 split phases
  const int ir = item / (DL / 4), ic4 = item % (DL / 4);
  float4 v[MAXS / 4];
  {
    const bool lv = live(ir);
    const float4 *pa = reinterpret_cast<const float4 *>(pacc + ((int64_t)(lv ? b0 + ir : 0) * splits * d.nq + g) * DL) + ic4;
    const int64_t as4 = (int64_t)d.nq * DL / 4;
#pragma unroll
    for (int u = 0; u < MAXS / 4; ++u) {
      const int sp = sph + 4 * u;
      v[u] = (lv && sp < splits) ? pa[sp * as4] : make_float4(0.f, 0.f, 0.f, 0.f);
    }
  }
  const int cg = tid % 8, ph = (tid / 8) % NPH, hl = tid / (8 * NPH);   // 8 output columns, latent phase, head
  bf16x8 w8[APC];
  {
    const bf16 *wb = wp + (int64_t)(g * HPQ + hl) * DL * DH + cg * 8;
#pragma unroll
    for (int i = 0; i < APC; ++i) w8[i] = *reinterpret_cast<const bf16x8 *>(wb + (int64_t)(ph * APC + i) * DH);
  }
  if (g == 0 && tid < ROWS && b0 + tid < batch) {
    const int b = b0 + tid, slot = slots ? slots[b] : b;
    if (slot >= 0 && slot < max_batch) {
      if (oldlen[b] >= 0) seq_lens[slot] = oldlen[b] + 1;
      else status[slot] = GTA_ERR_CACHE_FULL;
    }
  }
  // ---- log-sum-exp weights of the splits: one 32-lane half of wave 0 per row
  if (wave == 0) {
    float mx = m_s;
#pragma unroll
    for (int o = 16; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o, 64));
    const float e = m_s > -INFINITY ? exp2f(m_s - mx) : 0.f;
    float ls = e * l_s;
#pragma unroll
    for (int o = 16; o > 0; o >>= 1) ls += __shfl_xor(ls, o, 64);
    wt[lane / MAXS][lane % MAXS] = ls > 0.f ? e / ls : 0.f;
  }
  __syncthreads();
  {
    float4 a4 = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
    for (int u = 0; u < MAXS / 4; ++u) {
      const int sp = sph + 4 * u;
      const float w = sp < splits ? wt[ir][sp] : 0.f;
      if (w != 0.f) {   // a split without rows has weight 0 and an unwritten accumulator
        a4.x = fmaf(w, v[u].x, a4.x); a4.y = fmaf(w, v[u].y, a4.y);
        a4.z = fmaf(w, v[u].z, a4.z); a4.w = fmaf(w, v[u].w, a4.w);
      }
    }
    red4[sph][item] = a4;
  }
  __syncthreads();
  if (tid < ROWS * DL / 4) {
    const float4 x0 = red4[0][tid], x1 = red4[1][tid], x2 = red4[2][tid], x3 = red4[3][tid];
    float *dst = &Ls[0][0] + tid * 4;
    dst[0] = (x0.x + x1.x) + (x2.x + x3.x); dst[1] = (x0.y + x1.y) + (x2.y + x3.y);
    dst[2] = (x0.z + x1.z) + (x2.z + x3.z); dst[3] = (x0.w + x1.w) + (x2.w + x3.w);
  }
  __syncthreads();
  // ---- value decoder (Sec. 3.2) from the prefetched matrices, latent phases summed through LDS
#pragma unroll
  for (int r = 0; r < ROWS; ++r) {
    float z[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) z[e] = 0.f;
#pragma unroll
    for (int i = 0; i < APC; ++i) {
      const float lv = Ls[r][ph * APC + i];
#pragma unroll
      for (int e = 0; e < 8; ++e) z[e] = fmaf(lv, (float)w8[i][e], z[e]);
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) redz[ph][r][hl * DH + cg * 8 + e] = z[e];
  }
  __syncthreads();
#pragma unroll
  for (int o = 0; o < NOUT; ++o) {
    const int i = tid + o * 256, r = i / (HPQ * DH), c = i % (HPQ * DH);
    if (i >= ROWS * HPQ * DH || b0 + r >= batch) continue;
    float acc = 0.f;
#pragma unroll
    for (int q = 0; q < NPH; ++q) acc += redz[q][r][c];
    if (d.gate == kGateSigmoid) acc *= 1.0f / (1.0f + __expf(-gz[o]));
    else if (d.gate) acc *= gate_factor(d.gate, gz[o]);
    out[(int64_t)(b0 + r) * d.wg_w + g * HPQ * DH + c] = live(r) ? (TO)acc : (TO)0.f;
  }
}

// where the gate pre-activations come from: `nsum` terms at stride `kstride`, row pitch `ld`
struct GateSrc { const float *g; int nsum; int64_t kstride; int ld; };

// Large batches: the tail as a GEMM.  This kernel prepares its operands in one launch — blocks
// [0, n_q): log-sum-exp merge of the splits of one (sequence, map group) into the normalised group
// output, rounded to bf16 like the prefill path's (zero row for a full slot); blocks behind them: the
// gate pre-activations of the new token summed over the projection's split-K partials, bf16; block
// (0, b) also does the sequence's bookkeeping.  The value decoder then runs on the MFMA GEMM kernels.
__global__ __launch_bounds__(256) void decode_combine_gate_kernel(Dims d, const float *__restrict__ pacc,
                                                                  const float *__restrict__ pml,
                                                                  const int32_t *__restrict__ oldlen, int splits,
                                                                  GateSrc gs, bf16 *__restrict__ L, bf16 *__restrict__ G,
                                                                  int32_t *seq_lens, int32_t *status,
                                                                  const int32_t *__restrict__ slots, int max_batch) {
  extern __shared__ float wt[];   // [splits]
  const int tid = threadIdx.x, lane = tid & 63, b = blockIdx.y;
  if ((int)blockIdx.x >= d.nq) {   // gate columns, 8 per thread
    const int col = (((int)blockIdx.x - d.nq) * 256 + tid) * 8;
    if (col >= d.wg_w) return;
    float v[8] = {};
    for (int k = 0; k < gs.nsum; ++k) {
      const float *p = gs.g + k * gs.kstride + (int64_t)b * gs.ld + col;
      const float4 x0 = *reinterpret_cast<const float4 *>(p), x1 = *reinterpret_cast<const float4 *>(p + 4);
      v[0] += x0.x; v[1] += x0.y; v[2] += x0.z; v[3] += x0.w; v[4] += x1.x; v[5] += x1.y; v[6] += x1.z; v[7] += x1.w;
    }
    bf16 *o = G + (int64_t)b * d.wg_w + col;
#pragma unroll
    for (int e = 0; e < 8; ++e) o[e] = (bf16)v[e];
    return;
  }
  const int g = blockIdx.x;
  if (g == 0 && tid == 0) {
    const int slot = slots ? slots[b] : b;
    if (slot >= 0 && slot < max_batch) {
      if (oldlen[b] >= 0) seq_lens[slot] = oldlen[b] + 1;
      else status[slot] = GTA_ERR_CACHE_FULL;
    }
  }
  bf16 *Lr = L + ((int64_t)b * d.nq + g) * d.dl;
  if (oldlen[b] < 0) {
    for (int c = tid; c < d.dl; c += 256) Lr[c] = (bf16)0.f;
    return;
  }
  const float *pm = pml + ((int64_t)b * splits * d.nq + g) * 2;
  const int64_t ms = (int64_t)d.nq * 2;
  if (tid < 64) {   // one wave computes the weights
    float mx = -INFINITY;
    for (int s = lane; s < splits; s += 64) mx = fmaxf(mx, pm[s * ms]);
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o, 64));
    float ls = 0.f;
    for (int s = lane; s < splits; s += 64) {
      const float m = pm[s * ms];
      if (m > -INFINITY) ls += exp2f(m - mx) * pm[s * ms + 1];
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) ls += __shfl_xor(ls, o, 64);
    const float inv = 1.0f / ls;
    for (int s = lane; s < splits; s += 64) {
      const float m = pm[s * ms];
      wt[s] = m > -INFINITY ? exp2f(m - mx) * inv : 0.f;
    }
  }
  __syncthreads();
  const int64_t as = (int64_t)d.nq * d.dl;
  for (int c = tid; c < d.dl; c += 256) {
    const float *pa = pacc + ((int64_t)b * splits * d.nq + g) * d.dl + c;
    float a0 = 0.f;
    for (int s = 0; s < splits; ++s) a0 = fmaf(wt[s], pa[s * as], a0);
    Lr[c] = (bf16)a0;
  }
}

template <typename TO, int ROWS>
void launch_tail(const Dims &d, const float *pacc, const float *pml, const DecodeWs &ws, int batch, GateSrc gs,
                 const bf16 *wp, TO *out, const gta_cache &cache, const int32_t *slots, hipStream_t st) {
  dim3 grid(d.nh, (batch + ROWS - 1) / ROWS);
  const size_t red = (size_t)(8 * ROWS * d.dh > 2048 ? 8 * ROWS * d.dh : 2048);
  const size_t smem = ((size_t)ROWS * d.dl + red + (size_t)ROWS * ws.splits) * sizeof(float);
  // eight rows of a 1024-wide latent pass the 64 KiB a kernel gets without asking
  if (smem > 64 * 1024) allow_dynamic_lds((const void *)decode_tail_kernel<TO, ROWS>, 160 * 1024);
  decode_tail_kernel<TO, ROWS><<<grid, 512, smem, st>>>(d, pacc, pml, ws.oldlen, ws.splits, batch, gs.g, gs.nsum,
                                                        gs.kstride, gs.ld, wp, out, cache.seq_lens, cache.status,
                                                        slots, cache.max_batch);
}

template <typename TO>
void launch_tail_any(const Dims &d, const float *pacc, const float *pml, const DecodeWs &ws, int batch, GateSrc gs,
                     const bf16 *wp, TO *out, const gta_cache &cache, const int32_t *slots, hipStream_t st) {
  // about 512 workgroups (two per CU): one sequence per workgroup up to batch * n_h = 512, then 2, 4, 8.
  // Measured at the 1B shape, 8K context: batch 16 one-sequence kernel 9 us against 16 us with two rows;
  // batch 64 two rows 18 us against 31 us with eight (and a whole step of 205 us against 214 us with the
  // one-sequence kernel); batch 128 four rows 24 us against 30 us with two.
  const int rows = batch * d.nh / 512;
  if (rows < 2 && d.dl == 512 && d.dh == 128 && ws.splits <= 64) {
    decode_tail1_kernel<TO><<<dim3(d.nh, batch), 512, 0, st>>>(d, pacc, pml, ws.oldlen, ws.splits, gs.g, gs.nsum,
                                                               gs.kstride, gs.ld, wp, out, cache.seq_lens,
                                                               cache.status, slots, cache.max_batch);
    return;
  }
  if (d.dl == 128 && d.dh == 64 && (d.hpq == 1 || d.hpq == 2 || d.hpq == 4) && ws.splits <= 32) {
    const dim3 grid(d.nq, (batch + 1) / 2);
#define GTA_TAIL_NARROW(HPQ)                                                                                      \
    decode_tail_narrow_kernel<TO, HPQ><<<grid, 256, 0, st>>>(d, pacc, pml, ws.oldlen, ws.splits, batch, gs.g, gs.nsum, \
                                                            gs.kstride, gs.ld, wp, out, cache.seq_lens, cache.status, \
                                                            slots, cache.max_batch)
    if (d.hpq == 4) GTA_TAIL_NARROW(4);
    else if (d.hpq == 2) GTA_TAIL_NARROW(2);
    else GTA_TAIL_NARROW(1);
#undef GTA_TAIL_NARROW
    return;
  }
  if (rows >= 8) launch_tail<TO, 8>(d, pacc, pml, ws, batch, gs, wp, out, cache, slots, st);
  else if (rows >= 4) launch_tail<TO, 4>(d, pacc, pml, ws, batch, gs, wp, out, cache, slots, st);
  else if (rows >= 2) launch_tail<TO, 2>(d, pacc, pml, ws, batch, gs, wp, out, cache, slots, st);
  else launch_tail<TO, 1>(d, pacc, pml, ws, batch, gs, wp, out, cache, slots, st);
}

template <class S>
void launch_attn(const Dims &d, DecAttnArgs a, const RopeFreq &rf, int batch, hipStream_t st) {
  dim3 grid(a.splits, batch);
  decode_attn_kernel<S><<<grid, 256, 0, st>>>(a, rf);
}

typedef DecShape<128, 4, 1, 1, 1, 8, 2> Shape1B;      // 4 maps, 4 keys of 128, one latent of 512
typedef DecShape<128, 8, 1, 1, 2, 4, 1> ShapeWide;    // 8 maps, 8 keys of 128, one latent of 1024
// other groupings of heads of 128 on the same kernel (a key row and every latent row are multiples of 1 KiB):
typedef DecShape<128, 4, 2, 1, 1, 8, 2> ShapeQ8K4;    // 8 maps on 4 keys (two maps share a key), one latent of 512
typedef DecShape<128, 4, 1, 2, 1, 4, 1> ShapeC2;      // 4 maps, 4 keys, two latents of 512 (two maps per latent)
typedef DecShape<128, 4, 2, 2, 1, 4, 1> ShapeQ8K4C2;  // 8 maps on 4 keys and two latents of 512
typedef DecShape<128, 4, 1, 4, 1, 2, 1> ShapeC4;      // 4 maps, each with its own key and its own latent of 512
// X(shape) for every wide-row instantiation, in dispatch order
#define GTA_WIDE_DECODE_SHAPES(X) X(Shape1B) X(ShapeWide) X(ShapeQ8K4) X(ShapeC2) X(ShapeQ8K4C2) X(ShapeC4)

template <class S>
bool matches(const Dims &d) {
  return d.dh == S::DH && d.nk == S::NK && d.qpk == S::QPK && d.nc == S::NC && d.dl == S::DL;
}

}  // namespace

// one shared key of 64 and one latent of 128 with 3 / 5 / 6 maps, or two latents with 6 / 10 maps (the
// paper's 160M, 500M and 1B GTA models)
static bool narrow_shape(const Dims &d) {
  if (d.dh != 64 || d.nk != 1 || d.dl != 128) return false;
  return (d.nc == 1 && (d.nq == 3 || d.nq == 5 || d.nq == 6)) || (d.nc == 2 && (d.nq == 6 || d.nq == 10));
}

bool tuned_decode_supported(const Dims &d) {
  if (d.dtype != GTA_BF16) return false;
#define GTA_X(S) if (matches<S>(d)) return true;
  GTA_WIDE_DECODE_SHAPES(GTA_X)
#undef GTA_X
  return narrow_shape(d);
}

// Workgroups the split-K launch should have.  One per CU for the wide-row kernels and the two-latent
// narrow kernel: measured at the 1B shape with slot strides as the benchmark has them, 256 against 512
// workgroups: batch 8 at 32K rows 102 against 105 us per step, batch 16 at 8K 64 against 66, batch 32
// at 8K 110 against 111, batch 64 at 8K 197 against 199 (fewer partials to write and merge, longer
// slices per workgroup); the 8 x 128 + 1024 kernel and the two-latent narrow kernel keep only one
// workgroup per CU resident, so 512 would run in two rounds (163 -> 137 us, 82 -> 65 us).  The
// one-latent narrow kernel (384-byte rows, 50 MB per step) prefers two per CU: 41 against 44 us.
int tuned_decode_target_workgroups(const Dims &d) {
  if (d.dtype != GTA_BF16) return 512;
  return narrow_shape(d) && d.nc == 1 ? 512 : 256;
}

// The one-sequence tail kernel holds up to 64 splits; beyond that the general tail takes over, which
// costs more than the extra splits gain once there are at least 256 workgroups anyway (batch 4 at 32K
// rows: 67 us per step with 64 splits, 74 us with 128; batch 1 and 2 still gain from 128).
int tuned_decode_max_splits(const Dims &d, int batch) {
  const bool one_seq_tail = d.dtype == GTA_BF16 && d.dl == 512 && d.dh == 128 && batch * d.nh / 512 < 2;
  return one_seq_tail && batch >= 4 ? 64 : 1024;
}

// The streaming kernels take a page per scalar lookup: a step of up to 8 rows must not straddle pages.
bool tuned_decode_layout_ok(const gta_cache &cache) {
  if (!cache.block_table) return true;
  const int ps = cache.page_size;
  return ps >= 16 && (ps & (ps - 1)) == 0;
}

static DecAttnArgs attn_args(const Dims &d, const gta_cache &cache, const int32_t *slots, int batch, int splits,
                             float *part) {
  DecAttnArgs a{};
  a.batch = batch; a.wtot = d.wtot; a.rope = d.rope;
  a.kc = (bf16 *)cache.k; a.cc = (bf16 *)cache.c; a.seq_lens = cache.seq_lens; a.slots = slots;
  a.max_batch = cache.max_batch; a.max_seq = cache.max_seq;
  a.pm = page_map_of(cache);
  a.ps_shift = 0;
  while (a.pm.table && (1 << a.ps_shift) < a.pm.page_size) ++a.ps_shift;
  a.splits = splits; a.scale_log2e = d.scale * 1.4426950408889634f;
  a.pacc = part; a.pml = part + (int64_t)batch * splits * d.nq * d.dl;
  return a;
}

static void launch_attn_any(const Dims &d, const DecAttnArgs &a, const RopeFreq &rf, int batch, hipStream_t st) {
#define GTA_X(S) if (matches<S>(d)) { launch_attn<S>(d, a, rf, batch, st); return; }
  GTA_WIDE_DECODE_SHAPES(GTA_X)
#undef GTA_X
  if (d.nc == 2 && d.nq == 10) decode_narrow_kernel<10, 2><<<dim3(a.splits, batch), 256, 0, st>>>(a, rf);
  else if (d.nc == 2) decode_narrow_kernel<6, 2><<<dim3(a.splits, batch), 256, 0, st>>>(a, rf);
  else if (d.nq == 3) decode_narrow_kernel<3><<<dim3(a.splits, batch), 256, 0, st>>>(a, rf);
  else if (d.nq == 5) decode_narrow_kernel<5><<<dim3(a.splits, batch), 256, 0, st>>>(a, rf);
  else decode_narrow_kernel<6><<<dim3(a.splits, batch), 256, 0, st>>>(a, rf);
}

// q already rotated.  oldlen_in NULL: attend over the rows the caches hold now (stage call); otherwise
// over rows 0 .. oldlen_in[b].  oldlen_out (may equal oldlen_in) receives the newest row index or -1.
void tuned_decode_attention(const Dims &d, const float *q, const int32_t *oldlen_in, int32_t *oldlen_out,
                            const gta_cache &cache, const int32_t *slots, int batch, int splits, float *part,
                            hipStream_t st) {
  DecAttnArgs a = attn_args(d, cache, slots, batch, splits, part);
  a.q_direct = q; a.oldlen_in = oldlen_in; a.oldlen_out = oldlen_out;
  launch_attn_any(d, a, RopeFreq{}, batch, st);
}

void tuned_decode_combine(const Dims &d, const float *part, const int32_t *oldlen, int splits, int batch, float *L,
                          hipStream_t st) {
  const float *pml = part + (int64_t)batch * splits * d.nq * d.dl;
  decode_combine_kernel<<<dim3((d.dl + 255) / 256, d.nq, batch), 256, splits * sizeof(float), st>>>(
      d, part, pml, oldlen, splits, L);
}

int tuned_decode(const Dims &d, const gta_weights &w, const void *x_new, int batch, const gta_cache &cache,
                 const int32_t *slots, void *out, const DecodeWs &ws, hipStream_t st) {
  // Three launches: split-K projection of the new tokens (Sec. 3.2); attention, whose workgroups sum
  // the partials, rotate q and k at position seq_len and append the new rows themselves; the tail
  // (combine, value decoder, gate from the same partials, bookkeeping).
  GateSrc gs;
  if (gemm_shapes_supported(d)) {
    const int ks = skinny_ksplit(d, batch);
    launch_skinny_proj(d, w, x_new, batch, ws.praw, ks, st);
    RopeFreq rf{};
    for (int j = 0; j < d.dh / 2; ++j) rf.f[j] = pow(d.rope_base, -2.0 * (double)j / (double)d.dh);
    DecAttnArgs a = attn_args(d, cache, slots, batch, ws.splits, ws.part);
    a.praw = ws.praw; a.nsum = ks; a.oldlen_out = ws.oldlen;
    launch_attn_any(d, a, rf, batch, st);
    gs = GateSrc{ws.praw + d.wq_w + d.wk_w + d.wc_w, ks, (int64_t)batch * d.wtot, d.wtot};
  } else {
    generic_decode_project(d, w, x_new, batch, cache, slots, ws, st);
    tuned_decode_attention(d, ws.q, ws.oldlen, ws.oldlen, cache, slots, batch, ws.splits, ws.part, st);
    gs = GateSrc{ws.g, 1, 0, d.wg_w};
  }
  const float *pacc = ws.part;
  const float *pml = ws.part + (int64_t)batch * ws.splits * d.nq * d.dl;
  // Large batches: the per-row decoder of the tail kernels grows with the batch (32 us at 256 sequences,
  // 115 us at 1024 on the 1B shape); from 256 sequences on it runs as an MFMA GEMM on bf16 operands
  // (group outputs and gate pre-activations rounded as in prefill), behind one kernel that prepares them.
  if (batch >= kGemmTailBatch && gemm_shapes_supported(d) && d.wg_w % 8 == 0) {
    bf16 *Lb = reinterpret_cast<bf16 *>(ws.l), *Gb = reinterpret_cast<bf16 *>(ws.g);   // fp32-sized buffers, used as bf16
    const int gate_blocks = d.gate ? (d.wg_w / 8 + 255) / 256 : 0;
    decode_combine_gate_kernel<<<dim3(d.nq + gate_blocks, batch), 256, ws.splits * sizeof(float), st>>>(
        d, pacc, pml, ws.oldlen, ws.splits, gs, Lb, Gb, cache.seq_lens, cache.status, slots, cache.max_batch);
    if (w.wo) {
      bf16 *Ob = reinterpret_cast<bf16 *>(ws.o);
      launch_decoder_gemm(d, Lb, w.wp, Gb, Ob, batch, st);
      launch_plain_gemm(Ob, d.wg_w, batch, d.H, d.wg_w, w.wo, out, st);
    } else {
      launch_decoder_gemm(d, Lb, w.wp, Gb, out, batch, st);
    }
    return check_launch();
  }
  if (w.wo && gemm_shapes_supported(d)) {
    // Sec. 3.3 output projection on the MFMA GEMM (64-row tiles), heads rounded to bf16 as in prefill
    bf16 *Ob = reinterpret_cast<bf16 *>(ws.o);   // fp32-sized buffer, used as bf16
    launch_tail_any<bf16>(d, pacc, pml, ws, batch, gs, (const bf16 *)w.wp, Ob, cache, slots, st);
    launch_plain_gemm(Ob, d.wg_w, batch, d.H, d.wg_w, w.wo, out, st);
  } else if (w.wo) {
    launch_tail_any<float>(d, pacc, pml, ws, batch, gs, (const bf16 *)w.wp, ws.o, cache, slots, st);
    generic_out_proj_f32in(d, w, ws.o, batch, out, st);
  } else {
    launch_tail_any<bf16>(d, pacc, pml, ws, batch, gs, (const bf16 *)w.wp, (bf16 *)out, cache, slots, st);
  }
  return check_launch();
}

}  // namespace gta
