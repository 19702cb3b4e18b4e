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

template <class S>
__global__ __launch_bounds__(256, S::OCC) void decode_attn_kernel(const float *__restrict__ Q, const int32_t *__restrict__ oldlen,
                                                             const bf16 *__restrict__ kc, const bf16 *__restrict__ cc,
                                                             const int32_t *__restrict__ slots, int max_seq, int splits,
                                                             float scale_log2e, float *__restrict__ pacc,
                                                             float *__restrict__ pml) {
  constexpr int DH = S::DH, QPK = S::QPK, NQ = S::NQ, QPC = S::QPC, DL = S::DL, KCH = S::KCH, CCH = S::CCH;
  constexpr int GPL = S::GPL, LPG = S::LPG, R = S::R, DLC = S::DLC;
  constexpr int KROW = S::NK * DH / 8, CROW = S::NC * DL / 8;   // 16-byte words per cache row
  __shared__ float sm[kWaves][NQ], sl[kWaves][NQ];
  __shared__ float lacc[NQ * DL];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int s = blockIdx.x, b = blockIdx.y;
  const int old = oldlen[b];
  float *pa = pacc + (int64_t)(b * splits + s) * NQ * DL;
  float *pm = pml + (int64_t)(b * splits + s) * NQ * 2;
  if (old < 0) {   // slot full: the combine kernel zero-fills this sequence
    if (tid < NQ) { pm[2 * tid] = -INFINITY; pm[2 * tid + 1] = 0.f; }
    return;
  }
  const int n = old + 1;
  int chunk = (n + splits - 1) / splits;
  chunk = (chunk + kWaves * R - 1) / (kWaves * R) * (kWaves * R);
  const int j0 = min(n, s * chunk), j1 = min(n, j0 + chunk);
  const int slot = slots ? slots[b] : b;
  const u32x4 *Kp = reinterpret_cast<const u32x4 *>(kc + (int64_t)slot * max_seq * (S::NK * DH)) + lane;
  const u32x4 *Cp = reinterpret_cast<const u32x4 *>(cc + (int64_t)slot * max_seq * (S::NC * DL)) + lane;

  // this lane's slice of every query it scores against, pre-multiplied by scale * log2(e)
  float qf[KCH][QPK][8];
#pragma unroll
  for (int i = 0; i < KCH; ++i)
#pragma unroll
    for (int u = 0; u < QPK; ++u) {
      const int g = (i * GPL + lane / LPG) * QPK + u;
      const float *qp = Q + (int64_t)b * (NQ * DH) + g * DH + (lane % LPG) * 8;
#pragma unroll
      for (int e = 0; e < 8; ++e) qf[i][u][e] = qp[e] * scale_log2e;
    }
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

  const int nblk = (j1 - j0 + R - 1) / R;
  u32x4 kA[R][KCH], cA[R][CCH], kB[R][KCH], cB[R][CCH];

  auto load = [&](u32x4 (&kb)[R][KCH], u32x4 (&cb)[R][CCH], int blk) {
    const int jb = j0 + blk * R;
#pragma unroll
    for (int r = 0; r < R; ++r) {
      const int64_t j = min(jb + r, j1 - 1);   // rows past the slice re-read its last row; weight 0
#pragma unroll
      for (int i = 0; i < KCH; ++i) kb[r][i] = __builtin_nontemporal_load(Kp + j * KROW + i * 64);
#pragma unroll
      for (int i = 0; i < CCH; ++i) cb[r][i] = __builtin_nontemporal_load(Cp + j * CROW + i * 64);
    }
  };

  auto compute = [&](const u32x4 (&kb)[R][KCH], const u32x4 (&cb)[R][CCH], int blk) {
    const int nv = min(R, j1 - (j0 + blk * R));
    float p[R][KCH][QPK];
    // scores of R keys against this lane's groups (log2 domain)
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
      for (int i = 0; i < KCH; ++i) {
        float kf[8];
        unpack8(kb[r][i], kf);
#pragma unroll
        for (int u = 0; u < QPK; ++u) {
          float a = 0.f;
#pragma unroll
          for (int e = 0; e < 8; ++e) a = fmaf(qf[i][u][e], kf[e], a);
          a = group_sum<LPG>(a);
          p[r][i][u] = r < nv ? a : -INFINITY;
        }
      }
    // online softmax over the block
    float corr[KCH][QPK];
    bool changed = false;
#pragma unroll
    for (int i = 0; i < KCH; ++i)
#pragma unroll
      for (int u = 0; u < QPK; ++u) {
        float bm = p[0][i][u];
#pragma unroll
        for (int r = 1; r < R; ++r) bm = fmaxf(bm, p[r][i][u]);
        const float mn = fmaxf(m[i][u], bm);
        corr[i][u] = fast_exp2(m[i][u] - mn);
        changed |= (mn != m[i][u]);
        float ps = 0.f;
#pragma unroll
        for (int r = 0; r < R; ++r) { p[r][i][u] = fast_exp2(p[r][i][u] - mn); ps += p[r][i][u]; }
        l[i][u] = l[i][u] * corr[i][u] + ps;
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
    // L_g += p_g * c  for every map group fed by this latent chunk
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
      for (int j = 0; j < CCH; ++j) {
        float cf[8];
        unpack8(cb[r][j], cf);
#pragma unroll
        for (int v = 0; v < QPC; ++v) {
          const int g = (j / DLC) * QPC + v, t = g / QPK;
          const float pg = lane_bcast(p[r][t / GPL][g % QPK], (t % GPL) * LPG);
#pragma unroll
          for (int e = 0; e < 8; ++e) acc[j][v][e] = fmaf(pg, cf[e], acc[j][v][e]);
        }
      }
  };

  // waves interleave blocks of R keys; two register buffers keep the next block in flight
  int blk = wave;
  if (blk < nblk) load(kA, cA, blk);
  while (blk < nblk) {
    if (blk + kWaves < nblk) load(kB, cB, blk + kWaves);
    compute(kA, cA, blk);
    blk += kWaves;
    if (blk >= nblk) break;
    if (blk + kWaves < nblk) load(kA, cA, blk + kWaves);
    compute(kB, cB, blk);
    blk += kWaves;
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

// Value decoder and gate (Sec. 3.2) for one head and up to 8 sequences:
// O_i = (L_g W_{P,i}) * Sigmoid(gate pre-activation of the new token).
// 512 threads = d_h columns x (512 / d_h) slices of the latent dimension, reduced through LDS.
constexpr int kRows = 8;

template <typename TO>
__global__ __launch_bounds__(512) void decode_decoder_kernel(Dims d, const float *__restrict__ L, int batch,
                                                             const float *__restrict__ G,
                                                             const bf16 *__restrict__ wp, TO *__restrict__ out) {
  extern __shared__ float smem[];
  float *Ls = smem;                       // [kRows][dl]
  float *red = smem + kRows * d.dl;       // [nsl][kRows][dh]
  const int tid = threadIdx.x;
  const int head = blockIdx.x, g = head / d.hpq, b0 = blockIdx.y * kRows;
  for (int i = tid; i < kRows * d.dl; i += 512) {
    const int r = i / d.dl, c = i % d.dl, b = b0 + r;
    Ls[i] = b < batch ? L[((int64_t)b * d.nq + g) * d.dl + c] : 0.f;
  }
  __syncthreads();
  const int e = tid % d.dh, sl = tid / d.dh, nsl = 512 / d.dh;
  const int per = (d.dl + nsl - 1) / nsl;
  const int a0 = sl * per, a1 = min(d.dl, a0 + per);
  float z[kRows];
#pragma unroll
  for (int r = 0; r < kRows; ++r) z[r] = 0.f;
  const bf16 *wcol = wp + (int64_t)head * d.dl * d.dh + e;
#pragma unroll 4
  for (int a = a0; a < a1; ++a) {
    const float wv = (float)wcol[(int64_t)a * d.dh];
#pragma unroll
    for (int r = 0; r < kRows; ++r) z[r] = fmaf(Ls[r * d.dl + a], wv, z[r]);
  }
#pragma unroll
  for (int r = 0; r < kRows; ++r) red[(sl * kRows + r) * d.dh + e] = z[r];
  __syncthreads();
  for (int i = tid; i < kRows * d.dh; i += 512) {
    const int r = i / d.dh, ee = i % d.dh, b = b0 + r;
    if (b >= batch) continue;
    float v = 0.f;
    for (int q = 0; q < nsl; ++q) v += red[(q * kRows + r) * d.dh + ee];
    const int col = head * d.dh + ee;
    if (d.gate) v *= 1.0f / (1.0f + __expf(-G[(int64_t)b * d.wg_w + col]));
    out[(int64_t)b * d.wg_w + col] = (TO)v;
  }
}

template <class S>
void launch_attn(const Dims &d, const float *q, const int32_t *oldlen, const gta_cache &cache, const int32_t *slots,
                 int batch, int splits, float *pacc, float *pml, hipStream_t st) {
  dim3 grid(splits, batch);
  decode_attn_kernel<S><<<grid, 256, 0, st>>>(q, oldlen, (const bf16 *)cache.k, (const bf16 *)cache.c, slots,
                                             cache.max_seq, splits, d.scale * 1.4426950408889634f, pacc, pml);
}

typedef DecShape<128, 4, 1, 1, 1, 8, 2> Shape1B;      // 4 maps, 4 keys of 128, one latent of 512
typedef DecShape<128, 8, 1, 1, 2, 4, 1> ShapeWide;    // 8 maps, 8 keys of 128, one latent of 1024

template <class S>
bool matches(const Dims &d) {
  return d.dh == S::DH && d.nk == S::NK && d.qpk == S::QPK && d.nc == S::NC && d.dl == S::DL;
}

}  // namespace

bool tuned_decode_supported(const Dims &d) {
  if (d.dtype != GTA_BF16) return false;
  return matches<Shape1B>(d) || matches<ShapeWide>(d);
}

void tuned_decode_attention(const Dims &d, const float *q, const int32_t *oldlen, const gta_cache &cache,
                            const int32_t *slots, int batch, int splits, float *part, hipStream_t st) {
  float *pacc = part;
  float *pml = part + (int64_t)batch * splits * d.nq * d.dl;
  if (matches<Shape1B>(d)) launch_attn<Shape1B>(d, q, oldlen, cache, slots, batch, splits, pacc, pml, st);
  else launch_attn<ShapeWide>(d, q, oldlen, cache, slots, batch, splits, pacc, pml, st);
}

void tuned_decode_combine(const Dims &d, const float *part, const int32_t *oldlen, int splits, int batch, float *L,
                          hipStream_t st) {
  const float *pml = part + (int64_t)batch * splits * d.nq * d.dl;
  decode_combine_kernel<<<dim3((d.dl + 255) / 256, d.nq, batch), 256, splits * sizeof(float), st>>>(
      d, part, pml, oldlen, splits, L);
}

int tuned_decode(const Dims &d, const gta_weights &w, const void *x_new, int batch, const gta_cache &cache,
                 const int32_t *slots, void *out, const DecodeWs &ws, hipStream_t st) {
  // Sec. 3.2 projections of the new tokens, RoPE at position seq_len, append to the caches
  generic_decode_project(d, w, x_new, batch, cache, slots, ws, st);
  tuned_decode_attention(d, ws.q, ws.oldlen, cache, slots, batch, ws.splits, ws.part, st);
  tuned_decode_combine(d, ws.part, ws.oldlen, ws.splits, batch, ws.l, st);
  dim3 grid(d.nh, (batch + kRows - 1) / kRows);
  const size_t smem = (size_t)kRows * (d.dl + 512) * sizeof(float);
  if (w.wo) {
    decode_decoder_kernel<float><<<grid, 512, smem, st>>>(d, ws.l, batch, ws.g, (const bf16 *)w.wp, ws.o);
    generic_out_proj_f32in(d, w, ws.o, batch, out, st);
  } else {
    decode_decoder_kernel<bf16><<<grid, 512, smem, st>>>(d, ws.l, batch, ws.g, (const bf16 *)w.wp, (bf16 *)out);
  }
  launch_decode_commit(cache, slots, ws.oldlen, batch, st);
  return check_launch();
}

}  // namespace gta
