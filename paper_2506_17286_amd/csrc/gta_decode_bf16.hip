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

// Tail of the decode step in ONE launch, for one head and ROWS sequences per workgroup:
//   1. log-sum-exp weights of the context splits and the combined, normalised group output L_g,
//   2. value decoder and gate (Sec. 3.2): O_i = (L_g W_{P,i}) * Sigmoid(gate pre-activation of the
//      new token); 512 threads = d_h columns x (512 / d_h) slices of the latent dimension,
//   3. bookkeeping: seq_lens[slot] += 1, or the CACHE_FULL flag (head 0's workgroup only).
template <typename TO, int ROWS>
__global__ __launch_bounds__(512) void decode_tail_kernel(Dims d, const float *__restrict__ pacc,
                                                          const float *__restrict__ pml,
                                                          const int32_t *__restrict__ oldlen, int splits, int batch,
                                                          const float *__restrict__ G, const bf16 *__restrict__ wp,
                                                          TO *__restrict__ out, int32_t *seq_lens, int32_t *status,
                                                          const int32_t *__restrict__ slots, int max_batch) {
  extern __shared__ float smem[];
  float *Ls = smem;                          // [ROWS][dl]
  float *red = Ls + ROWS * d.dl;             // [8 waves][ROWS][dh] and, earlier, [4][128] float4
  float *wt = red + max(8 * ROWS * d.dh, 2048);   // [ROWS][splits]
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int head = blockIdx.x, g = head / d.hpq, b0 = blockIdx.y * ROWS;
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
  // combined group output: thread = (4 columns, one of 4 split phases); 8 independent 16-byte loads
  // in flight per thread, the 4 phases are summed through LDS
  const int64_t as4 = (int64_t)d.nq * d.dl / 4;
  const int nc4 = d.dl / 4;
  float4 *red4 = reinterpret_cast<float4 *>(red);          // [4 phases][nc4], reused below
  for (int r = 0; r < ROWS; ++r) {
    const int b = b0 + r;
    const bool live = b < batch && oldlen[b] >= 0;
    for (int c0 = 0; c0 < nc4; c0 += 128) {
      const int c4 = c0 + (tid & 127), ph = tid >> 7;
      float4 a = make_float4(0.f, 0.f, 0.f, 0.f);
      if (live && c4 < nc4) {
        const float4 *pa = reinterpret_cast<const float4 *>(pacc + ((int64_t)b * splits * d.nq + g) * d.dl) + c4;
        const float *w = wt + r * splits;
        for (int s0 = ph; s0 < splits; s0 += 32) {
          float4 v[8];
          float ww[8];
#pragma unroll
          for (int u = 0; u < 8; ++u) {
            const int s = s0 + 4 * u;
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
      red4[ph * 128 + (tid & 127)] = a;
      __syncthreads();
      if (tid < 128 && c4 < nc4) {
        const float4 x0 = red4[tid], x1 = red4[128 + tid], x2 = red4[256 + tid], x3 = red4[384 + tid];
        float4 o;
        o.x = (x0.x + x1.x) + (x2.x + x3.x); o.y = (x0.y + x1.y) + (x2.y + x3.y);
        o.z = (x0.z + x1.z) + (x2.z + x3.z); o.w = (x0.w + x1.w) + (x2.w + x3.w);
        reinterpret_cast<float4 *>(Ls + r * d.dl)[c4] = o;
      }
      __syncthreads();
    }
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
  for (int i = tid; i < ROWS * d.dh; i += 512) {
    const int r = i / d.dh, ee = i % d.dh, b = b0 + r;
    if (b >= batch) continue;
    float v = 0.f;
#pragma unroll
    for (int q = 0; q < 8; ++q) v += red[(q * ROWS + r) * d.dh + ee];
    const int col = head * d.dh + ee;
    if (d.gate) v *= 1.0f / (1.0f + __expf(-G[(int64_t)b * d.wg_w + col]));
    out[(int64_t)b * d.wg_w + col] = (TO)v;
  }
}

template <typename TO, int ROWS>
void launch_tail(const Dims &d, const float *pacc, const float *pml, const DecodeWs &ws, int batch, const bf16 *wp,
                 TO *out, const gta_cache &cache, const int32_t *slots, hipStream_t st) {
  dim3 grid(d.nh, (batch + ROWS - 1) / ROWS);
  const size_t red = (size_t)(8 * ROWS * d.dh > 2048 ? 8 * ROWS * d.dh : 2048);
  const size_t smem = ((size_t)ROWS * d.dl + red + (size_t)ROWS * ws.splits) * sizeof(float);
  decode_tail_kernel<TO, ROWS><<<grid, 512, smem, st>>>(d, pacc, pml, ws.oldlen, ws.splits, batch, ws.g, wp, out,
                                                        cache.seq_lens, cache.status, slots, cache.max_batch);
}

template <typename TO>
void launch_tail_any(const Dims &d, const float *pacc, const float *pml, const DecodeWs &ws, int batch,
                     const bf16 *wp, TO *out, const gta_cache &cache, const int32_t *slots, hipStream_t st) {
  // about 128 workgroups: one row per workgroup for small batches, up to 8 for large ones
  const int rows = batch * d.nh / 128;
  if (rows >= 8) launch_tail<TO, 8>(d, pacc, pml, ws, batch, wp, out, cache, slots, st);
  else if (rows >= 4) launch_tail<TO, 4>(d, pacc, pml, ws, batch, wp, out, cache, slots, st);
  else if (rows >= 2) launch_tail<TO, 2>(d, pacc, pml, ws, batch, wp, out, cache, slots, st);
  else launch_tail<TO, 1>(d, pacc, pml, ws, batch, wp, out, cache, slots, st);
}

// Sums the split-K partials of the new tokens' projections, rotates q and k at position
// seq_lens[slot] (App. B.1.1; angle reduced mod 2 pi in fp64, then fp32 sincos), appends the key and
// latent rows to the caches (App. B.1.3) and leaves q and the gate pre-activation in fp32.
struct RopeFreq { double f[64]; };   // base^(-2j/d_h), j < d_h/2 <= 64, computed on the host

__global__ __launch_bounds__(256) void decode_finalize_kernel(Dims d, RopeFreq rf, const float *__restrict__ part,
                                                              int nsum, int batch, float *__restrict__ Qo,
                                                              float *__restrict__ Go, int32_t *__restrict__ oldlen,
                                                              bf16 *__restrict__ kc, bf16 *__restrict__ cc,
                                                              const int32_t *__restrict__ seq_lens,
                                                              const int32_t *__restrict__ slots, int max_batch,
                                                              int max_seq) {
  const int64_t idx = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
  if (idx >= (int64_t)batch * d.wtot) return;
  const int b = (int)(idx / d.wtot), col = (int)(idx % d.wtot);
  const int slot = slots ? slots[b] : b;
  const bool slot_ok = slot >= 0 && slot < max_batch;
  const int p = slot_ok ? seq_lens[slot] : 0;
  const bool ok = slot_ok && p >= 0 && p < max_seq;
  if (col == 0) oldlen[b] = ok ? p : -1;
  if (!ok) return;
  const int64_t pstride = (int64_t)batch * d.wtot;
  const int qk_w = d.wq_w + d.wk_w;
  const int half = d.dh / 2, e = col % d.dh;
  const bool rot = d.rope && col < qk_w;
  const int64_t pidx = rot ? (e < half ? idx + half : idx - half) : idx;
  // all partial loads are independent: issue them together (nsum <= 16)
  float pv[16], pu[16];
#pragma unroll
  for (int s = 0; s < 16; ++s) {
    pv[s] = s < nsum ? part[s * pstride + idx] : 0.f;
    pu[s] = (rot && s < nsum) ? part[s * pstride + pidx] : 0.f;
  }
  float v = 0.f, u = 0.f;
#pragma unroll
  for (int s = 0; s < 16; ++s) { v += pv[s]; u += pu[s]; }
  if (rot) {
    const double ang = (double)p * rf.f[e % half];
    const double k = rint(ang * 0.15915494309189535);
    double r = fma(-k, 6.283185307179586, ang);
    r = fma(-k, 2.4492935982947064e-16, r);
    float sn, cs;
    sincosf((float)r, &sn, &cs);
    v = e < half ? v * cs - u * sn : v * cs + u * sn;
  }
  if (col < d.wq_w) {
    Qo[(int64_t)b * d.wq_w + col] = v;
  } else if (col < qk_w) {
    kc[((int64_t)slot * max_seq + p) * d.wk_w + (col - d.wq_w)] = (bf16)v;
  } else if (col < qk_w + d.wc_w) {
    cc[((int64_t)slot * max_seq + p) * d.wc_w + (col - qk_w)] = (bf16)v;
  } else {
    Go[(int64_t)b * d.wg_w + (col - qk_w - d.wc_w)] = v;
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
  if (gemm_shapes_supported(d)) {
    const int ks = skinny_ksplit(d, batch);
    launch_skinny_proj(d, w, x_new, batch, ws.praw, ks, st);
    RopeFreq rf;
    for (int j = 0; j < d.dh / 2; ++j) rf.f[j] = pow(d.rope_base, -2.0 * (double)j / (double)d.dh);
    const int64_t n = (int64_t)batch * d.wtot;
    decode_finalize_kernel<<<(unsigned)((n + 255) / 256), 256, 0, st>>>(
        d, rf, ws.praw, ks, batch, ws.q, ws.g, ws.oldlen, (bf16 *)cache.k, (bf16 *)cache.c, cache.seq_lens, slots,
        cache.max_batch, cache.max_seq);
  } else {
    generic_decode_project(d, w, x_new, batch, cache, slots, ws, st);
  }
  tuned_decode_attention(d, ws.q, ws.oldlen, cache, slots, batch, ws.splits, ws.part, st);
  const float *pacc = ws.part;
  const float *pml = ws.part + (int64_t)batch * ws.splits * d.nq * d.dl;
  if (w.wo) {
    launch_tail_any<float>(d, pacc, pml, ws, batch, (const bf16 *)w.wp, ws.o, cache, slots, st);
    generic_out_proj_f32in(d, w, ws.o, batch, out, st);
  } else {
    launch_tail_any<bf16>(d, pacc, pml, ws, batch, (const bf16 *)w.wp, (bf16 *)out, cache, slots, st);
  }
  return check_launch();
}

}  // namespace gta
