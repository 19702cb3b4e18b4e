// bf16 MFMA GEMMs of the GTA pass for gfx950 (fp32 accumulation):
//   * fused input projection  [Q | K | C | gate] = X . [W_Q | W_K | W_C | W_G]   (paper Sec. 3.2)
//     with RoPE on q and k (App. B.1.1) and the cache write (App. B.1.3) in the epilogue,
//   * value decoder  O_i = (L_{q(i)} W_{P,i}) * Sigmoid(gate)                     (Sec. 3.2),
//   * plain output projection  U = O . W_O                                         (Sec. 3.3).
//
// All weights are row-major [in, out], i.e. the contraction index is the SLOW index of the weight
// operand.  The kernel therefore computes the transposed tile D'[n][m] = sum_k W[k][n] X[m][k]:
// the MFMA row operand comes from the weight tile through the LDS transpose read of gfx950
// (ds_read_b64_tr_b16: each lane receives 4 consecutive k of one n), the MFMA column operand is
// a plain 16-byte LDS read of an X row.  Each lane then owns 4 consecutive output columns of one
// output row, which makes the RoPE pairing (j, j + d_h/2) lane-local.
//
// Workgroup tile BM x BN x BK with WGM x WGN waves of 32x32x16 MFMA tiles.  The 256 x 256 x 64 tiles
// (one wave of 128 x 128 per SIMD) run the hand-pipelined main loop below: two LDS stages, global
// loads two tiles ahead of the LDS writes in two register sets, one barrier per k-tile; their result
// is rounded to bf16, parked in LDS in output layout and written with 16-byte row-contiguous stores.
// The small tiles (64-row tiles of short prefills and of the decode step) take the plain two-stage
// loop and store straight from the accumulator layout.
#include <math.h>

#include <type_traits>

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

template <int BM_, int BN_, int BK_, int WGM_, int WGN_>
struct GemmTile {
  static constexpr int BM = BM_, BN = BN_, BK = BK_, WGM = WGM_, WGN = WGN_;
  static constexpr int WM = BM / WGM, WN = BN / WGN, TM = WM / 32, TN = WN / 32;
  static constexpr int NT = 64 * WGM * WGN;
  static constexpr int A_PITCH = BK * 2 + 16;    // bytes per X row: 16 * odd -> conflict-free b128 reads
  static constexpr int B_PITCH = BN * 2 + 64;    // bytes per weight k-row: == 64 mod 256 for the tr reads
  static constexpr int A_BYTES = BM * A_PITCH, B_BYTES = BK * B_PITCH, STAGE = A_BYTES + B_BYTES;
  static constexpr int SMEM = 2 * STAGE;
  static_assert(WM % 32 == 0 && WN % 32 == 0 && BK % 16 == 0, "tile");
};

// acc[tn][tm][r]:  n = n_wave + tn*32 + 8*(r/4) + 4*(lane/32) + r%4,  m = m_wave + tm*32 + lane%32
template <class T>
__device__ __forceinline__ void gemm_mainloop(const bf16 *__restrict__ A, int64_t lda, int M, int m0,
                                              const bf16 *__restrict__ B, int64_t ldb, int n0, int K, char *smem,
                                              f32x16 (&acc)[T::TN][T::TM]) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wn = wave % T::WGN, wm = wave / T::WGN;
  constexpr int A_CPR = T::BK / 8, A_RPP = T::NT / A_CPR, A_PASSES = T::BM / A_RPP;
  constexpr int B_CPR = T::BN / 8, B_RPP = T::NT / B_CPR, B_PASSES = T::BK / B_RPP;
  static_assert(T::BM % A_RPP == 0 && T::BK % B_RPP == 0 && A_PASSES >= 1 && B_PASSES >= 1, "staging");
  const int a_c = tid % A_CPR, a_r = tid / A_CPR;
  const int b_c = tid % B_CPR, b_r = tid / B_CPR;
  u32x4 ra[A_PASSES], rb[B_PASSES];

  auto gload = [&](int kt) {
#pragma unroll
    for (int i = 0; i < A_PASSES; ++i) {
      const int row = min(m0 + a_r + i * A_RPP, M - 1);
      ra[i] = *reinterpret_cast<const u32x4 *>(A + (int64_t)row * lda + kt * T::BK + a_c * 8);
    }
#pragma unroll
    for (int i = 0; i < B_PASSES; ++i) {
      const int krow = kt * T::BK + b_r + i * B_RPP;
      rb[i] = *reinterpret_cast<const u32x4 *>(B + (int64_t)krow * ldb + n0 + b_c * 8);
    }
  };
  auto sstore = [&](char *st) {
#pragma unroll
    for (int i = 0; i < A_PASSES; ++i)
      *reinterpret_cast<u32x4 *>(st + (a_r + i * A_RPP) * T::A_PITCH + a_c * 16) = ra[i];
#pragma unroll
    for (int i = 0; i < B_PASSES; ++i)
      *reinterpret_cast<u32x4 *>(st + T::A_BYTES + (b_r + i * B_RPP) * T::B_PITCH + b_c * 16) = rb[i];
  };
  // per-lane constant parts of the operand addresses
  const int xoff = (wm * T::WM + (lane & 31)) * T::A_PITCH + (lane >> 5) * 16;
  const int woff = T::A_BYTES + ((lane >> 5) * 8 + ((lane & 15) >> 2)) * T::B_PITCH +
                   (wn * T::WN + ((lane >> 4) & 1) * 16 + (lane & 3) * 4) * 2;
  auto compute = [&](const char *st) {
#pragma unroll
    for (int kk = 0; kk < T::BK / 16; ++kk) {
      bf16x8 xf[T::TM];
#pragma unroll
      for (int tm = 0; tm < T::TM; ++tm)
        xf[tm] = *reinterpret_cast<const bf16x8 *>(st + xoff + tm * 32 * T::A_PITCH + kk * 32);
#pragma unroll
      for (int tn = 0; tn < T::TN; ++tn) {
        const char *wp = st + woff + kk * 16 * T::B_PITCH + tn * 64;
        s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(wp));
        s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(wp + 4 * T::B_PITCH));
        s16x8 w8 = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        bf16x8 wf = __builtin_bit_cast(bf16x8, w8);
#pragma unroll
        for (int tm = 0; tm < T::TM; ++tm)
          acc[tn][tm] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf, xf[tm], acc[tn][tm], 0, 0, 0);
      }
    }
  };

  const int nk = K / T::BK;
  gload(0);
  sstore(smem);
  __syncthreads();
  for (int kt = 0; kt < nk; ++kt) {
    char *cur = smem + (kt & 1) * T::STAGE;
    char *nxt = smem + ((kt & 1) ^ 1) * T::STAGE;
    if (kt + 1 < nk) gload(kt + 1);
    compute(cur);
    if (kt + 1 < nk) sstore(nxt);
    __syncthreads();
  }
}

// ---- software-pipelined main loop for the big tiles --------------------------------------------
// One wave per SIMD owns a 128-wide accumulator tile, so nothing but the wave's own instruction
// stream can hide latencies.  The loop is therefore pipelined by hand on three levels:
//   * operand fragments of k-step kk+1 are read from LDS while the MFMAs of step kk run (two
//     fragment sets); the fragments of the next tile's first step are read during the last step;
//   * k-tile kt+1 is written to the other LDS stage during steps 0..2 of tile kt, and the one
//     workgroup barrier of the tile sits before the last step, whose MFMAs cover its skew;
//   * global loads run two tiles ahead of the LDS writes (two staging register sets): the loads of
//     tile kt+3 go out in steps 1..3, each into registers whose LDS write was issued one step before.
// Every step is one scheduling region in which the memory instructions are dealt out between the
// MFMAs (sched_group_barrier), so the matrix pipe always has the next MFMA queued and neither the
// LDS nor the vector-memory queue sees a burst.
// The last three k-tiles have nothing left to prefetch for the product; the caller may use the two
// staging sets that become free for a `tail` prefetch of 16 + 16 sixteen-byte chunks per thread
// (the decoder fetches its gate tile this way), which are handed back in r_tail0 / r_tail1.
template <class T>
struct PipeMap {
  static constexpr int A_CPR = T::BK / 8, A_RPP = T::NT / A_CPR, A_PASSES = T::BM / A_RPP;
  static constexpr int B_CPR = T::BN / 8, B_RPP = T::NT / B_CPR, B_PASSES = T::BK / B_RPP;
  static constexpr int KSTEPS = T::BK / 16;
  static_assert(T::BM % A_RPP == 0 && T::BK % B_RPP == 0 && A_PASSES >= 1 && B_PASSES >= 1, "staging");
  static_assert(KSTEPS == 4, "the step schedule below is written for four k-steps per tile");
};
template <class T>
struct PipeStage { u32x4 a[PipeMap<T>::A_PASSES], b[PipeMap<T>::B_PASSES]; };

enum : int { SG_MFMA = 0x008, SG_VMEM_READ = 0x020, SG_DS_READ = 0x100, SG_DS_WRITE = 0x200 };

// Schedule of one k-step: N_FRAG fragment reads of the next step go out one per MFMA, then N_W LDS
// writes and N_G global loads are dealt out over the remaining MFMAs.
template <int N_MFMA, int N_FRAG, int N_W, int N_G>
__device__ __forceinline__ void deal_step() {
  // MFMAs that carry fragment reads (one each if there are enough MFMAs, else half of the MFMAs with
  // several reads each); the others carry the LDS writes and global loads
  constexpr int F_SLOTS = N_MFMA > N_FRAG ? N_FRAG : N_MFMA / 2;
  constexpr int RPS = (N_FRAG + F_SLOTS - 1) / F_SLOTS;
  static_assert(F_SLOTS >= 1 && N_MFMA > F_SLOTS, "schedule");
#pragma unroll
  for (int i = 0; i < F_SLOTS; ++i) {
    __builtin_amdgcn_sched_group_barrier(SG_MFMA, 1, 0);
    __builtin_amdgcn_sched_group_barrier(SG_DS_READ, RPS, 0);
  }
  constexpr int rest = N_MFMA - F_SLOTS;
  constexpr int pw = (N_W + rest - 1) / rest, pg = (N_G + rest - 1) / rest;
#pragma unroll
  for (int i = 0; i < rest; ++i) {
    __builtin_amdgcn_sched_group_barrier(SG_MFMA, 1, 0);
    if constexpr (pw > 0) __builtin_amdgcn_sched_group_barrier(SG_DS_WRITE, pw, 0);
    if constexpr (pg > 0) __builtin_amdgcn_sched_group_barrier(SG_VMEM_READ, pg, 0);
  }
  __builtin_amdgcn_sched_barrier(0);
}

// Tail prefetch hook: chunk i (0..15) of tail set `set` is at gbase() + off(set, i) (wave-uniform) +
// thr_of(set, i) (per thread), all offsets in bytes.
struct NoTail {
  static constexpr bool active = false;
  __device__ const char *gbase() const { return nullptr; }
  __device__ unsigned off(int, int) const { return 0; }
  __device__ unsigned thr_of(int, int) const { return 0; }
};

// `Abase` points at row m0 of the row operand; `Bbase` + `boff` (bytes, per thread) at k-row
// tid / B_CPR of this thread's 8-column chunk of the weight operand.  K / BK must be even and >= 4.
template <class T, class Tail>
__device__ __forceinline__ void gemm_mainloop_pipe(const bf16 *__restrict__ Abase, int64_t lda, int rows_valid,
                                                   const bf16 *__restrict__ Bbase, unsigned boff, int64_t ldb,
                                                   int K, char *smem, f32x16 (&acc)[T::TN][T::TM],
                                                   PipeStage<T> &r_tail0, PipeStage<T> &r_tail1, const Tail &tail) {
  typedef PipeMap<T> P;
  typedef PipeStage<T> Stage;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wn = wave % T::WGN, wm = wave / T::WGN;
  const int a_c = tid % P::A_CPR, a_r = tid / P::A_CPR;
  const int b_c = tid % P::B_CPR, b_r = tid / P::B_CPR;
  // Addresses are a wave-uniform base plus ONE 32-bit per-thread offset.  Pass i of the row operand
  // covers rows i * A_RPP + a_r; ip is the last pass that holds a valid row.  Passes before it use the
  // full per-thread offset, pass ip and the (entirely invalid) passes after it use row ip * A_RPP +
  // min(a_r, last valid row of that pass): valid rows map to themselves, the rest stay in bounds.
  const int ip = (rows_valid - 1) / P::A_RPP;
  const unsigned athr = (unsigned)(a_r * lda + a_c * 8) * 2u;
  const unsigned athr_p = (unsigned)(min(a_r, rows_valid - 1 - ip * P::A_RPP) * lda + a_c * 8) * 2u;
  const char *Ab = reinterpret_cast<const char *>(Abase);
  const char *Bb = reinterpret_cast<const char *>(Bbase);
  const int nk = K / T::BK;

  struct Frags { bf16x8 x[T::TM], w[T::TN]; };
  // The 16 loads / LDS writes of a tile are split in three parts (6, 6, 4): A passes with
  // i % 3 == part, B passes with (i + 1) % 3 == part; part < 0 = all.
  // Tiles past the end of K are clamped to the last one (redundant loads, in bounds), except that
  // with a tail, tile nk+1 is tail set 0 and tile nk+2 tail set 1.  The choice is made with scalar
  // bit masks, not branches, so that every k-step stays one scheduling region.
  const unsigned a_pass_bytes = (unsigned)(P::A_RPP * lda * 2), b_pass_bytes = (unsigned)(P::B_RPP * ldb * 2);
  auto gload_part = [&](Stage &r, int kt, int part) {
    const bool tl = Tail::active && kt > nk;
    const int set = kt > nk + 1 ? 1 : 0;
    kt = min(kt, nk - 1);
    const char *ak = Ab + (int64_t)kt * (T::BK * 2);
    const char *bk = Bb + (int64_t)kt * T::BK * ldb * 2;
    const char *abase = tl ? tail.gbase() : ak, *bbase = tl ? tail.gbase() : bk;
#pragma unroll
    for (int i = 0; i < P::A_PASSES; ++i)
      if (part < 0 || i % 3 == part) {
        const unsigned o_tile = (unsigned)min(i, ip) * a_pass_bytes, o_tail = tail.off(set, i);
        const unsigned t_tile = i < ip ? athr : athr_p, t_tail = tail.thr_of(set, i);
        r.a[i] = *reinterpret_cast<const u32x4 *>(abase + (tl ? o_tail : o_tile) + (tl ? t_tail : t_tile));
      }
#pragma unroll
    for (int i = 0; i < P::B_PASSES; ++i)
      if (part < 0 || (i + 1) % 3 == part) {
        const unsigned o_tile = (unsigned)i * b_pass_bytes, o_tail = tail.off(set, P::A_PASSES + i);
        const unsigned t_tail = tail.thr_of(set, P::A_PASSES + i);
        r.b[i] = *reinterpret_cast<const u32x4 *>(bbase + (tl ? o_tail : o_tile) + (tl ? t_tail : boff));
      }
  };
  const int a_st = a_r * T::A_PITCH + a_c * 16, b_st = T::A_BYTES + b_r * T::B_PITCH + b_c * 16;
  auto sstore_part = [&](char *st, const Stage &r, int part) {
#pragma unroll
    for (int i = 0; i < P::A_PASSES; ++i)
      if (part < 0 || i % 3 == part) *reinterpret_cast<u32x4 *>(st + a_st + i * P::A_RPP * T::A_PITCH) = r.a[i];
#pragma unroll
    for (int i = 0; i < P::B_PASSES; ++i)
      if (part < 0 || (i + 1) % 3 == part)
        *reinterpret_cast<u32x4 *>(st + b_st + i * P::B_RPP * T::B_PITCH) = r.b[i];
  };
  const int xoff = (wm * T::WM + (lane & 31)) * T::A_PITCH + (lane >> 5) * 16;
  const int woff = T::A_BYTES + ((lane >> 5) * 8 + ((lane & 15) >> 2)) * T::B_PITCH +
                   (wn * T::WN + ((lane >> 4) & 1) * 16 + (lane & 3) * 4) * 2;
  auto load_frags = [&](Frags &f, const char *st, int kk) {
#pragma unroll
    for (int tm = 0; tm < T::TM; ++tm)
      f.x[tm] = *reinterpret_cast<const bf16x8 *>(st + xoff + tm * 32 * T::A_PITCH + kk * 32);
#pragma unroll
    for (int tn = 0; tn < T::TN; ++tn) {
      const char *wp = st + woff + kk * 16 * T::B_PITCH + tn * 64;
      s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(wp));
      s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(wp + 4 * T::B_PITCH));
      s16x8 w8 = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
      f.w[tn] = __builtin_bit_cast(bf16x8, w8);
    }
  };
  auto mma = [&](const Frags &f) {
#pragma unroll
    for (int tn = 0; tn < T::TN; ++tn)
#pragma unroll
      for (int tm = 0; tm < T::TM; ++tm)
        acc[tn][tm] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.w[tn], f.x[tm], acc[tn][tm], 0, 0, 0);
  };
  constexpr int N_MFMA = T::TM * T::TN, N_FRAG = T::TM + 2 * T::TN;

  Stage &r0 = r_tail1, &r1 = r_tail0;   // tile t is staged in r(t & 1); the tail sets end up in r1, r0
  Frags f0, f1;
  gload_part(r0, 0, -1);
  gload_part(r1, 1, -1);
  sstore_part(smem, r0, -1);
  gload_part(r0, 2, -1);
  __syncthreads();
  load_frags(f0, smem, 0);
  __builtin_amdgcn_sched_barrier(0);

  // tile kt is in `cur`; `rw` holds tile kt+1 and is refilled with tile kt+3 (or a tail set)
  auto tile = [&](char *cur, char *nxt, Stage &rw, int kt) {
    load_frags(f1, cur, 1);
    sstore_part(nxt, rw, 0);
    mma(f0);
    deal_step<N_MFMA, N_FRAG, 6, 0>();
    load_frags(f0, cur, 2);
    sstore_part(nxt, rw, 1);
    gload_part(rw, kt + 3, 0);
    mma(f1);
    deal_step<N_MFMA, N_FRAG, 6, 6>();
    load_frags(f1, cur, 3);
    sstore_part(nxt, rw, 2);
    gload_part(rw, kt + 3, 1);
    mma(f0);
    deal_step<N_MFMA, N_FRAG, 4, 6>();
    // tile kt+1 is complete and every wave is done reading `cur` once all waves pass this barrier
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
    load_frags(f0, nxt, 0);
    gload_part(rw, kt + 3, 2);
    mma(f1);
    deal_step<N_MFMA, N_FRAG, 0, 4>();
  };
  char *s0 = smem, *s1 = smem + T::STAGE;
  for (int kt = 0; kt < nk; kt += 2) {
    tile(s0, s1, r1, kt);
    tile(s1, s0, r0, kt + 1);
  }
}

template <class T>
__device__ __forceinline__ void zero_acc(f32x16 (&acc)[T::TN][T::TM]) {
#pragma unroll
  for (int tn = 0; tn < T::TN; ++tn)
#pragma unroll
    for (int tm = 0; tm < T::TM; ++tm)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[tn][tm][r] = 0.f;
}

__device__ __forceinline__ bf16x4 pack4(float a, float b, float c, float d) {
  bf16x4 v;
  v[0] = (bf16)a; v[1] = (bf16)b; v[2] = (bf16)c; v[3] = (bf16)d;
  return v;
}

// Workgroup -> tile mapping.  Consecutive workgroup ids land on different XCDs (8 of them, each with
// its own L2), and an XCD works through its ids in order, about 32 workgroups at a time.  The tiles are
// put in one global order -- blocks of 8 row strips x 4 column tiles, row strip fastest inside a block,
// blocks column-panel by column-panel inside a band of 8 row strips, band after band -- and XCD x takes
// the x-th eighth of that order: the 32 workgroups that run together on an XCD then form one block,
// share 8 X strips and 4 weight strips (every operand slice fetched into the L2 is used 4 or 8 times),
// whatever the numbers of row strips and column tiles are.  Edge blocks are simply smaller.
__device__ __forceinline__ void tile_of_block(int ntn, int ntm, int &mt, int &nt) {
  constexpr int RB = 8, PW = 4;
  const int nblk = ntn * ntm, id = blockIdx.x, per = nblk / 8;
  const int pos = id < per * 8 ? (id % 8) * per + id / 8 : id;   // the last nblk % 8 tiles keep their place
  const int band = pos / (RB * ntn);
  int rem = pos - band * RB * ntn;
  const int h = min(RB, ntm - band * RB);      // row strips of this band
  const int panel = rem / (h * PW);
  rem -= panel * h * PW;
  mt = band * RB + rem % h;
  nt = panel * PW + rem / h;
}

// ---- epilogue of the 256 x 256 tile through LDS -------------------------------------------------
// In the accumulator layout a lane owns 4 consecutive columns of one row, so direct stores would be
// 8 bytes wide and scattered over 32 rows per instruction.  The tile is therefore rounded to bf16,
// parked in LDS in output layout (row pitch 528 bytes) and written out with 16-byte stores in which
// 32 consecutive lanes cover one 512-byte row segment.
constexpr int kOutPitch = 256 * 2 + 16;

template <class T>
__device__ __forceinline__ int out_lds_offset(int tm, int tn, int rq) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wn = wave % T::WGN, wm = wave / T::WGN;
  return (wm * T::WM + tm * 32 + (lane & 31)) * kOutPitch + (wn * T::WN + tn * 32 + rq * 8 + (lane >> 5) * 4) * 2;
}

template <class T>
__device__ __forceinline__ void tile_to_lds(const f32x16 (&acc)[T::TN][T::TM], char *smem) {
  static_assert(T::BM == 256 && T::BN == 256 && T::SMEM >= 256 * kOutPitch, "epilogue staging");
#pragma unroll
  for (int tm = 0; tm < T::TM; ++tm)
#pragma unroll
    for (int tn = 0; tn < T::TN; ++tn)
#pragma unroll
      for (int rq = 0; rq < 4; ++rq)
        *reinterpret_cast<bf16x4 *>(smem + out_lds_offset<T>(tm, tn, rq)) =
            pack4(acc[tn][tm][rq * 4], acc[tn][tm][rq * 4 + 1], acc[tn][tm][rq * 4 + 2], acc[tn][tm][rq * 4 + 3]);
}

// calls f(row, chunk, value) for every 16-byte chunk (8 columns) of the staged tile: 32 lanes per row
template <int NT = 256, class F>
__device__ __forceinline__ void for_each_out_chunk(const char *smem, F f) {
  constexpr int RPP = NT / 32;   // rows per pass
  const int r0 = threadIdx.x >> 5, ch = threadIdx.x & 31;
#pragma unroll 4
  for (int it = 0; it < 256 / RPP; ++it) {
    const int r = it * RPP + r0;
    f(r, ch, *reinterpret_cast<const u32x4 *>(smem + r * kOutPitch + ch * 16));
  }
}

// ------------------------------------------------------------------------------ projection
constexpr int kHeadDim = 128;   // the RoPE epilogue is compiled for d_h = 128

struct ProjArgs {
  const bf16 *x; int64_t lda; int M, K;
  const bf16 *w[4]; int width[4];     // W_Q, W_K, W_C, W_G and their output widths
  bf16 *dst[4];                       // Q, K, C, gate pre-activation  [M, width]
  const int32_t *seq_id, *pos;        // per packed token
  const float2 *rope; int max_len;    // (cos, sin)[pos][j], NULL = no RoPE
  int rope_by_token;                  // chunked prefill: the table has one row per packed token instead
  int dh;
  bf16 *kcache, *ccache; const int32_t *slots; int max_batch, max_seq;   // kcache NULL = no cache write
  PageMap pm;                                                             // contiguous or block-table rows
};

template <class T>
__global__ __launch_bounds__(T::NT) void proj_gemm_kernel(ProjArgs a) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  const int wtot = a.width[0] + a.width[1] + a.width[2] + a.width[3];
  int mt, nt;
  tile_of_block(wtot / T::BN, (a.M + T::BM - 1) / T::BM, mt, nt);
  int n_glob = nt * T::BN, seg = 0;
  while (n_glob >= a.width[seg]) { n_glob -= a.width[seg]; ++seg; }   // widths are multiples of BN
  const int m0 = mt * T::BM;
  f32x16 acc[T::TN][T::TM];
  zero_acc<T>(acc);
  // positions of this lane's rows: asked for before the main loop (a tile of Q or K rotates by them right
  // after it: 0.8 us of load latency per tile otherwise), not at all by the big tiles that do not rotate
  const bool rotate = a.rope != nullptr && seg < 2;
  constexpr bool kBig = T::TM == 4 && T::TN == 4;
  int pos_of[T::TM];
  if (rotate || !kBig) {
#pragma unroll
    for (int tm = 0; tm < T::TM; ++tm)
      pos_of[tm] = a.pos[min(m0 + (int)(threadIdx.x >> 6) / T::WGN * T::WM + tm * 32 + (int)(threadIdx.x & 31), a.M - 1)];
  }
  if constexpr (T::TM == 4 && T::TN == 4) {
    const int ldb = a.width[seg];
    const unsigned boff = (unsigned)((threadIdx.x / (T::BN / 8)) * ldb + (threadIdx.x % (T::BN / 8)) * 8) * 2u;
    PipeStage<T> t0, t1;
    gemm_mainloop_pipe<T>(a.x + (int64_t)m0 * a.lda, a.lda, a.M - m0, a.w[seg] + n_glob, boff, ldb, a.K, smem, acc, t0, t1,
                          NoTail{});
  } else {
    gemm_mainloop<T>(a.x, a.lda, a.M, m0, a.w[seg], a.width[seg], n_glob, a.K, smem, acc);
  }

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wn = wave % T::WGN, wm = wave / T::WGN;
  const int nw = n_glob + wn * T::WN;            // first column of this wave inside its segment
  const int half = a.dh / 2;
  bf16 *cache = seg == 1 ? a.kcache : (seg == 2 ? a.ccache : nullptr);
  const int width = a.width[seg];
  if constexpr (kBig) {
    if (rotate) {
      // wave tile = one head: column j pairs with j + d_h/2.  32 groups of 4 pairs per lane (4 row blocks x
      // 2 column blocks x 4 register quads); the table values of a group are asked for two groups ahead of
      // their use (one after the other, every group would wait out a whole memory round trip: 9 us per tile)
      constexpr int tiles_half = kHeadDim / 64;
      static_assert(T::TN == 2 * tiles_half, "a wave tile of the rotating segments is one head wide");
      constexpr int G = T::TM * tiles_half * 4, AHEAD = 2;
      bool rot[T::TM];
      const float2 *trow[T::TM];
#pragma unroll
      for (int tm = 0; tm < T::TM; ++tm) {
        const int m = m0 + wm * T::WM + tm * 32 + (lane & 31), p = pos_of[tm];
        rot[tm] = m < a.M && (a.rope_by_token || p < a.max_len);
        // rows that do not rotate read row 0 of the table and keep their values
        trow[tm] = a.rope + (int64_t)(rot[tm] ? (a.rope_by_token ? m : p) : 0) * half + (lane >> 5) * 4;
      }
      float4 tv[AHEAD + 1][2];
      auto ask = [&](int g) {
        const int tm = g / (tiles_half * 4), tn = (g / 4) % tiles_half, rq = g % 4;
        const float4 *tp = reinterpret_cast<const float4 *>(trow[tm] + tn * 32 + rq * 8);
        tv[g % (AHEAD + 1)][0] = tp[0]; tv[g % (AHEAD + 1)][1] = tp[1];
      };
#pragma unroll
      for (int g = 0; g < AHEAD; ++g) ask(g);
#pragma unroll
      for (int g = 0; g < G; ++g) {
        if (g + AHEAD < G) ask(g + AHEAD);
        const int tm = g / (tiles_half * 4), tn = (g / 4) % tiles_half, rq = g % 4, tn_hi = tn + tiles_half;
        const float4 t0 = tv[g % (AHEAD + 1)][0], t1 = tv[g % (AHEAD + 1)][1];
        const float cs[4] = {t0.x, t0.z, t1.x, t1.z}, sn[4] = {t0.y, t0.w, t1.y, t1.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const float lo = acc[tn][tm][rq * 4 + i], hi = acc[tn_hi][tm][rq * 4 + i];
          acc[tn][tm][rq * 4 + i] = rot[tm] ? lo * cs[i] - hi * sn[i] : lo;
          acc[tn_hi][tm][rq * 4 + i] = rot[tm] ? hi * cs[i] + lo * sn[i] : hi;
        }
      }
    }
  }
  if constexpr (!kBig)
#pragma unroll
  for (int tm = 0; tm < T::TM; ++tm) {
    const int m = m0 + wm * T::WM + tm * 32 + (lane & 31);
    if (m >= a.M) continue;
    const int p = pos_of[tm];
    const int rrow = a.rope_by_token ? m : p;   // RoPE table row
    if (rotate && (a.rope_by_token || p < a.max_len)) {
      // wave tile spans whole heads (WN % d_h == 0); pair column j with j + d_h/2 of the same head
      constexpr int tiles_half = kHeadDim / 64, tiles_head = kHeadDim / 32;
#pragma unroll
      for (int tn = 0; tn < T::TN; ++tn) {
        if ((tn % tiles_head) >= tiles_half) continue;
        const int tn_hi = tn + tiles_half;
        if (tn_hi >= T::TN) continue;
#pragma unroll
        for (int rq = 0; rq < 4; ++rq) {
          const int j = (tn % tiles_head) * 32 + rq * 8 + (lane >> 5) * 4;
          const float4 *tp = reinterpret_cast<const float4 *>(a.rope + (int64_t)rrow * half + j);
          const float4 t0 = tp[0], t1 = tp[1];
          const float cs[4] = {t0.x, t0.z, t1.x, t1.z}, sn[4] = {t0.y, t0.w, t1.y, t1.w};
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const float lo = acc[tn][tm][rq * 4 + i], hi = acc[tn_hi][tm][rq * 4 + i];
            acc[tn][tm][rq * 4 + i] = lo * cs[i] - hi * sn[i];
            acc[tn_hi][tm][rq * 4 + i] = hi * cs[i] + lo * sn[i];
          }
        }
      }
    }
    bf16 *drow = a.dst[seg] + (int64_t)m * width + nw;
    bf16 *crow = nullptr;
    if (cache) {
      const int b = a.seq_id[m];
      const int slot = a.slots ? a.slots[b] : b;
      if (slot >= 0 && slot < a.max_batch && p >= 0 && p < a.max_seq) {
        const int64_t cr = cache_row(a.pm, a.max_seq, slot, p);
        if (cr >= 0) crow = cache + cr * width + nw;
      }
    }
#pragma unroll
    for (int tn = 0; tn < T::TN; ++tn)
#pragma unroll
      for (int rq = 0; rq < 4; ++rq) {
        const int n = tn * 32 + rq * 8 + (lane >> 5) * 4;
        const bf16x4 v = pack4(acc[tn][tm][rq * 4], acc[tn][tm][rq * 4 + 1], acc[tn][tm][rq * 4 + 2], acc[tn][tm][rq * 4 + 3]);
        *reinterpret_cast<bf16x4 *>(drow + n) = v;
        if (crow) *reinterpret_cast<bf16x4 *>(crow + n) = v;
      }
  }
  if constexpr (T::TM == 4 && T::TN == 4) {
    __syncthreads();                 // every wave is done with the operand stages
    tile_to_lds<T>(acc, smem);
    // cache row of every tile row (or -1), looked up once and shared through LDS
    int64_t *crow_of = reinterpret_cast<int64_t *>(smem + 256 * kOutPitch);
    static_assert(T::SMEM >= 256 * kOutPitch + 256 * 8, "epilogue staging");
    if (cache) {
      const int m = m0 + (int)threadIdx.x;
      int64_t cr = -1;
      if (m < a.M) {
        const int p = a.pos[m], b = a.seq_id[m];
        const int slot = a.slots ? a.slots[b] : b;
        if (slot >= 0 && slot < a.max_batch && p >= 0 && p < a.max_seq) cr = cache_row(a.pm, a.max_seq, slot, p);
      }
      crow_of[threadIdx.x] = cr;
    }
    __syncthreads();
    bf16 *dst = a.dst[seg] + n_glob;
    for_each_out_chunk(smem, [&](int r, int ch, u32x4 v) {
      const int m = m0 + r;
      if (m >= a.M) return;
      *reinterpret_cast<u32x4 *>(dst + (int64_t)m * width + ch * 8) = v;
      if (cache) {
        const int64_t cr = crow_of[r];
        if (cr >= 0) *reinterpret_cast<u32x4 *>(cache + cr * width + n_glob + ch * 8) = v;
      }
    });
  }
}

// ---- projection against packed weights -----------------------------------------------------------
// The four weight matrices are first copied side by side into one [H, Wtot] matrix, so that a
// 256-column tile may straddle Q | K | C | gate: this serves output widths that are multiples of 64
// but not of 256 (heads of 64, a single shared key).  Columns are routed to their outputs per
// 64-column group for RoPE (a head never straddles a group) and per 16-byte chunk for the stores.
// The packed row is padded with zero columns to a multiple of 256 (wpad); the last tile computes
// them and stores nothing for them.
__global__ void pack_weights_kernel(ProjArgs a, int wtot, int wpad, bf16 *dst) {
  const int cpr = wpad / 8;   // 16-byte chunks per packed row
  const int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
  if (i >= (int64_t)a.K * cpr) return;
  const int k = (int)(i / cpr);
  int col = (int)(i % cpr) * 8, seg = 0;
  u32x4 v = {0u, 0u, 0u, 0u};
  if (col < wtot) {
    while (col >= a.width[seg]) { col -= a.width[seg]; ++seg; }
    v = *reinterpret_cast<const u32x4 *>(a.w[seg] + (int64_t)k * a.width[seg] + col);
  }
  *reinterpret_cast<u32x4 *>(dst + i * 8) = v;
}

template <class T, int DH>
__global__ __launch_bounds__(T::NT) void proj_packed_kernel(ProjArgs a, const bf16 *wpack, int wpad) {
  static_assert(T::TM == 4 && T::TN == 4 && (DH == 64 || DH == 128), "tile");
  extern __shared__ __attribute__((aligned(16))) char smem[];
  const int b1 = a.width[0], b2 = b1 + a.width[1], b3 = b2 + a.width[2], wtot = b3 + a.width[3];
  int mt, nt;
  tile_of_block(wpad / T::BN, (a.M + T::BM - 1) / T::BM, mt, nt);
  const int m0 = mt * T::BM, n0 = nt * T::BN;
  f32x16 acc[T::TN][T::TM];
  zero_acc<T>(acc);
  {
    const unsigned boff = (unsigned)((threadIdx.x / (T::BN / 8)) * wpad + (threadIdx.x % (T::BN / 8)) * 8) * 2u;
    PipeStage<T> t0, t1;
    gemm_mainloop_pipe<T>(a.x + (int64_t)m0 * a.lda, a.lda, a.M - m0, wpack + n0, boff, wpad, a.K, smem, acc, t0, t1,
                          NoTail{});
  }
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wn = wave % T::WGN, wm = wave / T::WGN;
  if (a.rope && n0 < b2) {   // the tile holds q or k columns
    constexpr int half = DH / 2, tiles_half = DH / 64, tiles_head = DH / 32;
#pragma unroll
    for (int tm = 0; tm < T::TM; ++tm) {
      const int m = m0 + wm * T::WM + tm * 32 + (lane & 31);
      const int p = a.rope_by_token ? min(m, a.M - 1) : max(min(a.pos[min(m, a.M - 1)], a.max_len - 1), 0);   // RoPE table row
#pragma unroll
      for (int tn = 0; tn < T::TN; ++tn) {
        if ((tn % tiles_head) >= tiles_half) continue;
        const int tn_hi = tn + tiles_half;
        if (tn_hi >= T::TN) continue;
        // latent and gate columns of a straddling tile take the identity rotation (no branch: the
        // accumulators stay where they are)
        const bool rot = n0 + wn * T::WN + tn * 32 < b2;
#pragma unroll
        for (int rq = 0; rq < 4; ++rq) {
          const int j = (tn % tiles_head) * 32 + rq * 8 + (lane >> 5) * 4;
          const float4 *tp = reinterpret_cast<const float4 *>(a.rope + (int64_t)p * half + j);
          const float4 t0 = tp[0], t1 = tp[1];
          const float cs[4] = {t0.x, t0.z, t1.x, t1.z}, sn[4] = {t0.y, t0.w, t1.y, t1.w};
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const float c = rot ? cs[i] : 1.f, sv = rot ? sn[i] : 0.f;
            const float lo = acc[tn][tm][rq * 4 + i], hi = acc[tn_hi][tm][rq * 4 + i];
            acc[tn][tm][rq * 4 + i] = lo * c - hi * sv;
            acc[tn_hi][tm][rq * 4 + i] = hi * c + lo * sv;
          }
        }
      }
    }
  }
  __syncthreads();                 // every wave is done with the operand stages
  tile_to_lds<T>(acc, smem);
  int64_t *crow_of = reinterpret_cast<int64_t *>(smem + 256 * kOutPitch);
  if (a.kcache) {
    const int m = m0 + (int)threadIdx.x;
    int64_t cr = -1;
    if (m < a.M) {
      const int p = a.pos[m], b = a.seq_id[m];
      const int slot = a.slots ? a.slots[b] : b;
      if (slot >= 0 && slot < a.max_batch && p >= 0 && p < a.max_seq) cr = cache_row(a.pm, a.max_seq, slot, p);
    }
    crow_of[threadIdx.x] = cr;
  }
  __syncthreads();
  // a thread stores the same 16-byte chunk column of every row: its destination is fixed
  const int gcol = n0 + (threadIdx.x & 31) * 8;
  if (gcol >= wtot) return;        // zero padding of the packed row; no barrier follows
  const int seg = (gcol >= b1) + (gcol >= b2) + (gcol >= b3);
  const int lcol = gcol - (seg == 0 ? 0 : seg == 1 ? b1 : seg == 2 ? b2 : b3);
  const int width = a.width[seg];
  bf16 *dst = a.dst[seg] + lcol;
  bf16 *cache = !a.kcache ? nullptr : seg == 1 ? a.kcache + lcol : seg == 2 ? a.ccache + lcol : nullptr;
  for_each_out_chunk(smem, [&](int r, int, u32x4 v) {
    const int m = m0 + r;
    if (m >= a.M) return;
    *reinterpret_cast<u32x4 *>(dst + (int64_t)m * width) = v;
    if (cache) {
      const int64_t cr = crow_of[r];
      if (cr >= 0) *reinterpret_cast<u32x4 *>(cache + cr * width) = v;
    }
  });
}

// ------------------------------------------------------------------------------ value decoder
struct DecoderArgs {
  const bf16 *L; int64_t ldl; int M;          // [M, n_q*d_l] normalised group outputs
  const bf16 *wp; int dl, dh, hpq, nh;        // [n_h, d_l, d_h]
  const bf16 *g; int gate;                    // [M, n_h*d_h] gate pre-activation
  bf16 *out;                                  // [M, n_h*d_h]
};

template <class T>
__global__ __launch_bounds__(T::NT) void decoder_gemm_kernel(DecoderArgs a) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  const int tiles_per_head = a.dh / T::BN;     // BN divides d_h
  int mt, nt;
  tile_of_block(a.nh * tiles_per_head, (a.M + T::BM - 1) / T::BM, mt, nt);
  const int head = nt / tiles_per_head, n_in_head = (nt % tiles_per_head) * T::BN;
  const int m0 = mt * T::BM;
  f32x16 acc[T::TN][T::TM];
  zero_acc<T>(acc);
  gemm_mainloop<T>(a.L + (head / a.hpq) * a.dl, a.ldl, a.M, m0, a.wp + (int64_t)head * a.dl * a.dh, a.dh, n_in_head,
                   a.dl, smem, acc);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wn = wave % T::WGN, wm = wave / T::WGN;
  const int64_t ldo = (int64_t)a.nh * a.dh;
  const int col0 = head * a.dh + n_in_head + wn * T::WN;
#pragma unroll
  for (int tm = 0; tm < T::TM; ++tm) {
    const int m = m0 + wm * T::WM + tm * 32 + (lane & 31);
    if (m >= a.M) continue;
#pragma unroll
    for (int tn = 0; tn < T::TN; ++tn)
#pragma unroll
      for (int rq = 0; rq < 4; ++rq) {
        const int64_t o = (int64_t)m * ldo + col0 + tn * 32 + rq * 8 + (lane >> 5) * 4;
        float v[4] = {acc[tn][tm][rq * 4], acc[tn][tm][rq * 4 + 1], acc[tn][tm][rq * 4 + 2], acc[tn][tm][rq * 4 + 3]};
        if (a.gate) {
          const bf16x4 gz = *reinterpret_cast<const bf16x4 *>(a.g + o);
#pragma unroll
          for (int i = 0; i < 4; ++i)
            v[i] *= a.gate == kGateSigmoid ? 1.0f / (1.0f + __expf(-(float)gz[i])) : gate_factor(a.gate, (float)gz[i]);
        }
        *reinterpret_cast<bf16x4 *>(a.out + o) = pack4(v[0], v[1], v[2], v[3]);
      }
  }
}

// tail prefetch of the decoder: chunk (set*16 + i) of a thread is row (set*16 + i)*8 + tid/32 of the
// gate tile (rows past the end of the matrix re-read the last valid one)
struct GateTail {
  static constexpr bool active = true;
  const char *base; unsigned pass_bytes, thr, thr_p; int ip;   // ip: last 8-row pass with a valid row
  __device__ const char *gbase() const { return base; }
  __device__ unsigned off(int set, int i) const { return (unsigned)min(set * 16 + i, ip) * pass_bytes; }
  __device__ unsigned thr_of(int set, int i) const { return set * 16 + i < ip ? thr : thr_p; }
};

// Two heads of one map group per 256-wide tile (they share the row operand L_g), pipelined main
// loop.  The gate is applied to the fp32 accumulators: the gate tile is fetched with coalesced
// 16-byte loads into LDS in output layout, every lane reads the pre-activations of its own
// elements from there and puts the gated, rounded result back in the same place.
template <class T, bool GATE>
__global__ __launch_bounds__(T::NT) void decoder_pair_kernel(DecoderArgs a) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  int mt, nt;
  tile_of_block(a.nh / 2, (a.M + T::BM - 1) / T::BM, mt, nt);
  const int head = nt * 2, m0 = mt * T::BM;
  f32x16 acc[T::TN][T::TM];
  zero_acc<T>(acc);
  const int64_t ldo = (int64_t)a.nh * a.dh;
  const int col0 = head * a.dh;
  // the gate tile (32 chunks of 16 bytes per thread: rows it*8 + tid/32, chunk tid%32) is fetched by
  // the main loop's tail prefetch while the last two k-tiles are multiplied
  const int r0 = threadIdx.x >> 5, ch = threadIdx.x & 31;
  const int rows_valid = a.M - m0;
  // pass `it` covers rows it*8 + tid/32; rows past the last valid one are clamped to it (their outputs
  // are not stored)
  const int rv = min(rows_valid, T::BM);
  GateTail gate_tail;
  gate_tail.base = reinterpret_cast<const char *>(a.g + (int64_t)m0 * ldo + col0);
  gate_tail.pass_bytes = (unsigned)(8 * ldo * 2);
  gate_tail.ip = (rv - 1) / 8;
  gate_tail.thr = (unsigned)(r0 * ldo + ch * 8) * 2u;
  gate_tail.thr_p = (unsigned)(min(r0, (rv - 1) % 8) * ldo + ch * 8) * 2u;
  PipeStage<T> g0, g1;
  {
    const int b_c = threadIdx.x % (T::BN / 8), b_r = threadIdx.x / (T::BN / 8);
    const int col = b_c * 8;   // columns [0,128) belong to `head`, [128,256) to `head + 1`
    const unsigned boff = (unsigned)((col / 128) * a.dl * a.dh + b_r * a.dh + col % 128) * 2u;
    const bf16 *Ab = a.L + (int64_t)m0 * a.ldl + (head / a.hpq) * a.dl, *Bb = a.wp + (int64_t)head * a.dl * a.dh;
    if constexpr (GATE) gemm_mainloop_pipe<T>(Ab, a.ldl, rows_valid, Bb, boff, a.dh, a.dl, smem, acc, g0, g1, gate_tail);
    else gemm_mainloop_pipe<T>(Ab, a.ldl, rows_valid, Bb, boff, a.dh, a.dl, smem, acc, g0, g1, NoTail{});
  }
  __syncthreads();
  if constexpr (GATE) {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      *reinterpret_cast<u32x4 *>(smem + ((i) * 8 + r0) * kOutPitch + ch * 16) = g0.a[i];
      *reinterpret_cast<u32x4 *>(smem + ((8 + i) * 8 + r0) * kOutPitch + ch * 16) = g0.b[i];
      *reinterpret_cast<u32x4 *>(smem + ((16 + i) * 8 + r0) * kOutPitch + ch * 16) = g1.a[i];
      *reinterpret_cast<u32x4 *>(smem + ((24 + i) * 8 + r0) * kOutPitch + ch * 16) = g1.b[i];
    }
    __syncthreads();
  }
  // one row block (tm) at a time: all 16 gate reads of the block are issued before the first is used
  // the Sigmoid of the method takes the short path; the other nonlinearities a general one
  auto gate_rows = [&](auto sig_tag) {
    constexpr bool SIG = decltype(sig_tag)::value;
  #pragma unroll
    for (int tm = 0; tm < T::TM; ++tm) {
      bf16x4 gz[T::TN][4];
      if constexpr (GATE) {
  #pragma unroll
        for (int tn = 0; tn < T::TN; ++tn)
  #pragma unroll
          for (int rq = 0; rq < 4; ++rq) gz[tn][rq] = *reinterpret_cast<const bf16x4 *>(smem + out_lds_offset<T>(tm, tn, rq));
      }
  #pragma unroll
      for (int tn = 0; tn < T::TN; ++tn)
  #pragma unroll
        for (int rq = 0; rq < 4; ++rq) {
          float v[4] = {acc[tn][tm][rq * 4], acc[tn][tm][rq * 4 + 1], acc[tn][tm][rq * 4 + 2], acc[tn][tm][rq * 4 + 3]};
          if constexpr (GATE) {
  #pragma unroll
            for (int i = 0; i < 4; ++i)
              v[i] *= SIG ? __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-1.4426950408889634f * (float)gz[tn][rq][i]))
                          : gate_factor(a.gate, (float)gz[tn][rq][i]);
          }
          *reinterpret_cast<bf16x4 *>(smem + out_lds_offset<T>(tm, tn, rq)) = pack4(v[0], v[1], v[2], v[3]);
        }
    }
  };
  if (!GATE || a.gate == kGateSigmoid) gate_rows(std::true_type{});
  else gate_rows(std::false_type{});
  __syncthreads();
  for_each_out_chunk(smem, [&](int r, int ch, u32x4 v) {
    if (m0 + r < a.M) *reinterpret_cast<u32x4 *>(a.out + (int64_t)(m0 + r) * ldo + col0 + ch * 8) = v;
  });
}

// All 256 / d_h heads of one 256-wide tile share the row operand L_g (they lie in one map group);
// short contraction (d_l of 64 .. 192, or any multiple of 64): plain main loop.  The gate tile is
// fetched with coalesced 16-byte loads before the main loop starts and applied as above.
template <class T, bool GATE>
__global__ __launch_bounds__(T::NT) void decoder_multi_kernel(DecoderArgs a) {
  static_assert(T::BM == 256 && T::BN == 256 && T::NT == 256, "tile");
  extern __shared__ __attribute__((aligned(16))) char smem[];
  const int hpt = T::BN / a.dh;   // heads per tile
  int mt, nt;
  tile_of_block(a.nh / hpt, (a.M + T::BM - 1) / T::BM, mt, nt);
  const int head = nt * hpt, m0 = mt * T::BM;
  f32x16 acc[T::TN][T::TM];
  zero_acc<T>(acc);
  const int64_t ldo = (int64_t)a.nh * a.dh;
  const int col0 = head * a.dh;
  const int r0 = threadIdx.x >> 5, ch = threadIdx.x & 31;
  u32x4 gt[32];
  if constexpr (GATE) {
    const bf16 *gp = a.g + col0 + ch * 8;
#pragma unroll
    for (int it = 0; it < 32; ++it)
      gt[it] = *reinterpret_cast<const u32x4 *>(gp + (int64_t)min(m0 + it * 8 + r0, a.M - 1) * ldo);
  }
  {
    // column chunk -> head of the tile: the loop adds (chunk column) to the pointer it is given
    const int col = (threadIdx.x % (T::BN / 8)) * 8;
    const bf16 *Bt = a.wp + (int64_t)head * a.dl * a.dh + (int64_t)(col / a.dh) * a.dl * a.dh + (col % a.dh) - col;
    gemm_mainloop<T>(a.L + (head / a.hpq) * a.dl, a.ldl, a.M, m0, Bt, a.dh, 0, a.dl, smem, acc);
  }
  if constexpr (GATE) {
#pragma unroll
    for (int it = 0; it < 32; ++it) *reinterpret_cast<u32x4 *>(smem + (it * 8 + r0) * kOutPitch + ch * 16) = gt[it];
    __syncthreads();
  }
  // the Sigmoid of the method takes the short path; the other nonlinearities a general one
  auto gate_rows = [&](auto sig_tag) {
    constexpr bool SIG = decltype(sig_tag)::value;
  #pragma unroll
    for (int tm = 0; tm < T::TM; ++tm) {
      bf16x4 gz[T::TN][4];
      if constexpr (GATE) {
  #pragma unroll
        for (int tn = 0; tn < T::TN; ++tn)
  #pragma unroll
          for (int rq = 0; rq < 4; ++rq) gz[tn][rq] = *reinterpret_cast<const bf16x4 *>(smem + out_lds_offset<T>(tm, tn, rq));
      }
  #pragma unroll
      for (int tn = 0; tn < T::TN; ++tn)
  #pragma unroll
        for (int rq = 0; rq < 4; ++rq) {
          float v[4] = {acc[tn][tm][rq * 4], acc[tn][tm][rq * 4 + 1], acc[tn][tm][rq * 4 + 2], acc[tn][tm][rq * 4 + 3]};
          if constexpr (GATE) {
  #pragma unroll
            for (int i = 0; i < 4; ++i)
              v[i] *= SIG ? __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-1.4426950408889634f * (float)gz[tn][rq][i]))
                          : gate_factor(a.gate, (float)gz[tn][rq][i]);
          }
          *reinterpret_cast<bf16x4 *>(smem + out_lds_offset<T>(tm, tn, rq)) = pack4(v[0], v[1], v[2], v[3]);
        }
    }
  };
  if (!GATE || a.gate == kGateSigmoid) gate_rows(std::true_type{});
  else gate_rows(std::false_type{});
  __syncthreads();
  for_each_out_chunk(smem, [&](int r, int ch, u32x4 v) {
    if (m0 + r < a.M) *reinterpret_cast<u32x4 *>(a.out + (int64_t)(m0 + r) * ldo + col0 + ch * 8) = v;
  });
}

// ------------------------------------------------------------------------------ plain GEMM
struct PlainArgs { const bf16 *A; int64_t lda; int M, N, K; const bf16 *B; bf16 *C; };

template <class T>
__global__ __launch_bounds__(T::NT) void plain_gemm_kernel(PlainArgs a) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  int mt, nt;
  tile_of_block(a.N / T::BN, (a.M + T::BM - 1) / T::BM, mt, nt);
  const int m0 = mt * T::BM, n0 = nt * T::BN;
  f32x16 acc[T::TN][T::TM];
  zero_acc<T>(acc);
  if constexpr (T::BM == 256 && T::BN == 256) {
    const unsigned boff = (unsigned)((threadIdx.x / (T::BN / 8)) * a.N + (threadIdx.x % (T::BN / 8)) * 8) * 2u;
    PipeStage<T> t0, t1;
    gemm_mainloop_pipe<T>(a.A + (int64_t)m0 * a.lda, a.lda, a.M - m0, a.B + n0, boff, a.N, a.K, smem, acc, t0, t1, NoTail{});
  } else {
    gemm_mainloop<T>(a.A, a.lda, a.M, m0, a.B, a.N, n0, a.K, smem, acc);
  }
  if constexpr (T::BM == 256 && T::BN == 256) {
    __syncthreads();
    tile_to_lds<T>(acc, smem);
    __syncthreads();
    for_each_out_chunk<T::NT>(smem, [&](int r, int ch, u32x4 v) {
      if (m0 + r < a.M) *reinterpret_cast<u32x4 *>(a.C + (int64_t)(m0 + r) * a.N + n0 + ch * 8) = v;
    });
    return;
  }
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wn = wave % T::WGN, wm = wave / T::WGN;
#pragma unroll
  for (int tm = 0; tm < T::TM; ++tm) {
    const int m = m0 + wm * T::WM + tm * 32 + (lane & 31);
    if (m >= a.M) continue;
#pragma unroll
    for (int tn = 0; tn < T::TN; ++tn)
#pragma unroll
      for (int rq = 0; rq < 4; ++rq) {
        const int n = n0 + wn * T::WN + tn * 32 + rq * 8 + (lane >> 5) * 4;
        *reinterpret_cast<bf16x4 *>(a.C + (int64_t)m * a.N + n) =
            pack4(acc[tn][tm][rq * 4], acc[tn][tm][rq * 4 + 1], acc[tn][tm][rq * 4 + 2], acc[tn][tm][rq * 4 + 3]);
      }
  }
}

// ------------------------------------------------------------------------------ decode projection
// Few rows (one new token per sequence) against all four weight matrices: weight-streaming bound.
// Split-K over H so that several hundred workgroups pull on HBM at once; every (k-split, n-tile)
// writes an fp32 partial that the finalize kernel sums before RoPE / cache append.
struct SkinnyArgs {
  const bf16 *x; int64_t lda; int M, K;
  const bf16 *w[4]; int width[4];
  float *part;            // [ksplit, M, wtot]
  int ksplit, wtot;
};

template <class T>
__global__ __launch_bounds__(T::NT) void skinny_proj_kernel(SkinnyArgs a) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  const int ntn = a.wtot / T::BN, ntm = (a.M + T::BM - 1) / T::BM;
  const int ks = blockIdx.x / (ntn * ntm), rem = blockIdx.x % (ntn * ntm);
  const int mt = rem / ntn, nt = rem % ntn;
  int n_seg = nt * T::BN, seg = 0;
  while (n_seg >= a.width[seg]) { n_seg -= a.width[seg]; ++seg; }
  const int m0 = mt * T::BM, klen = a.K / a.ksplit, k0 = ks * klen;
  f32x16 acc[T::TN][T::TM];
  zero_acc<T>(acc);
  gemm_mainloop<T>(a.x + k0, a.lda, a.M, m0, a.w[seg] + (int64_t)k0 * a.width[seg], a.width[seg], n_seg, klen, smem, acc);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wn = wave % T::WGN, wm = wave / T::WGN;
  float *prow = a.part + (int64_t)ks * a.M * a.wtot;
#pragma unroll
  for (int tm = 0; tm < T::TM; ++tm) {
    const int m = m0 + wm * T::WM + tm * 32 + (lane & 31);
    if (m >= a.M) continue;
#pragma unroll
    for (int tn = 0; tn < T::TN; ++tn)
#pragma unroll
      for (int rq = 0; rq < 4; ++rq) {
        const int n = nt * T::BN + wn * T::WN + tn * 32 + rq * 8 + (lane >> 5) * 4;
        *reinterpret_cast<float4 *>(prow + (int64_t)m * a.wtot + n) =
            make_float4(acc[tn][tm][rq * 4], acc[tn][tm][rq * 4 + 1], acc[tn][tm][rq * 4 + 2], acc[tn][tm][rq * 4 + 3]);
      }
  }
}

// Short prefill (few hundred tokens): the 256 x 256 tiles would leave most CUs idle, so the projection
// runs as the split-K kernel above and this kernel finishes it: sums the partials, rotates q and k
// (App. B.1.1), rounds to bf16 and stores Q | K | C | gate rows and the cache rows (App. B.1.3).
// One thread per (token, 8 columns); a chunk never straddles the two halves of a head.
__global__ __launch_bounds__(256) void proj_small_finalize_kernel(ProjArgs a, const float *__restrict__ part, int ks) {
  const int b1 = a.width[0], b2 = b1 + a.width[1], b3 = b2 + a.width[2], wtot = b3 + a.width[3];
  const int cpr = wtot / 8;
  const int64_t idx = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
  if (idx >= (int64_t)a.M * cpr) return;
  const int m = (int)(idx / cpr), gcol = (int)(idx % cpr) * 8;
  const int seg = (gcol >= b1) + (gcol >= b2) + (gcol >= b3);
  const int lcol = gcol - (seg == 0 ? 0 : seg == 1 ? b1 : seg == 2 ? b2 : b3);
  const int64_t pstride = (int64_t)a.M * wtot;
  auto sum8 = [&](int col, float (&v)[8]) {
    const float *p = part + (int64_t)m * wtot + col;
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] = 0.f;
    for (int s = 0; s < ks; ++s) {
      const float4 x0 = *reinterpret_cast<const float4 *>(p + s * pstride), x1 = *reinterpret_cast<const float4 *>(p + s * pstride + 4);
      v[0] += x0.x; v[1] += x0.y; v[2] += x0.z; v[3] += x0.w; v[4] += x1.x; v[5] += x1.y; v[6] += x1.z; v[7] += x1.w;
    }
  };
  float v[8];
  sum8(gcol, v);
  const int p = a.pos[m];
  if (a.rope && seg < 2) {
    const int half = a.dh / 2, e = lcol % a.dh, lo = e < half;
    float o[8];
    sum8(lo ? gcol + half : gcol - half, o);
    const int row = a.rope_by_token ? m : max(min(p, a.max_len - 1), 0);
    const float2 *t = a.rope + (int64_t)row * half + e % half;
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] = lo ? v[i] * t[i].x - o[i] * t[i].y : v[i] * t[i].x + o[i] * t[i].y;
  }
  u32x4 w;
  {
    const bf16x4 a0 = pack4(v[0], v[1], v[2], v[3]), a1 = pack4(v[4], v[5], v[6], v[7]);
    typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
    const u32x2 r0 = __builtin_bit_cast(u32x2, a0);
    const u32x2 r1 = __builtin_bit_cast(u32x2, a1);
    w = u32x4{r0[0], r0[1], r1[0], r1[1]};
  }
  const int width = a.width[seg];
  *reinterpret_cast<u32x4 *>(a.dst[seg] + (int64_t)m * width + lcol) = w;
  if (a.kcache && (seg == 1 || seg == 2)) {
    const int b = a.seq_id[m];
    const int slot = a.slots ? a.slots[b] : b;
    if (slot >= 0 && slot < a.max_batch && p >= 0 && p < a.max_seq) {
      const int64_t cr = cache_row(a.pm, a.max_seq, slot, p);
      if (cr >= 0) *reinterpret_cast<u32x4 *>((seg == 1 ? a.kcache : a.ccache) + cr * width + lcol) = w;
    }
  }
}

typedef GemmTile<32, 128, 64, 1, 4> TileSkinny32;
typedef GemmTile<64, 128, 64, 1, 4> TileSkinny64;
typedef GemmTile<32, 64, 64, 1, 2> TileSkinny32N64;   // 64-wide tiles for widths that are not multiples of 128
typedef GemmTile<64, 64, 64, 2, 2> TileSkinny64N64;
typedef GemmTile<32, 32, 64, 1, 1> TileSkinny32N32;    // one wave per tile: the output projection of a decode step

typedef GemmTile<256, 256, 64, 2, 2> TileBig;    // wave tile 128 x 128
typedef GemmTile<256, 128, 64, 4, 1> TileHead;   // one 128-wide head per workgroup, wave tile 64(m) x 128(n)
typedef GemmTile<256, 64, 64, 4, 1> TileHead64;  // one 64-wide head per workgroup, wave tile 64(m) x 64(n)

template <class T, class K, class Args>
void launch(K kernel, const Args &a, int ntiles, hipStream_t st) {
  allow_dynamic_lds((const void *)kernel, T::SMEM);
  kernel<<<ntiles, T::NT, T::SMEM, st>>>(a);
}

}  // namespace

// The pipelined 256 x 256 tile against packed weights: widths in units of a 64-column group that
// holds whole heads, an even number (>= 4) of k-tiles.
static bool proj_packed_ok(const Dims &d) {
  if (d.dh != 64 && d.dh != 128) return false;
  if (d.wq_w % d.dh || d.wk_w % d.dh || d.wc_w % 64 || d.wg_w % 64 || d.wq_w % 64 || d.wk_w % 64) return false;
  if (d.dh == 128 && (d.wq_w % 128 || d.wk_w % 128 || d.wc_w % 128)) return false;   // head inside one wave tile
  return d.H % 128 == 0 && d.H >= 256;
}
static int proj_packed_width(const Dims &d) { return (d.wtot + 255) / 256 * 256; }
static bool proj_direct_ok(const Dims &d) {
  // RoPE pairing is lane-local only if a wave tile (128 columns) holds whole heads
  if (d.dh != 128) return false;
  return !(d.H % 64 || d.dl % 64 || d.wq_w % 128 || d.wk_w % 128 || d.wc_w % 128 || d.wg_w % 128);
}
static bool proj_direct_big(const Dims &d) {
  // the pipelined loop takes an even number (>= 4) of k-tiles
  return proj_direct_ok(d) && !(d.wq_w % 256 || d.wk_w % 256 || d.wc_w % 256 || d.wg_w % 256) && d.H % 128 == 0 && d.H >= 256;
}

bool gemm_shapes_supported(const Dims &d) {
  if (d.dtype != GTA_BF16) return false;
  if (d.H % 128) return false;   // H is also the output width of the W_O GEMM, tiled in 128 columns
  if (!proj_direct_ok(d) && !proj_packed_ok(d)) return false;
  if (d.dl % 64) return false;
  // row offsets inside a 256-row tile are kept in 32 bits
  if (d.H > (1 << 20) || (int64_t)d.nq * d.dl > (1 << 20) || d.wg_w > (1 << 20)) return false;
  return true;
}

size_t proj_packed_bytes(const Dims &d) {
  return d.dtype == GTA_BF16 && !proj_direct_big(d) && proj_packed_ok(d) ? (size_t)d.H * proj_packed_width(d) * 2 : 0;
}

static bool skinny_wide_tiles(const Dims &d);

// Short prefill: split-K projection on 64-row tiles plus a finalize kernel, as long as the 256-row tiles
// would fill at most half of the CUs (and up to 4096 tokens).  Measured, whole calls: 1B shape (20 column
// tiles) 1280 tokens 125 us against 147 us, 1536 tokens 140 against 158, 3072 tokens 244 against 220;
// the paper's layer (7 column tiles) 2048 tokens 110 against 127, 4096 tokens equal; the 8 x 128 + 1024
// shape (28 column tiles) 1500 tokens 256 against 216; the projection alone at the 1B shape: 128 tokens
// 11 us against 55 us, 1024 tokens 34 against 61.
static int proj_small_max_tokens(const Dims &d) {
  const int col_tiles = (d.wtot + 255) / 256;
  const int m = 128 / col_tiles * 256;
  return m < 4096 ? m : 4096;
}

int proj_small_ksplit(const Dims &d, int64_t M) {
  if (!gemm_shapes_supported(d) || M <= 0 || M > proj_small_max_tokens(d)) return 0;
  return skinny_ksplit(d, (int)M);
}

// Rows of fp32 partials [ksplit * M, W_tot] the short path needs at most, whatever M is:
// ksplit <= 768 / tiles + 1 with tiles = n_tiles * ceil(M / 64).
size_t proj_small_rows_bound(const Dims &d) {
  if (!gemm_shapes_supported(d)) return 0;
  const int ntn = d.wtot / (skinny_wide_tiles(d) ? 128 : 64);
  return (size_t)(768 * 64 / ntn + proj_small_max_tokens(d));
}

void launch_proj_gemm(const Dims &d, const gta_weights &w, const void *x, int M, const PrefillWs &ws,
                      const gta_cache *cache, const int32_t *slots, int max_len, hipStream_t st, bool rope_by_token) {
  ProjArgs a{};
  a.rope_by_token = rope_by_token ? 1 : 0;
  a.x = (const bf16 *)x; a.lda = d.H; a.M = M; a.K = d.H;
  const void *wm[4] = {w.wq, w.wk, w.wc, w.wg};
  const int wd[4] = {d.wq_w, d.wk_w, d.wc_w, d.wg_w};
  void *dst[4] = {ws.q, ws.k, ws.c, ws.g};
  for (int i = 0; i < 4; ++i) { a.w[i] = (const bf16 *)wm[i]; a.width[i] = wd[i]; a.dst[i] = (bf16 *)dst[i]; }
  a.seq_id = ws.seq_id; a.pos = ws.pos;
  a.rope = d.rope ? ws.rope : nullptr; a.max_len = max_len; a.dh = d.dh;
  if (cache) {
    a.kcache = (bf16 *)cache->k; a.ccache = (bf16 *)cache->c; a.slots = slots;
    a.max_batch = cache->max_batch; a.max_seq = cache->max_seq;
    a.pm = page_map_of(*cache);
  }
  if (const int ks = proj_small_ksplit(d, M)) {
    launch_skinny_proj(d, w, x, M, ws.praw, ks, st);
    const int64_t chunks = (int64_t)M * (d.wtot / 8);
    proj_small_finalize_kernel<<<(unsigned)((chunks + 255) / 256), 256, 0, st>>>(a, ws.praw, ks);
    return;
  }
  if (proj_direct_big(d)) {
    const int nt = (d.wtot / 256) * ((M + 255) / 256);
    launch<TileBig>(proj_gemm_kernel<TileBig>, a, nt, st);
  } else if (proj_packed_ok(d)) {
    bf16 *wpack = (bf16 *)ws.wpack;
    const int wpad = proj_packed_width(d);
    const int64_t chunks = (int64_t)d.H * (wpad / 8);
    pack_weights_kernel<<<(unsigned)((chunks + 255) / 256), 256, 0, st>>>(a, d.wtot, wpad, wpack);
    const int nt = (wpad / 256) * ((M + 255) / 256);
    const int which = d.dh == 64 ? 0 : 1;
    allow_dynamic_lds(which == 0 ? (const void *)proj_packed_kernel<TileBig, 64> : (const void *)proj_packed_kernel<TileBig, 128>,
                      TileBig::SMEM);
    if (which == 0) proj_packed_kernel<TileBig, 64><<<nt, TileBig::NT, TileBig::SMEM, st>>>(a, wpack, wpad);
    else proj_packed_kernel<TileBig, 128><<<nt, TileBig::NT, TileBig::SMEM, st>>>(a, wpack, wpad);
  } else {
    const int nt = (d.wtot / 128) * ((M + 255) / 256);
    launch<TileHead>(proj_gemm_kernel<TileHead>, a, nt, st);
  }
}

static bool skinny_wide_tiles(const Dims &d) { return !(d.wq_w % 128 || d.wk_w % 128 || d.wc_w % 128 || d.wg_w % 128); }

int skinny_ksplit(const Dims &d, int M) {
  const int ktiles = d.H / 64;
  const int bn = skinny_wide_tiles(d) ? 128 : 64;
  const int tiles = (d.wtot / bn) * ((M + 63) / 64);
  int want = (768 + tiles - 1) / tiles;
  if (want > 8) want = 8;
  int ks = 1;
  for (int c = 1; c <= want; ++c)
    if (ktiles % c == 0) ks = c;
  return ks;
}

// [M, wtot] = X . [W_Q | W_K | W_C | W_G] as `ksplit` fp32 partials (M small)
void launch_skinny_proj(const Dims &d, const gta_weights &w, const void *x, int M, float *part, int ksplit,
                        hipStream_t st) {
  SkinnyArgs a{};
  a.x = (const bf16 *)x; a.lda = d.H; a.M = M; a.K = d.H;
  const void *wm[4] = {w.wq, w.wk, w.wc, w.wg};
  const int wd[4] = {d.wq_w, d.wk_w, d.wc_w, d.wg_w};
  for (int i = 0; i < 4; ++i) { a.w[i] = (const bf16 *)wm[i]; a.width[i] = wd[i]; }
  a.part = part; a.ksplit = ksplit; a.wtot = d.wtot;
  if (skinny_wide_tiles(d)) {
    if (M <= 32) launch<TileSkinny32>(skinny_proj_kernel<TileSkinny32>, a, ksplit * (d.wtot / 128) * ((M + 31) / 32), st);
    else launch<TileSkinny64>(skinny_proj_kernel<TileSkinny64>, a, ksplit * (d.wtot / 128) * ((M + 63) / 64), st);
  } else {   // every width is a multiple of 64
    if (M <= 32) launch<TileSkinny32N64>(skinny_proj_kernel<TileSkinny32N64>, a, ksplit * (d.wtot / 64) * ((M + 31) / 32), st);
    else launch<TileSkinny64N64>(skinny_proj_kernel<TileSkinny64N64>, a, ksplit * (d.wtot / 64) * ((M + 63) / 64), st);
  }
}

void launch_decoder_gemm(const Dims &d, const void *L, const void *wp, const void *g, void *out, int M,
                         hipStream_t st) {
  DecoderArgs a{};
  a.L = (const bf16 *)L; a.ldl = (int64_t)d.nq * d.dl; a.M = M;
  a.wp = (const bf16 *)wp; a.dl = d.dl; a.dh = d.dh; a.hpq = d.hpq; a.nh = d.nh;
  a.g = (const bf16 *)g; a.gate = d.gate; a.out = (bf16 *)out;
  if ((M <= 1024 || proj_small_ksplit(d, M)) && (d.dh == 64 || d.dh == 128)) {   // short prefill: 64-row tiles, one head (or half of one) each
    if (d.dh == 128) launch<TileSkinny64>(decoder_gemm_kernel<TileSkinny64>, a, d.nh * ((M + 63) / 64), st);
    else launch<TileSkinny64N64>(decoder_gemm_kernel<TileSkinny64N64>, a, d.nh * ((M + 63) / 64), st);
    return;
  }
  if (d.dh == 128 && d.hpq % 2 == 0 && d.dl % 128 == 0 && d.dl >= 256) {
    if (d.gate) launch<TileBig>(decoder_pair_kernel<TileBig, true>, a, (d.nh / 2) * ((M + 255) / 256), st);
    else launch<TileBig>(decoder_pair_kernel<TileBig, false>, a, (d.nh / 2) * ((M + 255) / 256), st);
    return;
  }
  if ((d.dh == 64 || d.dh == 128) && d.hpq % (256 / d.dh) == 0) {
    const int nt = (d.nh * d.dh / 256) * ((M + 255) / 256);
    if (d.gate) launch<TileBig>(decoder_multi_kernel<TileBig, true>, a, nt, st);
    else launch<TileBig>(decoder_multi_kernel<TileBig, false>, a, nt, st);
  } else if (d.dh % 128 == 0) {
    launch<TileHead>(decoder_gemm_kernel<TileHead>, a, d.nh * (d.dh / 128) * ((M + 255) / 256), st);
  } else {   // heads of 64: one head per 64-wide tile
    launch<TileHead64>(decoder_gemm_kernel<TileHead64>, a, d.nh * (d.dh / 64) * ((M + 255) / 256), st);
  }
}

void launch_plain_gemm(const void *A, int64_t lda, int M, int N, int K, const void *B, void *C, hipStream_t st) {
  PlainArgs a{(const bf16 *)A, lda, M, N, K, (const bf16 *)B, (bf16 *)C};
  if (M <= 64 && N % 32 == 0) {
    // a decode step's few rows: 128-column tiles would be N / 128 workgroups (10 at the paper's layer, 14 us);
    // 32 x 32 tiles of one wave each give 4 to 8 times as many (11 us there, whole step 55 -> 52 us)
    launch<TileSkinny32N32>(plain_gemm_kernel<TileSkinny32N32>, a, (N / 32) * ((M + 31) / 32), st);
    return;
  }
  if (M <= 1024 && N % 128 == 0) {   // short prefill: 64-row tiles
    launch<TileSkinny64>(plain_gemm_kernel<TileSkinny64>, a, (N / 128) * ((M + 63) / 64), st);
    return;
  }
  if (N % 256 == 0 && K % 128 == 0 && K >= 256) launch<TileBig>(plain_gemm_kernel<TileBig>, a, (N / 256) * ((M + 255) / 256), st);
  else launch<TileHead>(plain_gemm_kernel<TileHead>, a, (N / 128) * ((M + 255) / 256), st);
}

}  // namespace gta
