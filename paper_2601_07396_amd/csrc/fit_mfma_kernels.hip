// Matrix-core versions of the two products with F in the basis fit (bf16 features as they are; float32 features
// split into bf16 high + low parts on the fly, see FPiece and fit_backproject_f32_kernel):
//   project      Y[N x l] = F * Q           Q stationary in registers (fit_project_mfma_kernel), or, for wide sketches
//                                           and split operands, shared through LDS by waves that split the rows
//                                           (fit_project_rows_kernel)
//   backproject  Z[D x l] += F[rows, :]^T * Y[rows, :]         (Z accumulators stationary in registers)
// Both stream F exactly once per column range of the sketch (one range up to width 128, two up to 256), in 16- or
// 32-row tiles, on v_mfma_f32_16x16x32_bf16 (operand layouts: see mfma_kernels.hip).  A projection that is followed by a back-projection hands Y over as
// packed bf16 operand words (pack_y_word) instead of float32 rows; the last projection of a fit writes float32 rows
// for the Gram matrix.  backproject stores Z directly when one workgroup covers all rows of a block and otherwise
// combines the partial results of its row groups with float atomics (it clears Z itself).
#include <type_traits>

#include "svdc_device.h"
#include "svdc_internal.h"

namespace svdc {

namespace {

constexpr int kWaves = 4;

__device__ __forceinline__ f32x4 mfma16(const u32x4& a, const u32x4& b, const f32x4& c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c,
                                                 0, 0, 0);
}

// Eight consecutive channels of one token as they are loaded, and as matrix-core operands.  bf16 features are the
// operand; float32 features are split into bf16 high + low parts when used (the products then take the high part
// against both parts of the other operand and the low part against its high part: about 16 significant bits).
template <typename T>
struct FPiece;
template <>
struct FPiece<bf16_t> {
  static constexpr bool kTwoParts = false;
  u32x4 w;
  __device__ __forceinline__ void load(const bf16_t* p) { w = *reinterpret_cast<const u32x4*>(p); }
  __device__ __forceinline__ void operands(u32x4* hi, u32x4* lo) const { *hi = w; *lo = w; }
  __device__ __forceinline__ float sumsq() const {
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const float x0 = bf16_lo(w[i]), x1 = bf16_hi(w[i]);
      s += x0 * x0 + x1 * x1;
    }
    return s;
  }
};
template <>
struct FPiece<float> {
  static constexpr bool kTwoParts = true;
  f32x4 x[2];
  __device__ __forceinline__ void load(const float* p) {
    x[0] = *reinterpret_cast<const f32x4*>(p);
    x[1] = *reinterpret_cast<const f32x4*>(p + 4);
  }
  __device__ __forceinline__ void operands(u32x4* hi, u32x4* lo) const {
    const float c8[8] = {x[0][0], x[0][1], x[0][2], x[0][3], x[1][0], x[1][1], x[1][2], x[1][3]};
    split_operand(c8, hi, lo);
  }
  __device__ __forceinline__ float sumsq() const {
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i) s += x[0][i] * x[0][i] + x[1][i] * x[1][i];
    return s;
  }
};

// Q [B, D, l] float32 -> bf16 high / low operand tiles (projection layout):
//   tile (cg, jt), lane (r, g), e  ->  Q[d = 32 cg + 8 g + e][j = 16 jt + r]   (0 for j >= l)
// Per block: hi array of D * LP elements followed by the lo array, LP = 16 KT.
// Q points at the first of the l columns to pack; ldq is the row stride of the whole matrix (sketches wider than 128
// are packed, and multiplied, as two column ranges).
// One workgroup per 32-channel chunk cg: its 32 rows of Q are read row by row (contiguous), staged in LDS, and
// written out as the chunk's KT operand words of 1 KB each (both parts), so that reads and writes are coalesced.
__global__ __launch_bounds__(256) void pack_q_kernel(const float* __restrict__ Q, uint16_t* __restrict__ P, int D,
                                                     int l, int KT, int ldq) {
  __shared__ float tile[32][129];   // [channel in the chunk][coefficient], l <= 128
  const int b = blockIdx.y, cg = blockIdx.x, t = threadIdx.x;
  const int LP = 16 * KT;
  const float* q = Q + ((int64_t)b * D + 32 * cg) * ldq;
  for (int idx = t; idx < 32 * LP; idx += 256) {
    const int d = idx / LP, j = idx % LP;
    tile[d][j] = j < l ? q[(int64_t)d * ldq + j] : 0.f;
  }
  __syncthreads();
  const int64_t per = (int64_t)D * LP;
  uint16_t* p = P + (int64_t)b * 2 * per + (int64_t)cg * KT * 512;
  for (int idx = t; idx < KT * 512; idx += 256) {
    const int e = idx & 7, lane = (idx >> 3) & 63, r = lane & 15, g = lane >> 4, jt = idx >> 9;
    const float x = tile[8 * g + e][16 * jt + r];
    const bf16_t hi = (bf16_t)x;
    const bf16_t lo = (bf16_t)(x - (float)hi);
    p[idx] = __builtin_bit_cast(uint16_t, hi);
    p[per + idx] = __builtin_bit_cast(uint16_t, lo);
  }
}

// Packed Y for the back-projection: Y rounded to bf16, already in the layout of its MFMA operand, so that the
// back-projection fetches an operand with one 16-byte load per lane instead of 8 scalar loads and 4 conversions.
// A 32-row step s and coefficient tile jt form one 1 KB word; lane (r, g), element e holds
//   Y[32 s + 16 (e / 4) + 4 g + e % 4][16 jt + r]      (0 for rows >= N),
// i.e. the lane's four accumulator rows of the step's first 16-row tile followed by those of the second.  The
// back-projection contracts over the rows of a step in this same order.  Index: ((b nsteps + s) KT + jt) 64 + lane.
__device__ __forceinline__ u32x4 pack_y_word(const f32x4& t0, const f32x4& t1, int row, int N) {
  f32x4 a = t0, c = t1;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    if (row + i >= N) a[i] = 0.f;
    if (row + 16 + i >= N) c[i] = 0.f;
  }
  return u32x4{pack_bf16(a[0], a[1]), pack_bf16(a[2], a[3]), pack_bf16(c[0], c[1]), pack_bf16(c[2], c[3])};
}

// ---------------------------------------------------------------------------
// project: Y = F Q for a group of TG 16-row tiles per workgroup, no atomics.
// The workgroup walks over the channel slabs (128 * NCW channels each); for one
// slab wave w keeps the Q operands of its NCW chunks (all KT coefficient tiles)
// in registers and streams the group's row tiles of that slab past them.  The
// partial products of all slabs accumulate in registers (TG x KT accumulators per
// wave); at the end the four waves' partial sums are added through LDS in a
// fixed order and stored once.
//   A operand = F tile   (m = token row, kk = channel)   -- the natural 16-byte row pieces
//   B operand = Q tile   (kk = channel, n = coefficient)
//   D[m = 4 g + i][n = r]  ->  Y[row 16 tile + 4 g + i][16 jt + r]
// FRO: also accumulate sum F^2 (for ||F||_F^2).
// ---------------------------------------------------------------------------
template <typename T, int NCW, int KT, int TG, bool SPLIT, bool FRO>
__global__ __launch_bounds__(256) void fit_project_mfma_kernel(const T* __restrict__ F,
                                                               const uint16_t* __restrict__ Qp, float* Y,
                                                               u32x4* Yp, double* fro_acc, int N, int D, int l,
                                                               int64_t ldf, int64_t bstride, int NS,
                                                               int groups_per_block, int ldy) {
  constexpr int PD = 2;
  static_assert(TG % PD == 0, "prefetch ring must divide the tile group");
  __shared__ f32x4 part[kWaves][2][KT][64];
  const int b = blockIdx.x / groups_per_block, rg = blockIdx.x % groups_per_block;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, r = lane & 15, g = lane >> 4;
  const int64_t per = (int64_t)D * KT * 16;
  const u32x4* Qhi = reinterpret_cast<const u32x4*>(Qp + (int64_t)b * 2 * per);
  const u32x4* Qlo = reinterpret_cast<const u32x4*>(Qp + (int64_t)b * 2 * per + per);
  const T* fbase = F + (int64_t)b * bstride + 8 * g;
  const int tile0 = rg * TG;
  const int ntiles = min(TG, (N + 15) / 16 - tile0);

  f32x4 acc[TG][KT];
#pragma unroll
  for (int t = 0; t < TG; ++t)
#pragma unroll
    for (int jt = 0; jt < KT; ++jt) acc[t][jt] = f32x4{0.f, 0.f, 0.f, 0.f};

  FPiece<T> fin[PD][NCW];
  auto load_tile = [&](int slab, int t, FPiece<T>(&fi)[NCW]) {
    const int row = min((tile0 + t) * 16 + r, N - 1);
    const int cg0 = (slab * kWaves + wave) * NCW;
#pragma unroll
    for (int c = 0; c < NCW; ++c) fi[c].load(fbase + (int64_t)row * ldf + 32 * (cg0 + c));
  };
#pragma unroll
  for (int u = 0; u < PD; ++u) load_tile(0, u, fin[u]);

  float ssq = 0.f;
  for (int slab = 0; slab < NS; ++slab) {
    const int cg0 = (slab * kWaves + wave) * NCW;
    u32x4 q_hi[NCW][KT], q_lo[NCW][KT];
#pragma unroll
    for (int c = 0; c < NCW; ++c)
#pragma unroll
      for (int jt = 0; jt < KT; ++jt) {
        const int64_t ti = (int64_t)(cg0 + c) * KT + jt;
        q_hi[c][jt] = Qhi[ti * 64 + lane];
        if (SPLIT) q_lo[c][jt] = Qlo[ti * 64 + lane];
      }
#pragma unroll
    for (int t = 0; t < TG; ++t) {
      const int u = t % PD;
      if (t < ntiles) {
#pragma unroll
        for (int c = 0; c < NCW; ++c) {
          u32x4 fh, fl;
          fin[u][c].operands(&fh, &fl);
#pragma unroll
          for (int jt = 0; jt < KT; ++jt) {
            acc[t][jt] = mfma16(fh, q_hi[c][jt], acc[t][jt]);
            if (FPiece<T>::kTwoParts) acc[t][jt] = mfma16(fl, q_hi[c][jt], acc[t][jt]);
            if (SPLIT) acc[t][jt] = mfma16(fh, q_lo[c][jt], acc[t][jt]);
          }
          if (FRO && (tile0 + t) * 16 + r < N) ssq += fin[u][c].sumsq();
        }
      }
      // refill this ring slot with the tile PD steps ahead (possibly in the next slab)
      if (t + PD < TG) {
        if (t + PD < ntiles) load_tile(slab, t + PD, fin[u]);
      } else if (slab + 1 < NS) {
        load_tile(slab + 1, t + PD - TG, fin[u]);
      }
    }
  }
  if (FRO) {
    const double s = wave_sum((double)ssq);
    if (lane == 0) atomicAdd(fro_acc + b, s);
  }

  // add the four waves' partial sums, two row tiles per round
  float* ybase = Y + (int64_t)b * N * ldy;
  const int nsteps = (N + 31) / 32;
#pragma unroll
  for (int rd = 0; rd < TG / 2; ++rd) {
#pragma unroll
    for (int tt = 0; tt < 2; ++tt)
#pragma unroll
      for (int jt = 0; jt < KT; ++jt) part[wave][tt][jt][lane] = acc[2 * rd + tt][jt];
    __syncthreads();
    if (Yp) {
      // packed output for the back-projection: the two tiles of this pass of the loop are one 32-row step (see pack_y_word)
      const int step = (tile0 + 2 * rd) / 2;
#pragma unroll
      for (int jt = 0; jt < KT; ++jt) {
        if ((jt % kWaves) != wave) continue;
        f32x4 s2[2];
#pragma unroll
        for (int tt = 0; tt < 2; ++tt) {
          f32x4 s = part[0][tt][jt][lane];
#pragma unroll
          for (int w = 1; w < kWaves; ++w) {
            const f32x4 p = part[w][tt][jt][lane];
            s[0] += p[0]; s[1] += p[1]; s[2] += p[2]; s[3] += p[3];
          }
          s2[tt] = s;
        }
        if (step < nsteps) Yp[(((int64_t)b * nsteps + step) * KT + jt) * 64 + lane] = pack_y_word(s2[0], s2[1], 32 * step + 4 * g, N);
      }
      __syncthreads();
      continue;
    }
#pragma unroll
    for (int item = 0; item < 2 * KT; ++item) {
      if ((item % kWaves) != wave) continue;
      const int tt = item / KT, jt = item % KT;
      f32x4 s = part[0][tt][jt][lane];
#pragma unroll
      for (int w = 1; w < kWaves; ++w) {
        const f32x4 p = part[w][tt][jt][lane];
        s[0] += p[0]; s[1] += p[1]; s[2] += p[2]; s[3] += p[3];
      }
      const int j = 16 * jt + r;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int row = (tile0 + 2 * rd + tt) * 16 + 4 * g + i;
        if (row < N && j < l) ybase[(int64_t)row * ldy + j] = s[i];
      }
    }
    __syncthreads();
  }
}

// ---------------------------------------------------------------------------
// project, row-split version for wide sketches: the four waves of a workgroup take different row tiles (RTW
// each) and all channels, so no partial sums have to be combined, and they share the Q operands through LDS:
// the operand words of a slab of SC 32-channel chunks are fetched once per workgroup (registers -> LDS, double
// buffered, one barrier per slab) and every wave reads them from there.  Per token row the packed sketch is then
// read from L2 once per 64 RTW rows and from LDS once per 16 RTW rows; with the operands stationary in registers
// (kernel above) it is read from L2 once per 64 rows, which at sketch width 128 is twice the bytes of F itself.
// Same operand roles and output mapping as above.  Measured at 57 x 4608 x 3072: 0.47 ms against 0.63 ms at width
// 128 (0.66 against 0.88 ms with split operands), 0.41 against 0.53 ms at width 64 with split operands; at width
// 64 with plain operands the register-stationary kernel stays ahead (0.36 against 0.42 ms).
// ---------------------------------------------------------------------------
template <typename T, int KT, int RTW, int SC, bool SPLIT, bool FRO>
__global__ __launch_bounds__(256) void fit_project_rows_kernel(const T* __restrict__ F,
                                                               const uint16_t* __restrict__ Qp, float* Y,
                                                               u32x4* Yp, double* fro_acc, int N, int D, int l,
                                                               int64_t ldf, int64_t bstride,
                                                               int groups_per_block, int ldy) {
  // Four chunks of F in flight per wave.  With split operands they are requested two at a time: the two 64-byte
  // pieces of a 128-byte line belong to neighbouring chunks, and asked for a whole chunk's work apart the line comes
  // from L2 twice (4 % slower).  With plain operands a slot is refilled as soon as its chunk is done (two chunks
  // in flight instead of four: 3 % slower at width 128).
  constexpr bool PAIRED = SPLIT;
  constexpr int PD = 4;
  static_assert(SC == 2 || SC == 4, "slab of 2 or 4 chunks");
  static_assert(PAIRED || SC == PD, "without pairing the ring slot of a chunk is its index in the slab");
  constexpr int NP = SPLIT ? 2 : 1;           // operand parts (high, low)
  constexpr int WPW = SC * KT / kWaves;       // operand words a wave stages per slab and part
  static_assert(SC * KT % kWaves == 0, "staging must divide among the waves");
  __shared__ u32x4 qs[2][NP][SC * KT][64];
  const int b = blockIdx.x / groups_per_block, rg = blockIdx.x % groups_per_block;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, r = lane & 15, g = lane >> 4;
  const int64_t per = (int64_t)D * KT * 16;
  const u32x4* Qhi = reinterpret_cast<const u32x4*>(Qp + (int64_t)b * 2 * per);
  const u32x4* Qlo = reinterpret_cast<const u32x4*>(Qp + (int64_t)b * 2 * per + per);
  const T* fbase = F + (int64_t)b * bstride + 8 * g;
  const int tile0 = (rg * kWaves + wave) * RTW;
  const int NS = D / (32 * SC), NC = D / 32;

  f32x4 acc[RTW][KT];
#pragma unroll
  for (int t = 0; t < RTW; ++t)
#pragma unroll
    for (int jt = 0; jt < KT; ++jt) acc[t][jt] = f32x4{0.f, 0.f, 0.f, 0.f};

  int64_t rowoff[RTW];
#pragma unroll
  for (int t = 0; t < RTW; ++t) rowoff[t] = (int64_t)min((tile0 + t) * 16 + r, N - 1) * ldf;
  FPiece<T> fin[PD][RTW];
  auto load_chunk = [&](int chunk, FPiece<T>(&fi)[RTW]) {
#pragma unroll
    for (int t = 0; t < RTW; ++t) fi[t].load(fbase + rowoff[t] + 32 * chunk);
  };
  u32x4 stg[NP][WPW];
  auto load_stage = [&](int slab) {
#pragma unroll
    for (int i = 0; i < WPW; ++i) {
      const int64_t w = (int64_t)slab * SC * KT + wave * WPW + i;
      stg[0][i] = Qhi[w * 64 + lane];
      if (SPLIT) stg[NP - 1][i] = Qlo[w * 64 + lane];
    }
  };
  auto store_stage = [&](int buf) {
#pragma unroll
    for (int i = 0; i < WPW; ++i)
#pragma unroll
      for (int p = 0; p < NP; ++p) qs[buf][p][wave * WPW + i][lane] = stg[p][i];
  };
  load_stage(0);
#pragma unroll
  for (int u = 0; u < PD; ++u) load_chunk(u, fin[u]);
  store_stage(0);
  __syncthreads();

  float ssq = 0.f;
  // one slab; with paired requests PAR = slab & 1 is a compile-time value, so that the ring slots are static
  auto do_slab = [&](int slab, auto par) {
    constexpr int PAR = decltype(par)::value;
    const int buf = PAIRED ? PAR : (slab & 1);
    if (slab + 1 < NS) load_stage(slab + 1);
#pragma unroll
    for (int c = 0; c < SC; ++c) {
      const int chunk = slab * SC + c;
      constexpr int kSlotBase = (PAR * SC) % PD;
      const int u = (kSlotBase + c) % PD;     // = chunk % PD
      u32x4 fh[RTW], fl[RTW];
#pragma unroll
      for (int t = 0; t < RTW; ++t) fin[u][t].operands(&fh[t], &fl[t]);
#pragma unroll
      for (int jt = 0; jt < KT; ++jt) {
        const u32x4 bh = qs[buf][0][c * KT + jt][lane];
        u32x4 bl;
        if (SPLIT) bl = qs[buf][NP - 1][c * KT + jt][lane];
#pragma unroll
        for (int t = 0; t < RTW; ++t) {
          acc[t][jt] = mfma16(fh[t], bh, acc[t][jt]);
          if (FPiece<T>::kTwoParts) acc[t][jt] = mfma16(fl[t], bh, acc[t][jt]);
          if (SPLIT) acc[t][jt] = mfma16(fh[t], bl, acc[t][jt]);
        }
      }
      if (FRO) {
#pragma unroll
        for (int t = 0; t < RTW; ++t)
          if ((tile0 + t) * 16 + r < N) ssq += fin[u][t].sumsq();
      }
      if constexpr (PAIRED) {
        if (c % 2 == 1) {                     // chunks c - 1 and c are done: refill both slots together
          if (chunk - 1 + PD < NC) load_chunk(chunk - 1 + PD, fin[(kSlotBase + c - 1) % PD]);
          if (chunk + PD < NC) load_chunk(chunk + PD, fin[u]);
        }
      } else {
        if (chunk + PD < NC) load_chunk(chunk + PD, fin[u]);
      }
    }
    if (slab + 1 < NS) store_stage(buf ^ 1);
    __syncthreads();
  };
  if constexpr (PAIRED) {
    for (int slab = 0; slab < NS; slab += 2) {
      do_slab(slab, std::integral_constant<int, 0>{});
      if (slab + 1 < NS) do_slab(slab + 1, std::integral_constant<int, 1>{});
    }
  } else {
    for (int slab = 0; slab < NS; ++slab) do_slab(slab, std::integral_constant<int, 0>{});
  }
  if (FRO) {
    const double s = wave_sum((double)ssq);
    if (lane == 0) atomicAdd(fro_acc + b, s);
  }
  if constexpr (RTW == 2) {
    if (Yp) {   // packed output for the back-projection: the wave's two tiles are one 32-row step
      const int nsteps = (N + 31) / 32, step = tile0 / 2;
      if (step < nsteps) {
#pragma unroll
        for (int jt = 0; jt < KT; ++jt)
          Yp[(((int64_t)b * nsteps + step) * KT + jt) * 64 + lane] = pack_y_word(acc[0][jt], acc[1][jt], 32 * step + 4 * g, N);
      }
      return;
    }
  }
  float* ybase = Y + (int64_t)b * N * ldy;
#pragma unroll
  for (int t = 0; t < RTW; ++t)
#pragma unroll
    for (int jt = 0; jt < KT; ++jt) {
      const int j = 16 * jt + r;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int row = (tile0 + t) * 16 + 4 * g + i;
        if (row < N && j < l) ybase[(int64_t)row * ldy + j] = acc[t][jt][i];
      }
    }
}

// ---------------------------------------------------------------------------
// backproject: Z[d][j] += sum_rows F[row][d] Y[row][j] over the workgroup's rows.
// The contraction runs over token rows, so both operands need 8 consecutive
// rows per lane:
//   A operand (m = channel, kk = row): a lane loads, for each of its 8 rows, the
//       32-bit word holding channels (2 r, 2 r + 1) of a 32-channel chunk and
//       regroups the low / high halves with v_perm into the operands of the
//       "even" (d = 2 r) and "odd" (d = 2 r + 1) channel tiles;
//   B operand (kk = row, n = coefficient): Y[row 8 g + e][16 jt + r] converted to bf16.
//   D[m = 4 g + i][n = r]  ->  Z[32 chunk + 2 (4 g + i) + parity][16 jt + r]
// Accumulators (NCW chunks x 2 parities x KT tiles) stay in registers over all rows.
// ---------------------------------------------------------------------------
// PACKED: Y comes as the operand words that the projection wrote (pack_y_word); the rows of a 32-row step are then
// contracted in that word's order, kk = 8 g + e  <->  row 16 (e / 4) + 4 g + e % 4.
template <int NCW, int KT, bool PACKED>
__global__ __launch_bounds__(256) void fit_backproject_mfma_kernel(const bf16_t* __restrict__ F,
                                                                   const float* __restrict__ Y,
                                                                   const u32x4* __restrict__ Yp, float* Z, int N,
                                                                   int D, int l, int64_t ldf, int64_t bstride,
                                                                   int NS, int groups_per_block,
                                                                   int rows_per_group, int ldy, int ldz) {
  const int slab = blockIdx.x % NS;
  const int rgb = blockIdx.x / NS;
  const int b = rgb / groups_per_block, rg = rgb % groups_per_block;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, r = lane & 15, g = lane >> 4;
  const int cg0 = (slab * kWaves + wave) * NCW;
  const uint32_t* fbase = reinterpret_cast<const uint32_t*>(F + (int64_t)b * bstride + 32 * cg0) + r;
  const int64_t ldw = ldf / 2;   // row stride in 32-bit words
  const float* ybase = Y + (int64_t)b * N * ldy;
  const int row_begin = rg * rows_per_group;
  const int row_end = min(N, row_begin + rows_per_group);

  f32x4 acc[NCW][2][KT];
#pragma unroll
  for (int c = 0; c < NCW; ++c)
#pragma unroll
    for (int p = 0; p < 2; ++p)
#pragma unroll
      for (int jt = 0; jt < KT; ++jt) acc[c][p][jt] = f32x4{0.f, 0.f, 0.f, 0.f};

  uint32_t fw[NCW][8];
  float yv[PACKED ? 1 : KT][8];
  u32x4 yw[PACKED ? KT : 1];
  const int nsteps = (N + 31) / 32;
  auto load_step = [&](int row0) {
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const int row = PACKED ? row0 + 16 * (e / 4) + 4 * g + e % 4 : row0 + 8 * g + e;
      const int rowc = min(row, N - 1);
#pragma unroll
      for (int c = 0; c < NCW; ++c) fw[c][e] = fbase[(int64_t)rowc * ldw + 16 * c];
      if constexpr (!PACKED) {
#pragma unroll
        for (int jt = 0; jt < KT; ++jt) {
          const int j = 16 * jt + r;
          yv[jt][e] = (row < row_end && j < l) ? ybase[(int64_t)row * ldy + j] : 0.f;
        }
      }
    }
    if constexpr (PACKED) {   // row groups start at multiples of 32 rows; rows >= N are zero in the packed words
#pragma unroll
      for (int jt = 0; jt < KT; ++jt) yw[jt] = Yp[(((int64_t)b * nsteps + row0 / 32) * KT + jt) * 64 + lane];
    }
  };
  if (row_begin < row_end) load_step(row_begin);
  for (int row0 = row_begin; row0 < row_end; row0 += 32) {
    u32x4 yop[KT];
#pragma unroll
    for (int jt = 0; jt < KT; ++jt) {
      if constexpr (PACKED)
        yop[jt] = yw[jt];
      else
        yop[jt] = u32x4{pack_bf16(yv[jt][0], yv[jt][1]), pack_bf16(yv[jt][2], yv[jt][3]),
                        pack_bf16(yv[jt][4], yv[jt][5]), pack_bf16(yv[jt][6], yv[jt][7])};
    }
    u32x4 fop[NCW][2];
#pragma unroll
    for (int c = 0; c < NCW; ++c)
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        fop[c][0][w] = __builtin_amdgcn_perm(fw[c][2 * w + 1], fw[c][2 * w], 0x05040100u);
        fop[c][1][w] = __builtin_amdgcn_perm(fw[c][2 * w + 1], fw[c][2 * w], 0x07060302u);
      }
    if (row0 + 32 < row_end) load_step(row0 + 32);
#pragma unroll
    for (int c = 0; c < NCW; ++c)
#pragma unroll
      for (int p = 0; p < 2; ++p)
#pragma unroll
        for (int jt = 0; jt < KT; ++jt) acc[c][p][jt] = mfma16(fop[c][p], yop[jt], acc[c][p][jt]);
  }

  float* zbase = Z + (int64_t)b * D * ldz;
#pragma unroll
  for (int c = 0; c < NCW; ++c)
#pragma unroll
    for (int p = 0; p < 2; ++p)
#pragma unroll
      for (int jt = 0; jt < KT; ++jt) {
        const int j = 16 * jt + r;
        if (j >= l) continue;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int d = 32 * (cg0 + c) + 2 * (4 * g + i) + p;
          // one row group per block: every element has a single writer
          if (groups_per_block == 1) zbase[(int64_t)d * ldz + j] = acc[c][p][jt][i];
          else atomicAdd(zbase + (int64_t)d * ldz + j, acc[c][p][jt][i]);
        }
      }
}

// ---------------------------------------------------------------------------
// backproject for float32 features: the same contraction, Z[d][j] += sum_rows F[row][d] Y[row][j], with both
// operands split into bf16 high + low parts on the fly (F_hi Y_hi + F_lo Y_hi + F_hi Y_lo).  A lane loads, for each
// of its 8 rows, the two float32 channels (2 r, 2 r + 1) of a chunk; Y comes as float32 rows.  Same output mapping
// and row-group scheme as the bf16 kernel.
// ---------------------------------------------------------------------------
template <int NCW, int KT>
__global__ __launch_bounds__(256) void fit_backproject_f32_kernel(const float* __restrict__ F,
                                                                  const float* __restrict__ Y, float* Z, int N,
                                                                  int D, int l, int64_t ldf, int64_t bstride,
                                                                  int NS, int groups_per_block, int rows_per_group,
                                                                  int ldy, int ldz) {
  const int slab = blockIdx.x % NS;
  const int rgb = blockIdx.x / NS;
  const int b = rgb / groups_per_block, rg = rgb % groups_per_block;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, r = lane & 15, g = lane >> 4;
  const int cg0 = (slab * kWaves + wave) * NCW;
  const f32x2* fbase = reinterpret_cast<const f32x2*>(F + (int64_t)b * bstride + 32 * cg0) + r;
  const int64_t ldw = ldf / 2;   // row stride in channel pairs
  const float* ybase = Y + (int64_t)b * N * ldy;
  const int row_begin = rg * rows_per_group;
  const int row_end = min(N, row_begin + rows_per_group);

  f32x4 acc[NCW][2][KT];
#pragma unroll
  for (int c = 0; c < NCW; ++c)
#pragma unroll
    for (int p = 0; p < 2; ++p)
#pragma unroll
      for (int jt = 0; jt < KT; ++jt) acc[c][p][jt] = f32x4{0.f, 0.f, 0.f, 0.f};

  f32x2 fw[NCW][8];
  float yv[KT][8];
  auto load_step = [&](int row0) {
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const int row = row0 + 8 * g + e;
      const int rowc = min(row, N - 1);
#pragma unroll
      for (int c = 0; c < NCW; ++c) {
        const f32x2 x = fbase[(int64_t)rowc * ldw + 16 * c];
        fw[c][e] = row < row_end ? x : f32x2{0.f, 0.f};
      }
#pragma unroll
      for (int jt = 0; jt < KT; ++jt) {
        const int j = 16 * jt + r;
        yv[jt][e] = (row < row_end && j < l) ? ybase[(int64_t)row * ldy + j] : 0.f;
      }
    }
  };
  if (row_begin < row_end) load_step(row_begin);
  for (int row0 = row_begin; row0 < row_end; row0 += 32) {
    u32x4 yhi[KT], ylo[KT];
#pragma unroll
    for (int jt = 0; jt < KT; ++jt) split_operand(yv[jt], &yhi[jt], &ylo[jt]);
    u32x4 fhi[NCW][2], flo[NCW][2];
#pragma unroll
    for (int c = 0; c < NCW; ++c)
#pragma unroll
      for (int p = 0; p < 2; ++p) {
        float c8[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) c8[e] = fw[c][e][p];
        split_operand(c8, &fhi[c][p], &flo[c][p]);
      }
    if (row0 + 32 < row_end) load_step(row0 + 32);
#pragma unroll
    for (int c = 0; c < NCW; ++c)
#pragma unroll
      for (int p = 0; p < 2; ++p)
#pragma unroll
        for (int jt = 0; jt < KT; ++jt) {
          acc[c][p][jt] = mfma16(fhi[c][p], yhi[jt], acc[c][p][jt]);
          acc[c][p][jt] = mfma16(flo[c][p], yhi[jt], acc[c][p][jt]);
          acc[c][p][jt] = mfma16(fhi[c][p], ylo[jt], acc[c][p][jt]);
        }
  }

  float* zbase = Z + (int64_t)b * D * ldz;
#pragma unroll
  for (int c = 0; c < NCW; ++c)
#pragma unroll
    for (int p = 0; p < 2; ++p)
#pragma unroll
      for (int jt = 0; jt < KT; ++jt) {
        const int j = 16 * jt + r;
        if (j >= l) continue;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int d = 32 * (cg0 + c) + 2 * (4 * g + i) + p;
          if (groups_per_block == 1) zbase[(int64_t)d * ldz + j] = acc[c][p][jt][i];
          else atomicAdd(zbase + (int64_t)d * ldz + j, acc[c][p][jt][i]);
        }
      }
}

template <int KT>
constexpr int width_for() { return KT <= 2 ? 12 : (KT == 4 ? 6 : 3); }

// Row strides of the whole Y / Z matrices when a call covers only a range of their columns (sketches wider than 128
// are multiplied as two column ranges), and whether Z has been cleared for atomic accumulation already.
struct Strides {
  int ldy, ldz;
  bool z_cleared;
};

template <typename T, int NCW, int KT>
void project_launch(const svdc_shape& s, int l, const void* F, const void* Qp, float* Y, u32x4* Yp,
                    double* fro_acc, bool split, Strides ld, hipStream_t st) {
  constexpr bool kF32 = std::is_same<T, float>::value;   // float32 features always take the split sketch
  // 4 row tiles per workgroup from sketch width 64 on: with a 4-chunk slab that is about 250 registers, so two
  // workgroups share a compute unit and one streams F while the other loads its Q operands (measured 8 % / 13 %
  // faster than 8 tiles x 6 chunks at 3072 channels, plain / split operands)
  constexpr int TG = KT <= 2 ? 8 : 4;
  // the split operand doubles the Q registers: halve the slab width when it is wide
  constexpr int NCWS = (NCW * KT > 12 && NCW % 2 == 0) ? NCW / 2 : NCW;
  const int ntile = (s.N + 15) / 16;
  const int gpb = (ntile + TG - 1) / TG;
  const unsigned grid = (unsigned)((int64_t)gpb * s.B);
  const T* f = (const T*)F;
  const uint16_t* q = (const uint16_t*)Qp;
  if (kF32) split = true;
  // wide sketches: rows split over the waves, Q shared through LDS
  if constexpr (KT >= 4) {
    constexpr int RTW = (KT == 8) ? 2 : 3;
    auto rows_grid = [&] { return (ntile + kWaves * RTW - 1) / (kWaves * RTW); };
    if (split) {
      constexpr int SC = (KT == 8) ? 2 : 4;
      const int g = rows_grid();
      if (fro_acc)
        fit_project_rows_kernel<T, KT, RTW, SC, true, true><<<(unsigned)((int64_t)g * s.B), 256, 0, st>>>(
            f, q, Y, Yp, fro_acc, s.N, s.D, l, s.ldf, s.block_stride, g, ld.ldy);
      else
        fit_project_rows_kernel<T, KT, RTW, SC, true, false><<<(unsigned)((int64_t)g * s.B), 256, 0, st>>>(
            f, q, Y, Yp, fro_acc, s.N, s.D, l, s.ldf, s.block_stride, g, ld.ldy);
      return;
    }
    if constexpr (KT == 8 && !kF32) {
      const int g = rows_grid();
      fit_project_rows_kernel<T, KT, RTW, 4, false, false><<<(unsigned)((int64_t)g * s.B), 256, 0, st>>>(
          f, q, Y, Yp, fro_acc, s.N, s.D, l, s.ldf, s.block_stride, g, ld.ldy);
      return;
    }
  }
  if (split) {
    const int NS = s.D / (128 * NCWS);
    if (fro_acc)
      fit_project_mfma_kernel<T, NCWS, KT, TG, true, true><<<grid, 256, 0, st>>>(
          f, q, Y, Yp, fro_acc, s.N, s.D, l, s.ldf, s.block_stride, NS, gpb, ld.ldy);
    else
      fit_project_mfma_kernel<T, NCWS, KT, TG, true, false><<<grid, 256, 0, st>>>(
          f, q, Y, Yp, fro_acc, s.N, s.D, l, s.ldf, s.block_stride, NS, gpb, ld.ldy);
  } else if constexpr (!kF32) {
    const int NS = s.D / (128 * NCW);
    fit_project_mfma_kernel<T, NCW, KT, TG, false, false><<<grid, 256, 0, st>>>(
        f, q, Y, Yp, fro_acc, s.N, s.D, l, s.ldf, s.block_stride, NS, gpb, ld.ldy);
  }
}

template <typename T, int NCW, int KT>
void backproject_launch(const svdc_shape& s, int l, const void* F, const float* Y, const u32x4* Yp, float* Z, int gpb, int rows,
                        Strides ld, hipStream_t st) {
  const int NS = s.D / (128 * NCW);
  const unsigned grid = (unsigned)((int64_t)NS * gpb * s.B);
  if constexpr (std::is_same<T, float>::value) {
    fit_backproject_f32_kernel<NCW, KT><<<grid, 256, 0, st>>>((const float*)F, Y, Z, s.N, s.D, l, s.ldf,
                                                              s.block_stride, NS, gpb, rows, ld.ldy, ld.ldz);
  } else {
    if (Yp)
      fit_backproject_mfma_kernel<NCW, KT, true><<<grid, 256, 0, st>>>((const bf16_t*)F, Y, Yp, Z, s.N, s.D, l, s.ldf,
                                                                      s.block_stride, NS, gpb, rows, ld.ldy, ld.ldz);
    else
      fit_backproject_mfma_kernel<NCW, KT, false><<<grid, 256, 0, st>>>((const bf16_t*)F, Y, Yp, Z, s.N, s.D, l, s.ldf,
                                                                       s.block_stride, NS, gpb, rows, ld.ldy, ld.ldz);
  }
}

__global__ void clear_f32_kernel(float* p, int64_t n) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0.0f;
}

// Row groups per block in backproject.  Partial sums of different groups meet in float atomics, which cost
// more than the parallelism they buy: one group per block as soon as the slabs of all blocks give about one
// workgroup per compute unit, otherwise just enough groups to reach that.
template <int NCW>
void backproject_groups(const svdc_shape& s, int* gpb, int* rows) {
  int dev = 0, cus = 256;
  if (hipGetDevice(&dev) != hipSuccess ||
      hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1)
    cus = 256;
  const int64_t slabs = (int64_t)(s.D / (128 * NCW)) * s.B;
  int g = (int)((cus + slabs / 2) / slabs);
  if (g < 1) g = 1;
  int r = ((s.N + g - 1) / g + 31) / 32 * 32;
  if (r < 32) r = 32;
  *rows = r;
  *gpb = (s.N + r - 1) / r;
}

// largest instantiated slab width (chunks per wave) that divides D / 128 and is at most `cap` (compile time: what
// the registers hold) and `maxw` (run time)
template <int cap, typename Fn12, typename Fn6, typename Fn4, typename Fn3, typename Fn2, typename Fn1>
void by_width(int m, int maxw, Fn12 f12, Fn6 f6, Fn4 f4, Fn3 f3, Fn2 f2, Fn1 f1) {
  if constexpr (cap >= 12) { if (maxw >= 12 && m % 12 == 0) return f12(); }
  if constexpr (cap >= 6) { if (maxw >= 6 && m % 6 == 0) return f6(); }
  if constexpr (cap >= 4) { if (maxw >= 4 && m % 4 == 0) return f4(); }
  if constexpr (cap >= 3) { if (maxw >= 3 && m % 3 == 0) return f3(); }
  if (maxw >= 2 && m % 2 == 0) return f2();
  return f1();
}

template <typename T, int KT>
void project_kt(const svdc_shape& s, int l, const void* F, const void* Qp, float* Y, u32x4* Yp, double* fro, bool split,
                Strides ld, hipStream_t st) {
  // float32 features hold 8 registers per piece in flight and always carry both sketch parts: narrower slabs
  constexpr int cap = std::is_same<T, float>::value ? 3 : (KT == 4 ? 4 : width_for<KT>());
  by_width<cap>(
      s.D / 128, cap, [&] { project_launch<T, (cap >= 12 ? 12 : 1), KT>(s, l, F, Qp, Y, Yp, fro, split, ld, st); },
      [&] { project_launch<T, (cap >= 6 ? 6 : 1), KT>(s, l, F, Qp, Y, Yp, fro, split, ld, st); },
      [&] { project_launch<T, (cap >= 4 ? 4 : 1), KT>(s, l, F, Qp, Y, Yp, fro, split, ld, st); },
      [&] { project_launch<T, (cap >= 3 ? 3 : 1), KT>(s, l, F, Qp, Y, Yp, fro, split, ld, st); },
      [&] { project_launch<T, 2, KT>(s, l, F, Qp, Y, Yp, fro, split, ld, st); },
      [&] { project_launch<T, 1, KT>(s, l, F, Qp, Y, Yp, fro, split, ld, st); });
}

template <typename T, int NCW, int KT>
void backproject_one(const svdc_shape& s, int l, const void* F, const float* Y, const u32x4* Yp, float* Z,
                     Strides ld, hipStream_t st) {
  int gpb, rows;
  backproject_groups<NCW>(s, &gpb, &rows);
  if (gpb > 1 && !ld.z_cleared) {   // atomics accumulate into Z (a single column range: Z is contiguous)
    const int64_t n = (int64_t)s.B * s.D * l;
    clear_f32_kernel<<<(unsigned)((n + 255) / 256), 256, 0, st>>>(Z, n);
  }
  backproject_launch<T, NCW, KT>(s, l, F, Y, Yp, Z, gpb, rows, ld, st);
}

// slab widths of the float32 back-projection (twice the registers per loaded row, two operand parts on each side)
template <int KT>
constexpr int width_for_f32() { return KT <= 2 ? 6 : (KT == 4 ? 3 : 2); }

template <typename T, int KT>
void backproject_kt(const svdc_shape& s, int l, const void* F, const float* Y, const u32x4* Yp, float* Z,
                    Strides ld, hipStream_t st) {
  constexpr int cap = std::is_same<T, float>::value ? width_for_f32<KT>() : width_for<KT>();
  // Small batches: narrower slabs give more workgroups without more row groups, whose partial sums meet in float
  // atomics (one per element and row group): the widest slab that still gives 64 slabs over all blocks, if any.
  // Measured at 4608 x 3072, width 64: 42 -> 15 us for one block, 55 -> 36 us for 4, 72 -> 53 us for 8; from 28
  // blocks on the widest slab is the fastest again.  Not for float32 features, whose back-projection reads and
  // splits Y as float32 rows once per slab (18432 x 3072, one block: 3.7 -> 4.7 ms per fit at width 128 when tried).
  constexpr int64_t kMinSlabs = 64;
  const int m = s.D / 128;
  int maxw = cap;
  if (!std::is_same<T, float>::value && Yp) {   // packed Y only: float32 rows of Y cost the same once per slab
    maxw = 1;
    for (int w : {2, 3, 4, 6, 12})
      if (w <= cap && m % w == 0 && (int64_t)(m / w) * s.B >= kMinSlabs) maxw = w;
  }
  by_width<cap>(
      s.D / 128, maxw, [&] { backproject_one<T, (cap >= 12 ? 12 : 1), KT>(s, l, F, Y, Yp, Z, ld, st); },
      [&] { backproject_one<T, (cap >= 6 ? 6 : 1), KT>(s, l, F, Y, Yp, Z, ld, st); },
      [&] { backproject_one<T, (cap >= 4 ? 4 : 1), KT>(s, l, F, Y, Yp, Z, ld, st); },
      [&] { backproject_one<T, (cap >= 3 ? 3 : 1), KT>(s, l, F, Y, Yp, Z, ld, st); },
      [&] { backproject_one<T, 2, KT>(s, l, F, Y, Yp, Z, ld, st); },
      [&] { backproject_one<T, 1, KT>(s, l, F, Y, Yp, Z, ld, st); });
}

// Sketches wider than 128 are handled as two column ranges (128 and the rest), each with the kernels of its own
// width: F is then read twice per product.
struct ColRange { int j0, l; };
inline int col_ranges(int l, ColRange (&r)[2]) {
  if (l <= 128) { r[0] = {0, l}; return 1; }
  r[0] = {0, 128};
  r[1] = {128, l - 128};
  return 2;
}
inline int kt_for(int l) { return l <= 16 ? 1 : (l <= 32 ? 2 : (l <= 64 ? 4 : 8)); }
inline size_t packed_q_bytes_one(const svdc_shape& s, int l) { return (size_t)s.B * 2 * s.D * kt_for(l) * 16 * sizeof(uint16_t); }
inline size_t packed_y_bytes_one(const svdc_shape& s, int l) { return (size_t)s.B * (((size_t)s.N + 31) / 32) * kt_for(l) * 1024; }

template <typename Fn>
void by_kt(int l, Fn fn) {
  if (l <= 16) fn(std::integral_constant<int, 1>{});
  else if (l <= 32) fn(std::integral_constant<int, 2>{});
  else if (l <= 64) fn(std::integral_constant<int, 4>{});
  else fn(std::integral_constant<int, 8>{});
}

}  // namespace

bool fit_mfma_supported(const svdc_shape& s, int l) {
  return (s.dtype == SVDC_BF16 || s.dtype == SVDC_F32) && s.D % 128 == 0 && l <= 256;
}

size_t fit_mfma_packed_q_bytes(const svdc_shape& s, int l) {
  ColRange r[2];
  const int n = col_ranges(l, r);
  size_t bytes = 0;
  for (int h = 0; h < n; ++h) bytes += packed_q_bytes_one(s, r[h].l);
  return bytes;
}

size_t fit_mfma_packed_y_bytes(const svdc_shape& s, int l) {
  ColRange r[2];
  const int n = col_ranges(l, r);
  size_t bytes = 0;
  for (int h = 0; h < n; ++h) bytes += packed_y_bytes_one(s, r[h].l);
  return bytes;
}

void fit_mfma_pack_q(const svdc_shape& s, int l, const float* Q, void* Qp, hipStream_t st) {
  ColRange r[2];
  const int n = col_ranges(l, r);
  char* out = static_cast<char*>(Qp);
  for (int h = 0; h < n; ++h) {
    const int KT = kt_for(r[h].l);
    pack_q_kernel<<<dim3((unsigned)(s.D / 32), s.B), 256, 0, st>>>(Q + r[h].j0, (uint16_t*)out, s.D, r[h].l, KT, l);
    out += packed_q_bytes_one(s, r[h].l);
  }
}

void fit_mfma_project(const svdc_shape& s, int l, const void* F, const void* Qp, float* Y, void* Ypacked, double* fro_acc,
                      bool split, hipStream_t st) {
  ColRange r[2];
  const int n = col_ranges(l, r);
  const char* qp = static_cast<const char*>(Qp);
  char* yp = static_cast<char*>(Ypacked);
  for (int h = 0; h < n; ++h) {
    const Strides ld{l, l, false};
    by_kt(r[h].l, [&](auto kt) {
      constexpr int KT = decltype(kt)::value;
      if (s.dtype == SVDC_F32)
        project_kt<float, KT>(s, r[h].l, F, qp, Y + r[h].j0, nullptr, h == 0 ? fro_acc : nullptr, true, ld, st);
      else
        project_kt<bf16_t, KT>(s, r[h].l, F, qp, Y + r[h].j0, (u32x4*)yp, h == 0 ? fro_acc : nullptr, split, ld, st);
    });
    qp += packed_q_bytes_one(s, r[h].l);
    if (yp) yp += packed_y_bytes_one(s, r[h].l);
  }
}

void fit_mfma_backproject(const svdc_shape& s, int l, const void* F, const float* Y, const void* Ypacked, float* Z,
                          hipStream_t st) {
  ColRange r[2];
  const int n = col_ranges(l, r);
  const char* yp = static_cast<const char*>(Ypacked);
  bool cleared = false;
  if (n > 1) {   // the column ranges interleave in memory: clear all of Z once, for whichever range accumulates
    const int64_t cnt = (int64_t)s.B * s.D * l;
    clear_f32_kernel<<<(unsigned)((cnt + 255) / 256), 256, 0, st>>>(Z, cnt);
    cleared = true;
  }
  for (int h = 0; h < n; ++h) {
    const Strides ld{l, l, cleared};
    by_kt(r[h].l, [&](auto kt) {
      constexpr int KT = decltype(kt)::value;
      if (s.dtype == SVDC_F32)
        backproject_kt<float, KT>(s, r[h].l, F, Y + r[h].j0, nullptr, Z + r[h].j0, ld, st);
      else
        backproject_kt<bf16_t, KT>(s, r[h].l, F, Y ? Y + r[h].j0 : nullptr, (const u32x4*)yp, Z + r[h].j0, ld, st);
    });
    if (yp) yp += packed_y_bytes_one(s, r[h].l);
  }
}

}  // namespace svdc
