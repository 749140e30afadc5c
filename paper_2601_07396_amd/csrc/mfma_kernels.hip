// Matrix-core (MFMA) kernels for bf16 and float32 features on gfx950 (float32 operands are split into bf16 parts).
//
// All contractions go through v_mfma_f32_16x16x32_bf16 (wave64):
//     D[m][n] += sum_kk A[m][kk] * B[kk][n],   m, n in 0..15, kk in 0..31
// operand layout per lane l (r = l % 16, g = l / 16):
//     A: 8 bf16 = A[m = r][kk = 8g .. 8g+7]        B: 8 bf16 = B[kk = 8g .. 8g+7][n = r]
//     D: 4 f32  = D[m = 4g .. 4g+3][n = r]
// The contraction index kk may be any fixed permutation of the mathematical
// index as long as A and B use the same one, and the rows of A (columns of B)
// may be any permutation of the output index.  The kernels below choose those
// permutations so that
//   * a lane's 16-byte piece of a feature row (8 consecutive hidden channels
//     of one token) is at once a global-memory vector load, an MFMA operand
//     and the position of the MFMA result it must be combined with, and
//   * the accumulators of the projection are, after conversion to bf16,
//     directly the operand of the reconstruction,
// so no value ever moves between lanes.
//
// Basis operands are pre-packed once per fitted basis (svdcache_pack_basis)
// as bf16 "high" and "low" parts (V = hi + lo to ~16 significant bits) in
// per-wavefront tiles of 64 lanes x 16 bytes.
#include <algorithm>
#include <cmath>

#include "svdc_device.h"
#include "svdc_internal.h"

namespace svdc {

namespace {

constexpr int kWavesPerGroup = 4;

__device__ __forceinline__ f32x4 mfma16(const u32x4& a, const u32x4& b, const f32x4& c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c,
                                                 0, 0, 0);
}

// Direct global-to-LDS load of 16 bytes per lane: lane l's bytes land at lds_wave_base + 16 l.  Counts in vmcnt
// like any other vector memory load; lds_wave_base must be the same in all lanes of the wave.
__device__ __forceinline__ void load_to_lds16(const void* gsrc_lane, void* lds_wave_base) {
  __builtin_amdgcn_global_load_lds(gsrc_lane, lds_wave_base, 16, 0, 0);
}

int num_compute_units() {
  int dev = 0, n = 0;
  if (hipGetDevice(&dev) != hipSuccess) return 256;
  if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) return 256;
  return n;
}

// rank padded to 32, 64 or 128 (one reconstruction MFMA contracts 32 coefficients)
__host__ __device__ inline int padded_rank(int k) { return k <= 32 ? 32 : (k <= 64 ? 64 : 128); }

// ---------------------------------------------------------------------------
// Packed basis.  Per block, four arrays of D * KP bf16 each (KP = padded rank):
//   P1hi, P1lo : projection operand.      tile (cg, jt) of 64 lanes x 8 bf16:
//                lane (r, g), e  ->  V[d = 32 cg + 8 g + e][j = 16 jt + r]
//   P2hi, P2lo : reconstruction operand, NEGATED.   tile (cg, t, kt):
//                lane (r, g), e  -> -V[d = 32 cg + 8 (r / 4) + 4 t + r % 4][j = 32 kt + 16 (e / 4) + 4 g + e % 4]
// with cg = d / 32 the 32-channel chunk, jt the 16-coefficient tile, t the
// half of the chunk, kt the 32-coefficient group.  Entries with j >= k are 0.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void pack_basis_kernel(const float* __restrict__ V, uint16_t* __restrict__ P,
                                                         int D, int k, int KP) {
  const int b = blockIdx.y;
  const int64_t per = (int64_t)D * KP;           // elements per array
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= per) return;
  const float* v = V + (int64_t)b * D * k;
  uint16_t* p = P + (int64_t)b * 4 * per;
  const int e = idx & 7, lane = (idx >> 3) & 63, r = lane & 15, g = lane >> 4;
  const int64_t tile = idx >> 9;
  {  // projection operand
    const int KT = KP / 16;
    const int jt = tile % KT, cg = tile / KT;
    const int d = 32 * cg + 8 * g + e, j = 16 * jt + r;
    const float x = j < k ? v[(int64_t)d * k + j] : 0.f;
    const bf16_t hi = (bf16_t)x;
    const bf16_t lo = (bf16_t)(x - (float)hi);
    p[idx] = __builtin_bit_cast(uint16_t, hi);
    p[per + idx] = __builtin_bit_cast(uint16_t, lo);
  }
  {  // reconstruction operand (negated so that the MFMA computes F - V C^T)
    const int KT2 = KP / 32;
    const int kt = tile % KT2, t = (tile / KT2) & 1, cg = tile / (2 * KT2);
    const int d = 32 * cg + 8 * (r >> 2) + 4 * t + (r & 3);
    const int j = 32 * kt + 16 * (e >> 2) + 4 * g + (e & 3);
    const float x = j < k ? -v[(int64_t)d * k + j] : 0.f;
    const bf16_t hi = (bf16_t)x;
    const bf16_t lo = (bf16_t)(x - (float)hi);
    p[2 * per + idx] = __builtin_bit_cast(uint16_t, hi);
    p[3 * per + idx] = __builtin_bit_cast(uint16_t, lo);
  }
}

// ---------------------------------------------------------------------------
// Packed coefficient state: S [B, N, k] float32 as the operand words of the cached step.  Per block, 16-row tile and
// group kt of 32 coefficients two words of 64 lanes x 16 bytes (bf16 high part, then low part) of -S:
//   lane (r, g), e  ->  -S[row = 16 tile + r][j = 32 kt + 16 (e / 4) + 4 g + e % 4]     (0 for row >= N, j >= k)
// word index ((b ntile + tile) KT2 + kt) 2 + part.  The full step writes the same words next to S when asked.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void pack_state_kernel(const float* __restrict__ S, u32x4* __restrict__ Sp, int N,
                                                         int k, int KT2, int64_t words_per_block) {
  const int b = blockIdx.y;
  const int64_t w = (int64_t)blockIdx.x * kWavesPerGroup + (threadIdx.x >> 6);   // (tile, kt)
  if (w >= words_per_block) return;
  const int lane = threadIdx.x & 63, r = lane & 15, g = lane >> 4;
  const int kt = (int)(w % KT2);
  const int64_t tile = w / KT2;
  const int64_t row = tile * 16 + r;
  float c8[8];
#pragma unroll
  for (int t = 0; t < 2; ++t) {
    const int j = 32 * kt + 16 * t + 4 * g;
    f32x4 x = {0.f, 0.f, 0.f, 0.f};
    if (row < N && j < k) x = *reinterpret_cast<const f32x4*>(S + ((int64_t)b * N + row) * k + j);
#pragma unroll
    for (int i = 0; i < 4; ++i) c8[4 * t + i] = -x[i];
  }
  u32x4 hi, lo;
  split_operand(c8, &hi, &lo);
  u32x4* out = Sp + ((int64_t)b * words_per_block + w) * 2 * 64 + lane;
  out[0] = hi;
  out[64] = lo;
}

// Eight consecutive channels of one token as they sit in memory and in registers.  bf16: 16 bytes,
// exact as an MFMA operand.  float32: 32 bytes; as an MFMA operand it is split into bf16 high + low parts.
template <typename T>
struct RowPiece;
template <>
struct RowPiece<bf16_t> {
  u32x4 w;
  __device__ __forceinline__ void load(const bf16_t* p) { w = *reinterpret_cast<const u32x4*>(p); }
  __device__ __forceinline__ f32x4 half(int t) const {
    return f32x4{bf16_lo(w[2 * t]), bf16_hi(w[2 * t]), bf16_lo(w[2 * t + 1]), bf16_hi(w[2 * t + 1])};
  }
  static __device__ __forceinline__ void store(bf16_t* p, const f32x4& x0, const f32x4& x1) {
    *reinterpret_cast<u32x4*>(p) =
        u32x4{pack_bf16(x0[0], x0[1]), pack_bf16(x0[2], x0[3]), pack_bf16(x1[0], x1[1]), pack_bf16(x1[2], x1[3])};
  }
};
template <>
struct RowPiece<float> {
  f32x4 x[2];
  __device__ __forceinline__ void load(const float* p) {
    x[0] = *reinterpret_cast<const f32x4*>(p);
    x[1] = *reinterpret_cast<const f32x4*>(p + 4);
  }
  __device__ __forceinline__ f32x4 half(int t) const { return x[t]; }
  static __device__ __forceinline__ void store(float* p, const f32x4& x0, const f32x4& x1) {
    *reinterpret_cast<f32x4*>(p) = x0;
    *reinterpret_cast<f32x4*>(p + 4) = x1;
  }
};

// ---------------------------------------------------------------------------
// Cached step (Sec. 3.5):  Fhat = S V^T + R   for bf16 R / Fhat.
//
// Basis-stationary: a wave keeps the (negated) reconstruction operands of NCW
// consecutive 32-channel chunks in registers and streams 16-row tiles of R past
// them, so the basis is read from L2 once per workgroup, not once per tile.
// A workgroup of 4 waves covers 4*NCW chunks (a "slab" of 128*NCW channels) and
// tiles_per_group row tiles; adjacent workgroup ids are adjacent slabs of the same
// rows.  Per tile and chunk: two MFMAs per 32 coefficients whose accumulator
// starts at R; the coefficient operand is -S (bf16 high + low parts), so the
// MFMA computes Fhat^T = R^T + (-V)(-S)^T.  PD tiles are kept in flight.
// EXT: the coefficient operand is sum_m w_m S_m over up to kMaxStates stored states (forecasters that are linear
// in them, Sec. 5.3) and a tensor X may be added to the result (Out = C_hat V^T + R + X).
// ---------------------------------------------------------------------------

// PS: the coefficient state comes as packed operand words (packed_state_kernel / the full step's second state
// output) instead of float32 rows: nothing is converted per tile.
// MSX, HX (EXT only): registers are held for MSX coefficient states per tile in flight, and for the added tensor only
// with HX -- a forecaster of two states that adds nothing should not pay for four states and a second row tile.
template <typename T, int NCW, int KT2, bool SPLIT, int PD, bool EXT, bool PS = false, int MSX = kMaxStates, bool HX = true>
__global__ __launch_bounds__(256) void forecast_mfma_kernel(const CoefStates cs, const uint16_t* __restrict__ P,
                                                            const T* R, const T* X, T* Fh, int N, int D, int k,
                                                            int64_t ldf, int64_t bstride, int NS,
                                                            int groups_per_block, int tiles_per_group) {
  static_assert(!(PS && EXT), "the packed state serves the plain cached step");
  const int slab = blockIdx.x % NS;
  const int rgb = blockIdx.x / NS;
  const int b = rgb / groups_per_block, rg = rgb % groups_per_block;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, r = lane & 15, g = lane >> 4;
  constexpr int KP = KT2 * 32;
  const int64_t per = (int64_t)D * KP;
  const u32x4* P2hi = reinterpret_cast<const u32x4*>(P + (int64_t)b * 4 * per + 2 * per);
  const u32x4* P2lo = reinterpret_cast<const u32x4*>(P + (int64_t)b * 4 * per + 3 * per);
  const int cg0 = (slab * kWavesPerGroup + wave) * NCW;
  const T* rbase = R + (int64_t)b * bstride + 32 * cg0 + 8 * g;
  T* obase = Fh + (int64_t)b * bstride + 32 * cg0 + 8 * g;
  // EXT: the coefficient forecast is sum_m w_m S_m over up to kMaxStates stored states, and a tensor X
  // (nullable) is added to the result; otherwise the single state cs.s[0] with weight one.
  constexpr int MS = EXT ? MSX : 1;
  const int ntile_block = (N + 15) / 16;
  const bool has_x = EXT && HX && X != nullptr;
  const T* xbase = has_x ? X + (int64_t)b * bstride + 32 * cg0 + 8 * g : nullptr;
  const int64_t soff = (int64_t)b * N * k;
  // Row tiles rg, rg + groups_per_block, ...: the workgroups of a block advance through its rows side by
  // side, which keeps the addresses in flight close together (measurably kinder to HBM than giving each
  // workgroup a contiguous range of tiles).
  const int ntiles = min(tiles_per_group, (ntile_block - rg + groups_per_block - 1) / groups_per_block);

  RowPiece<T> rin[PD][NCW];
  RowPiece<T> xin[PD][(EXT && HX) ? NCW : 1];
  f32x4 sraw[PD][PS ? 1 : MS][PS ? 1 : KT2][2];
  u32x4 spk[PD][PS ? KT2 : 1][2];   // packed state: high and low operand words
  const u32x4* spbase = PS ? reinterpret_cast<const u32x4*>(cs.s[0]) + (int64_t)b * ntile_block * KT2 * 2 * 64 + lane : nullptr;
  // lane (r, g) needs S[row][j = 32 kt + 16 t + 4 g + i], i = 0..3 (zero beyond k)
  auto load_tile = [&](int tile, int u) {
    const int row = min(tile * 16 + r, N - 1);
    if constexpr (PS) {
#pragma unroll
      for (int kt = 0; kt < KT2; ++kt)
#pragma unroll
        for (int part = 0; part < (SPLIT ? 2 : 1); ++part)
          spk[u][kt][part] = spbase[(((int64_t)tile * KT2 + kt) * 2 + part) * 64];
    }
#pragma unroll
    for (int ms = 0; ms < (PS ? 0 : MS); ++ms) {
      if (ms >= cs.m) break;
#pragma unroll
      for (int kt = 0; kt < KT2; ++kt)
#pragma unroll
        for (int t = 0; t < 2; ++t) {
          const int j = 32 * kt + 16 * t + 4 * g;
          sraw[u][ms][kt][t] = (j < k) ? *reinterpret_cast<const f32x4*>(cs.s[ms] + soff + (int64_t)row * k + j)
                                       : f32x4{0.f, 0.f, 0.f, 0.f};
        }
    }
#pragma unroll
    for (int c = 0; c < NCW; ++c) rin[u][c].load(rbase + (int64_t)row * ldf + 32 * c);
    if constexpr (EXT && HX) {
      if (has_x) {
#pragma unroll
        for (int c = 0; c < NCW; ++c) xin[u][c].load(xbase + (int64_t)row * ldf + 32 * c);
      }
    }
  };
#pragma unroll
  for (int u = 0; u < PD; ++u)
    if (u < ntiles) load_tile(rg + u * groups_per_block, u);

  u32x4 a_hi[NCW][2][KT2], a_lo[NCW][2][KT2];
#pragma unroll
  for (int c = 0; c < NCW; ++c)
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int kt = 0; kt < KT2; ++kt) {
        const int64_t ti = ((int64_t)(cg0 + c) * 2 + t) * KT2 + kt;
        a_hi[c][t][kt] = P2hi[ti * 64 + lane];
        if (SPLIT) a_lo[c][t][kt] = P2lo[ti * 64 + lane];
      }

  for (int it = 0; it < ntiles; it += PD) {
#pragma unroll
    for (int u = 0; u < PD; ++u) {
      if (it + u >= ntiles) continue;
      const int tile = rg + (it + u) * groups_per_block;
      u32x4 shi[KT2], slo[KT2];
#pragma unroll
      for (int kt = 0; kt < (PS ? KT2 : 0); ++kt) {
        shi[kt] = spk[u][kt][0];
        if (SPLIT) slo[kt] = spk[u][kt][1];
      }
#pragma unroll
      for (int kt = 0; kt < (PS ? 0 : KT2); ++kt) {
        float c8[8];
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            if constexpr (EXT) {
              float v = cs.w[0] * sraw[u][0][kt][t][i];
#pragma unroll
              for (int ms = 1; ms < MS; ++ms)
                if (ms < cs.m) v = __builtin_fmaf(cs.w[ms], sraw[u][ms][kt][t][i], v);
              c8[4 * t + i] = -v;
            } else {
              c8[4 * t + i] = -sraw[u][0][kt][t][i];
            }
          }
        split_operand(c8, &shi[kt], &slo[kt]);
      }
      const int row = tile * 16 + r;
#pragma unroll
      for (int c = 0; c < NCW; ++c) {
        f32x4 res[2];
#pragma unroll
        for (int t = 0; t < 2; ++t) {
          f32x4 acc = rin[u][c].half(t);
          if constexpr (EXT && HX) {
            if (has_x) {
              const f32x4 xa = xin[u][c].half(t);
              acc[0] += xa[0]; acc[1] += xa[1]; acc[2] += xa[2]; acc[3] += xa[3];
            }
          }
#pragma unroll
          for (int kt = 0; kt < KT2; ++kt) {
            acc = mfma16(a_hi[c][t][kt], shi[kt], acc);
            if (SPLIT) {
              acc = mfma16(a_hi[c][t][kt], slo[kt], acc);
              acc = mfma16(a_lo[c][t][kt], shi[kt], acc);
            }
          }
          res[t] = acc;
        }
        if (row < N) RowPiece<T>::store(obase + (int64_t)row * ldf + 32 * c, res[0], res[1]);
      }
      if (it + u + PD < ntiles) load_tile(tile + PD * groups_per_block, u);
    }
  }
}

// ---------------------------------------------------------------------------
// Full-compute step (Eq. 8-11) for bf16 F / R, one pass over F.
// Persistent workgroups (one per compute unit) walk over row tiles; a workgroup
// of 4 waves holds a tile of 16*RT token rows x D channels in registers: wave w
// keeps the channels [w D/4, (w+1) D/4) of all rows as packed bf16
// (RT * CH * 4 VGPRs, CH = D / 128 chunks of 32 channels).
//   phase 1  C^T partial = V^T F^T over the wave's channels (MFMA); the basis
//            operands stream from L2 through a ring of RD operand words so that
//            their latency is covered; partials of the 4 waves are summed through
//            LDS in a fixed order
//   EMA      wave w updates S (and writes C) for row tile w, w+4, ...
//   phase 2  R^T = F^T - V C^T per chunk: accumulator starts at F, A operand
//            is the negated basis, B operand is C (bf16 high [+ low] parts)
//   then     the next tile's rows are requested in one burst, so the loads are
//            in flight while nothing else of this wave waits behind them
// S1 / S2: use the low parts of the basis (and of C) in phase 1 / phase 2.
// REMA: the residual state is smoothed as well (ablation of Sec. 4.5): R = (1 - alpha_r) Rp + alpha_r (F - C V^T),
// with the previous residual Rp read chunk by chunk a few chunks ahead; Rp may be the buffer R.
// LT = 1 (bf16 only): one more row tile per workgroup tile lives in LDS, as an image of the registers it would
// occupy (96 KB at 3072 channels).  It arrives by direct global-to-LDS loads (lane l's 16 bytes land at
// base + 16 l), each wave reads back only what it loaded itself, and every basis operand then serves RT + 1
// row tiles: a third less basis traffic from L2 per token row at RT = 2.
// F and R may alias: a tile is completely on chip (registers, LDS) before it is overwritten.
// ---------------------------------------------------------------------------
template <typename T, int CH, int RT, int KT2, bool S1, bool S2, int RD, bool REMA, int LT = 0>
__global__ __launch_bounds__(256) void full_step_mfma_kernel(const T* F, const uint16_t* __restrict__ P,
                                                             T* R, const T* Rp, float alpha_r, float* S, float* C,
                                                             int N, int k, int64_t ldf, int64_t bstride,
                                                             float alpha, int init, int tiles_per_block,
                                                             int total, u32x4* Sp) {
  constexpr int KP = KT2 * 32, KT = KT2 * 2, D = CH * 128;
  constexpr int M = CH * KT;   // basis operand items per wave and phase (a high + a low 16-byte word per lane each)
  constexpr int RA = RT + LT;  // row tiles per workgroup tile: RT in registers, LT in LDS
  static_assert(LT == 0 || (LT == 1 && !REMA && sizeof(T) == 2), "the LDS row tile is for bf16 features, plain residual");
  __shared__ f32x4 part[kWavesPerGroup][KT][RA][64];
  __shared__ u32x4 ftile[LT ? kWavesPerGroup : 1][LT ? CH : 1][LT ? 64 : 1];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, r = lane & 15, g = lane >> 4;
  const int64_t per = (int64_t)D * KP;
  const int cg0 = wave * CH;
  int v = blockIdx.x;
  if (v >= total) return;

  // the wave's slab of the tile: 8 channels per lane per (row tile, chunk)
  constexpr bool kF32 = sizeof(T) == 4;
  RowPiece<T> f[RT][CH];
  auto load_f_chunk = [&](int vv, int c) {
    const int b = vv / tiles_per_block, tile = vv % tiles_per_block;
    const T* fbase = F + (int64_t)b * bstride + 32 * (cg0 + c) + 8 * g;
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
      const int row = min(tile * 16 * RA + 16 * rt + r, N - 1);
      f[rt][c].load(fbase + (int64_t)row * ldf);
    }
    if constexpr (LT > 0) {
      const int row = min(tile * 16 * RA + 16 * RT + r, N - 1);
      load_to_lds16(fbase + (int64_t)row * ldf, &ftile[wave][c][0]);
    }
  };
#pragma unroll
  for (int c = 0; c < CH; ++c) load_f_chunk(v, c);

  for (; v < total; v += gridDim.x) {
    const int b = v / tiles_per_block, tile = v % tiles_per_block;
    const u32x4* P1hi = reinterpret_cast<const u32x4*>(P + (int64_t)b * 4 * per) + lane;
    const u32x4* P1lo = reinterpret_cast<const u32x4*>(P + (int64_t)b * 4 * per + per) + lane;
    const u32x4* P2hi = reinterpret_cast<const u32x4*>(P + (int64_t)b * 4 * per + 2 * per) + lane;
    const u32x4* P2lo = reinterpret_cast<const u32x4*>(P + (int64_t)b * 4 * per + 3 * per) + lane;
    const int row0 = tile * 16 * RA;
    T* obase = R + (int64_t)b * bstride + 8 * g;

    // ---- phase 1: acc[jt][rt] = C^T[j = 16 jt + 4 g + i][row = 16 rt + r] over this wave's channels.
    // Operand item m = (chunk c, coefficient tile jt), consecutive in the packed basis; RD items in flight.
    const u32x4* p1h = P1hi + (int64_t)cg0 * KT * 64;
    const u32x4* p1l = P1lo + (int64_t)cg0 * KT * 64;
    u32x4 rh[RD], rl[RD];
#pragma unroll
    for (int m = 0; m < RD; ++m)
      if (m < M) {
        rh[m] = p1h[m * 64];
        if (S1) rl[m] = p1l[m * 64];
      }
    f32x4 acc[KT][RA];
#pragma unroll
    for (int jt = 0; jt < KT; ++jt)
#pragma unroll
      for (int rt = 0; rt < RA; ++rt) acc[jt][rt] = f32x4{0.f, 0.f, 0.f, 0.f};
    u32x4 lnext;            // the LDS row tile's piece of the next chunk, read one chunk ahead
    if constexpr (LT > 0) lnext = ftile[wave][0][lane];
    __builtin_amdgcn_sched_barrier(0);
    u32x4 bh[RA], bl[RA];   // feature operand of the current chunk: exact for bf16; high + low parts for float32
#pragma unroll
    for (int m = 0; m < M; ++m) {
      const int c = m / KT, jt = m % KT, slot = m % RD;
      if (jt == 0) {
        if constexpr (LT > 0) {
          bh[RT] = lnext;
          if (c + 1 < CH) lnext = ftile[wave][c + 1][lane];
        }
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) {
          if constexpr (kF32) {
            const f32x4 x0 = f[rt][c].half(0), x1 = f[rt][c].half(1);
            const float x8[8] = {x0[0], x0[1], x0[2], x0[3], x1[0], x1[1], x1[2], x1[3]};
            split_operand(x8, &bh[rt], &bl[rt]);
          } else {
            bh[rt] = f[rt][c].w;
          }
        }
      }
#pragma unroll
      for (int rt = 0; rt < RA; ++rt) {
        acc[jt][rt] = mfma16(rh[slot], bh[rt], acc[jt][rt]);
        if (kF32) acc[jt][rt] = mfma16(rh[slot], bl[rt], acc[jt][rt]);
        if (S1) acc[jt][rt] = mfma16(rl[slot], bh[rt], acc[jt][rt]);
      }
      if (m + RD < M) {
        rh[slot] = p1h[(m + RD) * 64];
        if (S1) rl[slot] = p1l[(m + RD) * 64];
      }
      __builtin_amdgcn_sched_barrier(0);
    }

    // REMA: the residual state is smoothed too, R = (1 - alpha_r) R_prev + alpha_r (F - C V^T); PR chunks of the
    // previous residual are kept in flight
    constexpr int PR = 4;
    RowPiece<T> rp[REMA ? PR : 1][REMA ? RT : 1];
    const T* pbase = REMA ? Rp + (int64_t)b * bstride + 8 * g : nullptr;
    auto load_prev = [&](int c) {
      if constexpr (REMA) {
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) {
          const int row = min(row0 + 16 * rt + r, N - 1);
          rp[c % PR][rt].load(pbase + (int64_t)row * ldf + 32 * (cg0 + c));
        }
      }
    };
    if constexpr (REMA) {
#pragma unroll
      for (int c = 0; c < PR; ++c)
        if (c < CH) load_prev(c);
    }

    // the first reconstruction operands are requested before the reduction so they arrive during it;
    // item n = (chunk c, half t, coefficient tile kt), again consecutive in memory
    const u32x4* p2h = P2hi + (int64_t)cg0 * 2 * KT2 * 64;
    const u32x4* p2l = P2lo + (int64_t)cg0 * 2 * KT2 * 64;
    u32x4 qh[RD], ql[RD];
#pragma unroll
    for (int n = 0; n < RD; ++n)
      if (n < M) {
        qh[n] = p2h[n * 64];
        if (S2) ql[n] = p2l[n * 64];
      }
    __builtin_amdgcn_sched_barrier(0);

    // sum the four partial products through LDS, same order in every wave
#pragma unroll
    for (int jt = 0; jt < KT; ++jt)
#pragma unroll
      for (int rt = 0; rt < RA; ++rt) part[wave][jt][rt][lane] = acc[jt][rt];
    __syncthreads();
#pragma unroll
    for (int jt = 0; jt < KT; ++jt)
#pragma unroll
      for (int rt = 0; rt < RA; ++rt) {
        f32x4 s = part[0][jt][rt][lane];
#pragma unroll
        for (int w = 1; w < kWavesPerGroup; ++w) {
          const f32x4 p = part[w][jt][rt][lane];
          s[0] += p[0]; s[1] += p[1]; s[2] += p[2]; s[3] += p[3];
        }
        acc[jt][rt] = s;
      }
    __syncthreads();   // the next tile reuses `part`

    // EMA update (Eq. 11, alpha = 1 - beta) and coefficient output, one wave per row tile.  Sp (nullable): the new
    // state also leaves as the cached step's operand words (negated, bf16 high + low parts; zeros beyond N and k).
    const int ntile_block = (N + 15) / 16;
#pragma unroll
    for (int rt = 0; rt < RA; ++rt) {
      if ((rt % kWavesPerGroup) != wave) continue;
      const int row = row0 + 16 * rt + r;
      const int tile16 = tile * RA + rt;
      if (tile16 >= ntile_block) continue;
      const int64_t srow = ((int64_t)b * N + min(row, N - 1)) * k;
      f32x4 snew[KT];
#pragma unroll
      for (int jt = 0; jt < KT; ++jt) {
        const int j = 16 * jt + 4 * g;
        snew[jt] = f32x4{0.f, 0.f, 0.f, 0.f};
        if (j >= k || row >= N) continue;   // k is a multiple of 4: a group of four is all inside or all outside
        const f32x4 c4 = acc[jt][rt];
        f32x4 s4 = c4;
        if (!init) {
          const f32x4 old = *reinterpret_cast<const f32x4*>(S + srow + j);
#pragma unroll
          for (int i = 0; i < 4; ++i) s4[i] = (1.f - alpha) * old[i] + alpha * c4[i];
        }
        *reinterpret_cast<f32x4*>(S + srow + j) = s4;
        if (C) *reinterpret_cast<f32x4*>(C + srow + j) = c4;
        snew[jt] = s4;
      }
      if (Sp) {
#pragma unroll
        for (int kt = 0; kt < KT2; ++kt) {
          float c8[8];
#pragma unroll
          for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int i = 0; i < 4; ++i) c8[4 * t + i] = -snew[2 * kt + t][i];
          u32x4 hi, lo;
          split_operand(c8, &hi, &lo);
          u32x4* w = Sp + ((((int64_t)b * ntile_block + tile16) * KT2 + kt) * 2) * 64 + lane;
          w[0] = hi;
          w[64] = lo;
        }
      }
    }

    // coefficient operand of the reconstruction: kk = 8 g + 4 t + i  <->  j = 32 kt + 16 t + 4 g + i
    u32x4 chi[RA][KT2], clo[RA][KT2];
#pragma unroll
    for (int rt = 0; rt < RA; ++rt)
#pragma unroll
      for (int kt = 0; kt < KT2; ++kt) {
        float c8[8];
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
          for (int i = 0; i < 4; ++i) c8[4 * t + i] = acc[2 * kt + t][rt][i];
        split_operand(c8, &chi[rt][kt], &clo[rt][kt]);
      }
    if constexpr (LT > 0) lnext = ftile[wave][0][lane];
    __builtin_amdgcn_sched_barrier(0);

    // ---- phase 2: residual, chunk by chunk
#pragma unroll
    for (int c = 0; c < CH; ++c) {
      f32x4 x[RA][2];
#pragma unroll
      for (int rt = 0; rt < RT; ++rt)
#pragma unroll
        for (int t = 0; t < 2; ++t) x[rt][t] = f[rt][c].half(t);
      if constexpr (LT > 0) {
        RowPiece<bf16_t> piece;
        piece.w = lnext;
        if (c + 1 < CH) lnext = ftile[wave][c + 1][lane];
#pragma unroll
        for (int t = 0; t < 2; ++t) x[RT][t] = piece.half(t);
      }
#pragma unroll
      for (int tk = 0; tk < 2 * KT2; ++tk) {
        const int t = tk / KT2, kt = tk % KT2, n = c * 2 * KT2 + tk, slot = n % RD;
#pragma unroll
        for (int rt = 0; rt < RA; ++rt) {
          x[rt][t] = mfma16(qh[slot], chi[rt][kt], x[rt][t]);
          if (S2) {
            x[rt][t] = mfma16(qh[slot], clo[rt][kt], x[rt][t]);
            x[rt][t] = mfma16(ql[slot], chi[rt][kt], x[rt][t]);
          }
        }
        if (n + RD < M) {
          qh[slot] = p2h[(n + RD) * 64];
          if (S2) ql[slot] = p2l[(n + RD) * 64];
        }
      }
#pragma unroll
      for (int rt = 0; rt < RA; ++rt) {
        if constexpr (REMA) {
#pragma unroll
          for (int t = 0; t < 2; ++t) {
            const f32x4 old = rp[c % PR][rt].half(t);
#pragma unroll
            for (int i = 0; i < 4; ++i) x[rt][t][i] = (1.f - alpha_r) * old[i] + alpha_r * x[rt][t][i];
          }
        }
        const int row = row0 + 16 * rt + r;
        if (row < N) RowPiece<T>::store(obase + (int64_t)row * ldf + 32 * (cg0 + c), x[rt][0], x[rt][1]);
      }
      if constexpr (REMA) {
        if (c + PR < CH) load_prev(c + PR);
      }
      __builtin_amdgcn_sched_barrier(0);
    }

    // request the next tile
    const int vn = v + (int)gridDim.x;
    if (vn < total) {
#pragma unroll
      for (int c = 0; c < CH; ++c) load_f_chunk(vn, c);
    }
  }
}


}  // namespace

bool mfma_shape_supported(const svdc_shape& s) {
  if (s.D % 128 != 0 || s.k > 128 || s.k % 4 != 0) return false;
  // hidden sizes 256, 512, 1024, 1152, 1536, 1920, 2048, 2560, 3072, 4096, 5120 (the full step is instantiated per width)
  switch (s.D / 128) {
    case 2: case 4: case 8: case 9: case 12: case 15: case 16: case 20: case 24: case 32: case 40: return true;
    default: return false;
  }
}

size_t mfma_packed_bytes(const svdc_shape& s) {
  return (size_t)s.B * 4 * s.D * padded_rank(s.k) * sizeof(uint16_t);
}

int32_t launch_pack_basis(const svdc_shape& s, const float* V, void* packed, hipStream_t st) {
  const int KP = padded_rank(s.k);
  const int64_t per = (int64_t)s.D * KP;
  dim3 grid((unsigned)((per + 255) / 256), s.B);
  pack_basis_kernel<<<grid, 256, 0, st>>>(V, (uint16_t*)packed, s.D, s.k, KP);
  return launch_status();
}

namespace {

template <typename T, int NCW, int KT2, bool SPLIT, int PD, bool EXT, bool PS = false>
int32_t forecast_launch(const svdc_shape& s, const CoefStates& cs, const void* packed, const void* R, const void* X,
                        void* Fhat, hipStream_t st) {
  const int NS = s.D / (128 * NCW);
  const int ntile = (s.N + 15) / 16;
  // Row tiles per workgroup: 6..16, chosen so that the workgroups fill whole rounds of the machine
  // (a grid of e.g. 16.03 x the number of compute units costs a 17th, nearly empty round).
  const int cus = num_compute_units();
  int tpg = 8;
  double best = 0.0;
  for (int cand = 16; cand >= 6; --cand) {
    const int64_t w = (int64_t)NS * ((ntile + cand - 1) / cand) * s.B;
    const double rounds = (double)w / cus;
    const double eff = rounds / std::ceil(rounds) * ((double)ntile / (cand * ((ntile + cand - 1) / cand)));
    if (eff > best + 1e-9) { best = eff; tpg = cand; }
  }
  const int gpb = (ntile + tpg - 1) / tpg;
  const int64_t grid = (int64_t)NS * gpb * s.B;
  if (grid > 0x7fffffff) return SVDC_E_SHAPE;
  auto launch = [&](auto kernel) {
    kernel<<<(unsigned)grid, 256, 0, st>>>(cs, (const uint16_t*)packed, (const T*)R, (const T*)X, (T*)Fhat, s.N, s.D,
                                           s.k, s.ldf, s.block_stride, NS, gpb, tpg);
  };
  if constexpr (EXT) {
    // registers for two or four states, with or without the added tensor
    if (cs.m <= 2) {
      if (X) launch(forecast_mfma_kernel<T, NCW, KT2, SPLIT, PD, true, false, 2, true>);
      else launch(forecast_mfma_kernel<T, NCW, KT2, SPLIT, PD, true, false, 2, false>);
    } else {
      if (X) launch(forecast_mfma_kernel<T, NCW, KT2, SPLIT, PD, true, false, kMaxStates, true>);
      else launch(forecast_mfma_kernel<T, NCW, KT2, SPLIT, PD, true, false, kMaxStates, false>);
    }
  } else {
    launch(forecast_mfma_kernel<T, NCW, KT2, SPLIT, PD, false, PS>);
  }
  return launch_status();
}

// widest slab per wave (NCW chunks) that divides D / 128 and keeps the basis operands in registers
template <typename T, int KT2, bool SPLIT, int PD, bool EXT, bool PS = false>
int32_t forecast_by_width(const svdc_shape& s, const CoefStates& cs, const void* packed, const void* R, const void* X,
                          void* Fhat, hipStream_t st) {
  // registers: basis operands 8 (16 with the low parts) per chunk and 32 coefficients, row pieces 4 (8 for f32)
  // (the extended kernel also holds up to 4 coefficient states and the added tensor per tile in flight)
  constexpr int kBudget = (SPLIT ? 12 : 24) / KT2 / (sizeof(T) == 4 ? 2 : 1) / (EXT && KT2 >= 2 ? 2 : 1);
  constexpr int kMax =
      kBudget >= 12 ? 12 : (kBudget >= 6 ? 6 : (kBudget >= 4 ? 4 : (kBudget >= 3 ? 3 : ((kBudget >= 2 || !EXT) ? 2 : 1))));
  const int m = s.D / 128;
  if constexpr (kMax >= 12) {
    if (m % 12 == 0) return forecast_launch<T, 12, KT2, SPLIT, PD, EXT, PS>(s, cs, packed, R, X, Fhat, st);
    // hidden sizes that 12 does not divide (1152 = 9 x 128, 2560 and 5120 = 20 and 40 x 128, 4096 = 32 x 128); only
    // the basic kernel, to bound the number of instantiations
    if constexpr (!EXT) {
      if (m % 10 == 0) return forecast_launch<T, 10, KT2, SPLIT, PD, EXT, PS>(s, cs, packed, R, X, Fhat, st);
      if (m % 9 == 0) return forecast_launch<T, 9, KT2, SPLIT, PD, EXT, PS>(s, cs, packed, R, X, Fhat, st);
      if (m % 8 == 0) return forecast_launch<T, 8, KT2, SPLIT, PD, EXT, PS>(s, cs, packed, R, X, Fhat, st);
    }
  }
  // bf16 features at rank 64 with split operands: the estimate above gives 6, but 8 chunks still fit (500 of the 512
  // registers, no spills); a workgroup then covers a third of a 3072-channel row instead of a quarter
  // (0.760 -> 0.725 ms at 57 x 4608 x 3072)
  if constexpr (kMax == 6 && KT2 == 2 && SPLIT && sizeof(T) == 2 && !EXT) {
    if (m % 8 == 0) return forecast_launch<T, 8, KT2, SPLIT, PD, EXT, PS>(s, cs, packed, R, X, Fhat, st);
  }
  if constexpr (kMax >= 6) {
    if (m % 6 == 0) return forecast_launch<T, 6, KT2, SPLIT, PD, EXT, PS>(s, cs, packed, R, X, Fhat, st);
    if constexpr (!EXT) {   // 1920 = 15 x 128
      if (m % 5 == 0) return forecast_launch<T, 5, KT2, SPLIT, PD, EXT, PS>(s, cs, packed, R, X, Fhat, st);
    }
  }
  if constexpr (kMax == 3 && KT2 == 4 && SPLIT && sizeof(T) == 2 && !EXT) {   // likewise 4 chunks at rank 128
    if (m % 4 == 0) return forecast_launch<T, 4, KT2, SPLIT, PD, EXT, PS>(s, cs, packed, R, X, Fhat, st);
  }
  if constexpr (kMax >= 4) {
    if (m % 4 == 0) return forecast_launch<T, 4, KT2, SPLIT, PD, EXT, PS>(s, cs, packed, R, X, Fhat, st);
  }
  if constexpr (kMax >= 3) {
    if (m % 3 == 0) return forecast_launch<T, 3, KT2, SPLIT, PD, EXT, PS>(s, cs, packed, R, X, Fhat, st);
  }
  if constexpr (kMax >= 2) {
    if (m % 2 == 0) return forecast_launch<T, 2, KT2, SPLIT, PD, EXT, PS>(s, cs, packed, R, X, Fhat, st);
  }
  return forecast_launch<T, 1, KT2, SPLIT, PD, EXT, PS>(s, cs, packed, R, X, Fhat, st);
}

template <typename T, int CH, int RT, int KT2, bool SPLIT, int RD, bool REMA, int LT = 0>
int32_t full_step_launch(const svdc_shape& s, const void* F, const void* packed, void* R, float* S, float* C,
                         float alpha, int init, ResidualEma re, hipStream_t st) {
  const int tiles = (s.N + 16 * (RT + LT) - 1) / (16 * (RT + LT));
  const int64_t total = (int64_t)tiles * s.B;
  if (total > 0x7fffffff) return SVDC_E_SHAPE;
  const int grid = (int)std::min<int64_t>(total, num_compute_units());
  full_step_mfma_kernel<T, CH, RT, KT2, SPLIT, SPLIT, RD, REMA, LT><<<grid, 256, 0, st>>>(
      (const T*)F, (const uint16_t*)packed, (T*)R, (const T*)re.prev, re.alpha_r, S, C, s.N, s.k, s.ldf,
      s.block_stride, alpha, init, tiles, (int)total, (u32x4*)re.packed_state);
  return launch_status();
}

// Row tiles per workgroup tile (RT) and depth of the basis-operand ring (RD items) for a feature width of
// CH * 128 channels, W = 1 (bf16) or 2 (float32) registers per channel pair and KT2 = padded rank / 32.
// Every basis byte is read once per tile, so the tile should have as many rows as the 512 registers of a lane
// allow: estimate = row pieces + accumulators + coefficient operands + ring + addressing and temporaries.
constexpr int full_step_regs(int CH, int W, int KT2, int RT, int RD) {
  return RT * CH * 4 * W + 2 * KT2 * RT * 4 + RT * KT2 * 12 + RD * 8 + (W == 2 ? RT * 8 + 70 : 0) + 46 +
         (KT2 == 4 ? 40 : 0);
}
constexpr int tile_rows(int CH, int W, int KT2) {
  if (CH == 24 && W == 1) return KT2 == 1 ? 3 : 2;   // measured at 3072 channels (FLUX, HunyuanVideo)
  for (int rt = 4; rt > 1; --rt)   // 2 KT2 rt <= 16: the reduction buffer (4 KB per accumulator) stays within 64 KB of LDS
    if (full_step_regs(CH, W, KT2, rt, 8) <= 450 && 2 * KT2 * rt <= 16) return rt;
  return 1;
}
constexpr int ring_depth(int CH, int W, int KT2) {
  const int rt = tile_rows(CH, W, KT2);
  int rd = KT2 == 1 ? 12 : (KT2 == 2 ? 16 : 8);   // measured best at 3072 channels
  if (CH == 24 && W == 1) return rd;
  while (rd > 2 && full_step_regs(CH, W, KT2, rt, rd) > 478) rd -= 2;
  return rd;
}

// A launch with fewer tiles than compute units leaves units idle: such small problems take tiles one step
// smaller (their packed-basis traffic does not matter at that size).
template <typename T, int CH, int KT2, bool SPLIT>
int32_t full_step_by_size(const svdc_shape& s, const void* F, const void* packed, void* R, float* S, float* C,
                          float alpha, int init, ResidualEma re, hipStream_t st) {
  constexpr int W = sizeof(T) == 4 ? 2 : 1;
  constexpr int RT = tile_rows(CH, W, KT2), RD = ring_depth(CH, W, KT2);
  // the variant that also smooths the residual keeps a few chunks of the previous residual in flight: one row
  // tile less
  if (re.prev) return full_step_launch<T, CH, (RT > 1 ? RT - 1 : 1), KT2, SPLIT, RD, true>(s, F, packed, R, S, C, alpha, init, re, st);
  // bf16 at 3072 channels, rank 33..64: a third row tile in LDS.  Measured at the HunyuanVideo shape: 4 % (split
  // operands) to 8 % (single operands) less time per launch, 8-10 % on a single 18432-row block.  At rank <= 32 the
  // packed-basis stream is small enough that a fourth tile gains nothing, at rank 128 the LDS tile only replaces
  // the second register tile at equal speed.  A taller tile can leave more of the last round of the persistent
  // grid empty, so the choice compares rounds x tile height x cost per row (0.92 of the register-only tile's).
  if constexpr (CH == 24 && W == 1 && KT2 == 2) {
    constexpr int RDL = SPLIT ? 12 : 16;
    const int64_t cus = num_compute_units();
    auto tile_count = [&](int ra) { return (int64_t)((s.N + 16 * ra - 1) / (16 * ra)) * s.B; };
    auto rounds = [&](int ra) { return (double)((tile_count(ra) + cus - 1) / cus); };
    if (tile_count(RT + 1) >= cus && rounds(RT + 1) * (RT + 1) * 0.92 <= rounds(RT) * RT)
      return full_step_launch<T, CH, RT, KT2, SPLIT, RDL, false, 1>(s, F, packed, R, S, C, alpha, init, re, st);
  }
  if constexpr (RT > 1) {
    const int64_t tiles = (int64_t)((s.N + 16 * RT - 1) / (16 * RT)) * s.B;
    if (tiles < num_compute_units())
      return full_step_launch<T, CH, RT - 1, KT2, SPLIT, RD, false>(s, F, packed, R, S, C, alpha, init, re, st);
  }
  return full_step_launch<T, CH, RT, KT2, SPLIT, RD, false>(s, F, packed, R, S, C, alpha, init, re, st);
}

template <typename T, int CH, bool SPLIT>
int32_t full_step_by_rank(const svdc_shape& s, const void* F, const void* packed, void* R, float* S, float* C,
                          float alpha, int init, ResidualEma re, hipStream_t st) {
  const int kp = padded_rank(s.k);
  if (kp == 32) return full_step_by_size<T, CH, 1, SPLIT>(s, F, packed, R, S, C, alpha, init, re, st);
  if (kp == 64) return full_step_by_size<T, CH, 2, SPLIT>(s, F, packed, R, S, C, alpha, init, re, st);
  return full_step_by_size<T, CH, 4, SPLIT>(s, F, packed, R, S, C, alpha, init, re, st);
}

template <typename T, bool SPLIT>
int32_t full_step_by_width(const svdc_shape& s, const void* F, const void* packed, void* R, float* S, float* C,
                           float alpha, int init, ResidualEma re, hipStream_t st) {
  switch (s.D / 128) {
    case 2: return full_step_by_rank<T, 2, SPLIT>(s, F, packed, R, S, C, alpha, init, re, st);
    case 4: return full_step_by_rank<T, 4, SPLIT>(s, F, packed, R, S, C, alpha, init, re, st);
    case 8: return full_step_by_rank<T, 8, SPLIT>(s, F, packed, R, S, C, alpha, init, re, st);
    case 9: return full_step_by_rank<T, 9, SPLIT>(s, F, packed, R, S, C, alpha, init, re, st);
    case 12: return full_step_by_rank<T, 12, SPLIT>(s, F, packed, R, S, C, alpha, init, re, st);
    case 15: return full_step_by_rank<T, 15, SPLIT>(s, F, packed, R, S, C, alpha, init, re, st);
    case 16: return full_step_by_rank<T, 16, SPLIT>(s, F, packed, R, S, C, alpha, init, re, st);
    case 20: return full_step_by_rank<T, 20, SPLIT>(s, F, packed, R, S, C, alpha, init, re, st);
    case 24: return full_step_by_rank<T, 24, SPLIT>(s, F, packed, R, S, C, alpha, init, re, st);
    case 32: return full_step_by_rank<T, 32, SPLIT>(s, F, packed, R, S, C, alpha, init, re, st);
    case 40: return full_step_by_rank<T, 40, SPLIT>(s, F, packed, R, S, C, alpha, init, re, st);
    default: return SVDC_E_SHAPE;
  }
}

}  // namespace

int32_t launch_full_step_mfma(const svdc_shape& s, const void* F, const void* packed, void* R, float* S,
                              float* C, float alpha, int init, ResidualEma re, hipStream_t st) {
  // float32 features always use the full operand split (a single bf16 operand would cost 8 of their 24 bits)
  if (s.dtype == SVDC_F32) return full_step_by_width<float, true>(s, F, packed, R, S, C, alpha, init, re, st);
  return s.precision == SVDC_PRECISE
             ? full_step_by_width<bf16_t, true>(s, F, packed, R, S, C, alpha, init, re, st)
             : full_step_by_width<bf16_t, false>(s, F, packed, R, S, C, alpha, init, re, st);
}

namespace {

template <bool EXT, bool PS = false>
int32_t forecast_dispatch(const svdc_shape& s, const CoefStates& cs, const void* packed, const void* R,
                          const void* X, void* Fhat, hipStream_t st) {
  const int kp = padded_rank(s.k);
  if (s.dtype == SVDC_F32) {
    if (kp == 32) return forecast_by_width<float, 1, true, 1, EXT, PS>(s, cs, packed, R, X, Fhat, st);
    if (kp == 64) return forecast_by_width<float, 2, true, 2, EXT, PS>(s, cs, packed, R, X, Fhat, st);
    return forecast_by_width<float, 4, true, 2, EXT, PS>(s, cs, packed, R, X, Fhat, st);
  }
  if (s.precision == SVDC_PRECISE) {
    if (kp == 32) return forecast_by_width<bf16_t, 1, true, 1, EXT, PS>(s, cs, packed, R, X, Fhat, st);
    // at rank 64 the matrix-core time per tile is no longer small next to its memory time: more tiles in flight
    if (kp == 64) return forecast_by_width<bf16_t, 2, true, (EXT ? 2 : 4), EXT, PS>(s, cs, packed, R, X, Fhat, st);
    return forecast_by_width<bf16_t, 4, true, 2, EXT, PS>(s, cs, packed, R, X, Fhat, st);
  }
  // at rank <= 32 the split-operand kernel is the faster one (its matrix-core work is hidden anyway)
  if (kp == 32) return forecast_by_width<bf16_t, 1, true, 1, EXT, PS>(s, cs, packed, R, X, Fhat, st);
  if (kp == 64) return forecast_by_width<bf16_t, 2, false, 2, EXT, PS>(s, cs, packed, R, X, Fhat, st);
  return forecast_by_width<bf16_t, 4, false, 2, EXT, PS>(s, cs, packed, R, X, Fhat, st);
}

}  // namespace

int32_t launch_forecast_mfma(const svdc_shape& s, const float* S, const void* packed, const void* R,
                             void* Fhat, hipStream_t st) {
  CoefStates cs{};
  cs.s[0] = S;
  cs.w[0] = 1.f;
  cs.m = 1;
  return forecast_dispatch<false>(s, cs, packed, R, nullptr, Fhat, st);
}

int32_t launch_forecast_combine_mfma(const svdc_shape& s, const CoefStates& cs, const void* packed, const void* R,
                                     const void* X, void* Out, hipStream_t st) {
  return forecast_dispatch<true>(s, cs, packed, R, X, Out, st);
}

size_t mfma_packed_state_bytes(const svdc_shape& s) {
  return (size_t)s.B * ((size_t)(s.N + 15) / 16) * (padded_rank(s.k) / 32) * 2 * 1024;
}

int32_t launch_pack_state(const svdc_shape& s, const float* S, void* Sp, hipStream_t st) {
  const int KT2 = padded_rank(s.k) / 32;
  const int64_t words = (int64_t)((s.N + 15) / 16) * KT2;
  dim3 grid((unsigned)((words + kWavesPerGroup - 1) / kWavesPerGroup), s.B);
  pack_state_kernel<<<grid, 256, 0, st>>>(S, (u32x4*)Sp, s.N, s.k, KT2, words);
  return launch_status();
}

int32_t launch_forecast_packed_mfma(const svdc_shape& s, const void* Sp, const void* packed, const void* R,
                                    void* Fhat, hipStream_t st) {
  CoefStates cs{};
  cs.s[0] = static_cast<const float*>(Sp);   // the kernel reads it as operand words
  cs.w[0] = 1.f;
  cs.m = 1;
  return forecast_dispatch<false, true>(s, cs, packed, R, nullptr, Fhat, st);
}

}  // namespace svdc
