// Basis fit (Sec. 3.2, Eq. 4-5): the k leading right singular vectors of F by
// randomized subspace iteration followed by a Rayleigh-Ritz step.
//
//   Q <- Omega                             Omega: D x l Gaussian, l = k + p
//   repeat q times:  Y = F Q;  Z = F^T Y;  Q <- orth(Z)       (one application of F^T F)
//   Y = F Q;  H = Y^T Y = L L^T;  L = W diag(sigma) X^T       (one-sided Jacobi on L, fp64: H = W diag(sigma^2) W^T)
//   V_k = Q W[:, :k],  sigma_k = sigma[:k]
//
// orth() is CholeskyQR applied twice; every l x l object (Gram matrices, Cholesky
// factors, Jacobi rotations) is float64 because Z = F^T F Q has the squared
// condition number of F's leading part and its Gram matrix squares it again.
// The tall matrices Q, Z (D x l) and Y (N x l) are float32.
//
// This file holds the small-matrix kernels, the host orchestration and the general (vector-ALU) versions of the two
// products with F; their matrix-core versions are in fit_mfma_kernels.hip.
#include <algorithm>
#include <utility>

#include <type_traits>

#include "svdc_device.h"
#include "svdc_internal.h"

namespace svdc {

// ---------------------------------------------------------------------------
// counter-based Gaussian test matrix
// ---------------------------------------------------------------------------
__device__ __forceinline__ uint64_t mix64(uint64_t x) {
  // 64-bit finaliser (xor-shift-multiply rounds); statistically adequate for a sketch matrix
  x ^= x >> 30; x *= 0xbf58476d1ce4e5b9ull;
  x ^= x >> 27; x *= 0x94d049bb133111ebull;
  x ^= x >> 31;
  return x;
}

__global__ void init_omega_kernel(float* Q, int64_t per_block, int64_t total, uint64_t seed) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= total) return;
  const uint64_t h = mix64(seed * 0x9e3779b97f4a7c15ull + (uint64_t)i + 1);
  const uint32_t a = (uint32_t)h, c = (uint32_t)(h >> 32);
  const float u1 = ((float)(a >> 8) + 0.5f) * (1.0f / 16777216.0f);   // (0,1)
  const float u2 = ((float)(c >> 8) + 0.5f) * (1.0f / 16777216.0f);
  Q[i] = sqrtf(-2.0f * __logf(u1)) * __cosf(6.283185307179586f * u2);  // Box-Muller
  (void)per_block;
}

__global__ void fill_zero_kernel(double* p, int64_t n) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0.0;
}
__global__ void fill_zero_f32_kernel(float* p, int64_t n) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0.f;
}

// ---------------------------------------------------------------------------
// products with F (general fp32 version)
//   TRANS = false:  Out[N x l]  = F[N x D] * Bm[D x l]
//   TRANS = true :  Out[D x l] += F^T      * Bm[N x l]   (rows of F split over grid.z, atomic accumulate)
// 64 x 64 output tile per workgroup, 4 x 4 per thread, 16-deep steps through LDS.
// ---------------------------------------------------------------------------
template <typename T, bool TRANS>
__global__ __launch_bounds__(256) void fit_gemm_kernel(const T* __restrict__ F, const float* __restrict__ Bm,
                                                       float* Out, int N, int D, int l, int64_t ldf,
                                                       int64_t bstride, int ksplit_len, int nsplit) {
  __shared__ float As[16][64 + 4];
  __shared__ float Bs[16][64 + 4];
  const int b = blockIdx.z / nsplit, split = blockIdx.z % nsplit;
  const int M = TRANS ? D : N, K = TRANS ? N : D;
  const int m0 = blockIdx.x * 64, j0 = blockIdx.y * 64;
  const int kbeg = split * ksplit_len, kend = min(K, kbeg + ksplit_len);
  const T* f = F + (int64_t)b * bstride;
  const float* bm = Bm + (int64_t)b * K * l;
  float* out = Out + (int64_t)b * M * l;
  const int t = threadIdx.x, tx = t & 15, ty = t >> 4;
  float acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = 0.f;

  for (int k0 = kbeg; k0 < kend; k0 += 16) {
    if (!TRANS) {
      const int m = t >> 2, kk = (t & 3) * 4;
      const int64_t row = m0 + m;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int kidx = k0 + kk + e;
        As[kk + e][m] = (row < M && kidx < kend) ? ld_elem(f, row * ldf + kidx) : 0.f;
      }
    } else {
      const int kk = t >> 4, m = (t & 15) * 4;
      const int64_t n = k0 + kk;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int d = m0 + m + e;
        As[kk][m + e] = (n < kend && d < M) ? ld_elem(f, n * ldf + d) : 0.f;
      }
    }
    {
      const int kk = t >> 4, j = (t & 15) * 4;
      const int64_t kidx = k0 + kk;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int col = j0 + j + e;
        Bs[kk][j + e] = (kidx < kend && col < l) ? bm[kidx * l + col] : 0.f;
      }
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < 16; ++kk) {
      float a[4], bb[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) a[i] = As[kk][ty * 4 + i];
#pragma unroll
      for (int j = 0; j < 4; ++j) bb[j] = Bs[kk][tx * 4 + j];
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] += a[i] * bb[j];
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int64_t row = m0 + ty * 4 + i;
    if (row >= M) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int col = j0 + tx * 4 + j;
      if (col >= l) continue;
      if (TRANS) atomicAdd(&out[row * l + col], acc[i][j]);
      else out[row * l + col] = acc[i][j];
    }
  }
}

// ---------------------------------------------------------------------------
// 64 x 64 x (4 K4) float64 product on the matrix cores (v_mfma_f64_16x16x4_f64), shared by the Gram matrices and the
// small tile products below.  Both operands sit in LDS with the contraction index as the row:
//   As[k][i] (row stride LDA), Bs[k][j] (row stride LDB),  acc += sum_k As[k][i] * Bs[k][j].
// Wave w of four takes the 32 x 32 quadrant (w / 2, w % 2) as 2 x 2 tiles of 16 x 16.  Lane layout of the
// instruction (checked on the device with one-hot operands):
//   A operand: lane -> A[i = lane % 16][k = lane / 16]        B operand: lane -> B[k = lane / 16][j = lane % 16]
//   D: lane, v  -> D[i = 4 v + lane / 16][j = lane % 16]
// so a lane reads As[4 k4 + lane / 16][i0 + lane % 16]: 16 consecutive doubles per group of 16 lanes, and with a row
// stride of 80 doubles the two groups of a half wave fall into different halves of the LDS banks.
// ---------------------------------------------------------------------------
typedef double f64x4 __attribute__((ext_vector_type(4)));
constexpr int kM64Stride = 80;

struct Quadrant {
  int i0, j0, m, kq;   // first row / column of the wave's quadrant, lane % 16, lane / 16
  __device__ __forceinline__ Quadrant() {
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    i0 = 32 * (wave >> 1); j0 = 32 * (wave & 1); m = lane & 15; kq = lane >> 4;
  }
  // row and column (inside the 64 x 64 tile) of element v of accumulator tile (a, b)
  __device__ __forceinline__ int row(int a, int v) const { return i0 + 16 * a + 4 * v + kq; }
  __device__ __forceinline__ int col(int b) const { return j0 + 16 * b + m; }
};

template <int K4>
__device__ __forceinline__ void mfma64_accumulate(const double* As, const double* Bs, const Quadrant& q,
                                                  f64x4 (&acc)[2][2]) {
#pragma unroll
  for (int k4 = 0; k4 < K4; ++k4) {
    const double* ar = As + (4 * k4 + q.kq) * kM64Stride + q.i0 + q.m;
    const double* br = Bs + (4 * k4 + q.kq) * kM64Stride + q.j0 + q.m;
    const double a0 = ar[0], a1 = ar[16], b0 = br[0], b1 = br[16];
    acc[0][0] = __builtin_amdgcn_mfma_f64_16x16x4f64(a0, b0, acc[0][0], 0, 0, 0);
    acc[0][1] = __builtin_amdgcn_mfma_f64_16x16x4f64(a0, b1, acc[0][1], 0, 0, 0);
    acc[1][0] = __builtin_amdgcn_mfma_f64_16x16x4f64(a1, b0, acc[1][0], 0, 0, 0);
    acc[1][1] = __builtin_amdgcn_mfma_f64_16x16x4f64(a1, b1, acc[1][1], 0, 0, 0);
  }
}

// ---------------------------------------------------------------------------
// Partial Gram matrices A^T A in float64, A float32 [rows x l]; rows split over grid.x, 64 x 64 tiles of the lower
// block triangle (tile row >= tile column) over grid.y: the factorisation that follows never reads the rest.
// 16 rows per step, staged in LDS as float64 (each value converted once); the next step's rows are fetched into
// registers while the current ones are multiplied.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void gram_f64_kernel(const float* __restrict__ A, double* G, int rows, int l,
                                                       int rows_per_slice) {
  __shared__ double Ai[16 * kM64Stride];
  __shared__ double Aj[16 * kM64Stride];
  const int b = blockIdx.z;
  int ti = 0;
  while ((ti + 1) * (ti + 2) / 2 <= (int)blockIdx.y) ++ti;
  const int tj = blockIdx.y - ti * (ti + 1) / 2;
  const float* a = A + (int64_t)b * rows * l;
  double* g = G + ((int64_t)b * gridDim.x + blockIdx.x) * l * l;   // partial Gram matrix of this row slice
  const int t = threadIdx.x;
  const int rbeg = blockIdx.x * rows_per_slice, rend = min(rows, rbeg + rows_per_slice);
  const Quadrant q;
  f64x4 acc[2][2];
#pragma unroll
  for (int x = 0; x < 2; ++x)
#pragma unroll
    for (int y = 0; y < 2; ++y) acc[x][y] = f64x4{0.0, 0.0, 0.0, 0.0};
  const bool vec = (l & 3) == 0;
  const int rr = t >> 4, c = (t & 15) * 4;
  const int ci = ti * 64 + c, cj = tj * 64 + c;
  float vi[4], vj[4];
  auto fetch = [&](int r0) {
    const int64_t r = r0 + rr;
#pragma unroll
    for (int e = 0; e < 4; ++e) { vi[e] = 0.f; vj[e] = 0.f; }
    if (r < rend) {
      if (vec) {
        if (ci < l) *reinterpret_cast<float4*>(vi) = *reinterpret_cast<const float4*>(a + r * l + ci);
        if (cj < l) *reinterpret_cast<float4*>(vj) = *reinterpret_cast<const float4*>(a + r * l + cj);
      } else {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          if (ci + e < l) vi[e] = a[r * l + ci + e];
          if (cj + e < l) vj[e] = a[r * l + cj + e];
        }
      }
    }
  };
  if (rbeg < rend) fetch(rbeg);
  for (int r0 = rbeg; r0 < rend; r0 += 16) {
    if (r0 > rbeg) __syncthreads();             // the previous step has been read by everybody
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      Ai[rr * kM64Stride + c + e] = (double)vi[e];
      Aj[rr * kM64Stride + c + e] = (double)vj[e];
    }
    __syncthreads();
    if (r0 + 16 < rend) fetch(r0 + 16);
    mfma64_accumulate<4>(Ai, Aj, q, acc);
  }
#pragma unroll
  for (int x = 0; x < 2; ++x)
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      const int gi = ti * 64 + q.row(x, v);
      if (gi >= l) continue;
#pragma unroll
      for (int y = 0; y < 2; ++y) {
        const int gj = tj * 64 + q.col(y);
        if (gj < l) g[(int64_t)gi * l + gj] = acc[x][y][v];
      }
    }
}

// G[b] = sum over the row slices of the partial Gram matrices, in slice order (no atomics: the same bits every run);
// lower block triangle only, like the partial matrices
__global__ __launch_bounds__(256) void gram_reduce_kernel(const double* __restrict__ part, double* G, int nslice,
                                                          int l) {
  const int b = blockIdx.y;
  const int64_t ll = (int64_t)l * l;
  const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (e >= ll || (e % l) / 64 > (e / l) / 64) return;
  const double* p = part + (int64_t)b * nslice * ll + e;
  double s = 0.0;
  for (int i = 0; i < nslice; ++i) s += p[(int64_t)i * ll];
  G[(int64_t)b * ll + e] = s;
}

// A pivot of the Cholesky factorisation below kRankTol x the largest diagonal entry of the Gram matrix means that a
// column of the sketch depends on the others to within (1e-6)^2, the round-off of the float32 sketch itself: the
// matrix has numerical rank < l.  The shift keeps the factorisation going (the result stays orthonormal, directions
// beyond the numerical rank are arbitrary) and the block's status word reports it.
constexpr double kRankTol = 1e-12;

// ---------------------------------------------------------------------------
// Register-blocked Cholesky factor for l <= 64, factor only: thread (ti, tj) of a 16 x 16 grid owns the 4 x 4 block
// (ti, tj) of the matrix in registers; a wave owns four block columns.  Right-looking by panels of 4 columns (one
// block column), two barriers per panel:
//   the thread on the diagonal factors its 4 x 4 block and publishes it,
//   the threads below it in the block column (the same wave) solve their blocks against it, X = B L_d^-T, and publish
//   the panel (64 rows x 4),
//   every thread below or on the diagonal and right of the panel subtracts the rank-4 product of the panel rows of
//   its block row and of its block column.
// (One column at a time, with the column published through LDS and a barrier per column, took three times as long:
// the per-column chain of barrier, pivot, reciprocal square root and rank-1 update is what costs, not the flops.)
//   G      in/out  [l x l] at row stride ld, block b at G + b * bstride: lower triangle = L with
//                  G + shift I = L L^T, upper triangle zeroed
//   rdiag  out     (nullable) 1 / L[i][i], block b at rdiag + b * rd_bstride
// The matrix may be a diagonal block of a larger one that is factored block by block (see chol_panel_kernel).
// ChoShift tells every step which shift to use: the first computes it from the whole diagonal, diag_n >= l
// entries, and stores it; the later ones, diag_n = 0, read it.  A later block is A_kk - L_k L_k^T with L_k the ku
// finished columns of its rows, given transposed: Ut [ku x l] at row stride ldut.
// ---------------------------------------------------------------------------
struct ChoShift {
  double* slot;        // per block (stride slot_bstride): the shift, written when diag_n > 0, read otherwise
  int64_t slot_bstride;
  int diag_n;          // diagonal entries of G (same ld) that define the shift
};
struct ChoUpdate {
  const double* Ut;    // nullable
  int64_t bstride;
  int ldut, ku;
};

template <int BS>
__global__ __launch_bounds__(256) void chol_reg_kernel(double* G, int64_t bstride, int ld, double* rdiag,
                                                       int64_t rd_bstride, int l, double rel_shift, int32_t* info,
                                                       ChoShift sh, ChoUpdate up) {
  static_assert(BS == 4, "4 x 4 blocks");
  constexpr int LM = 16 * BS;          // padded matrix size
  __shared__ double panel[LM][BS];     // the current block column of L, rows below its diagonal block
  __shared__ double dblk[BS][BS];      // its diagonal block: strict lower part, reciprocals of the diagonal on the diagonal
  __shared__ double s_shift;
  const int b = blockIdx.x, t = threadIdx.x, tj = t >> 4, ti = t & 15;
  double* g = G + (int64_t)b * bstride;
  if (t < kWave) {
    if (sh.diag_n > 0) {
      double mx = 0.0;
      for (int i = t; i < sh.diag_n; i += kWave) mx = fmax(mx, g[(int64_t)i * ld + i]);
#pragma unroll
      for (int o = 32; o > 0; o >>= 1) mx = fmax(mx, __shfl_xor(mx, o, kWave));
      if (t == 0) {
        s_shift = mx * rel_shift;
        if (sh.slot) sh.slot[(int64_t)b * sh.slot_bstride] = mx * rel_shift;
      }
    } else if (t == 0) {
      s_shift = sh.slot[(int64_t)b * sh.slot_bstride];
    }
  }
  __syncthreads();
  double a[BS][BS];
#pragma unroll
  for (int ii = 0; ii < BS; ++ii)
#pragma unroll
    for (int jj = 0; jj < BS; ++jj) {
      const int i = BS * ti + ii, j = BS * tj + jj;
      double v = (i < l && j < l) ? g[(int64_t)i * ld + j] : (i == j ? 1.0 : 0.0);   // identity padding
      if (i == j && i < l) v += s_shift;
      a[ii][jj] = v;
    }
  if (up.Ut && ti >= tj) {   // a -= L21 L21^T, from the transposed factor (rows of Ut are contiguous over i)
    const double* ut = up.Ut + (int64_t)b * up.bstride;
#pragma unroll 8
    for (int kk = 0; kk < up.ku; ++kk) {   // ku is a multiple of 64; unrolled so that the loads of several steps are in flight
      double ui[BS], uj[BS];
#pragma unroll
      for (int ii = 0; ii < BS; ++ii) ui[ii] = (BS * ti + ii < l) ? ut[(int64_t)kk * up.ldut + BS * ti + ii] : 0.0;
#pragma unroll
      for (int jj = 0; jj < BS; ++jj) uj[jj] = (BS * tj + jj < l) ? ut[(int64_t)kk * up.ldut + BS * tj + jj] : 0.0;
#pragma unroll
      for (int ii = 0; ii < BS; ++ii)
#pragma unroll
        for (int jj = 0; jj < BS; ++jj) a[ii][jj] -= ui[ii] * uj[jj];
    }
  }
  const double pivot_floor = s_shift * (kRankTol / rel_shift);
  bool dependent = false;
  const int nbk = (l + BS - 1) / BS;
  for (int cb = 0; cb < nbk; ++cb) {
    if (ti == cb && tj == cb) {        // factor the diagonal block in place (lower part), publish it
#pragma unroll
      for (int q = 0; q < BS; ++q) {
        dependent |= (BS * cb + q < l) && a[q][q] < pivot_floor;
        const double piv2 = fmax(a[q][q], 1e-300);
        // 1 / sqrt(piv2): hardware estimate refined by two Newton steps (an exact sqrt and a division per
        // column would dominate this kernel)
        double rs = __builtin_amdgcn_rsq(piv2);
        rs = rs * (1.5 - 0.5 * piv2 * rs * rs);
        rs = rs * (1.5 - 0.5 * piv2 * rs * rs);
        a[q][q] = piv2 * rs;
        dblk[q][q] = rs;
#pragma unroll
        for (int i = q + 1; i < BS; ++i) {
          a[i][q] *= rs;
          dblk[i][q] = a[i][q];
        }
#pragma unroll
        for (int j = q + 1; j < BS; ++j)
#pragma unroll
          for (int i = j; i < BS; ++i) a[i][j] -= a[i][q] * a[j][q];
      }
    }
    __syncthreads();
    if (tj == cb && ti > cb) {         // X = B L_d^-T, row by row; publish the panel
      const double r0 = dblk[0][0], r1 = dblk[1][1], r2 = dblk[2][2], r3 = dblk[3][3];
      const double l10 = dblk[1][0], l20 = dblk[2][0], l21 = dblk[2][1], l30 = dblk[3][0], l31 = dblk[3][1],
                   l32 = dblk[3][2];
#pragma unroll
      for (int ii = 0; ii < BS; ++ii) {
        const double x0 = a[ii][0] * r0;
        const double x1 = (a[ii][1] - x0 * l10) * r1;
        const double x2 = (a[ii][2] - x0 * l20 - x1 * l21) * r2;
        const double x3 = (a[ii][3] - x0 * l30 - x1 * l31 - x2 * l32) * r3;
        a[ii][0] = x0; a[ii][1] = x1; a[ii][2] = x2; a[ii][3] = x3;
        panel[BS * ti + ii][0] = x0; panel[BS * ti + ii][1] = x1;
        panel[BS * ti + ii][2] = x2; panel[BS * ti + ii][3] = x3;
      }
    }
    __syncthreads();
    if (tj > cb && ti >= tj) {         // rank-4 update of the blocks right of the panel
      double pi[BS][BS], pj[BS][BS];
#pragma unroll
      for (int ii = 0; ii < BS; ++ii)
#pragma unroll
        for (int q = 0; q < BS; ++q) {
          pi[ii][q] = panel[BS * ti + ii][q];
          pj[ii][q] = panel[BS * tj + ii][q];
        }
#pragma unroll
      for (int ii = 0; ii < BS; ++ii)
#pragma unroll
        for (int jj = 0; jj < BS; ++jj)
#pragma unroll
          for (int q = 0; q < BS; ++q) a[ii][jj] -= pi[ii][q] * pj[jj][q];
    }
  }
#pragma unroll
  for (int ii = 0; ii < BS; ++ii)
#pragma unroll
    for (int jj = 0; jj < BS; ++jj) {
      const int i = BS * ti + ii, j = BS * tj + jj;
      const double v = (j <= i) ? a[ii][jj] : 0.0;
      if (i < l && j < l) g[(int64_t)i * ld + j] = v;
      if (rdiag && i == j && i < l) rdiag[(int64_t)b * rd_bstride + i] = 1.0 / v;
    }
  // every thread on the diagonal has seen the pivots of its own block
  if (info && dependent) atomicOr(info + b, SVDC_FIT_RANK_DEFICIENT);
}

// ---------------------------------------------------------------------------
// 64 x 64 tile of a product A[64 x K] (float32 rows) * Bm[K x 64] (float64), accumulated in float64 on the matrix
// cores by one workgroup of 256 threads (mfma64_accumulate).  The inner dimension is walked in chunks of 32 staged in
// LDS as float64, A transposed to [k][r]; the next chunk's elements are fetched into registers before the current one
// is multiplied, so their latency is hidden behind the arithmetic.
//   load_a(r, k)  element (r, k) of A, 0 outside        load_b(k, j)  element (k, j) of Bm, 0 outside
//   emit(r, j, x) called for every element (r, j) of the tile that this lane holds
// ---------------------------------------------------------------------------
constexpr int kTileK = 32;
struct TileGemmLds {
  double Bs[kTileK * kM64Stride];          // [k][j]
  double As[kTileK * (kM64Stride + 1)];    // [k][r], odd stride: the transposing stores of a wave spread over the banks
};

template <typename LoadA, typename LoadB, typename Emit>
__device__ __forceinline__ void tile_gemm_64x64(int K, LoadA load_a, LoadB load_b, TileGemmLds& lds, Emit emit) {
  constexpr int LA = kM64Stride + 1;
  const int t = threadIdx.x;
  // staging role of this thread: 8 elements of each operand per chunk
  const int ar = t >> 5, ak = t & 31;          // A: rows ar + 8 e, column ak
  const int bk = t >> 6, bj = t & 63;          // B: rows bk + 4 e, column bj
  float ra[8];
  double rb[8];
  auto fetch = [&](int k0) {
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      ra[e] = load_a(ar + 8 * e, k0 + ak);
      rb[e] = load_b(k0 + bk + 4 * e, bj);
    }
  };
  const Quadrant q;
  f64x4 acc[2][2];
#pragma unroll
  for (int x = 0; x < 2; ++x)
#pragma unroll
    for (int y = 0; y < 2; ++y) acc[x][y] = f64x4{0.0, 0.0, 0.0, 0.0};
  fetch(0);
  for (int k0 = 0; k0 < K; k0 += kTileK) {
    if (k0 > 0) __syncthreads();               // the previous chunk has been read by everybody
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      lds.As[ak * LA + ar + 8 * e] = (double)ra[e];
      lds.Bs[(bk + 4 * e) * kM64Stride + bj] = rb[e];
    }
    __syncthreads();
    if (k0 + kTileK < K) fetch(k0 + kTileK);
#pragma unroll
    for (int k4 = 0; k4 < kTileK / 4; ++k4) {
      const double* arow = lds.As + (4 * k4 + q.kq) * LA + q.i0 + q.m;
      const double* brow = lds.Bs + (4 * k4 + q.kq) * kM64Stride + q.j0 + q.m;
      const double a0 = arow[0], a1 = arow[16], b0 = brow[0], b1 = brow[16];
      acc[0][0] = __builtin_amdgcn_mfma_f64_16x16x4f64(a0, b0, acc[0][0], 0, 0, 0);
      acc[0][1] = __builtin_amdgcn_mfma_f64_16x16x4f64(a0, b1, acc[0][1], 0, 0, 0);
      acc[1][0] = __builtin_amdgcn_mfma_f64_16x16x4f64(a1, b0, acc[1][0], 0, 0, 0);
      acc[1][1] = __builtin_amdgcn_mfma_f64_16x16x4f64(a1, b1, acc[1][1], 0, 0, 0);
    }
  }
#pragma unroll
  for (int x = 0; x < 2; ++x)
#pragma unroll
    for (int v = 0; v < 4; ++v)
#pragma unroll
      for (int y = 0; y < 2; ++y) emit(q.row(x, v), q.col(y), acc[x][y][v]);
}

// ---------------------------------------------------------------------------
// Out[rows x m] (float32) = In[rows x l] (float32) * M[l x m] (float64, row stride ldm), 64 x 64 tiles.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void rows_times_small_kernel(const float* __restrict__ In,
                                                               const double* __restrict__ M, float* Out,
                                                               int rows, int l, int m, int ldm) {
  __shared__ TileGemmLds lds;
  const int b = blockIdx.z;
  const float* in = In + (int64_t)b * rows * l;
  const double* mm = M + (int64_t)b * l * ldm;
  float* out = Out + (int64_t)b * rows * m;
  const int r0 = blockIdx.x * 64, j0 = blockIdx.y * 64;
  tile_gemm_64x64(
      l, [&](int r, int k) { return (r0 + r < rows && k < l) ? in[(int64_t)(r0 + r) * l + k] : 0.f; },
      [&](int k, int j) { return (k < l && j0 + j < m) ? mm[(int64_t)k * ldm + j0 + j] : 0.0; }, lds,
      [&](int r, int j, double x) {
        if (r0 + r < rows && j0 + j < m) out[(int64_t)(r0 + r) * m + j0 + j] = (float)x;
      });
}

// ---------------------------------------------------------------------------
// Out = In * L^-T by forward substitution, one thread per row:
//   q_j = (z_j - sum_{i<j} q_i L[j][i]) / L[j][j]
// L (float64 Cholesky factor, lower) and the reciprocals of its diagonal are read
// from LDS as broadcasts; the row lives in registers.  l <= LMAX <= 64: wider factors are applied block by block
// (cholqr_apply).
// The l columns may be a column range of wider rows (row stride ld_io, In and Out already offset to the range's
// first column) and L a diagonal block of a larger factor (row stride ldl, block b at Lfac + b * l_bstride).  In may
// be the same buffer as Out: a thread reads its whole row before it writes.
// ---------------------------------------------------------------------------
template <int LMAX>
__global__ __launch_bounds__(256) void tri_solve_rows_kernel(const float* In, const double* __restrict__ Lfac,
                                                             const double* __restrict__ rdiag, float* Out,
                                                             int rows, int l, int ld_io, int ldl,
                                                             int64_t l_bstride, int64_t rd_bstride) {
  const int b = blockIdx.y, t = threadIdx.x;
  // every thread reads the same element of L at the same time: the factor is staged in LDS and read as
  // broadcasts (as scalar loads its 32 KB at l = 64 overflow the scalar cache)
  __shared__ double Lf[LMAX * LMAX];
  __shared__ double rd[LMAX];
  // rows of L at a compile-time stride: every LDS offset below is then a constant and neighbouring elements of a
  // row are fetched by one wide read
  for (int e = t; e < l * l; e += 256) Lf[(e / l) * LMAX + e % l] = Lfac[(int64_t)b * l_bstride + (int64_t)(e / l) * ldl + e % l];
  if (t < l) rd[t] = rdiag[(int64_t)b * rd_bstride + t];
  __syncthreads();
  const int64_t row = (int64_t)blockIdx.x * 256 + t;
  if (row >= rows) return;
  const float* in = In + ((int64_t)b * rows + row) * ld_io;
  float* out = Out + ((int64_t)b * rows + row) * ld_io;
  double q[LMAX];
  const bool vec = ((l | ld_io) & 3) == 0;   // rows (and column ranges that start at a multiple of 4) are then 16-byte aligned
  if (vec) {
#pragma unroll
    for (int j = 0; j < LMAX; j += 4) {
      float4 x = make_float4(0.f, 0.f, 0.f, 0.f);
      if (j < l) x = *reinterpret_cast<const float4*>(in + j);
      q[j] = x.x; q[j + 1] = x.y; q[j + 2] = x.z; q[j + 3] = x.w;
    }
  } else {
#pragma unroll
    for (int j = 0; j < LMAX; ++j) q[j] = (j < l) ? (double)in[j] : 0.0;
  }
#pragma unroll
  for (int j = 0; j < LMAX; ++j) {
    if (j < l) {
      double s = q[j];
#pragma unroll
      for (int i = 0; i < j; ++i) s -= q[i] * Lf[j * LMAX + i];
      q[j] = s * rd[j];
    }
  }
  if (vec) {
#pragma unroll
    for (int j = 0; j < LMAX; j += 4)
      if (j < l) *reinterpret_cast<float4*>(out + j) = make_float4((float)q[j], (float)q[j + 1], (float)q[j + 2], (float)q[j + 3]);
  } else {
#pragma unroll
    for (int j = 0; j < LMAX; ++j)
      if (j < l) out[j] = (float)q[j];
  }
}

// ---------------------------------------------------------------------------
// Blocked Cholesky factorisation for l > 64, left-looking over column blocks of 64: for block k at columns c0..c0+63
//   L_kk = chol(A_kk - sum_{c < c0} L[k, c] L[k, c]^T)                     (chol_reg_kernel with its update)
//   L_ik = (A_ik - sum_{c < c0} L[i, c] L[k, c]^T) L_kk^-T  for rows i below  (this kernel)
// The finished columns are kept twice, as L in the lower triangle and as L^T in the upper one (G[c][r] = L[r][c]):
// every product above then reads rows of the upper triangle, contiguous over the output index.
// A workgroup takes 64 rows of the panel: all 256 threads form the 64 x 64 update (4 x 4 per thread, float64), then
// 64 threads solve one row each against L_kk staged in LDS.
// ---------------------------------------------------------------------------
constexpr int kCholBlock = 64;

__global__ __launch_bounds__(256) void chol_panel_kernel(double* G, const double* __restrict__ rdiag,
                                                         int64_t rd_bstride, int l, int c0) {
  constexpr int H = kCholBlock, LT = H + 1;
  __shared__ double T[H * LT];     // [row][j]
  __shared__ double Lk[H * H];     // [j][i]
  __shared__ double rd[H];
  const int b = blockIdx.y, t = threadIdx.x;
  double* g = G + (int64_t)b * l * l;
  const int r0 = c0 + H + blockIdx.x * H;          // first row of this workgroup
  for (int e = t; e < H * H; e += 256) Lk[e] = g[(int64_t)(c0 + e / H) * l + c0 + e % H];
  if (t < H) rd[t] = rdiag[(int64_t)b * rd_bstride + c0 + t];
  const int ty = t >> 4, tx = t & 15;
  double acc[4][4];
#pragma unroll
  for (int ii = 0; ii < 4; ++ii)
#pragma unroll
    for (int jj = 0; jj < 4; ++jj) acc[ii][jj] = 0.0;
  int ri[4];
#pragma unroll
  for (int ii = 0; ii < 4; ++ii) ri[ii] = min(r0 + 4 * ty + ii, l - 1);
#pragma unroll 8
  for (int c = 0; c < c0; ++c) {
    const double* gc = g + (int64_t)c * l;
    double av[4], bv[4];
#pragma unroll
    for (int ii = 0; ii < 4; ++ii) av[ii] = gc[ri[ii]];
#pragma unroll
    for (int jj = 0; jj < 4; ++jj) bv[jj] = gc[c0 + tx + 16 * jj];
#pragma unroll
    for (int ii = 0; ii < 4; ++ii)
#pragma unroll
      for (int jj = 0; jj < 4; ++jj) acc[ii][jj] += av[ii] * bv[jj];
  }
#pragma unroll
  for (int ii = 0; ii < 4; ++ii)
#pragma unroll
    for (int jj = 0; jj < 4; ++jj)
      T[(4 * ty + ii) * LT + tx + 16 * jj] = g[(int64_t)ri[ii] * l + c0 + tx + 16 * jj] - acc[ii][jj];
  __syncthreads();
  const int row = r0 + t;
  if (t >= H || row >= l) return;
  double q[H];
#pragma unroll
  for (int j = 0; j < H; ++j) q[j] = T[t * LT + j];
#pragma unroll
  for (int j = 0; j < H; ++j) {
    double s = q[j];
#pragma unroll
    for (int i = 0; i < j; ++i) s -= q[i] * Lk[j * H + i];
    q[j] = s * rd[j];
  }
#pragma unroll
  for (int j = 0; j < H; ++j) {
    g[(int64_t)row * l + c0 + j] = q[j];
    g[(int64_t)(c0 + j) * l + row] = q[j];
  }
}

// ---------------------------------------------------------------------------
// Out[:, c0 + j] = In[:, c0 + j] - sum_{c < c0} Out[:, c] * L[c0 + j][c],  j < w: the update step of Out = In L^-T by
// column blocks, between the triangular solves of the blocks (tri_solve_rows_kernel).  L^T is read from the upper
// triangle of G.  A workgroup takes 64 rows x the block's columns (tile_gemm_64x64).
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void rows_minus_product_kernel(const float* __restrict__ In, float* Out,
                                                                 const double* __restrict__ G, int rows, int l,
                                                                 int c0, int w) {
  __shared__ TileGemmLds lds;
  const int b = blockIdx.y;
  const float* in = In + (int64_t)b * rows * l;
  float* out = Out + (int64_t)b * rows * l;
  const double* g = G + (int64_t)b * l * l;
  const int r0 = blockIdx.x * 64;
  tile_gemm_64x64(
      c0, [&](int r, int k) { return (r0 + r < rows && k < c0) ? out[(int64_t)(r0 + r) * l + k] : 0.f; },
      [&](int k, int j) { return (k < c0 && j < w) ? g[(int64_t)k * l + c0 + j] : 0.0; }, lds,
      [&](int r, int j, double x) {
        const int64_t at = (int64_t)(r0 + r) * l + c0 + j;
        if (r0 + r < rows && j < w) out[at] = (float)((double)in[at] - x);
      });
}

// ---------------------------------------------------------------------------
// Eigenvectors of H = L L^T by a one-sided (Hestenes) Jacobi SVD of the Cholesky factor L itself (l x l, float64),
// one workgroup per block: plane rotations on column pairs until all columns are orthogonal, with a round-robin
// ordering so that l/2 disjoint pairs are rotated concurrently.  L J_1 J_2 ... = U diag(sigma): the final columns,
// normalised, are the LEFT singular vectors of L, which are the eigenvectors of H -- so the rotations are never
// accumulated (half the work and half the storage of a Jacobi on L^T that tracks its right vectors), and working on
// the columns of L instead of those of L^T means diagonalising L^T L, which is one step of the Cholesky-LR iteration
// closer to diagonal than H = L L^T: fewer sweeps.
//   Lfac  in   [l x l] lower-triangular Cholesky factor of H = Y^T Y
//   Wout  out  [l x l] row-major, column r = eigenvector of H of rank r (descending eigenvalue)
//   sigma out  [k] leading singular values of Y = square roots of the eigenvalues
// Columns whose norm is at round-off level (a rank-deficient sketch, kept factorisable by the diagonal shift) are
// still orthogonalised relative to their own norm, so the normalised set stays orthonormal.
// ---------------------------------------------------------------------------
// x from the lane that the DPP control word selects (both halves of the double)
template <int CTRL>
__device__ __forceinline__ double dpp_move(double x) {
  const int lo = __double2loint(x), hi = __double2hiint(x);
  return __hiloint2double(__builtin_amdgcn_update_dpp(hi, hi, CTRL, 0xf, 0xf, true),
                          __builtin_amdgcn_update_dpp(lo, lo, CTRL, 0xf, 0xf, true));
}
// Sum over aligned groups of min(width, 16) lanes (width a power of two); every lane of a group gets the sum.
// Lane i adds lane i^1, then i^2 (quad permutations); once the quads are uniform, mirroring a half row (i <-> 7-i)
// and then a row (i <-> 15-i) brings in the other quads.
template <int WIDTH>
__device__ __forceinline__ double row_sum(double x) {
  if constexpr (WIDTH >= 2) x += dpp_move<0xB1>(x);    // quad_perm [1,0,3,2]
  if constexpr (WIDTH >= 4) x += dpp_move<0x4E>(x);    // quad_perm [2,3,0,1]
  if constexpr (WIDTH >= 8) x += dpp_move<0x141>(x);   // row_half_mirror
  if constexpr (WIDTH >= 16) x += dpp_move<0x140>(x);  // row_mirror
  return x;
}

constexpr int kJacobiThreads = 512;

// One plane rotation of the one-sided Jacobi: the TP lanes of a pair (lane gl of TP, a compile-time power of two:
// with a run-time width every level of the sums below is a branch) make columns ap and aq (length l, in LDS)
// orthogonal.  A lane handles exactly NE elements of a column, NE >= ceil(l / tp), so the element loops
// unroll with a fixed trip count, their LDS loads are issued together, and the elements stay in registers between
// the dot products and the rotation.  A rotation sets *rot, and *big when the cosine of the angle between the
// columns was above 3.2e-5 (flags in registers: the caller publishes them once per sweep).
// PAD: the columns are stored with TP * NE elements, zero beyond l (zeros stay zero under a rotation), so that no
// load or store needs a bounds check (each conditional store is a branch).
template <int NE, int TP, bool PAD>
__device__ __forceinline__ void jacobi_rotate(double* ap, double* aq, int l, int gl, int* rot, int* big) {
  constexpr int tp = TP;
  double al = 0.0, be = 0.0, ga = 0.0;
  double xs[NE], ys[NE];
#pragma unroll
  for (int e = 0; e < NE; ++e) {
    const int r = gl + e * tp;
    xs[e] = (PAD || r < l) ? ap[r] : 0.0;
    ys[e] = (PAD || r < l) ? aq[r] : 0.0;
  }
#pragma unroll
  for (int e = 0; e < NE; ++e) {
    al += xs[e] * xs[e]; be += ys[e] * ys[e]; ga += xs[e] * ys[e];
  }
  // sums over the tp lanes of the pair: inside a row of 16 lanes with data-parallel-primitive moves (no LDS
  // round trip as in a shuffle), across rows with shuffles
  al = row_sum<TP>(al); be = row_sum<TP>(be); ga = row_sum<TP>(ga);
#pragma unroll
  for (int o = tp >> 1; o >= 16; o >>= 1) {
    al += __shfl_xor(al, o, kWave);
    be += __shfl_xor(be, o, kWave);
    ga += __shfl_xor(ga, o, kWave);
  }
  // rotate when the columns are not yet orthogonal to 1e-7 (compared in squares, no sqrt): the outputs are
  // float32, and a sweep that finds nothing above the threshold ends the iteration
  if (ga * ga > 1e-14 * al * be) {
    // The rotation ANGLE only steers convergence, so tan(theta) is computed in float32; cos and sin
    // are then formed in float64 so that the rotation is orthogonal to double round-off.
    const double zd = (be - al) * 0.5 * __builtin_amdgcn_rcp(ga);     // approximate reciprocal is enough
    double tt;
    if (fabs(zd) < 1e15) {
      const float zeta = (float)zd;
      tt = (double)((zeta >= 0.f ? 1.f : -1.f) / (fabsf(zeta) + sqrtf(1.f + zeta * zeta)));
    } else {
      tt = 0.5 * __builtin_amdgcn_rcp(zd);
    }
    const double n2 = 1.0 + tt * tt;
    double cs = __builtin_amdgcn_rsq(n2);
    cs = cs * (1.5 - 0.5 * n2 * cs * cs);
    cs = cs * (1.5 - 0.5 * n2 * cs * cs);
    const double sn = cs * tt;
#pragma unroll
    for (int e = 0; e < NE; ++e) {
      const int r = gl + e * tp;
      if (PAD || r < l) {
        ap[r] = cs * xs[e] - sn * ys[e];
        aq[r] = sn * xs[e] + cs * ys[e];
      }
    }
    *rot = 1;
    if (ga * ga > 1e-9 * al * be) *big = 1;
  }
}

// players p, q of pair `group` in step `step` of a round-robin over `le` players (le even): le - 1 steps pair
// everybody with everybody once
__device__ __forceinline__ void round_robin_pair(int le, int step, int group, int* p, int* q) {
  if (group == 0) { *p = le - 1; *q = step % (le - 1); }
  else { *p = (step + group) % (le - 1); *q = (step + (le - 1) - group) % (le - 1); }
}

// The same pairing followed step by step without divisions (a remainder by a run-time divisor costs about as many
// instructions as the rest of a rotation): start(le, group) gives the pair of step 0, next() that of the step after.
struct RoundRobin {
  int p, q, m;
  bool fixed;   // group 0 keeps player le - 1
  __device__ __forceinline__ void start(int le, int group) {
    m = le - 1;
    fixed = group == 0;
    p = fixed ? le - 1 : group;      // group <= le / 2 - 1 < m
    q = fixed ? 0 : m - group;
  }
  __device__ __forceinline__ void next() {
    if (!fixed) p = p + 1 == m ? 0 : p + 1;
    q = q + 1 == m ? 0 : q + 1;
  }
};

// Whole matrix in LDS (l <= 138), one workgroup per block.
template <int NE, int NT, int TP, bool PAD>
__global__ __launch_bounds__(NT) void jacobi_kernel(const double* __restrict__ Lfac, double* Wout, float* sigma,
                                                     int l, int k, const double* fro_acc, float* fro2,
                                                     int max_sweeps, int32_t* info) {
  extern __shared__ double dyn_lds[];
  __shared__ double nrm[256];
  __shared__ int s_rot, s_big;
  const int b = blockIdx.x, t = threadIdx.x;
  const double* Lf = Lfac + (int64_t)b * l * l;
  // column stride: odd, so that concurrently rotated columns spread over the LDS banks
  const int la = PAD ? TP * NE + 1 : l + 1;
  double* A = dyn_lds;    // column-major
  for (int idx = t; idx < l * l; idx += NT) {
    const int r = idx / l, c = idx % l;
    A[c * la + r] = (c <= r) ? Lf[idx] : 0.0;   // A = L
  }
  if (PAD) {
    const int np = la - l;
    for (int idx = t; idx < l * np; idx += NT) A[(idx / np) * la + l + idx % np] = 0.0;
  }
  if (t == 0 && fro2) fro2[b] = (float)fro_acc[b];
  __syncthreads();

  const int le = (l + 1) & ~1;         // players in the round-robin (one dummy if l is odd)
  const int npairs = le / 2;           // <= 69; the host picks TP with TP * npairs <= NT
  const int group = t / TP, gl = t % TP;
  const bool active = group < npairs;

  bool converged = false;
  for (int sweep = 0; sweep < max_sweeps; ++sweep) {
    if (t == 0) { s_rot = 0; s_big = 0; }
    __syncthreads();
    int my_rot = 0, my_big = 0;
    RoundRobin rr;
    rr.start(le, active ? group : 0);
    for (int step = 0; step < le - 1; ++step) {
      if (active && rr.p < l && rr.q < l) jacobi_rotate<NE, TP, PAD>(A + rr.p * la, A + rr.q * la, l, gl, &my_rot, &my_big);
      rr.next();
      __syncthreads();
    }
    if (my_rot && gl == 0) atomicOr(&s_rot, 1);
    if (my_big && gl == 0) atomicOr(&s_big, 1);
    __syncthreads();
    const int rot = s_rot, big = s_big;
    __syncthreads();
    // Done when a sweep rotates nothing -- or only pairs whose cosine was below 3.2e-5: cyclic Jacobi converges
    // quadratically, so what such a sweep leaves behind is of the order of the square of that, far below the 1e-7
    // threshold, and the sweep that would merely confirm it (a seventh of the kernel's time) is not run.
    if (rot == 0 || big == 0) { converged = true; break; }
  }
  if (t == 0 && !converged && info) atomicOr(info + b, SVDC_FIT_JACOBI_CAPPED);

  for (int j = t; j < l; j += NT) {
    double s = 0.0;
    for (int r = 0; r < l; ++r) s += A[(int64_t)j * la + r] * A[(int64_t)j * la + r];
    nrm[j] = s;
  }
  __syncthreads();
  double* wo = Wout + (int64_t)b * l * l;
  for (int j = t; j < l; j += NT) {
    const double nj = nrm[j];
    int rank = 0;
    for (int i = 0; i < l; ++i) rank += (nrm[i] > nj || (nrm[i] == nj && i < j)) ? 1 : 0;
    if (rank < k) sigma[(int64_t)b * k + rank] = (float)sqrt(nj);
    const double inv = nj > 0.0 ? 1.0 / sqrt(nj) : 0.0;
    for (int i = 0; i < l; ++i) wo[(int64_t)i * l + rank] = A[(int64_t)j * la + i] * inv;
  }
}

// ---------------------------------------------------------------------------
// The same Jacobi for 138 < l <= 256, where the matrix (l x l float64) no longer fits the LDS of one workgroup: by
// column blocks.  The columns form nb = ceil(l / 32) blocks; a round-robin over the blocks pairs every block with
// every other once per sweep, and the pairs of one round-robin step are disjoint, so one launch handles a step with
// one workgroup per block pair: it brings the pair's 64 columns into LDS, rotates every pair across the two blocks
// (32 rounds of 32 concurrent pairs, 16 lanes per pair; in the first step of a sweep every pair among the 64 columns,
// 63 rounds, which covers the pairs inside the blocks) and writes them back: each pair of columns once per sweep.
// The working matrix A lives in global memory column by column (A[c * l + r]); the very first launch reads its
// columns from the Cholesky factor instead.  Convergence is tracked per block in three rotating counters cnt[b][0..2]: the launches of sweep s count
// the rotations with a cosine above 3.2e-5 in cnt[s % 3], return at once when cnt[(s - 1) % 3] is zero (the previous
// sweep found nothing: converged, and it stays so because nothing is counted any more), and the first launch of the
// sweep clears cnt[(s + 1) % 3] for the next one.  jacobi_finish_kernel then sorts and normalises.
// ---------------------------------------------------------------------------
constexpr int kJbCols = 32;

template <int NE>
__global__ __launch_bounds__(kJacobiThreads) void jacobi_block_kernel(const double* __restrict__ Lfac, double* gA, int l,
                                                                      int step, int sweep, int first, int* cnt) {
  extern __shared__ double dyn_lds[];
  __shared__ int s_rot, s_big;
  constexpr int NT = kJacobiThreads, NC = 2 * kJbCols, TP = NT / kJbCols;   // 64 local columns, 16 lanes per pair
  static_assert(TP == 16, "lanes per pair");
  const int b = blockIdx.y, t = threadIdx.x;
  int* c3 = cnt + 4 * b;
  if (blockIdx.x == 0 && step == 0 && t == 0) c3[(sweep + 1) % 3] = 0;
  if (sweep > 0 && c3[(sweep + 2) % 3] == 0) return;   // uniform over the workgroup
  const int nb = (l + kJbCols - 1) / kJbCols, nbe = (nb + 1) & ~1;
  int bi, bj;
  round_robin_pair(nbe, step, blockIdx.x, &bi, &bj);
  constexpr int la = TP * NE + 1;                       // columns padded with zeros to TP * NE elements
  double* A = dyn_lds;                                  // [NC][la]
  double* ga = gA + (int64_t)b * l * l;
  // global column of local column c (>= l: none)
  auto gcol = [&](int c) { const int blk = c < kJbCols ? bi : bj; return blk < nb ? blk * kJbCols + (c & (kJbCols - 1)) : l; };
  if (first) {
    const double* Lf = Lfac + (int64_t)b * l * l;
    for (int idx = t; idx < l * NC; idx += NT) {
      const int r = idx / NC, c = idx % NC, gc = gcol(c);
      if (gc < l) A[c * la + r] = (gc <= r) ? Lf[(int64_t)r * l + gc] : 0.0;
    }
  } else {
    for (int idx = t; idx < NC * l; idx += NT) {
      const int c = idx / l, r = idx % l, gc = gcol(c);
      if (gc < l) A[c * la + r] = ga[(int64_t)gc * l + r];
    }
  }
  for (int idx = t; idx < NC * (la - l); idx += NT) A[(idx / (la - l)) * la + l + idx % (la - l)] = 0.0;
  if (t == 0) { s_rot = 0; s_big = 0; }
  __syncthreads();
  const int group = t / TP, gl = t % TP;
  int my_rot = 0, my_big = 0;
  if (step == 0) {
    // first step of a sweep: every pair among the 64 columns, i.e. also the pairs inside each block (every block is
    // in exactly one pair of step 0)
    RoundRobin rr;
    rr.start(NC, group);
    for (int st = 0; st < NC - 1; ++st) {
      if (gcol(rr.p) < l && gcol(rr.q) < l) jacobi_rotate<NE, TP, true>(A + rr.p * la, A + rr.q * la, l, gl, &my_rot, &my_big);
      rr.next();
      __syncthreads();
    }
  } else {
    // later steps: only the pairs across the two blocks, column i of the first with column (i + st) mod 32 of the second
    const bool ok_p = gcol(group) < l;
    for (int st = 0; st < kJbCols; ++st) {
      const int q = kJbCols + ((group + st) & (kJbCols - 1));
      if (ok_p && gcol(q) < l) jacobi_rotate<NE, TP, true>(A + group * la, A + q * la, l, gl, &my_rot, &my_big);
      __syncthreads();
    }
  }
  if (my_big && gl == 0) atomicAdd(&s_big, 1);
  __syncthreads();
  for (int idx = t; idx < NC * l; idx += NT) {
    const int c = idx / l, r = idx % l, gc = gcol(c);
    if (gc < l) ga[(int64_t)gc * l + r] = A[c * la + r];
  }
  if (t == 0 && s_big > 0) atomicAdd(&c3[sweep % 3], s_big);
}

// Column norms -> singular values, rank order, normalised eigenvectors (same outputs as jacobi_kernel), one
// workgroup per block, one wave per column at a time.
__global__ __launch_bounds__(256) void jacobi_finish_kernel(const double* __restrict__ gA, double* Wout, float* sigma,
                                                            int l, int k, const double* fro_acc, float* fro2,
                                                            int max_sweeps, const int* cnt, int32_t* info) {
  __shared__ double nrm[256];
  const int b = blockIdx.x, t = threadIdx.x, wave = t >> 6, lane = t & 63;
  const double* A = gA + (int64_t)b * l * l;
  if (t == 0) {
    if (fro2) fro2[b] = (float)fro_acc[b];
    // the last sweep still found rotations to do
    if (info && cnt[4 * b + (max_sweeps - 1) % 3] != 0) atomicOr(info + b, SVDC_FIT_JACOBI_CAPPED);
  }
  for (int j = wave; j < l; j += 4) {
    double s = 0.0;
    for (int r = lane; r < l; r += kWave) s += A[(int64_t)j * l + r] * A[(int64_t)j * l + r];
    s = wave_sum(s);
    if (lane == 0) nrm[j] = s;
  }
  __syncthreads();
  double* wo = Wout + (int64_t)b * l * l;
  for (int j = wave; j < l; j += 4) {
    const double nj = nrm[j];
    int rank = 0;
    for (int i = lane; i < l; i += kWave) rank += (nrm[i] > nj || (nrm[i] == nj && i < j)) ? 1 : 0;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) rank += __shfl_xor(rank, o, kWave);
    if (lane == 0 && rank < k) sigma[(int64_t)b * k + rank] = (float)sqrt(nj);
    const double inv = nj > 0.0 ? 1.0 / sqrt(nj) : 0.0;
    for (int i = lane; i < l; i += kWave) wo[(int64_t)i * l + rank] = A[(int64_t)j * l + i] * inv;
  }
}

// ---------------------------------------------------------------------------
// sum of squares of F[b] in float64 (||F||_F^2 for the energy rule, Eq. 6)
// ---------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void sumsq_kernel(const T* __restrict__ F, double* acc, int N, int D,
                                                    int64_t ldf, int64_t bstride, int rows_per_group) {
  __shared__ double part[4];
  const int b = blockIdx.y, t = threadIdx.x;
  const T* f = F + (int64_t)b * bstride;
  const int r0 = blockIdx.x * rows_per_group, r1 = min(N, r0 + rows_per_group);
  double s = 0.0;
  for (int r = r0; r < r1; ++r)
    for (int d = t; d < D; d += 256) {
      const float x = ld_elem(f, (int64_t)r * ldf + d);
      s += (double)x * (double)x;
    }
  s = wave_sum(s);
  if ((t & 63) == 0) part[t >> 6] = s;
  __syncthreads();
  if (t == 0) atomicAdd(&acc[b], part[0] + part[1] + part[2] + part[3]);
}

// ---------------------------------------------------------------------------
// host orchestration
// ---------------------------------------------------------------------------
static size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

constexpr size_t kLdsBudget = 150 * 1024;  // dynamic LDS a single workgroup may take (160 KB per CU)
constexpr int kGramSlices = 16;   // row slices whose partial Gram matrices are summed in a fixed order

bool make_fit_plan(const svdc_shape& s, const svdc_fit_params* p, FitPlan* plan) {
  int pp = p ? p->oversample_p : 0;
  int q = p ? p->power_iters_q : 0;
  if (pp < -1 || q < -1 || pp > 4096 || q > 64) return false;
  if (pp == 0) pp = s.k;
  if (pp == -1) pp = 0;
  if (q == 0) q = (s.dtype == SVDC_BF16) ? 3 : 5;
  if (q == -1) q = 0;
  int l = s.k + pp;
  l = std::min(l, std::min(s.N, s.D));
  l = std::min(l, 256);
  if (l < s.k) return false;  // k > 256 is not supported by the fit
  plan->l = l;
  plan->q = q;
  plan->seed = p ? p->seed : 0;
  const int sweeps = p ? p->jacobi_max_sweeps : 0;
  if (sweeps < 0 || sweeps > 1000) return false;
  // default cap: 40 sweeps; 20 for the Jacobi by column blocks (l > 138), which takes 8-9 and whose launches are
  // issued up to the cap (those after convergence return at once, but are not free)
  plan->max_sweeps = sweeps == 0 ? ((size_t)l * (l + 1) * sizeof(double) <= kLdsBudget ? 40 : 20) : sweeps;
  size_t off = 0;
  const size_t B = s.B;
  plan->off_Q = off; off = align_up(off + B * s.D * l * sizeof(float), 256);
  plan->off_Z = off; off = align_up(off + B * s.D * l * sizeof(float), 256);
  // Y as float32 rows; the matrix-core path also keeps its packed bf16 form there between a projection and the
  // back-projection that follows (never both at once)
  size_t y_bytes = B * (size_t)s.N * l * sizeof(float);
  if (fit_mfma_supported(s, l)) y_bytes = std::max(y_bytes, fit_mfma_packed_y_bytes(s, l));
  plan->off_Y = off; off = align_up(off + y_bytes, 256);
  plan->off_G = off; off = align_up(off + B * l * l * sizeof(double), 256);
  plan->off_Gp = off; off = align_up(off + B * kGramSlices * (size_t)l * l * sizeof(double), 256);
  plan->off_M = off; off = align_up(off + B * l * l * sizeof(double), 256);
  plan->off_W = off; off = align_up(off + B * l * l * sizeof(double), 256);   // Jacobi matrix when l > 138
  // ||F||_F^2 accumulators (B doubles) followed by the status words (B int32, see svdcache_fit_status_offset)
  plan->off_misc = off; off = align_up(off + B * sizeof(double), 256);
  plan->off_info = off; off = align_up(off + B * sizeof(int32_t), 256);
  // convergence counters of the Jacobi by column blocks (4 int32 per block); cleared together with the two above
  plan->off_jcnt = off; off = align_up(off + B * 4 * sizeof(int32_t), 256);
  plan->mfma = fit_mfma_supported(s, l);
  plan->off_Qp = off;
  if (plan->mfma) off = align_up(off + fit_mfma_packed_q_bytes(s, l), 256);
  plan->total = off;
  return true;
}

namespace {


int32_t set_dyn_lds(const void* fn, size_t bytes) {
  if (bytes <= 48 * 1024) return SVDC_OK;
  return hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes) == hipSuccess
             ? SVDC_OK : SVDC_E_HIP;
}

void zero_f64(double* p, int64_t n, hipStream_t st) {
  fill_zero_kernel<<<(unsigned)((n + 255) / 256), 256, 0, st>>>(p, n);
}
void zero_f32(float* p, int64_t n, hipStream_t st) {
  fill_zero_f32_kernel<<<(unsigned)((n + 255) / 256), 256, 0, st>>>(p, n);
}

template <typename T>
void gemm_fq(const svdc_shape& s, int l, const T* F, const float* Q, float* Y, hipStream_t st) {
  dim3 grid((s.N + 63) / 64, (l + 63) / 64, s.B);
  fit_gemm_kernel<T, false><<<grid, 256, 0, st>>>(F, Q, Y, s.N, s.D, l, s.ldf, s.block_stride, s.D, 1);
}
template <typename T>
void gemm_fty(const svdc_shape& s, int l, const T* F, const float* Y, float* Z, hipStream_t st) {
  zero_f32(Z, (int64_t)s.B * s.D * l, st);
  const int split_len = 1024;
  const int nsplit = (s.N + split_len - 1) / split_len;
  dim3 grid((s.D + 63) / 64, (l + 63) / 64, s.B * nsplit);
  fit_gemm_kernel<T, true><<<grid, 256, 0, st>>>(F, Y, Z, s.N, s.D, l, s.ldf, s.block_stride, split_len, nsplit);
}

void gram(const float* A, double* G, double* Gpart, int B, int rows, int l, hipStream_t st) {
  const int ntile = (l + 63) / 64;
  int rows_per_slice = ((rows + kGramSlices - 1) / kGramSlices + 15) / 16 * 16;
  if (rows_per_slice < 64) rows_per_slice = 64;
  const int nslice = (rows + rows_per_slice - 1) / rows_per_slice;
  dim3 grid(nslice, ntile * (ntile + 1) / 2, B);
  gram_f64_kernel<<<grid, 256, 0, st>>>(A, Gpart, rows, l, rows_per_slice);
  const int64_t ll = (int64_t)l * l;
  gram_reduce_kernel<<<dim3((unsigned)((ll + 255) / 256), B), 256, 0, st>>>(Gpart, G, nslice, l);
}

// Cholesky factor of G + shift I in place, l <= 256: L in the lower triangle; for l > 64 the strict upper triangle
// holds L^T outside the 64 x 64 diagonal blocks (whose upper halves are zeroed).  scratch (block stride l * l
// doubles): receives the reciprocal diagonal in its first l entries per block when not null; REQUIRED for l > 64,
// where entry [l] carries the diagonal shift from the first block's factorisation to the later ones.
int32_t chol_factor(double* G, int B, int l, int32_t* info, hipStream_t st, double* scratch) {
  const int64_t ll = (int64_t)l * l;
  constexpr int H = kCholBlock;
  if (l <= H) {
    chol_reg_kernel<4><<<B, 256, 0, st>>>(G, ll, l, scratch, ll, l, 1e-14, info, ChoShift{nullptr, 0, l},
                                          ChoUpdate{nullptr, 0, 0, 0});
    return SVDC_OK;
  }
  if (!scratch) return SVDC_E_NULL;
  for (int c0 = 0; c0 < l; c0 += H) {
    const int w = std::min(H, l - c0);
    chol_reg_kernel<4><<<B, 256, 0, st>>>(G + (int64_t)c0 * l + c0, ll, l, scratch + c0, ll, w, 1e-14, info,
                                          ChoShift{scratch + l, ll, c0 == 0 ? l : 0},
                                          ChoUpdate{c0 ? G + c0 : nullptr, ll, l, c0});
    if (c0 + w < l) chol_panel_kernel<<<dim3((l - c0 - w + H - 1) / H, B), 256, 0, st>>>(G, scratch, ll, l, c0);
  }
  return SVDC_OK;
}

// Out[rows x m] = In[rows x l] * M[l x m]
int32_t rows_times_small(const float* In, const double* M, float* Out, int B, int rows, int l, int m, int ldm,
                         hipStream_t st) {
  dim3 grid((rows + 63) / 64, (m + 63) / 64, B);
  rows_times_small_kernel<<<grid, 256, 0, st>>>(In, M, Out, rows, l, m, ldm);
  return SVDC_OK;
}

// Orthonormalise the columns of Zin by CholeskyQR (Gram matrix and Cholesky factor in float64).
// One pass leaves the result in Qout and is accurate to about eps32 * cond(Zin): enough to keep the
// power iteration well conditioned.  two_pass repeats the step on the result (CholeskyQR2), giving
// orthonormality at float32 round-off; the result is then back in Zin.
// Out = In * L^-T with L the Cholesky factor of In^T In (left in G by chol_factor)
int32_t cholqr_apply(const float* In, float* Out, double* G, double* M, int B, int rows, int l, int32_t* info,
                     hipStream_t st) {
  const int64_t ll = (int64_t)l * l;
  // M receives the reciprocal diagonal of L (its first l entries per block)
  if (chol_factor(G, B, l, info, st, M) != SVDC_OK) return SVDC_E_HIP;
  // by column blocks of 64: Out_j = (In_j - sum_{i < j} Out_i L_ji^T) L_jj^-T
  constexpr int H = kCholBlock;
  const dim3 grid((rows + 255) / 256, B);
  for (int c0 = 0; c0 < l; c0 += H) {
    const int w = std::min(H, l - c0);
    const float* src = In;
    if (c0 > 0) {
      rows_minus_product_kernel<<<dim3((rows + H - 1) / H, B), 256, 0, st>>>(In, Out, G, rows, l, c0, w);
      src = Out;
    }
    const double* lkk = G + (int64_t)c0 * l + c0;
    if (w <= 16) tri_solve_rows_kernel<16><<<grid, 256, 0, st>>>(src + c0, lkk, M + c0, Out + c0, rows, w, l, l, ll, ll);
    else if (w <= 32) tri_solve_rows_kernel<32><<<grid, 256, 0, st>>>(src + c0, lkk, M + c0, Out + c0, rows, w, l, l, ll, ll);
    else tri_solve_rows_kernel<64><<<grid, 256, 0, st>>>(src + c0, lkk, M + c0, Out + c0, rows, w, l, l, ll, ll);
  }
  return SVDC_OK;
}

int32_t orth(float* Zin, float* Qout, double* G, double* Gpart, double* M, int B, int rows, int l, bool two_pass,
             int32_t* info, hipStream_t st) {
  gram(Zin, G, Gpart, B, rows, l, st);
  if (cholqr_apply(Zin, Qout, G, M, B, rows, l, info, st) != SVDC_OK) return SVDC_E_HIP;
  if (!two_pass) return SVDC_OK;
  // the second pass factors a matrix that is already orthonormal to float32 round-off: only the first one can
  // meet a dependent column
  gram(Qout, G, Gpart, B, rows, l, st);
  return cholqr_apply(Qout, Zin, G, M, B, rows, l, nullptr, st);
}

template <typename T>
int32_t run_fit_typed(const svdc_shape& s, const FitPlan& pl, const T* F, float* V, float* sigma, float* fro2,
                      char* ws, hipStream_t st) {
  const int l = pl.l, B = s.B;
  float* Q = (float*)(ws + pl.off_Q);
  float* Z = (float*)(ws + pl.off_Z);
  float* Y = (float*)(ws + pl.off_Y);
  double* G = (double*)(ws + pl.off_G);
  double* Gp = (double*)(ws + pl.off_Gp);
  double* M = (double*)(ws + pl.off_M);
  double* Wg = (double*)(ws + pl.off_W);
  double* misc = (double*)(ws + pl.off_misc);
  int32_t* info = (int32_t*)(ws + pl.off_info);

  const int64_t nq = (int64_t)B * s.D * l;
  // fro accumulators, status words and Jacobi counters are adjacent 256-byte aligned areas: one fill clears them all
  zero_f64(misc, (int64_t)((pl.off_jcnt - pl.off_misc) + align_up((size_t)B * 4 * sizeof(int32_t), 8)) / 8, st);
  // With power iterations the Gaussian test matrix (D x l) is used as it is: its columns are well conditioned
  // and every product F^T F Q is re-orthonormalised afterwards.  With none, the sketch is Z = F^T Omega with a
  // Gaussian Omega (N x l) -- the plain randomized range finder, exact when rank(F) <= l -- and Q <- orth(Z), two
  // passes, goes straight into the Rayleigh-Ritz step.
  if (pl.q == 0) {
    const int64_t ny = (int64_t)B * s.N * l;
    init_omega_kernel<<<(unsigned)((ny + 255) / 256), 256, 0, st>>>(Y, (int64_t)s.N * l, ny, pl.seed);
    if (pl.mfma) fit_mfma_backproject(s, l, F, Y, nullptr, Z, st);
    else gemm_fty<T>(s, l, F, Y, Z, st);
    if (orth(Z, Q, G, Gp, M, B, s.D, l, true, info, st) != SVDC_OK) return SVDC_E_HIP;
    std::swap(Q, Z);
  } else {
    init_omega_kernel<<<(unsigned)((nq + 255) / 256), 256, 0, st>>>(Q, (int64_t)s.D * l, nq, pl.seed);
  }

  void* Qp = ws + pl.off_Qp;
  const bool want_fro = fro2 != nullptr;
  bool fro_done = false;
  // Y = F Q.  The last product feeds the Rayleigh-Ritz step and uses the full-precision operand split.
  // float32 features: every product splits both operands, and Y stays float32 rows between the two products
  constexpr bool kF32 = std::is_same<T, float>::value;
  auto project = [&](bool last) {
    if (pl.mfma) {
      fit_mfma_pack_q(s, l, Q, Qp, st);
      fit_mfma_project(s, l, F, Qp, Y, (last || kF32) ? nullptr : (void*)Y, (last && want_fro) ? misc : nullptr,
                       last || kF32, st);
      if (last && want_fro) fro_done = true;
    } else {
      gemm_fq<T>(s, l, F, Q, Y, st);
    }
  };
  for (int it = 0; it < pl.q; ++it) {
    project(false);
    if (pl.mfma) {
      fit_mfma_backproject(s, l, F, Y, kF32 ? nullptr : Y, Z, st);   // bf16: Y holds the packed form here
    } else {
      gemm_fty<T>(s, l, F, Y, Z, st);
    }
    const bool last_it = it + 1 == pl.q;
    if (orth(Z, Q, G, Gp, M, B, s.D, l, last_it, info, st) != SVDC_OK) return SVDC_E_HIP;
    if (last_it) std::swap(Q, Z);
  }

  // Rayleigh-Ritz on span(Q)
  project(true);
  gram(Y, G, Gp, B, s.N, l, st);
  if (chol_factor(G, B, l, info, st, M) != SVDC_OK) return SVDC_E_HIP;   // M: scratch until the Jacobi writes it
  if (want_fro && !fro_done) {
    const int rpg = 64;
    sumsq_kernel<T><<<dim3((s.N + rpg - 1) / rpg, B), 256, 0, st>>>(F, misc, s.N, s.D, s.ldf, s.block_stride, rpg);
  }
  int32_t jrc = SVDC_OK;
  if ((size_t)l * (l + 1) * sizeof(double) <= kLdsBudget) {   // l <= 138: the whole matrix in the LDS of one workgroup
    // lanes per pair: the largest power of two <= 64 with pairs x lanes <= threads (1024 threads from 33 pairs on),
    // and the elements of a column per lane that follow from it; columns padded to lanes x elements up to l = 128
    const int npairs = ((l + 1) & ~1) / 2;
    auto launch = [&](auto kernel, int nt, int la) -> int32_t {
      const size_t mat = (size_t)l * la * sizeof(double);
      if (set_dyn_lds((const void*)kernel, mat) != SVDC_OK) return SVDC_E_HIP;
      kernel<<<B, nt, mat, st>>>(G, M, sigma, l, s.k, misc, fro2, pl.max_sweeps, info);
      return SVDC_OK;
    };
    constexpr int NT = kJacobiThreads;
    if (npairs <= 8) jrc = launch(jacobi_kernel<1, NT, 64, true>, NT, 65);             // l <= 16
    else if (npairs <= 16) jrc = launch(jacobi_kernel<1, NT, 32, true>, NT, 33);       // l <= 32
    else if (npairs <= 32) jrc = launch(jacobi_kernel<4, NT, 16, true>, NT, 65);       // l <= 64
    else if (npairs <= 64) jrc = launch(jacobi_kernel<8, 1024, 16, true>, 1024, 129);  // l <= 128
    else jrc = launch(jacobi_kernel<18, 1024, 8, false>, 1024, l + 1);                 // l <= 138
  } else {                                          // by column blocks, one launch per round-robin step
    const int nb = (l + kJbCols - 1) / kJbCols, nbe = (nb + 1) & ~1;
    const size_t lds = (size_t)2 * kJbCols * (l <= 192 ? 193 : 257) * sizeof(double);   // columns of 16 lanes x 12 or 16
    int* cnt = (int*)(ws + pl.off_jcnt);
    auto sweeps = [&](auto kernel) -> int32_t {
      if (set_dyn_lds((const void*)kernel, lds) != SVDC_OK) return SVDC_E_HIP;
      for (int sweep = 0; sweep < pl.max_sweeps; ++sweep)
        for (int step = 0; step < nbe - 1; ++step)
          kernel<<<dim3(nbe / 2, B), kJacobiThreads, lds, st>>>(G, Wg, l, step, sweep, sweep == 0 && step == 0, cnt);
      return SVDC_OK;
    };
    jrc = l <= 192 ? sweeps(jacobi_block_kernel<12>) : sweeps(jacobi_block_kernel<16>);
    jacobi_finish_kernel<<<B, 256, 0, st>>>(Wg, M, sigma, l, s.k, misc, fro2, pl.max_sweeps, cnt, info);
  }
  if (jrc != SVDC_OK) return jrc;
  if (rows_times_small(Q, M, V, B, s.D, l, s.k, l, st) != SVDC_OK) return SVDC_E_HIP;
  return launch_status();
}

}  // namespace

int32_t run_fit(const svdc_shape& s, const FitPlan& plan, const void* F, float* V, float* sigma, float* fro2,
                void* workspace, hipStream_t st) {
  if (s.dtype == SVDC_BF16)
    return run_fit_typed<bf16_t>(s, plan, (const bf16_t*)F, V, sigma, fro2, (char*)workspace, st);
  return run_fit_typed<float>(s, plan, (const float*)F, V, sigma, fro2, (char*)workspace, st);
}

}  // namespace svdc
