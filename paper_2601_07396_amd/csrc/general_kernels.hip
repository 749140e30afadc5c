// General (any shape, any k <= 1024) kernels for the full-compute step and the
// cached step.  Plain fp32 vector arithmetic, one wavefront per token row.
// They are the fallback for shapes the matrix-core kernels do not cover (hidden sizes that are not one of the
// instantiated multiples of 128, ranks above 128 or not a multiple of 4), for either storage type.
#include "svdc_device.h"
#include "svdc_internal.h"

namespace svdc {

constexpr int kRowsPerGroup = 4;   // one wave64 per row, 256 threads
constexpr int kMaxRank = 1024;     // coefficients of one row staged in LDS
constexpr int kChunk = 32;         // columns of V handled per projection pass

// Full-compute step (Eq. 8-11): C = F V, R = F - C V^T, EMA update of S.
// F and R may alias (in place): each element of a row is read before it is written.
template <typename T>
__global__ __launch_bounds__(256) void full_step_general_kernel(const T* F, const float* __restrict__ V, T* R,
                                                                const T* Rp, float alpha_r, float* S, float* C,
                                                                int N, int D, int k, int64_t ldf, int64_t bstride,
                                                                float alpha, int init) {
  __shared__ float csh[kRowsPerGroup][kMaxRank];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int b = blockIdx.y;
  const int64_t row = (int64_t)blockIdx.x * kRowsPerGroup + wave;
  const bool valid = row < N;  // uniform within the wave
  const T* f = F + (int64_t)b * bstride + (valid ? row : 0) * ldf;
  T* r = R + (int64_t)b * bstride + (valid ? row : 0) * ldf;
  const float* v = V + (int64_t)b * D * k;
  const bool vec4 = (k & 3) == 0;

  if (valid) {
    // projection, kChunk columns of V at a time; each lane owns a stripe of d
    for (int jc = 0; jc < k; jc += kChunk) {
      const int jn = min(kChunk, k - jc);
      float acc[kChunk];
#pragma unroll
      for (int j = 0; j < kChunk; ++j) acc[j] = 0.f;
      if (vec4) {
        for (int d = lane; d < D; d += kWave) {
          const float x = ld_elem(f, d);
          const float4* vp = reinterpret_cast<const float4*>(v + (int64_t)d * k + jc);
#pragma unroll
          for (int g = 0; g < kChunk / 4; ++g) {
            if (g * 4 < jn) {
              const float4 w = vp[g];
              acc[4 * g + 0] += x * w.x;
              acc[4 * g + 1] += x * w.y;
              acc[4 * g + 2] += x * w.z;
              acc[4 * g + 3] += x * w.w;
            }
          }
        }
      } else {
        for (int d = lane; d < D; d += kWave) {
          const float x = ld_elem(f, d);
          const float* vp = v + (int64_t)d * k + jc;
#pragma unroll
          for (int j = 0; j < kChunk; ++j)
            if (j < jn) acc[j] += x * vp[j];
        }
      }
      float mine = 0.f;
#pragma unroll
      for (int j = 0; j < kChunk; ++j) {
        const float t = wave_sum(acc[j]);
        if (lane == j) mine = t;
      }
      if (lane < jn) csh[wave][jc + lane] = mine;
    }
  }
  __syncthreads();
  if (!valid) return;

  // EMA update of the coefficient state (Eq. 11 with alpha = 1 - beta)
  const int64_t srow = ((int64_t)b * N + row) * k;
  for (int j = lane; j < k; j += kWave) {
    const float c = csh[wave][j];
    const float s = init ? c : (1.f - alpha) * S[srow + j] + alpha * c;
    S[srow + j] = s;
    if (C) C[srow + j] = c;
  }

  // residual R = F - C V^T (Eq. 10)
  const float* cw = csh[wave];
  for (int d = lane; d < D; d += kWave) {
    float acc = 0.f;
    const float* vp = v + (int64_t)d * k;
    if (vec4) {
      for (int j = 0; j < k; j += 4) {
        const float4 w = *reinterpret_cast<const float4*>(vp + j);
        acc += cw[j] * w.x + cw[j + 1] * w.y + cw[j + 2] * w.z + cw[j + 3] * w.w;
      }
    } else {
      for (int j = 0; j < k; ++j) acc += cw[j] * vp[j];
    }
    float rnew = ld_elem(f, d) - acc;
    // optional smoothing of the residual state (Rp: previous residual, may be the buffer R itself)
    if (Rp) rnew = (1.f - alpha_r) * ld_elem(Rp + (int64_t)b * bstride + row * ldf, d) + alpha_r * rnew;
    st_elem(r, d, rnew);
  }
}

// Cached step (Sec. 3.5): Fhat = C_hat V^T + R [+ X] with the coefficient forecast C_hat = sum_m w_m S_m
// (one state with weight one is the paper's EMA forecast).  X is nullable; Fhat may alias R or X.
template <typename T>
__global__ __launch_bounds__(256) void forecast_general_kernel(const CoefStates cs, const float* __restrict__ V,
                                                               const T* R, const T* X, T* Fh, int N, int D, int k,
                                                               int64_t ldf, int64_t bstride) {
  __shared__ float ssh[kRowsPerGroup][kMaxRank];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int b = blockIdx.y;
  const int64_t row = (int64_t)blockIdx.x * kRowsPerGroup + wave;
  const bool valid = row < N;
  if (valid) {
    const int64_t srow = ((int64_t)b * N + row) * k;
    for (int j = lane; j < k; j += kWave) {
      float c = cs.w[0] * cs.s[0][srow + j];
      for (int m = 1; m < cs.m; ++m) c = __builtin_fmaf(cs.w[m], cs.s[m][srow + j], c);
      ssh[wave][j] = c;
    }
  }
  __syncthreads();
  if (!valid) return;
  const T* r = R + (int64_t)b * bstride + row * ldf;
  const T* x = X ? X + (int64_t)b * bstride + row * ldf : nullptr;
  T* o = Fh + (int64_t)b * bstride + row * ldf;
  const float* v = V + (int64_t)b * D * k;
  const float* sw = ssh[wave];
  const bool vec4 = (k & 3) == 0;
  for (int d = lane; d < D; d += kWave) {
    float acc = 0.f;
    const float* vp = v + (int64_t)d * k;
    if (vec4) {
      for (int j = 0; j < k; j += 4) {
        const float4 w = *reinterpret_cast<const float4*>(vp + j);
        acc += sw[j] * w.x + sw[j + 1] * w.y + sw[j + 2] * w.z + sw[j + 3] * w.w;
      }
    } else {
      for (int j = 0; j < k; ++j) acc += sw[j] * vp[j];
    }
    float base = ld_elem(r, d);
    if (x) base += ld_elem(x, d);
    st_elem(o, d, base + acc);
  }
}

int32_t launch_full_step_general(const svdc_shape& s, const void* F, const float* V, void* R, float* S,
                                 float* C, float alpha, int init, ResidualEma re, hipStream_t st) {
  dim3 grid((s.N + kRowsPerGroup - 1) / kRowsPerGroup, s.B), block(256);
  if (s.dtype == SVDC_BF16)
    full_step_general_kernel<bf16_t><<<grid, block, 0, st>>>((const bf16_t*)F, V, (bf16_t*)R, (const bf16_t*)re.prev,
                                                           re.alpha_r, S, C, s.N, s.D, s.k, s.ldf, s.block_stride,
                                                           alpha, init);
  else
    full_step_general_kernel<float><<<grid, block, 0, st>>>((const float*)F, V, (float*)R, (const float*)re.prev,
                                                          re.alpha_r, S, C, s.N, s.D, s.k, s.ldf, s.block_stride,
                                                          alpha, init);
  return launch_status();
}

int32_t launch_forecast_general(const svdc_shape& s, const CoefStates& cs, const float* V, const void* R,
                                const void* X, void* Out, hipStream_t st) {
  dim3 grid((s.N + kRowsPerGroup - 1) / kRowsPerGroup, s.B), block(256);
  if (s.dtype == SVDC_BF16)
    forecast_general_kernel<bf16_t><<<grid, block, 0, st>>>(cs, V, (const bf16_t*)R, (const bf16_t*)X, (bf16_t*)Out,
                                                          s.N, s.D, s.k, s.ldf, s.block_stride);
  else
    forecast_general_kernel<float><<<grid, block, 0, st>>>(cs, V, (const float*)R, (const float*)X, (float*)Out, s.N,
                                                         s.D, s.k, s.ldf, s.block_stride);
  return launch_status();
}

// ---------------------------------------------------------------------------
// Rank selection by retained energy (Eq. 6) from the leading singular values and ||F||_F^2:
// k* = smallest count whose squared singular values sum to at least tau * ||F||_F^2, in float64, summed left to
// right.  One thread per block (k <= 1024 values).
// ---------------------------------------------------------------------------
__global__ void select_rank_kernel(const float* __restrict__ sigma, const float* __restrict__ fro2, float tau,
                                   int32_t* k_star, int32_t* reached, int B, int k) {
  const int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b >= B) return;
  const double thr = (double)tau * (double)fro2[b];
  double acc = 0.0;
  int ks = k, ok = 0;
  for (int i = 0; i < k; ++i) {
    const double s = (double)sigma[(int64_t)b * k + i];
    acc = acc + s * s;
    if (acc >= thr) {
      ks = i + 1;
      ok = 1;
      break;
    }
  }
  k_star[b] = ks;
  if (reached) reached[b] = ok;
}

// zero the columns j >= k_star[b] of V[b] (and of sigma[b])
__global__ __launch_bounds__(256) void truncate_basis_kernel(float* V, float* sigma, const int32_t* __restrict__ k_star,
                                                             int D, int k) {
  const int b = blockIdx.y;
  const int ks = k_star[b];
  const int64_t n = (int64_t)D * k;
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx < n && (int)(idx % k) >= ks) V[(int64_t)b * n + idx] = 0.f;
  if (sigma && idx < k && idx >= ks) sigma[(int64_t)b * k + idx] = 0.f;
}

int32_t launch_select_rank(int B, int k, const float* sigma, const float* fro2, float tau, int32_t* k_star,
                           int32_t* reached, hipStream_t st) {
  select_rank_kernel<<<(B + 63) / 64, 64, 0, st>>>(sigma, fro2, tau, k_star, reached, B, k);
  return launch_status();
}

int32_t launch_truncate_basis(const svdc_shape& s, float* V, float* sigma, const int32_t* k_star, hipStream_t st) {
  const int64_t n = (int64_t)s.D * s.k;
  dim3 grid((unsigned)((n + 255) / 256), s.B);
  truncate_basis_kernel<<<grid, 256, 0, st>>>(V, sigma, k_star, s.D, s.k);
  return launch_status();
}

}  // namespace svdc
