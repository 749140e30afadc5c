// Basis reuse across prompts and re-basing of the coefficient state (Sec. 3.3, Fig. 1(b)).
// All three kernels touch only the D x k bases and the N x k states, never the features.
#include "svdc_device.h"
#include "svdc_internal.h"

namespace svdc {

namespace {

constexpr int kOvRows = 16;      // rows of M per workgroup
constexpr int kOvDepth = 32;     // channels staged per step
constexpr int kOvMaxRank = 128;  // overlap / re-basing work up to this rank

// M[b][i][j] = sum_d V_old[b][d][i] * V_new[b][d][j].  Grid (ceil(k / 16), B); thread (ti, tj) of the
// 16 x 16 arrangement owns M[i0 + ti][tj + 16 c], c = 0..7.  The sum runs over d in ascending order.
template <int KC>   // column tiles of 16 that hold data: ceil(k / 16), a compile-time loop bound
__global__ __launch_bounds__(256) void basis_overlap_kernel(const float* __restrict__ Vo,
                                                            const float* __restrict__ Vn, float* M, int D, int k) {
  __shared__ float so[kOvDepth][kOvRows + 1];
  __shared__ float sn[kOvDepth][kOvMaxRank + 1];
  const int b = blockIdx.y, i0 = blockIdx.x * kOvRows, t = threadIdx.x, ti = t >> 4, tj = t & 15;
  const float* vo = Vo + (int64_t)b * D * k;
  const float* vn = Vn + (int64_t)b * D * k;
  float acc[KC];
#pragma unroll
  for (int c = 0; c < KC; ++c) acc[c] = 0.f;
  for (int d0 = 0; d0 < D; d0 += kOvDepth) {
    for (int e = t; e < kOvDepth * kOvRows; e += 256) {
      const int dd = e / kOvRows, ii = e % kOvRows, d = d0 + dd, i = i0 + ii;
      so[dd][ii] = (d < D && i < k) ? vo[(int64_t)d * k + i] : 0.f;
    }
    for (int e = t; e < kOvDepth * 16 * KC; e += 256) {       // columns beyond k are staged as zeros
      const int dd = e / (16 * KC), jj = e % (16 * KC), d = d0 + dd;
      sn[dd][jj] = (d < D && jj < k) ? vn[(int64_t)d * k + jj] : 0.f;
    }
    __syncthreads();
#pragma unroll 8
    for (int dd = 0; dd < kOvDepth; ++dd) {
      const float a = so[dd][ti];
#pragma unroll
      for (int c = 0; c < KC; ++c) acc[c] = __builtin_fmaf(a, sn[dd][tj + 16 * c], acc[c]);
    }
    __syncthreads();
  }
  if (i0 + ti < k) {
#pragma unroll
    for (int c = 0; c < KC; ++c)
      if (tj + 16 * c < k) M[((int64_t)b * k + i0 + ti) * k + tj + 16 * c] = acc[c];
  }
}

// S_out[row][j] = sum_i S_in[row][i] * M[i][j]: one wavefront per row, M of the block in LDS.  S_out may
// be S_in: a row is staged in LDS completely before it is written.  Every wave of a workgroup runs the same
// number of iterations (rows beyond N are skipped by predicate), so the barriers are uniform.
__global__ __launch_bounds__(256) void rebase_state_kernel(const float* __restrict__ M, const float* Sin, float* Sout,
                                                           int N, int k, int rows_per_group) {
  extern __shared__ float lds[];
  float* m = lds;                       // [k][k]
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  float* srow = lds + k * k + wave * k;
  const int b = blockIdx.y;
  for (int e = threadIdx.x; e < k * k; e += 256) m[e] = M[(int64_t)b * k * k + e];
  const int r0 = blockIdx.x * rows_per_group;
  for (int rr = 0; rr < rows_per_group; rr += 4) {
    const int row = r0 + rr + wave;
    const bool valid = row < N && rr + wave < rows_per_group;
    const int64_t off = ((int64_t)b * N + row) * k;
    __syncthreads();                    // M loaded / previous row consumed
    if (valid)
      for (int j = lane; j < k; j += kWave) srow[j] = Sin[off + j];
    __syncthreads();
    if (valid)
      for (int j = lane; j < k; j += kWave) {
        float acc = 0.f;
        for (int i = 0; i < k; ++i) acc = __builtin_fmaf(srow[i], m[i * k + j], acc);
        Sout[off + j] = acc;
      }
  }
}

// Fig. 1(b): cosine similarity times magnitude similarity for every pair of basis directions and for the two
// singular-value vectors.  One workgroup per block; wave w takes the directions w, w + 4, ...
__global__ __launch_bounds__(256) void basis_similarity_kernel(const float* __restrict__ Va,
                                                               const float* __restrict__ sa,
                                                               const float* __restrict__ Vb,
                                                               const float* __restrict__ sb, float* sim_dir,
                                                               float* sim_sigma, int D, int k) {
  const int b = blockIdx.x, wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const float* va = Va + (int64_t)b * D * k;
  const float* vb = Vb + (int64_t)b * D * k;
  auto score = [](double dot, double na2, double nb2, bool take_abs) -> float {
    if (!(na2 > 0.0) || !(nb2 > 0.0)) return 0.f;
    const double na = sqrt(na2), nb = sqrt(nb2);
    const double c = (take_abs ? fabs(dot) : dot) / (na * nb);
    return (float)(c * (na < nb ? na / nb : nb / na));
  };
  for (int j = wave; j < k; j += 4) {
    double dot = 0.0, na = 0.0, nb = 0.0;
    for (int d = lane; d < D; d += kWave) {
      const double x = va[(int64_t)d * k + j], y = vb[(int64_t)d * k + j];
      dot += x * y; na += x * x; nb += y * y;
    }
    dot = wave_sum(dot); na = wave_sum(na); nb = wave_sum(nb);
    if (lane == 0) sim_dir[(int64_t)b * k + j] = score(dot, na, nb, true);
  }
  if (wave == 0 && sim_sigma) {
    double dot = 0.0, na = 0.0, nb = 0.0;
    for (int j = lane; j < k; j += kWave) {
      const double x = sa[(int64_t)b * k + j], y = sb[(int64_t)b * k + j];
      dot += x * y; na += x * x; nb += y * y;
    }
    dot = wave_sum(dot); na = wave_sum(na); nb = wave_sum(nb);
    if (lane == 0) sim_sigma[b] = score(dot, na, nb, false);
  }
}

}  // namespace

bool rebase_rank_supported(int k) { return k >= 1 && k <= kOvMaxRank; }

int32_t launch_basis_overlap(const svdc_shape& s, const float* V_old, const float* V_new, float* M, hipStream_t st) {
  dim3 grid((s.k + kOvRows - 1) / kOvRows, s.B);
  switch ((s.k + 15) / 16) {
    case 1: basis_overlap_kernel<1><<<grid, 256, 0, st>>>(V_old, V_new, M, s.D, s.k); break;
    case 2: basis_overlap_kernel<2><<<grid, 256, 0, st>>>(V_old, V_new, M, s.D, s.k); break;
    case 3: basis_overlap_kernel<3><<<grid, 256, 0, st>>>(V_old, V_new, M, s.D, s.k); break;
    case 4: basis_overlap_kernel<4><<<grid, 256, 0, st>>>(V_old, V_new, M, s.D, s.k); break;
    case 5: basis_overlap_kernel<5><<<grid, 256, 0, st>>>(V_old, V_new, M, s.D, s.k); break;
    case 6: basis_overlap_kernel<6><<<grid, 256, 0, st>>>(V_old, V_new, M, s.D, s.k); break;
    case 7: basis_overlap_kernel<7><<<grid, 256, 0, st>>>(V_old, V_new, M, s.D, s.k); break;
    default: basis_overlap_kernel<8><<<grid, 256, 0, st>>>(V_old, V_new, M, s.D, s.k); break;
  }
  return launch_status();
}

int32_t launch_rebase_state(const svdc_shape& s, const float* M, const float* S_in, float* S_out, hipStream_t st) {
  const size_t lds = ((size_t)s.k * s.k + 4 * (size_t)s.k) * sizeof(float);
  if (lds > 48 * 1024 &&
      hipFuncSetAttribute((const void*)rebase_state_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) !=
          hipSuccess)
    return SVDC_E_HIP;
  const int rows_per_group = 64;
  dim3 grid((s.N + rows_per_group - 1) / rows_per_group, s.B);
  rebase_state_kernel<<<grid, 256, lds, st>>>(M, S_in, S_out, s.N, s.k, rows_per_group);
  return launch_status();
}

int32_t launch_basis_similarity(const svdc_shape& s, const float* V_a, const float* sigma_a, const float* V_b,
                                const float* sigma_b, float* sim_dir, float* sim_sigma, hipStream_t st) {
  basis_similarity_kernel<<<s.B, 256, 0, st>>>(V_a, sigma_a, V_b, sigma_b, sim_dir, sim_sigma, s.D, s.k);
  return launch_status();
}

}  // namespace svdc
