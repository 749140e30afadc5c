// C ABI of libsvdcache: argument validation and dispatch.  See include/svdcache.h.
#include <stdint.h>

#include <mutex>

#include "svdc_internal.h"

using namespace svdc;

// Workspace of svdcache_fit_basis_static: one array per GPU, part of the loaded code object, so the entry point
// never allocates.  In host code this name is only a handle for hipGetSymbolAddress; the device address it resolves
// to (per device) is what kernels get.
static __device__ __align__(256) unsigned char scratch[SVDC_STATIC_SCRATCH_BYTES];

namespace {

bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

int32_t check_shape(const svdc_shape* s) {
  if (!s) return SVDC_E_NULL;
  if (s->dtype != SVDC_F32 && s->dtype != SVDC_BF16) return SVDC_E_DTYPE;
  if (s->precision != SVDC_PRECISE && s->precision != SVDC_FAST) return SVDC_E_PARAM;
  if (s->B < 1 || s->B > 65535 || s->N < 1 || s->D < 1 || s->k < 1) return SVDC_E_SHAPE;
  if (s->N > (1 << 30) || s->D > (1 << 30)) return SVDC_E_SHAPE;   // tile counts such as (N + 31) / 32 stay in int
  if (s->k > s->N || s->k > s->D || s->k > 1024) return SVDC_E_SHAPE;
  // At most 2^48 elements from the first to the last block: more than any device holds, and small enough
  // that no offset or byte count computed from these strides leaves the int64 range.
  constexpr int64_t kMaxElems = int64_t(1) << 48;
  if (s->ldf < s->D || s->ldf > kMaxElems / s->N) return SVDC_E_SHAPE;
  if (s->block_stride < (int64_t)(s->N - 1) * s->ldf + s->D || s->block_stride > kMaxElems / s->B) return SVDC_E_SHAPE;
  const int64_t unit = s->dtype == SVDC_BF16 ? 8 : 4;
  if (s->D % unit || s->ldf % unit || s->block_stride % unit) return SVDC_E_ALIGN;
  return SVDC_OK;
}

constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices];   // device address of `scratch` on each device, resolved on first use
std::mutex g_scratch_mutex;

// Address of the current device's copy of `scratch` (looked up once per device, with that device current).
int32_t static_scratch(void** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return SVDC_E_HIP;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return SVDC_E_HIP;
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return SVDC_OK;
}

__global__ void copy_status_kernel(const int32_t* __restrict__ src, int32_t* __restrict__ dst, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) dst[i] = src[i];
}

}  // namespace

extern "C" {

int32_t svdcache_version(void) { return 300; }   // 0.3.0: fit status words, svdcache_workspace_bytes

const char* svdcache_strerror(int32_t status) {
  switch (status) {
    case SVDC_OK: return "ok";
    case SVDC_E_NULL: return "a required pointer is NULL";
    case SVDC_E_SHAPE: return "shape, stride or rank out of the supported range";
    case SVDC_E_DTYPE: return "unknown dtype";
    case SVDC_E_ALIGN: return "pointer or stride not aligned as documented";
    case SVDC_E_PARAM: return "parameter out of range";
    case SVDC_E_WORKSPACE: return "workspace or packed-basis buffer too small";
    case SVDC_E_HIP: return "HIP runtime call or kernel launch failed";
    default: return "unknown status";
  }
}

size_t svdcache_fit_workspace_bytes(const svdc_shape* shape, const svdc_fit_params* params) {
  FitPlan plan;
  if (check_shape(shape) != SVDC_OK || !make_fit_plan(*shape, params, &plan)) return 0;
  return plan.total;
}

size_t svdcache_workspace_bytes(const svdc_shape* shape, const svdc_fit_params* params) {
  return svdcache_fit_workspace_bytes(shape, params);
}

size_t svdcache_fit_status_offset(const svdc_shape* shape, const svdc_fit_params* params) {
  FitPlan plan;
  if (check_shape(shape) != SVDC_OK || !make_fit_plan(*shape, params, &plan)) return 0;
  return plan.off_info;
}

size_t svdcache_packed_basis_bytes(const svdc_shape* shape) {
  if (check_shape(shape) != SVDC_OK || !mfma_shape_supported(*shape)) return 0;
  return mfma_packed_bytes(*shape);
}

int32_t svdcache_has_mfma_path(const svdc_shape* shape) {
  return check_shape(shape) == SVDC_OK && mfma_shape_supported(*shape) ? 1 : 0;
}

int32_t svdcache_fit_basis(const svdc_shape* shape, const svdc_fit_params* params, const void* F, float* V,
                           float* sigma, float* fro2, void* workspace, size_t workspace_bytes, void* stream) {
  int32_t rc = check_shape(shape);
  if (rc != SVDC_OK) return rc;
  if (!F || !V || !sigma || !workspace) return SVDC_E_NULL;
  if (!aligned(F, 16) || !aligned(V, 16) || !aligned(workspace, 256)) return SVDC_E_ALIGN;
  FitPlan plan;
  if (shape->k > 256) return SVDC_E_SHAPE;
  if (!make_fit_plan(*shape, params, &plan)) return SVDC_E_PARAM;
  if (workspace_bytes < plan.total) return SVDC_E_WORKSPACE;
  return run_fit(*shape, plan, F, V, sigma, fro2, workspace, (hipStream_t)stream);
}

int32_t svdcache_fit_basis_static(const svdc_shape* shape, const svdc_fit_params* params, const void* F, float* V,
                                  float* sigma, float* fro2, int32_t* status, void* stream) {
  int32_t rc = check_shape(shape);
  if (rc != SVDC_OK) return rc;
  if (!F || !V || !sigma) return SVDC_E_NULL;
  if (!aligned(F, 16) || !aligned(V, 16) || (status && !aligned(status, 4))) return SVDC_E_ALIGN;
  FitPlan plan;
  if (shape->k > 256) return SVDC_E_SHAPE;
  if (!make_fit_plan(*shape, params, &plan)) return SVDC_E_PARAM;
  if (plan.total > (size_t)SVDC_STATIC_SCRATCH_BYTES) return SVDC_E_WORKSPACE;
  void* ws = nullptr;
  rc = static_scratch(&ws);
  if (rc != SVDC_OK) return rc;
  // the fit clears what must start at zero (accumulators, status words) with fill kernels of its own
  rc = run_fit(*shape, plan, F, V, sigma, fro2, ws, (hipStream_t)stream);
  if (rc != SVDC_OK || !status) return rc;
  copy_status_kernel<<<(shape->B + 255) / 256, 256, 0, (hipStream_t)stream>>>(
      reinterpret_cast<const int32_t*>(static_cast<const char*>(ws) + plan.off_info), status, shape->B);
  return launch_status();
}

int32_t svdcache_pack_basis(const svdc_shape* shape, const float* V, void* packed, size_t packed_bytes,
                            void* stream) {
  int32_t rc = check_shape(shape);
  if (rc != SVDC_OK) return rc;
  if (!V || !packed) return SVDC_E_NULL;
  if (!mfma_shape_supported(*shape)) return SVDC_E_SHAPE;
  if (!aligned(V, 16) || !aligned(packed, 256)) return SVDC_E_ALIGN;
  if (packed_bytes < mfma_packed_bytes(*shape)) return SVDC_E_WORKSPACE;
  return launch_pack_basis(*shape, V, packed, (hipStream_t)stream);
}

int32_t svdcache_full_step(const svdc_shape* shape, const void* F, const float* V, const void* packed, void* R,
                           float* S, float* C, float alpha, int32_t init, void* stream) {
  int32_t rc = check_shape(shape);
  if (rc != SVDC_OK) return rc;
  if (!F || !V || !R || !S) return SVDC_E_NULL;
  if (!(alpha > 0.f && alpha <= 1.f)) return SVDC_E_PARAM;
  if (!aligned(F, 16) || !aligned(R, 16) || !aligned(V, 16) || !aligned(S, 16) || (C && !aligned(C, 16)))
    return SVDC_E_ALIGN;
  if (packed && mfma_shape_supported(*shape)) {
    if (!aligned(packed, 256)) return SVDC_E_ALIGN;
    return launch_full_step_mfma(*shape, F, packed, R, S, C, alpha, init != 0, ResidualEma{}, (hipStream_t)stream);
  }
  return launch_full_step_general(*shape, F, V, R, S, C, alpha, init != 0, ResidualEma{}, (hipStream_t)stream);
}

int32_t svdcache_full_step_residual_ema(const svdc_shape* shape, const void* F, const float* V, const void* packed,
                                        const void* R_prev, void* R, float* S, float* C, float alpha,
                                        float alpha_r, int32_t init, void* stream) {
  int32_t rc = check_shape(shape);
  if (rc != SVDC_OK) return rc;
  if (!F || !V || !R || !S) return SVDC_E_NULL;
  if (!(alpha > 0.f && alpha <= 1.f) || !(alpha_r > 0.f && alpha_r <= 1.f)) return SVDC_E_PARAM;
  ResidualEma re;
  if (init == 0 && alpha_r < 1.f) {
    if (!R_prev) return SVDC_E_NULL;
    // the previous residual is read while the new one is written: it may be the output buffer (updated in
    // place) but then the output cannot also be the feature buffer
    if (R_prev == F) return SVDC_E_PARAM;
    if (!aligned(R_prev, 16)) return SVDC_E_ALIGN;
    re.prev = R_prev;
    re.alpha_r = alpha_r;
  }
  if (!aligned(F, 16) || !aligned(R, 16) || !aligned(V, 16) || !aligned(S, 16) || (C && !aligned(C, 16)))
    return SVDC_E_ALIGN;
  if (packed && mfma_shape_supported(*shape)) {
    if (!aligned(packed, 256)) return SVDC_E_ALIGN;
    return launch_full_step_mfma(*shape, F, packed, R, S, C, alpha, init != 0, re, (hipStream_t)stream);
  }
  return launch_full_step_general(*shape, F, V, R, S, C, alpha, init != 0, re, (hipStream_t)stream);
}

int32_t svdcache_forecast(const svdc_shape* shape, const float* S, const float* V, const void* packed,
                          const void* R, void* Fhat, void* stream) {
  int32_t rc = check_shape(shape);
  if (rc != SVDC_OK) return rc;
  if (!S || !V || !R || !Fhat) return SVDC_E_NULL;
  if (!aligned(R, 16) || !aligned(Fhat, 16) || !aligned(V, 16) || !aligned(S, 16)) return SVDC_E_ALIGN;
  if (packed && mfma_shape_supported(*shape)) {
    if (!aligned(packed, 256)) return SVDC_E_ALIGN;
    return launch_forecast_mfma(*shape, S, packed, R, Fhat, (hipStream_t)stream);
  }
  CoefStates cs{};
  cs.s[0] = S;
  cs.w[0] = 1.f;
  cs.m = 1;
  return launch_forecast_general(*shape, cs, V, R, nullptr, Fhat, (hipStream_t)stream);
}

size_t svdcache_packed_state_bytes(const svdc_shape* shape) {
  if (check_shape(shape) != SVDC_OK || !mfma_shape_supported(*shape)) return 0;
  return mfma_packed_state_bytes(*shape);
}

int32_t svdcache_pack_state(const svdc_shape* shape, const float* S, void* S_packed, size_t S_packed_bytes,
                            void* stream) {
  int32_t rc = check_shape(shape);
  if (rc != SVDC_OK) return rc;
  if (!S || !S_packed) return SVDC_E_NULL;
  if (!mfma_shape_supported(*shape)) return SVDC_E_SHAPE;
  if (!aligned(S, 16) || !aligned(S_packed, 256)) return SVDC_E_ALIGN;
  if (S_packed_bytes < mfma_packed_state_bytes(*shape)) return SVDC_E_WORKSPACE;
  return launch_pack_state(*shape, S, S_packed, (hipStream_t)stream);
}

int32_t svdcache_full_step_packed(const svdc_shape* shape, const void* F, const float* V, const void* packed, void* R,
                                  float* S, float* C, void* S_packed, size_t S_packed_bytes, float alpha,
                                  int32_t init, void* stream) {
  int32_t rc = check_shape(shape);
  if (rc != SVDC_OK) return rc;
  if (!F || !V || !R || !S || !packed || !S_packed) return SVDC_E_NULL;
  if (!(alpha > 0.f && alpha <= 1.f)) return SVDC_E_PARAM;
  if (!mfma_shape_supported(*shape)) return SVDC_E_SHAPE;
  if (!aligned(F, 16) || !aligned(R, 16) || !aligned(V, 16) || !aligned(S, 16) || (C && !aligned(C, 16)) ||
      !aligned(packed, 256) || !aligned(S_packed, 256))
    return SVDC_E_ALIGN;
  if (S_packed_bytes < mfma_packed_state_bytes(*shape)) return SVDC_E_WORKSPACE;
  ResidualEma re;
  re.packed_state = S_packed;
  return launch_full_step_mfma(*shape, F, packed, R, S, C, alpha, init != 0, re, (hipStream_t)stream);
}

int32_t svdcache_forecast_packed(const svdc_shape* shape, const void* S_packed, const void* packed, const void* R,
                                 void* Fhat, void* stream) {
  int32_t rc = check_shape(shape);
  if (rc != SVDC_OK) return rc;
  if (!S_packed || !packed || !R || !Fhat) return SVDC_E_NULL;
  if (!mfma_shape_supported(*shape)) return SVDC_E_SHAPE;
  if (!aligned(R, 16) || !aligned(Fhat, 16) || !aligned(packed, 256) || !aligned(S_packed, 256)) return SVDC_E_ALIGN;
  return launch_forecast_packed_mfma(*shape, S_packed, packed, R, Fhat, (hipStream_t)stream);
}

int32_t svdcache_select_rank(int32_t B, int32_t k, const float* sigma, const float* fro2, float tau,
                             int32_t* k_star, int32_t* reached, void* stream) {
  if (!sigma || !fro2 || !k_star) return SVDC_E_NULL;
  if (B < 1 || k < 1 || k > 1024) return SVDC_E_SHAPE;
  if (!(tau > 0.f && tau <= 1.f)) return SVDC_E_PARAM;
  return launch_select_rank(B, k, sigma, fro2, tau, k_star, reached, (hipStream_t)stream);
}

int32_t svdcache_truncate_basis(const svdc_shape* shape, float* V, float* sigma, const int32_t* k_star,
                                void* stream) {
  int32_t rc = check_shape(shape);
  if (rc != SVDC_OK) return rc;
  if (!V || !k_star) return SVDC_E_NULL;
  return launch_truncate_basis(*shape, V, sigma, k_star, (hipStream_t)stream);
}

int32_t svdcache_extrapolation_weights(int32_t order, double offset, double interval, float* weights) {
  if (!weights) return SVDC_E_NULL;
  const auto finite = [](double v) { return v - v == 0.0; };   // false for NaN and for +-inf
  if (order < 0 || order >= SVDC_MAX_STATES || interval == 0.0 || !finite(interval) || !finite(offset))
    return SVDC_E_PARAM;
  // Lagrange weights at x = offset / interval for the nodes 0, -1, ..., -order
  const double x = offset / interval;
  for (int m = 0; m <= order; ++m) {
    double w = 1.0;
    for (int i = 0; i <= order; ++i)
      if (i != m) w *= (x + i) / (double)(i - m);
    weights[m] = (float)w;
  }
  return SVDC_OK;
}

int32_t svdcache_forecast_combine(const svdc_shape* shape, int32_t num_states, const float* const* S_list,
                                  const float* weights, const float* V, const void* packed, const void* R,
                                  const void* X, void* Out, void* stream) {
  int32_t rc = check_shape(shape);
  if (rc != SVDC_OK) return rc;
  if (!S_list || !weights || !V || !R || !Out) return SVDC_E_NULL;
  if (num_states < 1 || num_states > SVDC_MAX_STATES) return SVDC_E_PARAM;
  CoefStates cs{};
  cs.m = num_states;
  for (int m = 0; m < num_states; ++m) {
    if (!S_list[m]) return SVDC_E_NULL;
    if (!aligned(S_list[m], 16)) return SVDC_E_ALIGN;
    if (!(weights[m] == weights[m])) return SVDC_E_PARAM;   // NaN
    cs.s[m] = S_list[m];
    cs.w[m] = weights[m];
  }
  if (!aligned(R, 16) || !aligned(Out, 16) || !aligned(V, 16) || (X && !aligned(X, 16))) return SVDC_E_ALIGN;
  if (packed && mfma_shape_supported(*shape)) {
    if (!aligned(packed, 256)) return SVDC_E_ALIGN;
    return launch_forecast_combine_mfma(*shape, cs, packed, R, X, Out, (hipStream_t)stream);
  }
  return launch_forecast_general(*shape, cs, V, R, X, Out, (hipStream_t)stream);
}

int32_t svdcache_basis_overlap(const svdc_shape* shape, const float* V_old, const float* V_new, float* M,
                               void* stream) {
  int32_t rc = check_shape(shape);
  if (rc != SVDC_OK) return rc;
  if (!V_old || !V_new || !M) return SVDC_E_NULL;
  if (!rebase_rank_supported(shape->k)) return SVDC_E_SHAPE;
  return launch_basis_overlap(*shape, V_old, V_new, M, (hipStream_t)stream);
}

int32_t svdcache_rebase_state(const svdc_shape* shape, const float* M, const float* S_in, float* S_out,
                              void* stream) {
  int32_t rc = check_shape(shape);
  if (rc != SVDC_OK) return rc;
  if (!M || !S_in || !S_out) return SVDC_E_NULL;
  if (!rebase_rank_supported(shape->k)) return SVDC_E_SHAPE;
  return launch_rebase_state(*shape, M, S_in, S_out, (hipStream_t)stream);
}

int32_t svdcache_basis_similarity(const svdc_shape* shape, const float* V_a, const float* sigma_a,
                                  const float* V_b, const float* sigma_b, float* sim_dir, float* sim_sigma,
                                  void* stream) {
  int32_t rc = check_shape(shape);
  if (rc != SVDC_OK) return rc;
  if (!V_a || !V_b || !sim_dir) return SVDC_E_NULL;
  if (sim_sigma && (!sigma_a || !sigma_b)) return SVDC_E_NULL;
  return launch_basis_similarity(*shape, V_a, sigma_a, V_b, sigma_b, sim_dir, sim_sigma, (hipStream_t)stream);
}

}  // extern "C"
