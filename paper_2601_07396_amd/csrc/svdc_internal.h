// Host-side declarations shared between the translation units of libsvdcache.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/svdcache.h"

namespace svdc {

inline int32_t launch_status() { return hipGetLastError() == hipSuccess ? SVDC_OK : SVDC_E_HIP; }

// ---- general (any-shape) kernels: general_kernels.hip -----------------------
int32_t launch_full_step_general(const svdc_shape& s, const void* F, const float* V, void* R, float* S,
                                 float* C, float alpha, int init, hipStream_t st);
int32_t launch_forecast_general(const svdc_shape& s, const float* S, const float* V, const void* R,
                                void* Fhat, hipStream_t st);

// ---- matrix-core kernels: mfma_kernels.hip -----------------------------------
bool mfma_shape_supported(const svdc_shape& s);
size_t mfma_packed_bytes(const svdc_shape& s);
int32_t launch_pack_basis(const svdc_shape& s, const float* V, void* packed, hipStream_t st);
int32_t launch_full_step_mfma(const svdc_shape& s, const void* F, const void* packed, void* R, float* S,
                              float* C, float alpha, int init, hipStream_t st);
int32_t launch_forecast_mfma(const svdc_shape& s, const float* S, const void* packed, const void* R,
                             void* Fhat, hipStream_t st);

// ---- basis fit: fit_kernels.hip ------------------------------------------------
struct FitPlan {
  int l;          // sketch width
  int q;          // power iterations
  uint64_t seed;
  size_t off_Q, off_Z, off_Y, off_G, off_M, off_W, off_misc, off_Qp, total;
  bool mfma;      // products with F on the matrix cores
};
bool make_fit_plan(const svdc_shape& s, const svdc_fit_params* p, FitPlan* plan);
int32_t run_fit(const svdc_shape& s, const FitPlan& plan, const void* F, float* V, float* sigma, float* fro2,
                void* workspace, hipStream_t st);

// ---- matrix-core products of the basis fit: fit_mfma_kernels.hip ------------------------
bool fit_mfma_supported(const svdc_shape& s, int l);
size_t fit_mfma_packed_q_bytes(const svdc_shape& s, int l);
void fit_mfma_pack_q(const svdc_shape& s, int l, const float* Q, void* Qp, hipStream_t st);
// Y = F Q;  fro_acc (nullable) += ||F||_F^2;  split: bf16 high + low parts of Q
void fit_mfma_project(const svdc_shape& s, int l, const void* F, const void* Qp, float* Y, double* fro_acc,
                      bool split, hipStream_t st);
// Z = F^T Y
void fit_mfma_backproject(const svdc_shape& s, int l, const void* F, const float* Y, float* Z, hipStream_t st);

}  // namespace svdc
