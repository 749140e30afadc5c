// Host-side declarations shared between the translation units of libsvdcache.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/svdcache.h"

namespace svdc {

inline int32_t launch_status() { return hipGetLastError() == hipSuccess ? SVDC_OK : SVDC_E_HIP; }

// Coefficient states of a forecaster that is linear in them: C_hat = sum_{i < m} w[i] * s[i] (device pointers,
// each [B, N, k] float32).  Passed to kernels by value.
constexpr int kMaxStates = SVDC_MAX_STATES;
struct CoefStates {
  const float* s[kMaxStates];
  float w[kMaxStates];
  int m;
};

// ---- general (any-shape) kernels: general_kernels.hip -----------------------
// Optional smoothing of the residual state: R = (1 - alpha_r) prev + alpha_r (F - C V^T); prev == nullptr: plain.
struct ResidualEma {
  const void* prev = nullptr;
  float alpha_r = 1.f;
  void* packed_state = nullptr;   // matrix-core full step only: second output of the new state, as operand words
};
int32_t launch_full_step_general(const svdc_shape& s, const void* F, const float* V, void* R, float* S,
                                 float* C, float alpha, int init, ResidualEma re, hipStream_t st);
// Out = (sum_m w_m S_m) V^T + R [+ X]   (X nullable)
int32_t launch_forecast_general(const svdc_shape& s, const CoefStates& cs, const float* V, const void* R,
                                const void* X, void* Out, hipStream_t st);
// rank selection by retained energy and truncation of a fitted basis to per-block ranks
int32_t launch_select_rank(int B, int k, const float* sigma, const float* fro2, float tau, int32_t* k_star,
                           int32_t* reached, hipStream_t st);
int32_t launch_truncate_basis(const svdc_shape& s, float* V, float* sigma, const int32_t* k_star, hipStream_t st);

// ---- basis reuse and re-basing: basis_kernels.hip ------------------------------------------
bool rebase_rank_supported(int k);
int32_t launch_basis_overlap(const svdc_shape& s, const float* V_old, const float* V_new, float* M, hipStream_t st);
int32_t launch_rebase_state(const svdc_shape& s, const float* M, const float* S_in, float* S_out, hipStream_t st);
int32_t launch_basis_similarity(const svdc_shape& s, const float* V_a, const float* sigma_a, const float* V_b,
                                const float* sigma_b, float* sim_dir, float* sim_sigma, hipStream_t st);

// ---- matrix-core kernels: mfma_kernels.hip -----------------------------------
bool mfma_shape_supported(const svdc_shape& s);
size_t mfma_packed_bytes(const svdc_shape& s);
int32_t launch_pack_basis(const svdc_shape& s, const float* V, void* packed, hipStream_t st);
int32_t launch_full_step_mfma(const svdc_shape& s, const void* F, const void* packed, void* R, float* S,
                              float* C, float alpha, int init, ResidualEma re, hipStream_t st);
int32_t launch_forecast_mfma(const svdc_shape& s, const float* S, const void* packed, const void* R,
                             void* Fhat, hipStream_t st);
// Coefficient state as the cached step's operand words (bf16 high + low parts of -S, tiled per 16 rows)
size_t mfma_packed_state_bytes(const svdc_shape& s);
int32_t launch_pack_state(const svdc_shape& s, const float* S, void* Sp, hipStream_t st);
int32_t launch_forecast_packed_mfma(const svdc_shape& s, const void* Sp, const void* packed, const void* R,
                                    void* Fhat, hipStream_t st);
int32_t launch_forecast_combine_mfma(const svdc_shape& s, const CoefStates& cs, const void* packed, const void* R,
                                     const void* X, void* Out, hipStream_t st);

// ---- basis fit: fit_kernels.hip ------------------------------------------------
struct FitPlan {
  int l;          // sketch width
  int q;          // power iterations
  uint64_t seed;
  int max_sweeps; // cap on the Jacobi sweeps
  size_t off_Q, off_Z, off_Y, off_G, off_Gp, off_M, off_W, off_misc, off_info, off_jcnt, off_Qp, total;
  bool mfma;      // products with F on the matrix cores
};
bool make_fit_plan(const svdc_shape& s, const svdc_fit_params* p, FitPlan* plan);
int32_t run_fit(const svdc_shape& s, const FitPlan& plan, const void* F, float* V, float* sigma, float* fro2,
                void* workspace, hipStream_t st);

// ---- matrix-core products of the basis fit: fit_mfma_kernels.hip ------------------------
bool fit_mfma_supported(const svdc_shape& s, int l);
size_t fit_mfma_packed_q_bytes(const svdc_shape& s, int l);
void fit_mfma_pack_q(const svdc_shape& s, int l, const float* Q, void* Qp, hipStream_t st);
// Bytes of Y rounded to bf16 in the operand layout of the back-projection (written by fit_mfma_project when asked)
size_t fit_mfma_packed_y_bytes(const svdc_shape& s, int l);
// Y = F Q;  fro_acc (nullable) += ||F||_F^2;  split: bf16 high + low parts of Q.
// Ypacked != nullptr (plain operands only): the result goes there in packed bf16 form and Y is not written.
void fit_mfma_project(const svdc_shape& s, int l, const void* F, const void* Qp, float* Y, void* Ypacked,
                      double* fro_acc, bool split, hipStream_t st);
// Z = F^T Y, with Y as float32 rows or (Ypacked != nullptr) in the packed form
void fit_mfma_backproject(const svdc_shape& s, int l, const void* F, const float* Y, const void* Ypacked, float* Z,
                          hipStream_t st);

}  // namespace svdc
