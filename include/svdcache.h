/*
 * svdcache.h -- C ABI of the SVD-Cache hot path for AMD MI355X (gfx950).
 *
 * The library implements the per-block, per-timestep cache step of
 * "Forecast the Principal, Stabilize the Residual" (SVD-Cache):
 *
 *   svdcache_fit_basis   rank-k right-singular basis V_k and singular values of
 *                        a feature matrix F (Sec. 3.2, Eq. 4-5; the "one-time
 *                        SVD" of Sec. 3.3)
 *   svdcache_full_step   full-compute step: C = F V_k, R = F - C V_k^T,
 *                        EMA update of the coefficient state (Eq. 8-11)
 *   svdcache_forecast    cached step: Fhat = S V_k^T + R (Sec. 3.4-3.5)
 *                        (svdcache_full_step_packed / svdcache_forecast_packed: the same two calls with the state
 *                        handed over in the reader's operand format)
 *
 * all batched over B independent blocks of equal shape, and around them
 *
 *   svdcache_select_rank / svdcache_truncate_basis       rank by retained energy (Eq. 6), per-block ranks
 *   svdcache_forecast_combine / svdcache_extrapolation_weights
 *                                                        cached step with forecasters linear in stored
 *                                                        coefficient states, optional fused add (Sec. 5.3)
 *   svdcache_full_step_residual_ema                      full step that smooths the residual too (Sec. 4.5)
 *   svdcache_basis_overlap / svdcache_rebase_state / svdcache_basis_similarity
 *                                                        basis reuse across prompts and refits (Sec. 3.3)
 *
 * General conventions
 *   - Every data pointer is a DEVICE pointer (HIP global memory) unless the
 *     argument is documented as "host".  The structs are host memory.
 *   - The caller owns every buffer.  The library never allocates or frees
 *     device memory and keeps no state between calls.
 *   - Calls only enqueue work on `stream` (a hipStream_t passed as void*;
 *     NULL = the default stream) and return; results are ready once the stream
 *     has been synchronised.  Buffers must stay alive until then.
 *   - Errors found on the host (null pointer, bad shape, alignment, parameter
 *     range, workspace too small) are returned before anything is launched.
 *     No exceptions cross this boundary.
 *   - Matrices are dense row-major.  F, R, Fhat: [B, N, D] with row stride
 *     `ldf` and block stride `block_stride` (both in elements), element type
 *     `dtype`.  V: [B, D, k] float32 contiguous (k fastest).  S, C: [B, N, k]
 *     float32 contiguous.  sigma: [B, k] float32.
 */
#ifndef SVDCACHE_H
#define SVDCACHE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* storage type of F, R and Fhat; arithmetic always accumulates in float32 or wider */
typedef enum { SVDC_F32 = 0, SVDC_BF16 = 1 } svdc_dtype;

/* Arithmetic of the bf16 matrix-core kernels (ignored by the float32 / general kernels).
 *   SVDC_PRECISE  V, C and S enter the products as bf16 high + low parts (about 16 significant
 *                 bits): results differ from exact float32 products by ~1e-5 relative.
 *   SVDC_FAST     single bf16 operands in the full step and the cached step: one third of the
 *                 matrix-core work and half the basis traffic; the error of R is about
 *                 1.1e-3 * ||C V^T|| / ||R|| relative (5e-3 when the residual holds 5 % of the energy). */
typedef enum { SVDC_PRECISE = 0, SVDC_FAST = 1 } svdc_precision;

typedef enum {
  SVDC_OK = 0,
  SVDC_E_NULL = -1,      /* a required pointer is NULL                          */
  SVDC_E_SHAPE = -2,     /* B,N,D,k, strides or ranks out of the supported range */
  SVDC_E_DTYPE = -3,     /* unknown dtype                                        */
  SVDC_E_ALIGN = -4,     /* pointer or stride not aligned as documented          */
  SVDC_E_PARAM = -5,     /* alpha, oversampling, iteration count out of range    */
  SVDC_E_WORKSPACE = -6, /* workspace / packed-basis buffer too small            */
  SVDC_E_HIP = -7        /* a HIP runtime call or kernel launch failed           */
} svdc_status;

/* Most coefficient states a linear forecaster may combine (svdcache_forecast_combine). */
#define SVDC_MAX_STATES 4

/* One batched problem: B independent blocks of identical shape.
 *   1 <= B <= 65535;  N, D <= 2^30;  1 <= k <= min(N, D), k <= 1024;  ldf >= D;  block_stride >= (N-1)*ldf + D;
 *   N*ldf and B*block_stride at most 2^48 elements (SVDC_E_SHAPE beyond).
 *   Base pointers of F/R/Fhat must be 16-byte aligned; with dtype BF16, D, ldf
 *   and block_stride must be multiples of 8 elements, with F32 multiples of 4. */
typedef struct {
  int32_t B, N, D, k;
  int64_t ldf;
  int64_t block_stride;
  int32_t dtype;     /* svdc_dtype */
  int32_t precision; /* svdc_precision; 0 = SVDC_PRECISE */
} svdc_shape;

/* Parameters of the randomized basis fit.  Zero-initialise for defaults. */
typedef struct {
  int32_t oversample_p;  /* sketch width l = k + p (clamped to min(N, D), at most 256); 0 -> p = k, -1 -> p = 0 */
  int32_t power_iters_q; /* applications of F^T F to the Gaussian sketch before the Rayleigh-Ritz step; 0 -> 3 (bf16) /
                            5 (f32); -1 -> none: the sketch is F^T Omega alone (plain randomized range finder, two
                            products with F in all; exact when rank(F) <= l, crude when the spectrum decays slowly) */
  uint64_t seed;         /* seed of the Gaussian test matrix                     */
  int32_t jacobi_max_sweeps; /* cap on the sweeps of the small SVD; 0 -> 40 (20 for sketch widths above 138); a sweep
                                that rotates nothing ends it: 6-9 sweeps in practice; at most 1000 */
  int32_t reserved;      /* set to 0 */
} svdc_fit_params;

/* Per-block status word of a basis fit (int32, bitwise OR of the flags below), written into the workspace at
 * svdcache_fit_status_offset().  0 = nothing to report.  Neither flag is an error: the call returns SVDC_OK, V is
 * orthonormal and sigma_j = ||F v_j||, but the caller may want to know. */
#define SVDC_FIT_JACOBI_CAPPED 1   /* the small SVD stopped at jacobi_max_sweeps before a sweep without rotations: sigma
                                      and V are those of the last sweep (still orthonormal), not converged */
#define SVDC_FIT_RANK_DEFICIENT 2  /* a Cholesky pivot fell to the round-off level of the float32 sketch (1e-12 x the
                                      largest diagonal entry of its Gram matrix): F, or F^T F applied to the sketch,
                                      has numerical rank < l.  The diagonal shift keeps the factorisation going; the
                                      directions beyond the numerical rank are arbitrary (their sigma is ~0) */

/* Library version (major*10000 + minor*100 + patch). */
int32_t svdcache_version(void);

/* Human-readable text for a status code (static storage, never NULL). */
const char* svdcache_strerror(int32_t status);

/* Bytes of device workspace svdcache_fit_basis needs for this shape and these
 * parameters (params may be NULL = defaults).  Returns 0 for an invalid shape.
 * svdcache_fit_workspace_bytes is the same function under its longer name. */
size_t svdcache_workspace_bytes(const svdc_shape* shape, const svdc_fit_params* params);
size_t svdcache_fit_workspace_bytes(const svdc_shape* shape, const svdc_fit_params* params);

/* Byte offset, inside the workspace of svdcache_fit_basis, of the B int32 status words (SVDC_FIT_* flags) that
 * the fit of this shape with these parameters writes, one per block.  Valid once the stream has been
 * synchronised after the fit and until the workspace is reused.  Returns 0 for an invalid shape (the words never
 * sit at offset 0). */
size_t svdcache_fit_status_offset(const svdc_shape* shape, const svdc_fit_params* params);

/* Bytes of the packed copy of the basis that the matrix-core kernels read
 * (see svdcache_pack_basis).  Returns 0 when the shape has no matrix-core
 * path; the step functions then take packed = NULL. */
size_t svdcache_packed_basis_bytes(const svdc_shape* shape);

/* 1 if full_step / forecast run their matrix-core (MFMA) kernels for this
 * shape when a packed basis is supplied, 0 if they use the general kernels.
 * The matrix-core kernels cover k <= 128 with k a multiple of 4 and D one of 256, 512, 1024, 1152, 1536, 1920, 2048,
 * 2560, 3072, 4096, 5120, for both dtypes. */
int32_t svdcache_has_mfma_path(const svdc_shape* shape);

/* Basis fit (Sec. 3.2, Eq. 4-5): the k leading right singular vectors of each
 * F[b] and their singular values, by randomized subspace iteration with a
 * Rayleigh-Ritz step (an approximation of the truncated SVD whose error is
 * controlled by oversample_p and power_iters_q).
 *   F       in   [B,N,D] dtype
 *   V       out  [B,D,k] float32, orthonormal columns, ordered by descending sigma
 *   sigma   out  [B,k]   float32, descending
 *   fro2    out  [B]     float32, ||F[b]||_F^2 (denominator of the energy rule, Eq. 6); may be NULL
 *   workspace    device scratch of at least svdcache_fit_workspace_bytes() bytes, 256-byte aligned
 * Signs of the columns of V are arbitrary.  Several launches on `stream`.  Numerical events that are not errors (a
 * capped small SVD, a rank-deficient sketch) are reported per block in the workspace: svdcache_fit_status_offset. */
int32_t svdcache_fit_basis(const svdc_shape* shape, const svdc_fit_params* params,
                           const void* F, float* V, float* sigma, float* fro2,
                           void* workspace, size_t workspace_bytes, void* stream);

/* The basis fit for callers that cannot allocate device memory or hand over a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same computation, arguments and results as
 * svdcache_fit_basis, but the workspace is a static device array of SVDC_STATIC_SCRATCH_BYTES inside the library
 * (each GPU the library runs on holds its own copy until the process ends); the call allocates and frees nothing.
 *   status  out  [B] int32 device, the SVDC_FIT_* status words of the blocks; may be NULL
 * Problems whose workspace (svdcache_workspace_bytes) exceeds SVDC_STATIC_SCRATCH_BYTES are refused with
 * SVDC_E_WORKSPACE before anything is launched: at the default parameters 32 MiB hold 8 blocks of 4608 x 3072 at
 * rank 32, 3 at rank 64, or one at rank 128.  The device that owns `stream` must be the current device.  All calls on one GPU
 * share that GPU's array: calls that overlap in time on one GPU (different streams, different threads) race and must
 * be serialised by the caller; consecutive calls on one stream are fine (the fit overwrites or clears every part of
 * the array it reads).  The first call on a device looks up the array's address (no allocation). */
#define SVDC_STATIC_SCRATCH_BYTES (32u << 20)
int32_t svdcache_fit_basis_static(const svdc_shape* shape, const svdc_fit_params* params,
                                  const void* F, float* V, float* sigma, float* fro2, int32_t* status,
                                  void* stream);

/* Re-lay V [B,D,k] float32 into the operand format of the matrix-core kernels
 * (bf16 high and low parts, tiled per 64-lane wavefront).  The packed buffer
 * is opaque, belongs to the caller, and stays valid for as long as V is
 * unchanged: pack once per fitted basis, reuse at every timestep.
 *   packed  out  svdcache_packed_basis_bytes(shape) bytes, 256-byte aligned */
int32_t svdcache_pack_basis(const svdc_shape* shape, const float* V, void* packed,
                            size_t packed_bytes, void* stream);

/* Full-compute step (Eq. 8-11), one pass over F:
 *   C = F V                       coefficients in the cached basis (sigma of Eq. 8-9 cancels)
 *   R = F - C V^T                 residual (Eq. 10)
 *   S = C                         if init != 0 (first full step)
 *   S = (1-alpha) S + alpha C     otherwise; alpha = 1 - beta of Eq. 11 (beta = 0.9 <-> alpha = 0.1)
 *   F       in      [B,N,D] dtype
 *   V       in      [B,D,k] float32 (used as given, not re-orthonormalised)
 *   packed  in      packed copy of the same V, or NULL (general kernel)
 *   R       out     [B,N,D] dtype; may be the same buffer as F (in place)
 *   S       in/out  [B,N,k] float32 (not read when init != 0)
 *   C       out     [B,N,k] float32; may be NULL
 *   alpha   in (0, 1] */
int32_t svdcache_full_step(const svdc_shape* shape, const void* F, const float* V,
                           const void* packed, void* R, float* S, float* C,
                           float alpha, int32_t init, void* stream);

/* Cached step (Sec. 3.4 last paragraph, Sec. 3.5): the EMA state is the forecast
 * of the principal coefficients and the residual is reused:
 *   Fhat = S V^T + R
 *   S in [B,N,k] float32;  V in [B,D,k] float32;  packed as above or NULL;
 *   R in [B,N,D] dtype;  Fhat out [B,N,D] dtype, may be the same buffer as R
 *   if the caller no longer needs R. */
int32_t svdcache_forecast(const svdc_shape* shape, const float* S, const float* V,
                          const void* packed, const void* R, void* Fhat, void* stream);

/* Coefficient state in the operand format of the matrix-core cached step (Sec. 3.4-3.5: the state that is read at
 * every cached step changes only at full steps, so it is laid out for the reader once, by the writer).  The packed
 * state is an opaque caller-owned buffer of svdcache_packed_state_bytes(shape) bytes, 256-byte aligned: bf16 high
 * and low parts of S (about 16 significant bits, the same values the cached step forms from float32 S), tiled per
 * 16 token rows.  It is a COPY for the cached step: S [B,N,k] float32 stays the state of record (the EMA update
 * reads and writes it).
 *
 * svdcache_packed_state_bytes   0 when the shape has no matrix-core path (then there is no packed state)
 * svdcache_pack_state           S_packed <- S, for a state that did not come from svdcache_full_step_packed
 * svdcache_full_step_packed     svdcache_full_step that also writes the packed copy of the NEW state S (same
 *                               arguments otherwise; `packed` must be given; SVDC_E_SHAPE without a matrix-core path)
 * svdcache_forecast_packed      svdcache_forecast reading the packed state: Fhat = S V^T + R, bit for bit the result
 *                               of svdcache_forecast on the float32 state it was packed from */
size_t svdcache_packed_state_bytes(const svdc_shape* shape);
int32_t svdcache_pack_state(const svdc_shape* shape, const float* S, void* S_packed, size_t S_packed_bytes,
                            void* stream);
int32_t svdcache_full_step_packed(const svdc_shape* shape, const void* F, const float* V, const void* packed,
                                  void* R, float* S, float* C, void* S_packed, size_t S_packed_bytes, float alpha,
                                  int32_t init, void* stream);
int32_t svdcache_forecast_packed(const svdc_shape* shape, const void* S_packed, const void* packed, const void* R,
                                 void* Fhat, void* stream);

/* Rank selection by retained energy (Sec. 3.2, Eq. 6; threshold tau about 0.85 in Sec. 4.5):
 * per block the smallest k* <= k with  sum_{i <= k*} sigma_i^2  >=  tau * fro2,  where fro2 = ||F||_F^2 is the
 * energy of ALL singular values (the fro2 output of svdcache_fit_basis).  Decided in float64, partial sums
 * formed left to right.
 *   sigma    in   [B,k] float32, descending (as returned by the fit)
 *   fro2     in   [B]   float32
 *   tau      in   (0, 1]
 *   k_star   out  [B] int32, in 1..k
 *   reached  out  [B] int32, nullable: 1 if the threshold was reached within the k fitted values, else 0
 *                 (then k_star = k: the basis was fitted with too small a rank for this tau) */
int32_t svdcache_select_rank(int32_t B, int32_t k, const float* sigma, const float* fro2, float tau,
                             int32_t* k_star, int32_t* reached, void* stream);

/* Per-block ranks inside one batched problem: zero the columns j >= k_star[b] of V[b] (and the entries of
 * sigma[b], nullable).  A full / cached step with the truncated basis IS the rank-k_star[b] step of block b
 * (the extra coefficients are identically zero), so blocks of different rank share one launch.  Pack the
 * basis again afterwards.
 *   V in/out [B,D,k] float32;  sigma in/out [B,k] float32 or NULL;  k_star in [B] int32, each in 0..k */
int32_t svdcache_truncate_basis(const svdc_shape* shape, float* V, float* sigma, const int32_t* k_star,
                                void* stream);

/* Weights of polynomial extrapolation from equally spaced past states (HOST function, no GPU work):
 * weights[m], m = 0..order, such that sum_m weights[m] * x(t - m*interval) is the value at t + offset of the
 * polynomial of degree `order` through x(t), x(t - interval), ..., x(t - order*interval).  order 0 is plain
 * reuse, order 1 the linear trend.  This is how a finite-difference forecaster applied to the principal
 * coefficients (Sec. 5.3) enters svdcache_forecast_combine.
 *   order in 0..SVDC_MAX_STATES-1;  offset and interval finite, interval != 0 (SVDC_E_PARAM otherwise);
 *   weights: host array of order+1 floats */
int32_t svdcache_extrapolation_weights(int32_t order, double offset, double interval, float* weights);

/* Cached step with a forecaster that is linear in stored coefficient states (Sec. 5.3: other predictors
 * applied to the low-rank part; Sec. 3.5 for the reconstruction):
 *   C_hat = sum_{m < num_states} weights[m] * S_list[m]
 *   Out   = C_hat V^T + R [+ X]
 * One state with weight 1 is svdcache_forecast.  One pass over R (and X), no intermediate buffers.
 *   num_states  1..SVDC_MAX_STATES
 *   S_list      HOST array of num_states device pointers, each [B,N,k] float32 (e.g. the C outputs of the
 *               last full steps, or EMA states)
 *   weights     HOST array of num_states floats
 *   V, packed   as in svdcache_forecast
 *   R           in  [B,N,D] dtype
 *   X           in  [B,N,D] dtype or NULL: a tensor the forecast is added to (the hidden state of a residual
 *               connection), so that the forecast itself never has to be written and read back
 *   Out         out [B,N,D] dtype; may be the same buffer as R or as X */
int32_t svdcache_forecast_combine(const svdc_shape* shape, int32_t num_states, const float* const* S_list,
                                  const float* weights, const float* V, const void* packed, const void* R,
                                  const void* X, void* Out, void* stream);

/* Full-compute step that smooths the residual state as well (the "EMA on both parts" variant of the ablation
 * in Sec. 4.5 / Fig. 5(c); the paper's method reuses the latest residual, which is alpha_r = 1):
 *   C, S as in svdcache_full_step;
 *   R = F - C V^T                                        if init != 0 or alpha_r == 1
 *   R = (1 - alpha_r) R_prev + alpha_r (F - C V^T)       otherwise
 *   R_prev  in   [B,N,D] dtype; may be NULL when it is not read; may be the buffer R (state updated in place),
 *                but must not be the buffer F
 *   alpha_r in (0, 1]; all other arguments as in svdcache_full_step (R may be the buffer F when R_prev is
 *   a third buffer or is not read) */
int32_t svdcache_full_step_residual_ema(const svdc_shape* shape, const void* F, const float* V,
                                        const void* packed, const void* R_prev, void* R, float* S, float* C,
                                        float alpha, float alpha_r, int32_t init, void* stream);

/* Basis reuse and re-basing (Sec. 3.3: one basis, fitted once, serves other prompts; Fig. 1(b): it stays
 * similar across prompts).  When a basis IS refitted, the coefficient state fitted to the old basis is carried
 * over instead of being dropped:
 *
 * svdcache_basis_overlap   M[b] = V_old[b]^T V_new[b]           ([B,k,k] float32, row i = old direction i)
 * svdcache_rebase_state    S_out[b] = S_in[b] M[b]              the coefficients of S_in V_old^T in the new basis
 *                                                               (exact when both bases span the same subspace)
 * svdcache_basis_similarity  cosine similarity times magnitude similarity, as plotted in Fig. 1(b):
 *                          sim_dir[b][j] = |<a,b>| / (|a||b|) * min(|a|,|b|) / max(|a|,|b|) for a, b = column j of
 *                          V_a[b], V_b[b]; sim_sigma[b] the same (signed cosine) for the singular-value vectors.
 *                          Values above about 0.8 mean the cached basis can be reused.
 * The shape argument supplies B, D, k (overlap, similarity) or B, N, k (rebase); k <= 128 for overlap and rebase.
 * S_out may be S_in.  sim_sigma (and then sigma_a, sigma_b) may be NULL. */
int32_t svdcache_basis_overlap(const svdc_shape* shape, const float* V_old, const float* V_new, float* M,
                               void* stream);
int32_t svdcache_rebase_state(const svdc_shape* shape, const float* M, const float* S_in, float* S_out,
                              void* stream);
int32_t svdcache_basis_similarity(const svdc_shape* shape, const float* V_a, const float* sigma_a,
                                  const float* V_b, const float* sigma_b, float* sim_dir, float* sim_sigma,
                                  void* stream);

#ifdef __cplusplus
}
#endif
#endif /* SVDCACHE_H */
