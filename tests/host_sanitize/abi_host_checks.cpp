// Host-side exercise of the C ABI for a build with AddressSanitizer and UndefinedBehaviorSanitizer on
// the host code: every path below returns before any GPU call (argument validation, size queries,
// weight computation), so it runs on a machine without a GPU.  Exit status 0 = all checks held; the
// sanitizers abort the process on a finding.
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <limits>
#include <vector>

#include "svdcache.h"

static int failures = 0;
#define EXPECT(cond)                                                        \
  do {                                                                      \
    if (!(cond)) {                                                          \
      std::fprintf(stderr, "line %d: expectation failed: %s\n", __LINE__, #cond); \
      ++failures;                                                           \
    }                                                                       \
  } while (0)

static svdc_shape make_shape(int32_t B, int32_t N, int32_t D, int32_t k, int32_t dtype) {
  svdc_shape s;
  std::memset(&s, 0, sizeof s);
  s.B = B; s.N = N; s.D = D; s.k = k;
  s.ldf = D;
  s.block_stride = (int64_t)N * D;
  s.dtype = dtype;
  s.precision = SVDC_PRECISE;
  return s;
}

int main() {
  void* const p = reinterpret_cast<void*>(uintptr_t(4096));      // aligned, never dereferenced
  void* const q = reinterpret_cast<void*>(uintptr_t(8192));
  void* const odd = reinterpret_cast<void*>(uintptr_t(4100));
  float* const pf = static_cast<float*>(p);
  float* const qf = static_cast<float*>(q);

  EXPECT(svdcache_version() > 0);
  for (int32_t code = -40; code <= 4; ++code) EXPECT(svdcache_strerror(code) != nullptr && std::strlen(svdcache_strerror(code)) > 0);
  EXPECT(std::strcmp(svdcache_strerror(std::numeric_limits<int32_t>::min()), "unknown status") == 0);

  // size queries over ordinary, degenerate and extreme shapes (the arithmetic must not overflow)
  const int32_t big = std::numeric_limits<int32_t>::max();
  const int32_t Bs[] = {1, 2, 57, 60, 65535, 65536, 0, -1};
  const int32_t Ns[] = {1, 15, 16, 64, 4608, 119056, big, 0, -7};
  const int32_t Ds[] = {8, 64, 128, 1024, 3072, 8192, big - 127, big, 0};
  const int32_t ks[] = {1, 8, 32, 64, 128, 129, 256, 257, 1024, 1025, big, 0, -3};
  for (int32_t dtype : {(int32_t)SVDC_F32, (int32_t)SVDC_BF16, 7})
    for (int32_t B : Bs) for (int32_t N : Ns) for (int32_t D : Ds) for (int32_t k : ks) {
      svdc_shape s = make_shape(B, N, D, k, dtype);
      const size_t pk = svdcache_packed_basis_bytes(&s);
      const int32_t has = svdcache_has_mfma_path(&s);
      EXPECT((pk > 0) == (has == 1));
      for (int32_t pp : {0, -1, 5, 300, big, -9}) for (int32_t qq : {0, -1, 2, 1000, -9}) {
        svdc_fit_params fp{}; fp.oversample_p = pp; fp.power_iters_q = qq; fp.seed = 1;
        fp.jacobi_max_sweeps = (pp == 5) ? qq : 0;
        const size_t need = svdcache_fit_workspace_bytes(&s, &fp);
        EXPECT(svdcache_workspace_bytes(&s, &fp) == need);
        const size_t off = svdcache_fit_status_offset(&s, &fp);
        EXPECT((need == 0) == (off == 0));
        if (need) EXPECT(off % 256 == 0 && off + sizeof(int32_t) * (size_t)s.B <= need);
      }
      (void)svdcache_fit_workspace_bytes(&s, nullptr);
      // the step entry points see the same shapes with a misaligned pointer: they must refuse, whatever the shape
      EXPECT(svdcache_forecast(&s, pf, pf, nullptr, odd, q, nullptr) < 0);
      EXPECT(svdcache_full_step(&s, odd, pf, nullptr, q, pf, nullptr, 0.5f, 1, nullptr) < 0);
    }
  // strides at the end of the int64 range
  for (int64_t ldf : {(int64_t)64, (int64_t)1 << 40, std::numeric_limits<int64_t>::max() - 7, std::numeric_limits<int64_t>::max(), (int64_t)-64})
    for (int64_t bs : {(int64_t)64 * 64, (int64_t)1 << 62, std::numeric_limits<int64_t>::max() - 7, std::numeric_limits<int64_t>::max(), (int64_t)-8}) {
      svdc_shape s = make_shape(2, 64, 64, 8, SVDC_BF16);
      s.ldf = ldf; s.block_stride = bs;
      (void)svdcache_fit_workspace_bytes(&s, nullptr);
      (void)svdcache_packed_basis_bytes(&s);
      EXPECT(svdcache_forecast(&s, pf, pf, nullptr, odd, q, nullptr) < 0);
    }

  // null / parameter / alignment / workspace refusals of every entry point
  svdc_shape s = make_shape(1, 64, 64, 8, SVDC_F32);
  EXPECT(svdcache_full_step(nullptr, p, pf, nullptr, q, pf, nullptr, 0.5f, 1, nullptr) == SVDC_E_NULL);
  EXPECT(svdcache_full_step(&s, nullptr, pf, nullptr, q, pf, nullptr, 0.5f, 1, nullptr) == SVDC_E_NULL);
  for (float a : {0.f, -1.f, 1.0001f, std::nanf(""), INFINITY})
    EXPECT(svdcache_full_step(&s, p, pf, nullptr, q, pf, nullptr, a, 1, nullptr) == SVDC_E_PARAM);
  EXPECT(svdcache_forecast(&s, pf, pf, nullptr, nullptr, q, nullptr) == SVDC_E_NULL);
  const size_t need = svdcache_fit_workspace_bytes(&s, nullptr);
  EXPECT(need > 0);
  EXPECT(svdcache_fit_basis(&s, nullptr, p, pf, pf, nullptr, q, need - 1, nullptr) == SVDC_E_WORKSPACE);
  EXPECT(svdcache_fit_basis(&s, nullptr, p, pf, pf, nullptr, nullptr, need, nullptr) == SVDC_E_NULL);
  EXPECT(svdcache_fit_basis(&s, nullptr, p, pf, pf, nullptr, odd, need, nullptr) == SVDC_E_ALIGN);
  EXPECT(svdcache_pack_basis(&s, pf, p, 0, nullptr) < 0);
  EXPECT(svdcache_full_step_residual_ema(&s, p, pf, nullptr, nullptr, q, pf, nullptr, 0.5f, 0.5f, 0, nullptr) == SVDC_E_NULL);
  EXPECT(svdcache_full_step_residual_ema(&s, p, pf, nullptr, p, q, pf, nullptr, 0.5f, 0.5f, 0, nullptr) == SVDC_E_PARAM);
  EXPECT(svdcache_full_step_residual_ema(&s, p, pf, nullptr, q, q, pf, nullptr, 0.5f, 2.f, 0, nullptr) == SVDC_E_PARAM);

  int32_t* const pi = static_cast<int32_t*>(p);
  EXPECT(svdcache_select_rank(1, 4, nullptr, pf, 0.85f, pi, nullptr, nullptr) == SVDC_E_NULL);
  EXPECT(svdcache_select_rank(0, 4, pf, pf, 0.85f, pi, nullptr, nullptr) == SVDC_E_SHAPE);
  EXPECT(svdcache_select_rank(big, big, pf, pf, 0.85f, pi, nullptr, nullptr) == SVDC_E_SHAPE);
  EXPECT(svdcache_select_rank(1, 4, pf, pf, std::nanf(""), pi, nullptr, nullptr) == SVDC_E_PARAM);
  EXPECT(svdcache_truncate_basis(&s, nullptr, nullptr, pi, nullptr) == SVDC_E_NULL);
  EXPECT(svdcache_truncate_basis(nullptr, pf, nullptr, pi, nullptr) == SVDC_E_NULL);

  // extrapolation weights: host arithmetic; each set sums to one and reproduces polynomials of its order
  for (int32_t order = 0; order < SVDC_MAX_STATES; ++order)
    for (double off : {0.0, 1.0, 2.5, 5.0, -4.0, 1e6})
      for (double itv : {1.0, 3.0, 6.0, 1e-3}) {
        float w[SVDC_MAX_STATES] = {0, 0, 0, 0};
        EXPECT(svdcache_extrapolation_weights(order, off, itv, w) == SVDC_OK);
        double sum = 0, scale = 0;
        for (int m = 0; m <= order; ++m) { sum += w[m]; scale += std::fabs(w[m]); }
        EXPECT(std::fabs(sum - 1.0) <= 1e-6 * scale);
      }
  float w4[SVDC_MAX_STATES];
  EXPECT(svdcache_extrapolation_weights(1, 1.0, 6.0, nullptr) == SVDC_E_NULL);
  EXPECT(svdcache_extrapolation_weights(SVDC_MAX_STATES, 1.0, 6.0, w4) == SVDC_E_PARAM);
  EXPECT(svdcache_extrapolation_weights(-1, 1.0, 6.0, w4) == SVDC_E_PARAM);
  EXPECT(svdcache_extrapolation_weights(big, 1.0, 6.0, w4) == SVDC_E_PARAM);
  EXPECT(svdcache_extrapolation_weights(1, 1.0, 0.0, w4) == SVDC_E_PARAM);
  EXPECT(svdcache_extrapolation_weights(1, std::nan(""), 6.0, w4) == SVDC_E_PARAM);
  EXPECT(svdcache_extrapolation_weights(1, 1.0, INFINITY, w4) == SVDC_E_PARAM);

  // combination of states: list validation reads exactly num_states entries of each host array
  {
    std::vector<const float*> list(SVDC_MAX_STATES, pf);
    std::vector<float> w(SVDC_MAX_STATES, 0.25f);
    EXPECT(svdcache_forecast_combine(&s, 0, list.data(), w.data(), pf, nullptr, p, nullptr, q, nullptr) == SVDC_E_PARAM);
    EXPECT(svdcache_forecast_combine(&s, SVDC_MAX_STATES + 1, list.data(), w.data(), pf, nullptr, p, nullptr, q, nullptr) == SVDC_E_PARAM);
    EXPECT(svdcache_forecast_combine(&s, big, list.data(), w.data(), pf, nullptr, p, nullptr, q, nullptr) == SVDC_E_PARAM);
    EXPECT(svdcache_forecast_combine(&s, 1, nullptr, w.data(), pf, nullptr, p, nullptr, q, nullptr) == SVDC_E_NULL);
    std::vector<const float*> one(1, static_cast<const float*>(odd));   // exactly one entry: reading a second is an overrun
    std::vector<float> w1(1, 1.f);
    EXPECT(svdcache_forecast_combine(&s, 1, one.data(), w1.data(), pf, nullptr, p, nullptr, q, nullptr) == SVDC_E_ALIGN);
    one[0] = nullptr;
    EXPECT(svdcache_forecast_combine(&s, 1, one.data(), w1.data(), pf, nullptr, p, nullptr, q, nullptr) == SVDC_E_NULL);
    one[0] = pf; w1[0] = std::nanf("");
    EXPECT(svdcache_forecast_combine(&s, 1, one.data(), w1.data(), pf, nullptr, p, nullptr, q, nullptr) == SVDC_E_PARAM);
  }

  // basis reuse
  EXPECT(svdcache_basis_overlap(&s, nullptr, pf, qf, nullptr) == SVDC_E_NULL);
  EXPECT(svdcache_rebase_state(&s, pf, nullptr, qf, nullptr) == SVDC_E_NULL);
  EXPECT(svdcache_basis_similarity(&s, pf, nullptr, nullptr, nullptr, qf, nullptr, nullptr) == SVDC_E_NULL);
  svdc_shape wide = make_shape(1, 2048, 2048, 1024, SVDC_F32);
  EXPECT(svdcache_basis_overlap(&wide, pf, pf, qf, nullptr) == SVDC_E_SHAPE);
  EXPECT(svdcache_rebase_state(&wide, pf, pf, qf, nullptr) == SVDC_E_SHAPE);

  if (failures) {
    std::fprintf(stderr, "%d host ABI expectation(s) failed\n", failures);
    return 1;
  }
  std::puts("host ABI checks passed");
  return 0;
}
