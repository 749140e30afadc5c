// Matrix-core (MFMA) kernels for bf16 features -- placeholder until the fast path lands.
#include "svdc_device.h"
#include "svdc_internal.h"

namespace svdc {

bool mfma_shape_supported(const svdc_shape&) { return false; }
size_t mfma_packed_bytes(const svdc_shape&) { return 0; }
int32_t launch_pack_basis(const svdc_shape&, const float*, void*, hipStream_t) { return SVDC_E_SHAPE; }
int32_t launch_full_step_mfma(const svdc_shape&, const void*, const void*, void*, float*, float*, float, int,
                              hipStream_t) { return SVDC_E_SHAPE; }
int32_t launch_forecast_mfma(const svdc_shape&, const float*, const void*, const void*, void*, hipStream_t) {
  return SVDC_E_SHAPE;
}

}  // namespace svdc
