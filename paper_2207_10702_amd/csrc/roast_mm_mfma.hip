// bf16 MFMA ROAST-MM kernels (placeholder until the tuned kernels land: every shape falls back to
// the generic kernels).
#include "roast_internal.hpp"

namespace roast {

roast_status mfma_mm_fwd(const MMArgs&, const void*, int64_t, const float*, void*, int64_t, hipStream_t) {
  return ROAST_ERR_UNSUPPORTED;
}
roast_status mfma_mm_bwd_dx(const MMArgs&, const void*, int64_t, const float*, void*, int64_t, hipStream_t) {
  return ROAST_ERR_UNSUPPORTED;
}
roast_status mfma_mm_bwd_dM(const MMArgs&, const void*, int64_t, const void*, int64_t, float*, float*, int,
                            hipStream_t) {
  return ROAST_ERR_UNSUPPORTED;
}

}  // namespace roast
