#include "hb_internal.h"
namespace hb {
bool lmhead_mfma_supports(int32_t, int32_t, int32_t, int32_t) { return false; }
hipError_t launch_lmhead_mfma(int32_t, int32_t, int32_t, const void *, const void *, unsigned long long *,
                              hipStream_t) {
  return hipErrorNotSupported;
}
}  // namespace hb
