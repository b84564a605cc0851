#include "hb_internal.h"
namespace hb {
bool attn_mfma_supports(const hb_attn_desc &) { return false; }
hipError_t launch_attn_mfma(const hb_attn_desc &, const AttnPlan &, const void *, const void *, const void *,
                            const void *, const void *, const int32_t *, const int32_t *, const int32_t *,
                            const int32_t *, void *, float *, float *, float *, hipStream_t) {
  return hipErrorNotSupported;
}
}  // namespace hb
