// bf16 MFMA attention (placeholder until the fused kernels land).
#include "common.h"
#include "kernels.h"
namespace dp {
bool attn_mfma_supported(int, int) { return false; }
hipError_t launch_attn_fwd_mfma(int, int, int, int, int, const void *, void *, float *, hipStream_t) {
  return hipErrorNotSupported;
}
hipError_t launch_attn_bwd_mfma(int, int, int, int, int, const void *, const void *, const float *, const void *,
                                void *, float *, hipStream_t) {
  return hipErrorNotSupported;
}
}  // namespace dp
