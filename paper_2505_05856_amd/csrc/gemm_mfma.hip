// bf16 MFMA GEMM (placeholder until the tiled kernels land: nothing is supported,
// so callers take the vector-ALU path).
#include "common.h"
#include "kernels.h"
namespace dp {
bool gemm_mfma_supported(const GemmArgs &) { return false; }
hipError_t launch_gemm_mfma(const GemmArgs &, hipStream_t) { return hipErrorNotSupported; }
}  // namespace dp
