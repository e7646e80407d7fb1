#include "gemm_mfma.h"
namespace tp {
bool mfma_fprop_supported(int, int, int) { return false; }
bool mfma_dgrad_supported(int, int, int) { return false; }
bool mfma_wgrad_supported(int, int, int) { return false; }
hipError_t mfma_fprop(hipStream_t, int, int, int, const uint16_t*, const uint16_t*, const float*, int, uint16_t*, uint16_t*) { return hipErrorNotSupported; }
hipError_t mfma_dgrad(hipStream_t, int, int, int, const uint16_t*, const uint16_t*, const uint16_t*, int, uint16_t*) { return hipErrorNotSupported; }
hipError_t mfma_wgrad(hipStream_t, int, int, int, const uint16_t*, const uint16_t*, float*) { return hipErrorNotSupported; }
}
