// bf16 MFMA GEMMs (fp32 accumulate) for gfx950.  The *_supported predicates state the shapes
// each kernel takes; everything else goes to the generic SIMT kernel.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace tp {

bool mfma_fprop_supported(int M, int N, int K);
bool mfma_dgrad_supported(int M, int N, int K);
bool mfma_wgrad_supported(int M, int N, int K);

hipError_t mfma_fprop(hipStream_t s, int M, int N, int K, const uint16_t* x, const uint16_t* W, const float* bias,
                      int act, uint16_t* z_out, uint16_t* a_out);
hipError_t mfma_dgrad(hipStream_t s, int M, int N, int K, const uint16_t* dz, const uint16_t* Wb,
                      const uint16_t* z_prev, int act_prev, uint16_t* out);
hipError_t mfma_wgrad(hipStream_t s, int M, int N, int K, const uint16_t* dz, const uint16_t* x, float* gW);

}  // namespace tp
