// bf16 MFMA GEMMs (fp32 accumulate) for gfx950.  The *_supported predicates state the shapes
// each kernel takes; everything else goes to the generic SIMT kernel.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace tp {

bool mfma_fprop_supported(int M, int N, int K);
bool mfma_dgrad_supported(int M, int N, int K);
bool mfma_wgrad_supported(int M, int N, int K);

// Tuning hook: force tile configuration `cfg` for product 0 = fprop, 1 = dgrad, 2 = wgrad
// (-1 = back to the heuristic).
void mfma_set_config(int product, int cfg);


// d_out receives act'(z) (what the backward pass multiplies with), a_out = act(z).  If x_copy is
// not null (16-byte aligned, like x) the launch also leaves a copy of x there.
// addend (or null): an [M x N] tensor added to the rounded activation -- the residual add that follows the layer.
hipError_t mfma_fprop(hipStream_t s, int M, int N, int K, const uint16_t* x, const uint16_t* W, const float* bias,
                      int act, uint16_t* d_out, uint16_t* a_out, uint16_t* x_copy, const uint16_t* addend = nullptr);
// out = (dz Wb) (.) d_prev, d_prev = saved act'(z) of the previous layer or null; relu_mask = 1: d_prev holds that layer's
// ReLU output instead and the factor is (output > 0).
hipError_t mfma_dgrad(hipStream_t s, int M, int N, int K, const uint16_t* dz, const uint16_t* Wb,
                      const uint16_t* d_prev, uint16_t* out, int relu_mask = 0);
// partial: scratch of mfma_wgrad_scratch_floats(M, N, K) floats, or null.  A gradient with too few output tiles to
// fill the chip is formed over several ranges of the M rows into `partial` and summed in a fixed order.
hipError_t mfma_wgrad(hipStream_t s, int M, int N, int K, const uint16_t* dz, const uint16_t* x, float* gW, float* partial);
size_t mfma_wgrad_scratch_floats(int M, int N, int K);

}  // namespace tp
