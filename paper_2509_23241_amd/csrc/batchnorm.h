// Batch normalisation in training mode on [rows x C] activations (row = one position of one sample of
// the micro-batch the call sees): per-channel statistics over the rows, scale, shift, activation.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace tp {

// a = act(gamma (x - mean)/sqrt(var + 1e-5) + beta), d = act' of the same pre-activation (d_out may be null);
// stats[2c] = mean_c, stats[2c+1] = 1/sqrt(var_c + eps) are kept for the backward pass.  Mean and variance are
// formed from sums of x - x[0][c] and its square (the shift keeps E[d^2] - E[d]^2 away from cancellation), or in two passes
// over registers in the slab kernels.  scratch: batchnorm_scratch_floats(rows, C) floats.
// addend (null: none; only where batchnorm_fwd_add_supported): the residual add that follows a normalisation without
// activation of its own, fused: a = act(bf16(normalised) + addend), d = act' of the same sum.
hipError_t launch_batchnorm_fwd(hipStream_t s, int elt, size_t rows, int C, const void* x, const float* gamma, const float* beta,
                                int act, void* a_out, void* d_out, float* stats, float* scratch, const void* addend = nullptr);
bool batchnorm_fwd_add_supported(int elt, size_t rows, int C);
// dy: gradient with respect to the normalised, scaled and shifted value (the activation's derivative already
// applied).  All nseg micro-batches of a mini-batch at once: segment q = rows [q*rows, (q+1)*rows) of dy, x, dx with
// its own statistics stats[q][2C]; sums[q][0..C) = sum dy * xhat, sums[q][C..2C) = sum dy of that segment (its share of
// dgamma, dbeta).  The scale of the backward pass is alpha*gamma_s + beta_c*gamma_l, formed in fp32.
// scratch: batchnorm_scratch_floats(rows, C, nseg) floats.
hipError_t launch_batchnorm_bwd(hipStream_t s, int elt, size_t rows, int C, int nseg, const void* dy, const void* x, const float* stats,
                                const float* gamma_s, const float* gamma_l, float alpha, float beta_c, void* dx, float* sums,
                                float* scratch);
size_t batchnorm_scratch_floats(size_t rows, int C, int nseg = 1);
// The backward pass of all nseg micro-batches of a mini-batch in one launch (bf16, small layers): segment q =
// rows [q*rows, (q+1)*rows) of dy, x, dx with its own statistics stats[q][2C]; sums[q][0..C) = sum dy * xhat and
// sums[q][C..2C) = sum dy of that segment; dx_sums (may be null): [nseg][C] column sums of each segment's dx as
// stored.  hipErrorNotSupported (nothing launched) for shapes it does not take.
bool batchnorm_fused_bwd_supported(int elt, size_t rows, int C);
hipError_t launch_batchnorm_bwd_fused(hipStream_t s, int elt, size_t rows, int C, int nseg, const void* dy, const void* x,
                                      const float* stats, const float* gamma_s, const float* gamma_l, float alpha, float beta_c,
                                      void* dx, float* sums, float* dx_sums = nullptr);

// out = act(a + b), d_out = act'(a + b) (null: not kept)
hipError_t launch_add_act(hipStream_t s, int elt, size_t count, const void* a, const void* b, int act, void* out, void* d_out);

}  // namespace tp
