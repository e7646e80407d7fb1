// Layers of the transformer-shaped stage: layer normalisation, causal multi-head self-attention and
// the residual add.  Activations are [rows x D] matrices (row = one token) in the stage's activation
// type (elt: 0 fp32, 1 bf16); statistics and parameter gradients are fp32.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace tp {

// y = gamma * (x - mean) / sqrt(var + eps) + beta per row; stats[2*r] = mean, stats[2*r+1] = 1/sqrt(var+eps).
hipError_t launch_layernorm_fwd(hipStream_t s, int elt, size_t rows, int D, const void* x, const float* gamma,
                                const float* beta, void* y, float* stats);
// dx, dgamma, dbeta of the above.  The scale the backward pass uses is alpha*gamma_s + beta_c*gamma_l
// (the intermediate weight of the method, formed on the fly in fp32; pass gamma_l twice with 1, 0 for
// the plain case).  partials: scratch of layernorm_scratch_floats(rows, D) floats.
// addend (null: none; only where layernorm_bwd_add_supported and all pointers are 16-byte aligned): a tensor of dx's shape
// that is added to the rounded dx -- the gradient that went around a residual branch which starts in front of this layer.
hipError_t launch_layernorm_bwd(hipStream_t s, int elt, size_t rows, int D, const void* dy, const void* x,
                                const float* stats, const float* gamma_s, const float* gamma_l, float alpha, float beta_c,
                                void* dx, float* dgamma, float* dbeta, float* partials, const void* addend = nullptr);
bool layernorm_bwd_add_supported(int elt, int D);
size_t layernorm_scratch_floats(size_t rows, int D);

// out = a + b, elementwise (out may alias a or b)
hipError_t launch_add(hipStream_t s, int elt, size_t count, const void* a, const void* b, void* out);

// qkv: [seqs*S x 3*D] (queries | keys | values, head h in columns h*dh..), out: [seqs*S x D],
// lse: [seqs*heads*S] log-sum-exp of the scaled scores of each query (kept for the backward pass).
// scratch (may be null): attention_scratch_bytes(elt, seqs, S, heads, dh) bytes let bf16 shapes the matrix-core
// kernels take run there; without it, and for every other shape, the wavefront kernels run.
hipError_t launch_attention_fwd(hipStream_t s, int elt, int seqs, int S, int heads, int dh, const void* qkv, void* out,
                                float* lse, void* scratch, size_t scratch_bytes);
size_t attention_scratch_bytes(int elt, int seqs, int S, int heads, int dh);
// dqkv: [seqs*S x 3*D] from dout, the saved qkv, the saved output and lse.
hipError_t launch_attention_bwd(hipStream_t s, int elt, int seqs, int S, int heads, int dh, const void* qkv, const void* out,
                                const void* dout, const float* lse, void* dqkv, void* scratch, size_t scratch_bytes);
// head widths the attention kernels take
bool attention_supported(int S, int heads, int dh);

// Matrix-core attention (bf16; kernels_attention_mfma.hip): same arguments and results as the two
// launchers above, plus scratch for the transient score matrices (attention_mfma_scratch_bytes for the
// largest number of sequences a call will see; a smaller scratch makes the call work in smaller chunks).
// Fused forward (head widths 64 and 128, tokens a multiple of 64): online softmax, no score matrix in memory, no scratch.
bool attention_flash_fwd_supported(int seqs, int S, int heads, int dh);
hipError_t attention_flash_fwd(hipStream_t s, int seqs, int S, int heads, int dh, const uint16_t* qkv, uint16_t* out, float* lse);
// Fused backward for the same shapes: two launches (dQ; dK and dV) that recompute the probabilities from lse, after a
// small kernel that forms delta = dO . O per token and head into `scratch` (attention_flash_bwd_scratch_bytes).
size_t attention_flash_bwd_scratch_bytes(int seqs, int S, int heads);
hipError_t attention_flash_bwd(hipStream_t s, int seqs, int S, int heads, int dh, const uint16_t* qkv, const uint16_t* out,
                               const uint16_t* dout, const float* lse, uint16_t* dqkv, void* scratch, size_t scratch_bytes);
bool attention_mfma_supported(int S, int heads, int dh);
size_t attention_mfma_scratch_bytes(int seqs, int S, int heads);
hipError_t attention_mfma_fwd(hipStream_t s, int seqs, int S, int heads, int dh, const uint16_t* qkv, uint16_t* out, float* lse,
                              void* scratch, size_t scratch_bytes);
hipError_t attention_mfma_bwd(hipStream_t s, int seqs, int S, int heads, int dh, const uint16_t* qkv, const uint16_t* dout,
                              const float* lse, uint16_t* dqkv, void* scratch, size_t scratch_bytes);

}  // namespace tp
