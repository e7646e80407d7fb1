// Internal launch interface between the C ABI (stage_api.cpp) and the HIP kernels.
// Everything here enqueues on the given stream and returns the launch status; nothing
// synchronises.  "elt" is the activation element type: 0 = fp32, 1 = bf16 (raw uint16).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <vector>

namespace tp {

enum Elt : int { ELT_F32 = 0, ELT_BF16 = 1 };
enum Act : int { ACT_NONE = 0, ACT_RELU = 1, ACT_GELU = 2 };

// z = x W^T + bias ; a = act(z) ; d = act'(z).   x:[M x K] W:[N x K] (elt), bias: fp32[N].
// d_out (what the backward pass multiplies with) may be null; a_out is always written.
// Both [M x N] in elt.  If x_copy is not null the launch also leaves a copy of x there (fused
// into the GEMM where the kernel supports it, a separate copy otherwise).
// addend (null: none; only where fprop_add_supported, 16-byte aligned): an [M x N] tensor added to the rounded
// activation, i.e. the residual add that follows the layer.
hipError_t launch_fprop(hipStream_t s, int elt, int M, int N, int K, const void* x, const void* W,
                        const float* bias, int act, void* d_out, void* a_out, void* x_copy, const void* addend = nullptr);
bool fprop_add_supported(int elt, int M, int N, int K);

// out = (dz W_b) (.) d_prev   dz:[M x N] W_b:[N x K] d_prev:[M x K] saved act'(z), or null.
hipError_t launch_dgrad(hipStream_t s, int elt, int M, int N, int K, const void* dz, const void* Wb,
                        const void* d_prev, void* out, int relu_mask = 0);

// gW = dz^T x  (fp32 [N x K]).
// partial: scratch of wgrad_scratch_floats(elt, M, N, K) floats (may be null when that is 0)
hipError_t launch_wgrad(hipStream_t s, int elt, int M, int N, int K, const void* dz, const void* x, float* gW, float* partial);
size_t wgrad_scratch_floats(int elt, int M, int N, int K);

// gb = column sums of dz[M x N] (fp32 [N]).
// partials: scratch of at least colsum_scratch_floats(M, N) floats.
hipError_t launch_colsum(hipStream_t s, int elt, int M, int N, const void* dz, float* gb, float* partials);
size_t colsum_scratch_floats(int M, int N);
// out[i] = sum over z < splits of partial[z*count + i], i < count; fixed summation order.
hipError_t launch_sum_partials(hipStream_t s, size_t count, int splits, const float* partial, float* out);
// the same with partial row z starting at partial + z*stride
hipError_t launch_sum_partials_strided(hipStream_t s, size_t count, int splits, const float* partial, size_t stride,
                                       float* out);
// Sums put off: while a sink is set on the calling thread, the two calls above (also where another launcher makes
// them) append their job to it and launch nothing; launch_sum_jobs then forms all of them in one launch per 96
// jobs, with the bits the separate launches would have given.  The caller keeps every job's partials untouched, and
// reads no result, until that launch has run.
struct SumJob {
  const float* partial;
  float* out;
  size_t count, stride;
  int splits;
};
void set_sum_sink(std::vector<SumJob>* sink);
hipError_t launch_sum_jobs(hipStream_t s, const SumJob* jobs, size_t njobs);

// dz = dy (.) d    all [rows x cols] in elt; d = saved act'(z).
// relu_mask = 1: d holds a ReLU output instead of its derivative; the factor is (d > 0).
// add (may be null): the gradient is dy + add, rounded to elt, before it is multiplied.  All pointers 16-byte aligned.
hipError_t launch_act_backward(hipStream_t s, int elt, size_t count, const void* dy, const void* d, void* dz, int relu_mask = 0,
                               const void* add = nullptr);

// The two in one pass over dy: dz = dy (.) d as launch_act_backward forms it, gb = column sums of that dz as
// launch_colsum forms them (same partial layout, same scratch).  Only where act_backward_colsum_supported and all three
// tensors are 16-byte aligned; hipErrorNotSupported (nothing launched) otherwise.
bool act_backward_colsum_supported(int elt, int N);
hipError_t launch_act_backward_colsum(hipStream_t s, int elt, int M, int N, const void* dy, const void* d, void* dz,
                                      int relu_mask, float* gb, float* partials);

// Device-to-device copy of `bytes` bytes.
hipError_t launch_copy(hipStream_t s, const void* src, void* dst, size_t bytes);

// Softmax cross-entropy over `rows` rows of `classes` logits; dlogits = (softmax-onehot)/rows,
// *loss = mean of the row losses.  row_loss: scratch of `rows` floats.
hipError_t launch_softmax_ce(hipStream_t s, int elt, int rows, int classes, const void* logits,
                             const int32_t* labels, void* dlogits, float* row_loss, float* loss);

// fp32 -> elt conversion of `count` elements (compute copy of a weight version).
hipError_t launch_convert(hipStream_t s, int elt, size_t count, const float* src, void* dst);

// W_b = alpha * W_stale + beta * W_latest  (fp32 in, elt out).
hipError_t launch_blend(hipStream_t s, int elt, size_t count, const float* w_stale,
                        const float* w_latest, float alpha, float beta, void* wb);

// The fused pass over the parameters of a stage:
//   m      <- mu*m + g
//   w_new  <- w_old - lr*m          (w_new may alias w_old)
//   wfwd   <- elt(w_new)            (skipped when wfwd == null)
//   wb     <- elt(alpha*w_stale + beta*w_new)   (skipped when wb == null)
// and the reductions TP_DIAG_* written as doubles to diag[0..3].
// partials: scratch of at least update_scratch_floats() floats.
struct UpdateArgs {
  size_t count;
  const float* g;
  float* m;
  const float* w_old;
  float* w_new;
  const float* w_stale;  // null => no blend
  void* wfwd;
  void* wb;
  float lr, mu, alpha, beta;
  float* partials;
  double* diag;
};
hipError_t launch_update(hipStream_t s, int elt, const UpdateArgs& a);
size_t update_scratch_floats();
// Device address, on the current GPU, of the library's own update_scratch_floats() floats of block partials
// (a file-scope device array; looked up once per device).  Allocates nothing.
hipError_t update_static_scratch(float** out, size_t* floats);

}  // namespace tp
