// Batch normalisation (training mode) and the residual add with activation of the bottleneck-shaped stage.
// Column statistics are formed by blocks of 64 columns x a chunk of rows (lanes along the columns: every
// row read is one contiguous segment), block partials are added in a fixed order by the shared
// partial-sum kernel.  Plain streaming kernels; the layer is bound by reading x three times in the forward
// pass and twice in the backward pass.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <algorithm>

#include "batchnorm.h"
#include "device_utils.h"
#include "kernels.h"

namespace tp {

namespace {

constexpr int kThreads = 256;
constexpr float kBnEps = 1e-5f;

inline int bn_chunk_rows(size_t rows) { return (int)std::max<size_t>(16, (rows + 255) / 256); }
inline int bn_chunks(size_t rows) { return (int)((rows + bn_chunk_rows(rows) - 1) / bn_chunk_rows(rows)); }

// MODE 0: sum x          MODE 1: sum (x - mean)^2, mean = totals[c] / rows
// MODE 2: sum dy * xhat (out[0..C)) and sum dy (out[C..2C)), xhat from stats
template <typename T, int MODE>
__global__ __launch_bounds__(kThreads) void bn_colsum_kernel(size_t rows, int C, int chunk_rows, const T* __restrict__ x,
                                                             const T* __restrict__ dy, const float* __restrict__ aux,
                                                             float* __restrict__ partial) {
  __shared__ float sm[2][4][64];
  const int cl = threadIdx.x & 63, rl = threadIdx.x >> 6;
  const int c = blockIdx.x * 64 + cl;
  const size_t r0 = (size_t)blockIdx.y * chunk_rows;
  const size_t r1 = std::min(rows, r0 + chunk_rows);
  float s0 = 0.f, s1 = 0.f;
  if (c < C) {
    float mean = 0.f, rstd = 0.f;
    if (MODE == 1) mean = aux[c] / (float)rows;
    if (MODE == 2) { mean = aux[2 * c]; rstd = aux[2 * c + 1]; }
    for (size_t r = r0 + rl; r < r1; r += 4) {
      const float v = to_float(x[r * C + c]);
      if (MODE == 0) s0 += v;
      if (MODE == 1) s0 += (v - mean) * (v - mean);
      if (MODE == 2) {
        const float g = to_float(dy[r * C + c]);
        s0 += g * (v - mean) * rstd;
        s1 += g;
      }
    }
  }
  sm[0][rl][cl] = s0;
  sm[1][rl][cl] = s1;
  __syncthreads();
  if (rl == 0 && c < C) {
    const size_t width = MODE == 2 ? 2 * (size_t)C : (size_t)C;
    partial[blockIdx.y * width + c] = sm[0][0][cl] + sm[0][1][cl] + sm[0][2][cl] + sm[0][3][cl];
    if (MODE == 2) partial[blockIdx.y * width + C + c] = sm[1][0][cl] + sm[1][1][cl] + sm[1][2][cl] + sm[1][3][cl];
  }
}

template <typename T>
__global__ __launch_bounds__(kThreads) void bn_normalize_kernel(size_t rows, int C, const T* __restrict__ x,
                                                                const float* __restrict__ sum_x, const float* __restrict__ sum_sq,
                                                                const float* __restrict__ gamma, const float* __restrict__ beta,
                                                                int act, T* __restrict__ a_out, T* __restrict__ d_out,
                                                                float* __restrict__ stats) {
  const size_t total = rows * C;
  const size_t stride = (size_t)gridDim.x * kThreads;
  for (size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x; i < total; i += stride) {
    const int c = (int)(i % C);
    const float mean = sum_x[c] / (float)rows;
    const float rstd = rsqrtf(sum_sq[c] / (float)rows + kBnEps);
    const float z = fmaf((to_float(x[i]) - mean) * rstd, gamma[c], beta[c]);
    a_out[i] = from_float<T>(act_forward(z, act));
    if (d_out) d_out[i] = from_float<T>(act_derivative(z, act));
    if (i < (size_t)C) {  // the first row's threads also record the statistics
      stats[2 * c] = mean;
      stats[2 * c + 1] = rstd;
    }
  }
}

template <typename T>
__global__ __launch_bounds__(kThreads) void bn_dx_kernel(size_t rows, int C, const T* __restrict__ dy, const T* __restrict__ x,
                                                         const float* __restrict__ stats, const float* __restrict__ sums,
                                                         const float* __restrict__ gamma_s, const float* __restrict__ gamma_l,
                                                         float alpha, float beta_c, T* __restrict__ dx) {
  const size_t total = rows * C;
  const size_t stride = (size_t)gridDim.x * kThreads;
  const float inv_rows = 1.f / (float)rows;
  for (size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x; i < total; i += stride) {
    const int c = (int)(i % C);
    const float mean = stats[2 * c], rstd = stats[2 * c + 1];
    const float g = fmaf(alpha, gamma_s[c], beta_c * gamma_l[c]);
    const float xh = (to_float(x[i]) - mean) * rstd;
    dx[i] = from_float<T>(g * rstd * (to_float(dy[i]) - (sums[C + c] + xh * sums[c]) * inv_rows));
  }
}

template <typename T>
__global__ __launch_bounds__(kThreads) void add_act_kernel(size_t count, const T* a, const T* b, int act, T* out, T* d_out) {
  const size_t stride = (size_t)gridDim.x * kThreads;
  for (size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x; i < count; i += stride) {
    const float z = to_float(a[i]) + to_float(b[i]);
    out[i] = from_float<T>(act_forward(z, act));
    if (d_out) d_out[i] = from_float<T>(act_derivative(z, act));
  }
}

inline unsigned stream_grid(size_t count) { return (unsigned)std::min<size_t>(std::max<size_t>((count + kThreads - 1) / kThreads, 1), 8192); }

template <typename T>
hipError_t bn_fwd_typed(hipStream_t s, size_t rows, int C, const T* x, const float* gamma, const float* beta, int act, T* a_out,
                        T* d_out, float* stats, float* scratch) {
  const int cr = bn_chunk_rows(rows), chunks = bn_chunks(rows);
  float* partial = scratch;                          // [chunks][C]
  float* sum_x = scratch + (size_t)chunks * 2 * C;   // [C]
  float* sum_sq = sum_x + C;                         // [C]
  const dim3 grid((C + 63) / 64, chunks);
  hipLaunchKernelGGL((bn_colsum_kernel<T, 0>), grid, dim3(kThreads), 0, s, rows, C, cr, x, (const T*)nullptr, (const float*)nullptr,
                     partial);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  e = launch_sum_partials(s, (size_t)C, chunks, partial, sum_x);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL((bn_colsum_kernel<T, 1>), grid, dim3(kThreads), 0, s, rows, C, cr, x, (const T*)nullptr, (const float*)sum_x,
                     partial);
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  e = launch_sum_partials(s, (size_t)C, chunks, partial, sum_sq);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(bn_normalize_kernel<T>, dim3(stream_grid(rows * C)), dim3(kThreads), 0, s, rows, C, x, sum_x, sum_sq, gamma, beta,
                     act, a_out, d_out, stats);
  return hipGetLastError();
}

template <typename T>
hipError_t bn_bwd_typed(hipStream_t s, size_t rows, int C, const T* dy, const T* x, const float* stats, const float* gamma_s,
                        const float* gamma_l, float alpha, float beta_c, T* dx, float* sums, float* scratch) {
  const int cr = bn_chunk_rows(rows), chunks = bn_chunks(rows);
  const dim3 grid((C + 63) / 64, chunks);
  hipLaunchKernelGGL((bn_colsum_kernel<T, 2>), grid, dim3(kThreads), 0, s, rows, C, cr, x, dy, stats, scratch);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  e = launch_sum_partials(s, 2 * (size_t)C, chunks, scratch, sums);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(bn_dx_kernel<T>, dim3(stream_grid(rows * C)), dim3(kThreads), 0, s, rows, C, dy, x, stats, sums, gamma_s, gamma_l,
                     alpha, beta_c, dx);
  return hipGetLastError();
}

}  // namespace

size_t batchnorm_scratch_floats(size_t rows, int C) { return ((size_t)bn_chunks(rows) * 2 + 2) * C; }

hipError_t launch_batchnorm_fwd(hipStream_t s, int elt, size_t rows, int C, const void* x, const float* gamma, const float* beta,
                                int act, void* a_out, void* d_out, float* stats, float* scratch) {
  if (elt == ELT_BF16)
    return bn_fwd_typed<uint16_t>(s, rows, C, (const uint16_t*)x, gamma, beta, act, (uint16_t*)a_out, (uint16_t*)d_out, stats, scratch);
  return bn_fwd_typed<float>(s, rows, C, (const float*)x, gamma, beta, act, (float*)a_out, (float*)d_out, stats, scratch);
}

hipError_t launch_batchnorm_bwd(hipStream_t s, int elt, size_t rows, int C, const void* dy, const void* x, const float* stats,
                                const float* gamma_s, const float* gamma_l, float alpha, float beta_c, void* dx, float* sums,
                                float* scratch) {
  if (elt == ELT_BF16)
    return bn_bwd_typed<uint16_t>(s, rows, C, (const uint16_t*)dy, (const uint16_t*)x, stats, gamma_s, gamma_l, alpha, beta_c,
                                  (uint16_t*)dx, sums, scratch);
  return bn_bwd_typed<float>(s, rows, C, (const float*)dy, (const float*)x, stats, gamma_s, gamma_l, alpha, beta_c, (float*)dx, sums,
                             scratch);
}

hipError_t launch_add_act(hipStream_t s, int elt, size_t count, const void* a, const void* b, int act, void* out, void* d_out) {
  if (elt == ELT_BF16)
    hipLaunchKernelGGL(add_act_kernel<uint16_t>, dim3(stream_grid(count)), dim3(kThreads), 0, s, count, (const uint16_t*)a,
                       (const uint16_t*)b, act, (uint16_t*)out, (uint16_t*)d_out);
  else
    hipLaunchKernelGGL(add_act_kernel<float>, dim3(stream_grid(count)), dim3(kThreads), 0, s, count, (const float*)a, (const float*)b,
                       act, (float*)out, (float*)d_out);
  return hipGetLastError();
}

}  // namespace tp
