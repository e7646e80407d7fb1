// Batch normalisation (training mode) and the residual add with activation of the bottleneck-shaped stage.
// Two families.  Streaming kernels (any type and size): column statistics are formed by blocks of 64 columns x
// a chunk of rows (lanes along the columns: every row read is one contiguous segment), block partials are
// added in a fixed order by the shared partial-sum kernel; mean and variance come from one pass over x (sums
// of x - x[0][c] and of its square), so x is read twice in the forward pass and twice in the backward pass; the
// backward pass takes all micro-batches of a mini-batch in the same three launches.  Slab kernels (bf16, up to 2048 rows per micro-batch): one launch per layer, the values
// stay in registers between the passes; above that size the streaming kernels are faster.
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

// MODE 0: sum d and sum d^2 with d = x - x[0][c] (out[0..C), out[C..2C)): mean and variance from ONE pass; the shift by the
//         channel's first value keeps the subtraction var = E[d^2] - E[d]^2 away from cancellation
// MODE 2: sum dy * xhat (out[0..C)) and sum dy (out[C..2C)), xhat from stats
// blockIdx.z = segment (micro-batch) q: rows [q*rows, (q+1)*rows), statistics aux[q][2C]; the partial sums of row chunk k
// go to partial[(k*nseg + q)][2C], so that one strided sum over k finishes all segments.
template <typename T, int MODE>
__global__ __launch_bounds__(kThreads) void bn_colsum_kernel(size_t rows, int C, int chunk_rows, const T* __restrict__ x,
                                                             const T* __restrict__ dy, const float* __restrict__ aux,
                                                             float* __restrict__ partial) {
  __shared__ float sm[2][4][64];
  const int cl = threadIdx.x & 63, rl = threadIdx.x >> 6;
  const int c = blockIdx.x * 64 + cl;
  const size_t seg = blockIdx.z, nseg = gridDim.z;
  x += seg * rows * C;
  if (MODE == 2) { dy += seg * rows * C; aux += seg * 2 * C; }
  const size_t r0 = (size_t)blockIdx.y * chunk_rows;
  const size_t r1 = std::min(rows, r0 + chunk_rows);
  float s0 = 0.f, s1 = 0.f;
  if (c < C) {
    float mean = 0.f, rstd = 0.f;
    if (MODE == 0) mean = to_float(x[c]);
    if (MODE == 2) { mean = aux[2 * c]; rstd = aux[2 * c + 1]; }
    for (size_t r = r0 + rl; r < r1; r += 4) {
      const float v = to_float(x[r * C + c]);
      if (MODE == 0) {
        s0 += v - mean;
        s1 = fmaf(v - mean, v - mean, s1);
      }
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
    float* out = partial + ((size_t)blockIdx.y * nseg + seg) * 2 * C;
    out[c] = sm[0][0][cl] + sm[0][1][cl] + sm[0][2][cl] + sm[0][3][cl];
    out[C + c] = sm[1][0][cl] + sm[1][1][cl] + sm[1][2][cl] + sm[1][3][cl];
  }
}

// The same for bf16 with C % 8 == 0 in 16-byte units: a workgroup covers 128 channels (16 lanes of 8) x 16 rows per
// step; the sixteen row lanes of a channel meet in LDS in a fixed order.  Same partial layout.
__device__ __forceinline__ void bn_unpack8(const uint4& u, float (&f)[8]) {
  const uint32_t w[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    f[2 * j] = __uint_as_float(w[j] << 16);
    f[2 * j + 1] = __uint_as_float(w[j] & 0xffff0000u);
  }
}
template <int MODE>
__global__ __launch_bounds__(kThreads) void bn_colsum_vec_kernel(size_t rows, int C, int chunk_rows, const uint16_t* __restrict__ x,
                                                                 const uint16_t* __restrict__ dy, const float* __restrict__ aux,
                                                                 float* __restrict__ partial) {
  __shared__ float sm[2][16][128 + 4];
  const int cl = threadIdx.x & 15, rl = threadIdx.x >> 4;
  const int c = blockIdx.x * 128 + cl * 8;
  const size_t seg = blockIdx.z, nseg = gridDim.z;
  x += seg * rows * C;
  if (MODE == 2) { dy += seg * rows * C; aux += seg * 2 * C; }
  const size_t r0 = (size_t)blockIdx.y * chunk_rows;
  const size_t r1 = std::min(rows, r0 + chunk_rows);
  float s0[8], s1[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) s0[j] = s1[j] = 0.f;
  if (c < C) {
    float mean[8], rstd[8];
    if (MODE == 0) {
      bn_unpack8(*reinterpret_cast<const uint4*>(x + c), mean);
    } else {
#pragma unroll
      for (int j = 0; j < 8; ++j) { mean[j] = aux[2 * (c + j)]; rstd[j] = aux[2 * (c + j) + 1]; }
    }
#pragma unroll 2
    for (size_t r = r0 + rl; r < r1; r += 16) {
      float v[8], g[8];
      bn_unpack8(*reinterpret_cast<const uint4*>(x + r * C + c), v);
      if (MODE == 2) bn_unpack8(*reinterpret_cast<const uint4*>(dy + r * C + c), g);
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        if (MODE == 0) {
          s0[j] += v[j] - mean[j];
          s1[j] = fmaf(v[j] - mean[j], v[j] - mean[j], s1[j]);
        } else {
          s0[j] += g[j] * (v[j] - mean[j]) * rstd[j];
          s1[j] += g[j];
        }
      }
    }
  }
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    sm[0][rl][cl * 8 + j] = s0[j];
    sm[1][rl][cl * 8 + j] = s1[j];
  }
  __syncthreads();
  if (threadIdx.x < 128 && blockIdx.x * 128 + threadIdx.x < C) {
    float a = 0.f, b = 0.f;
#pragma unroll
    for (int k = 0; k < 16; ++k) {
      a += sm[0][k][threadIdx.x];
      b += sm[1][k][threadIdx.x];
    }
    float* out = partial + ((size_t)blockIdx.y * nseg + seg) * 2 * C;
    out[blockIdx.x * 128 + threadIdx.x] = a;
    out[C + blockIdx.x * 128 + threadIdx.x] = b;
  }
}

// partial[chunk][0..C) = sum d, [C..2C) = sum d^2 over the chunk's rows (d = x - x[0][c])  ->  stats[2c] = mean,
// stats[2c+1] = 1/sqrt(var + eps).  16 channels per workgroup: lane (g, c) adds chunks g, g + 16, ... of channel c, the
// sixteen results meet in LDS in a fixed order.
template <typename T>
__global__ __launch_bounds__(kThreads) void bn_finalize_sum_kernel(size_t rows, int C, int chunks, const T* __restrict__ x,
                                                                   const float* __restrict__ partial, float* __restrict__ stats) {
  __shared__ float sm[2][16][16];
  const int cl = threadIdx.x & 15, g = threadIdx.x >> 4;
  const int c = blockIdx.x * 16 + cl;
  float s0 = 0.f, s1 = 0.f;
  if (c < C) {
#pragma unroll 4
    for (int k = g; k < chunks; k += 16) {
      s0 += partial[(size_t)k * 2 * C + c];
      s1 += partial[(size_t)k * 2 * C + C + c];
    }
  }
  sm[0][g][cl] = s0;
  sm[1][g][cl] = s1;
  __syncthreads();
  if (g == 0 && c < C) {
    float a = 0.f, b = 0.f;
#pragma unroll
    for (int k = 0; k < 16; ++k) {
      a += sm[0][k][cl];
      b += sm[1][k][cl];
    }
    const float inv = 1.f / (float)rows;
    const float md = a * inv;
    const float var = fmaxf(b * inv - md * md, 0.f);
    stats[2 * c] = to_float(x[c]) + md;
    stats[2 * c + 1] = rsqrtf(var + kBnEps);
  }
}

template <typename T>
__global__ __launch_bounds__(kThreads) void bn_normalize_kernel(size_t rows, int C, const T* __restrict__ x,
                                                                const float* __restrict__ stats,
                                                                const float* __restrict__ gamma, const float* __restrict__ beta,
                                                                int act, T* __restrict__ a_out, T* __restrict__ d_out) {
  const size_t total = rows * C;
  const size_t stride = (size_t)gridDim.x * kThreads;
  for (size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x; i < total; i += stride) {
    const int c = (int)(i % C);
    const float z = fmaf((to_float(x[i]) - stats[2 * c]) * stats[2 * c + 1], gamma[c], beta[c]);
    a_out[i] = from_float<T>(act_forward(z, act));
    if (d_out) d_out[i] = from_float<T>(act_derivative(z, act));
  }
}

// all segments at once: element i belongs to segment i / (rows*C)
template <typename T>
__global__ __launch_bounds__(kThreads) void bn_dx_kernel(size_t rows, int C, size_t nseg, const T* __restrict__ dy, const T* __restrict__ x,
                                                         const float* __restrict__ stats, const float* __restrict__ sums,
                                                         const float* __restrict__ gamma_s, const float* __restrict__ gamma_l,
                                                         float alpha, float beta_c, T* __restrict__ dx) {
  const size_t per = rows * C, total = per * nseg;
  const size_t stride = (size_t)gridDim.x * kThreads;
  const float inv_rows = 1.f / (float)rows;
  for (size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x; i < total; i += stride) {
    const size_t q = i / per;
    const int c = (int)(i % C);
    const float* st = stats + q * 2 * C;
    const float* sq = sums + q * 2 * C;
    const float mean = st[2 * c], rstd = st[2 * c + 1];
    const float g = fmaf(alpha, gamma_s[c], beta_c * gamma_l[c]);
    const float xh = (to_float(x[i]) - mean) * rstd;
    dx[i] = from_float<T>(g * rstd * (to_float(dy[i]) - (sq[C + c] + xh * sq[c]) * inv_rows));
  }
}

// bf16, C a multiple of 8: the two elementwise kernels with 16 bytes per lane
__global__ __launch_bounds__(kThreads) void bn_normalize_vec_kernel(size_t rows, int C, const uint16_t* __restrict__ x,
                                                                    const float* __restrict__ stats,
                                                                    const float* __restrict__ gamma, const float* __restrict__ beta,
                                                                    int act, const uint16_t* __restrict__ addend,
                                                                    uint16_t* __restrict__ a_out, uint16_t* __restrict__ d_out);
__global__ __launch_bounds__(kThreads) void bn_dx_vec_kernel(size_t rows, int C, size_t nseg, const uint16_t* __restrict__ dy,
                                                             const uint16_t* __restrict__ x, const float* __restrict__ stats,
                                                             const float* __restrict__ sums, const float* __restrict__ gamma_s,
                                                             const float* __restrict__ gamma_l, float alpha, float beta_c,
                                                             uint16_t* __restrict__ dx);

// ---- slab kernels (bf16, small layers) -----------------------------------------------------------------
// One workgroup of 1024 lanes owns W adjacent 16-byte units of every row (8 * W channels) for ALL rows the
// statistics run over: lane t takes unit t % W of rows t / W, t / W + 1024 / W, ... and keeps them in registers.
// The passes of the layer -- mean, centred variance, normalise (forward); the column sums, dx (backward) -- then
// cost one read of the slab and one launch instead of five (forward) or three per micro-batch (backward; the sums
// over the micro-batches stay a launch of their own).  For the layers of a bottleneck stage (a few MB per call) the
// launches, not the bytes, were what took the time.  W = 1 in the forward kernel, 2 in the backward kernel of layers
// with more than 1024 rows (the launchers say why).  Workgroups are renumbered so that those of one XCD (every eighth
// workgroup id) take neighbouring slabs: the 128-byte lines they share then meet in one L2 (without it the forward
// kernel at W = 2 took 18.6 us instead of 14.5 us).
constexpr int kSlabThreads = 1024, kSlabWaves = kSlabThreads / 64;

__device__ __forceinline__ int slab_of_block(int b, int nblocks) {
  return (nblocks & 7) ? b : (b & 7) * (nblocks >> 3) + (b >> 3);
}

// Sums NV values per lane over the lanes that hold the same unit t % W, in a fixed order; every lane gets the totals
// of its unit.  The values go through LDS as [NV][1024] with the lanes of one unit next to each other: thread (v, p)
// adds 16 neighbouring entries of quantity v, the 64 / W threads of one unit finish with a butterfly.
template <int NV, int W>
__device__ __forceinline__ void slab_sum(float (&v)[NV], float* red /* [NV][kSlabThreads] + [NV][W] */) {
  static_assert(NV * 64 <= kSlabThreads, "one wave per quantity");
  constexpr int kSeg = kSlabThreads / W;  // lanes per unit
  constexpr int kTpu = 64 / W;            // adding threads per unit
  const int t = threadIdx.x;
  const int at = (t % W) * kSeg + t / W;
  __syncthreads();  // the previous totals have been read
#pragma unroll
  for (int i = 0; i < NV; ++i) red[i * kSlabThreads + at] = v[i];
  __syncthreads();
  if (t < NV * 64) {
    const int q = t >> 6, p = t & 63;
    const float4* src = reinterpret_cast<const float4*>(red + q * kSlabThreads + p * 16);
    float a = 0.f;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const float4 f = src[k];
      a += (f.x + f.y) + (f.z + f.w);
    }
#pragma unroll
    for (int off = kTpu / 2; off > 0; off >>= 1) a += __shfl_xor(a, off, 64);
    if (p % kTpu == 0) red[NV * kSlabThreads + q * W + p / kTpu] = a;
  }
  __syncthreads();
#pragma unroll
  for (int i = 0; i < NV; ++i) v[i] = red[NV * kSlabThreads + i * W + t % W];
}

__device__ __forceinline__ void unpack8(const uint4& u, float (&f)[8]) {
  const uint32_t w[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    f[2 * j] = __uint_as_float(w[j] << 16);
    f[2 * j + 1] = __uint_as_float(w[j] & 0xffff0000u);
  }
}
__device__ __forceinline__ uint4 pack8(const float (&f)[8]) {
  return make_uint4(pack_bf16x2(f[0], f[1]), pack_bf16x2(f[2], f[3]), pack_bf16x2(f[4], f[5]), pack_bf16x2(f[6], f[7]));
}

// The launchers give these two kernels a grid whose stride (threads of the grid, in 16-byte units) is a multiple of
// the units per row, so a lane stays on the same 8 channels for all its rows and reads their statistics and affine
// parameters once (fetched per element they were 32-48 extra loads for every 16 bytes of x: 14 us for a layer the
// kernel now streams in a few).  addend (or null): the kept tensor of a residual add that follows a normalisation
// without activation -- the result is act(bf16(bn(x)) + addend), as the slab kernel forms it.
__global__ __launch_bounds__(kThreads) void bn_normalize_vec_kernel(size_t rows, int C, const uint16_t* __restrict__ x,
                                                                    const float* __restrict__ stats,
                                                                    const float* __restrict__ gamma, const float* __restrict__ beta,
                                                                    int act, const uint16_t* __restrict__ addend,
                                                                    uint16_t* __restrict__ a_out, uint16_t* __restrict__ d_out) {
  const size_t nvec = rows * C / 8;
  const int cv = C / 8;
  const size_t stride = (size_t)gridDim.x * kThreads;  // a multiple of cv
  const size_t first = (size_t)blockIdx.x * kThreads + threadIdx.x;
  const int c0 = (int)(first % cv) * 8;
  float mean[8], rstd[8], ga[8], be[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    mean[j] = stats[2 * (c0 + j)];
    rstd[j] = stats[2 * (c0 + j) + 1];
    ga[j] = gamma[c0 + j];
    be[j] = beta[c0 + j];
  }
#pragma unroll 2
  for (size_t i = first; i < nvec; i += stride) {
    float f[8], a[8], d[8], sk[8];
    unpack8(reinterpret_cast<const uint4*>(x)[i], f);
    if (addend) unpack8(reinterpret_cast<const uint4*>(addend)[i], sk);
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      float z = fmaf((f[j] - mean[j]) * rstd[j], ga[j], be[j]);
      if (addend) z = bf16_to_float(float_to_bf16(z)) + sk[j];
      a[j] = act_forward(z, act);
      d[j] = act_derivative(z, act);
    }
    reinterpret_cast<uint4*>(a_out)[i] = pack8(a);
    if (d_out) reinterpret_cast<uint4*>(d_out)[i] = pack8(d);
  }
}

// grid.y = segment (micro-batch)
__global__ __launch_bounds__(kThreads) void bn_dx_vec_kernel(size_t rows, int C, size_t nseg, const uint16_t* __restrict__ dy,
                                                             const uint16_t* __restrict__ x, const float* __restrict__ stats,
                                                             const float* __restrict__ sums, const float* __restrict__ gamma_s,
                                                             const float* __restrict__ gamma_l, float alpha, float beta_c,
                                                             uint16_t* __restrict__ dx) {
  const size_t per = rows * C / 8;
  const int cv = C / 8;
  const size_t q = blockIdx.y;
  const size_t stride = (size_t)gridDim.x * kThreads;  // a multiple of cv
  const size_t first = (size_t)blockIdx.x * kThreads + threadIdx.x;
  const int c0 = (int)(first % cv) * 8;
  const float inv_rows = 1.f / (float)rows;
  const float* st = stats + q * 2 * C;
  const float* sq = sums + q * 2 * C;
  float mean[8], rstd[8], gr[8], s_xh[8], s_dy[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    const int c = c0 + j;
    mean[j] = st[2 * c];
    rstd[j] = st[2 * c + 1];
    gr[j] = fmaf(alpha, gamma_s[c], beta_c * gamma_l[c]) * rstd[j];
    s_xh[j] = sq[c];
    s_dy[j] = sq[C + c];
  }
  const uint4* xs = reinterpret_cast<const uint4*>(x) + q * per;
  const uint4* ds = reinterpret_cast<const uint4*>(dy) + q * per;
  uint4* os = reinterpret_cast<uint4*>(dx) + q * per;
#pragma unroll 2
  for (size_t i = first; i < per; i += stride) {
    float fx[8], fd[8], o[8];
    unpack8(xs[i], fx);
    unpack8(ds[i], fd);
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const float xh = (fx[j] - mean[j]) * rstd[j];
      o[j] = gr[j] * (fd[j] - (s_dy[j] + xh * s_xh[j]) * inv_rows);
    }
    os[i] = pack8(o);
  }
}

template <int NL, int W>
__global__ __launch_bounds__(kSlabThreads) void bn_fwd_slab_kernel(int rows, int C, const uint16_t* __restrict__ x,
                                                                   const float* __restrict__ gamma,
                                                                   const float* __restrict__ beta, int act,
                                                                   const uint16_t* __restrict__ addend,
                                                                   uint16_t* __restrict__ a_out, uint16_t* __restrict__ d_out,
                                                                   float* __restrict__ stats) {
  __shared__ __attribute__((aligned(16))) float red[8 * kSlabThreads + 8 * W];
  constexpr int kRowsPerPass = kSlabThreads / W;
  const int r0 = threadIdx.x / W;
  const int c0 = slab_of_block(blockIdx.x, gridDim.x) * 8 * W + 8 * (threadIdx.x % W);
  // everything this lane will read is requested up front, the tensor of a fused residual add included: fetched
  // where it is used, its rows would arrive one memory latency after the other at the end of the kernel
  uint4 v[NL], va[NL];
#pragma unroll
  for (int i = 0; i < NL; ++i) {
    const int r = i * kRowsPerPass + r0;
    v[i] = r < rows ? *reinterpret_cast<const uint4*>(x + (size_t)r * C + c0) : make_uint4(0, 0, 0, 0);
    va[i] = (addend && r < rows) ? *reinterpret_cast<const uint4*>(addend + (size_t)r * C + c0) : make_uint4(0, 0, 0, 0);
  }
  const float inv_rows = 1.f / (float)rows;
  float mean[8], rstd[8], s[8], ga[8], be[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    s[j] = 0.f;
    ga[j] = gamma[c0 + j];
    be[j] = beta[c0 + j];
  }
#pragma unroll
  for (int i = 0; i < NL; ++i) {  // rows past the end hold zeros
    float f[8];
    unpack8(v[i], f);
#pragma unroll
    for (int j = 0; j < 8; ++j) s[j] += f[j];
  }
  slab_sum<8, W>(s, red);
#pragma unroll
  for (int j = 0; j < 8; ++j) { mean[j] = s[j] * inv_rows; s[j] = 0.f; }
#pragma unroll
  for (int i = 0; i < NL; ++i) {
    if (i * kRowsPerPass + r0 >= rows) continue;
    float f[8];
    unpack8(v[i], f);
#pragma unroll
    for (int j = 0; j < 8; ++j) s[j] = fmaf(f[j] - mean[j], f[j] - mean[j], s[j]);
  }
  slab_sum<8, W>(s, red);
#pragma unroll
  for (int j = 0; j < 8; ++j) rstd[j] = rsqrtf(s[j] * inv_rows + kBnEps);
  if (r0 == 0) {
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      stats[2 * (c0 + j)] = mean[j];
      stats[2 * (c0 + j) + 1] = rstd[j];
    }
  }
#pragma unroll
  for (int i = 0; i < NL; ++i) {
    const int r = i * kRowsPerPass + r0;
    if (r >= rows) continue;
    float f[8], a[8], d[8], sk[8];
    unpack8(v[i], f);
    unpack8(va[i], sk);
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      float z = fmaf((f[j] - mean[j]) * rstd[j], ga[j], be[j]);
      // with an addend the normalisation itself has no activation: its result takes the bf16 rounding it would get
      // as a stored tensor, then act(. + addend) is the residual add that follows it in the layer list
      if (addend) z = bf16_to_float(float_to_bf16(z)) + sk[j];
      a[j] = act_forward(z, act);
      d[j] = act_derivative(z, act);
    }
    *reinterpret_cast<uint4*>(a_out + (size_t)r * C + c0) = pack8(a);
    if (d_out) *reinterpret_cast<uint4*>(d_out + (size_t)r * C + c0) = pack8(d);
  }
}

// All micro-batches of a mini-batch in one launch: blockIdx.y = q owns rows [q*rows, (q+1)*rows) with its own
// statistics stats[q][2C]; its column sums go to sums[q][0..C) (dy * xhat) and sums[q][C..2C) (dy).  dx_sums (may be
// null): dx_sums[q][0..C) = column sums of the segment's dx as stored (rounded to bf16) -- the bias gradient of the
// layer in front, which then needs no pass of its own over dx.
template <int NL, int W>
__global__ __launch_bounds__(kSlabThreads) void bn_bwd_slab_kernel(int rows, int C, const uint16_t* __restrict__ dy,
                                                                   const uint16_t* __restrict__ x, const float* __restrict__ stats,
                                                                   const float* __restrict__ gamma_s,
                                                                   const float* __restrict__ gamma_l, float alpha, float beta_c,
                                                                   uint16_t* __restrict__ dx, float* __restrict__ sums,
                                                                   float* __restrict__ dx_sums) {
  __shared__ __attribute__((aligned(16))) float red[16 * kSlabThreads + 16 * W];
  constexpr int kRowsPerPass = kSlabThreads / W;
  const int r0 = threadIdx.x / W;
  const int c0 = slab_of_block(blockIdx.x, gridDim.x) * 8 * W + 8 * (threadIdx.x % W);
  const int q = blockIdx.y;
  const float inv_rows = 1.f / (float)rows;
  const size_t base = (size_t)q * rows * C + c0;
  uint4 vx[NL], vd[NL];
#pragma unroll
  for (int i = 0; i < NL; ++i) {
    const int r = i * kRowsPerPass + r0;
    vx[i] = r < rows ? *reinterpret_cast<const uint4*>(x + base + (size_t)r * C) : make_uint4(0, 0, 0, 0);
    vd[i] = r < rows ? *reinterpret_cast<const uint4*>(dy + base + (size_t)r * C) : make_uint4(0, 0, 0, 0);
  }
  float g[8], mean[8], rstd[8], s[16];
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    g[j] = fmaf(alpha, gamma_s[c0 + j], beta_c * gamma_l[c0 + j]);
    mean[j] = stats[(size_t)q * 2 * C + 2 * (c0 + j)];
    rstd[j] = stats[(size_t)q * 2 * C + 2 * (c0 + j) + 1];
    s[j] = s[8 + j] = 0.f;
  }
#pragma unroll
  for (int i = 0; i < NL; ++i) {  // rows past the end: dy = 0 adds nothing
    float fx[8], fd[8];
    unpack8(vx[i], fx);
    unpack8(vd[i], fd);
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      s[j] = fmaf(fd[j], (fx[j] - mean[j]) * rstd[j], s[j]);
      s[8 + j] += fd[j];
    }
  }
  slab_sum<16, W>(s, red);
  if (r0 == 0) {
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      sums[(size_t)q * 2 * C + c0 + j] = s[j];
      sums[(size_t)q * 2 * C + C + c0 + j] = s[8 + j];
    }
  }
  float t[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int i = 0; i < NL; ++i) {
    const int r = i * kRowsPerPass + r0;
    if (r >= rows) continue;
    float fx[8], fd[8], o[8];
    unpack8(vx[i], fx);
    unpack8(vd[i], fd);
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const float xh = (fx[j] - mean[j]) * rstd[j];
      o[j] = g[j] * rstd[j] * (fd[j] - (s[8 + j] + xh * s[j]) * inv_rows);
    }
    const uint4 packed = pack8(o);
    *reinterpret_cast<uint4*>(dx + base + (size_t)r * C) = packed;
    unpack8(packed, o);
#pragma unroll
    for (int j = 0; j < 8; ++j) t[j] += o[j];
  }
  if (dx_sums) {  // the same for every lane of the workgroup
    slab_sum<8, W>(t, red);
    if (r0 == 0) {
#pragma unroll
      for (int j = 0; j < 8; ++j) dx_sums[(size_t)q * C + c0 + j] = t[j];
    }
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

// Workgroups for the 16-byte kernels: enough for `units` 16-byte units at two per lane, at most 4096, and such that
// the threads of the grid are a multiple of the units per row (a lane then stays on the same channels).
inline unsigned vec_grid(size_t units, int units_per_row) {
  size_t a = (size_t)units_per_row, b = kThreads;
  while (b) { const size_t t = a % b; a = b; b = t; }  // a = gcd(units_per_row, 256)
  const size_t mult = (size_t)units_per_row / a;
  size_t g = std::min<size_t>(std::max<size_t>((units + 2 * kThreads - 1) / (2 * kThreads), 1), 4096);
  g = (g + mult - 1) / mult * mult;
  return (unsigned)g;
}

inline bool vec_ok(int es, int C, const void* p0, const void* p1, const void* p2) {
  return es == 2 && C % 8 == 0 && ((((uintptr_t)p0 | (uintptr_t)p1 | (uintptr_t)p2) & 15) == 0);
}

// scratch: [chunks][2C] partial sums
template <typename T>
hipError_t bn_fwd_typed(hipStream_t s, size_t rows, int C, const T* x, const float* gamma, const float* beta, int act, T* a_out,
                        T* d_out, float* stats, float* scratch, const T* addend) {
  const bool vec = vec_ok(sizeof(T), C, x, a_out, d_out) && (((uintptr_t)addend) & 15) == 0;
  if (addend && !vec) return hipErrorNotSupported;
  const int cr = bn_chunk_rows(rows), chunks = bn_chunks(rows);
  float* partial = scratch;
  if (sizeof(T) == 2 && C % 8 == 0 && (((uintptr_t)x) & 15) == 0)
    hipLaunchKernelGGL(bn_colsum_vec_kernel<0>, dim3((C + 127) / 128, chunks, 1), dim3(kThreads), 0, s, rows, C, cr, (const uint16_t*)x,
                       (const uint16_t*)nullptr, (const float*)nullptr, partial);
  else
    hipLaunchKernelGGL((bn_colsum_kernel<T, 0>), dim3((C + 63) / 64, chunks, 1), dim3(kThreads), 0, s, rows, C, cr, x, (const T*)nullptr,
                       (const float*)nullptr, partial);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(bn_finalize_sum_kernel<T>, dim3((C + 15) / 16), dim3(kThreads), 0, s, rows, C, chunks, x, partial, stats);
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (vec)
    hipLaunchKernelGGL(bn_normalize_vec_kernel, dim3(vec_grid(rows * C / 8, C / 8)), dim3(kThreads), 0, s, rows, C, (const uint16_t*)x,
                       stats, gamma, beta, act, (const uint16_t*)addend, (uint16_t*)a_out, (uint16_t*)d_out);
  else
    hipLaunchKernelGGL(bn_normalize_kernel<T>, dim3(stream_grid(rows * C)), dim3(kThreads), 0, s, rows, C, x, stats, gamma, beta, act,
                       a_out, d_out);
  return hipGetLastError();
}

// all nseg segments in three launches; scratch: [chunks][nseg][2C] partial sums; sums: [nseg][2C]
template <typename T>
hipError_t bn_bwd_typed(hipStream_t s, size_t rows, int C, int nseg, const T* dy, const T* x, const float* stats, const float* gamma_s,
                        const float* gamma_l, float alpha, float beta_c, T* dx, float* sums, float* scratch) {
  const int cr = bn_chunk_rows(rows), chunks = bn_chunks(rows);
  if (sizeof(T) == 2 && C % 8 == 0 && ((((uintptr_t)x | (uintptr_t)dy)) & 15) == 0)
    hipLaunchKernelGGL(bn_colsum_vec_kernel<2>, dim3((C + 127) / 128, chunks, nseg), dim3(kThreads), 0, s, rows, C, cr, (const uint16_t*)x,
                       (const uint16_t*)dy, stats, scratch);
  else
    hipLaunchKernelGGL((bn_colsum_kernel<T, 2>), dim3((C + 63) / 64, chunks, nseg), dim3(kThreads), 0, s, rows, C, cr, x, dy, stats, scratch);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  e = launch_sum_partials(s, (size_t)nseg * 2 * C, chunks, scratch, sums);
  if (e != hipSuccess) return e;
  if (vec_ok(sizeof(T), C, x, dy, dx))
    hipLaunchKernelGGL(bn_dx_vec_kernel, dim3(vec_grid(rows * C / 8, C / 8), nseg), dim3(kThreads), 0, s, rows, C, (size_t)nseg,
                       (const uint16_t*)dy, (const uint16_t*)x, stats, sums, gamma_s, gamma_l, alpha, beta_c, (uint16_t*)dx);
  else
    hipLaunchKernelGGL(bn_dx_kernel<T>, dim3(stream_grid(rows * C * nseg)), dim3(kThreads), 0, s, rows, C, (size_t)nseg, dy, x, stats, sums,
                       gamma_s, gamma_l, alpha, beta_c, dx);
  return hipGetLastError();
}

// Rows per micro-batch the slab kernels take (beyond that the streaming kernels are faster) and the loads per lane (a
// power of two) that cover `rows` when a workgroup owns `width` 16-byte units of every row.
constexpr size_t kSlabMaxRows = 2048;
inline int slab_loads(size_t rows, int width) {
  const size_t rows_per_pass = kSlabThreads / width;
  int nl = 1;
  while ((size_t)nl * rows_per_pass < rows) nl *= 2;
  return nl;
}

}  // namespace

size_t batchnorm_scratch_floats(size_t rows, int C, int nseg) { return ((size_t)bn_chunks(rows) * std::max(nseg, 1) + 1) * 2 * C; }

bool batchnorm_fused_bwd_supported(int elt, size_t rows, int C) {
  return elt == ELT_BF16 && C % 8 == 0 && rows >= 1 && rows <= kSlabMaxRows && rows * C < (1ull << 31);
}

hipError_t launch_batchnorm_bwd_fused(hipStream_t s, int elt, size_t rows, int C, int nseg, const void* dy, const void* x,
                                      const float* stats, const float* gamma_s, const float* gamma_l, float alpha, float beta_c,
                                      void* dx, float* sums, float* dx_sums) {
  if (!batchnorm_fused_bwd_supported(elt, rows, C) || nseg < 1 || nseg > 65535) return hipErrorNotSupported;
  // 32 bytes per row where a micro-batch has more than 1024 rows and the channels allow it (measured on the layers of
  // a bottleneck group, 2048 rows: 16.0 us against 19.0 us at 16 bytes per row; 64 bytes per row would need eight loads
  // of x and of dy per lane, more than the 128 registers of a lane in a 1024-lane workgroup hold)
  const int W = (C % 16 == 0 && rows > (size_t)kSlabThreads) ? 2 : 1;
  const dim3 grid(C / (8 * W), nseg);
#define TP_BN_BWD(NL, W)                                                                                                     \
  hipLaunchKernelGGL((bn_bwd_slab_kernel<NL, W>), grid, dim3(kSlabThreads), 0, s, (int)rows, C, (const uint16_t*)dy,        \
                     (const uint16_t*)x, stats, gamma_s, gamma_l, alpha, beta_c, (uint16_t*)dx, sums, dx_sums)
  if (W == 2) TP_BN_BWD(4, 2);
  else if (slab_loads(rows, 1) == 1) TP_BN_BWD(1, 1);
  else TP_BN_BWD(2, 1);
#undef TP_BN_BWD
  return hipGetLastError();
}

// bf16 with whole 16-byte units of channels: the slab kernel up to kSlabMaxRows rows, the streaming normalise beyond
bool batchnorm_fwd_add_supported(int elt, size_t rows, int C) {
  return elt == ELT_BF16 && C % 8 == 0 && rows >= 1 && rows * C < (1ull << 31);
}
inline bool batchnorm_fwd_slab(int elt, size_t rows, int C) {
  return elt == ELT_BF16 && C % 8 == 0 && rows >= 1 && rows <= kSlabMaxRows && rows * C < (1ull << 31);
}

hipError_t launch_batchnorm_fwd(hipStream_t s, int elt, size_t rows, int C, const void* x, const float* gamma, const float* beta,
                                int act, void* a_out, void* d_out, float* stats, float* scratch, const void* addend) {
  if (addend && !batchnorm_fwd_add_supported(elt, rows, C)) return hipErrorNotSupported;
  if (batchnorm_fwd_slab(elt, rows, C)) {
    // 16 bytes per row: wider slabs, which pay in the backward kernel, were slower here on the layers of a bottleneck
    // group (C = 1024, 2048 rows: 14.5 us at 32 bytes per row against 10.9 us), where x has just been written by another
    // kernel and more workgroups fetch it from more CUs
#define TP_BN_FWD(NL, W)                                                                                                     \
  hipLaunchKernelGGL((bn_fwd_slab_kernel<NL, W>), dim3(C / (8 * W)), dim3(kSlabThreads), 0, s, (int)rows, C, (const uint16_t*)x, \
                     gamma, beta, act, (const uint16_t*)addend, (uint16_t*)a_out, (uint16_t*)d_out, stats)
    if (slab_loads(rows, 1) == 1) TP_BN_FWD(1, 1); else TP_BN_FWD(2, 1);
#undef TP_BN_FWD
    return hipGetLastError();
  }
  if (elt == ELT_BF16)
    return bn_fwd_typed<uint16_t>(s, rows, C, (const uint16_t*)x, gamma, beta, act, (uint16_t*)a_out, (uint16_t*)d_out, stats, scratch,
                                  (const uint16_t*)addend);
  return bn_fwd_typed<float>(s, rows, C, (const float*)x, gamma, beta, act, (float*)a_out, (float*)d_out, stats, scratch,
                             (const float*)nullptr);
}

hipError_t launch_batchnorm_bwd(hipStream_t s, int elt, size_t rows, int C, int nseg, const void* dy, const void* x, const float* stats,
                                const float* gamma_s, const float* gamma_l, float alpha, float beta_c, void* dx, float* sums,
                                float* scratch) {
  if (nseg < 1 || nseg > 65535) return hipErrorInvalidValue;
  if (elt == ELT_BF16)
    return bn_bwd_typed<uint16_t>(s, rows, C, nseg, (const uint16_t*)dy, (const uint16_t*)x, stats, gamma_s, gamma_l, alpha, beta_c,
                                  (uint16_t*)dx, sums, scratch);
  return bn_bwd_typed<float>(s, rows, C, nseg, (const float*)dy, (const float*)x, stats, gamma_s, gamma_l, alpha, beta_c, (float*)dx,
                             sums, scratch);
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
