// GEMM launchers of a stage: fprop (z = x W^T + b, a = act(z)), dgrad (dx = dz W_b, fused with
// the previous layer's activation derivative) and wgrad (dW = dz^T x, db = column sums of dz).
//
// This file holds the shape-generic, bounds-checked SIMT kernel (fp32 FMA, LDS-tiled) that
// serves the fp32 mode and any bf16 shape the MFMA kernels do not take, and the dispatch
// between the two.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <algorithm>

#include "device_utils.h"
#include "gemm_mfma.h"
#include "kernels.h"

namespace tp {

namespace {

constexpr int BM = 64, BN = 64, BK = 16, kThreads = 256;

enum Epi : int { EPI_STORE_F32 = 0, EPI_FPROP = 1, EPI_DGRAD = 2 };

struct EpiArgs {
  float* c_f32;        // EPI_STORE_F32: [M x N] fp32
  const float* bias;   // EPI_FPROP
  void* d_out;         // EPI_FPROP: optional act'(z)
  void* a_out;         // EPI_FPROP: activation; EPI_DGRAD: output
  const void* d_prev;  // EPI_DGRAD: optional saved act'(z) of the previous layer
  int act;
  int relu_mask;       // EPI_DGRAD: d_prev holds the ReLU output, the factor is (output > 0)
};

// C(m,n) = sum_k A[m*sam + k*sak] * B[k*sbk + n*sbn], 64x64 tile per block, 4x4 per thread.
template <typename T, int EPI>
__global__ __launch_bounds__(kThreads) void gemm_simt_kernel(int M, int N, int K, const T* __restrict__ A, long sam,
                                                             long sak, const T* __restrict__ B, long sbk, long sbn,
                                                             EpiArgs e) {
  __shared__ float As[BK][BM + 4];
  __shared__ float Bs[BK][BN + 4];
  const int t = threadIdx.x;
  const int tx = t & 15, ty = t >> 4;
  const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
  float acc[4][4] = {};
  const bool a_kfast = sak == 1, b_kfast = sbk == 1;
  for (int k0 = 0; k0 < K; k0 += BK) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int el = t + i * kThreads;
      int m, k;
      if (a_kfast) { k = el & (BK - 1); m = el >> 4; } else { m = el & (BM - 1); k = el >> 6; }
      float v = 0.f;
      if (m0 + m < M && k0 + k < K) v = to_float(A[(long)(m0 + m) * sam + (long)(k0 + k) * sak]);
      As[k][m] = v;
      int n, kb;
      if (b_kfast) { kb = el & (BK - 1); n = el >> 4; } else { n = el & (BN - 1); kb = el >> 6; }
      float w = 0.f;
      if (n0 + n < N && k0 + kb < K) w = to_float(B[(long)(k0 + kb) * sbk + (long)(n0 + n) * sbn]);
      Bs[kb][n] = w;
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < BK; ++k) {
      const float4 a = *reinterpret_cast<const float4*>(&As[k][ty * 4]);
      const float4 b = *reinterpret_cast<const float4*>(&Bs[k][tx * 4]);
      const float av[4] = {a.x, a.y, a.z, a.w};
      const float bv[4] = {b.x, b.y, b.z, b.w};
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(av[i], bv[j], acc[i][j]);
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int m = m0 + ty * 4 + i;
    if (m >= M) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int n = n0 + tx * 4 + j;
      if (n >= N) continue;
      const size_t idx = (size_t)m * N + n;
      float v = acc[i][j];
      if (EPI == EPI_STORE_F32) {
        e.c_f32[idx] = v;
      } else if (EPI == EPI_FPROP) {
        v += e.bias[n];
        if (e.d_out) ((T*)e.d_out)[idx] = from_float<T>(act_derivative(v, e.act));
        ((T*)e.a_out)[idx] = from_float<T>(act_forward(v, e.act));
      } else {
        if (e.d_prev) {
          const float dp = to_float(((const T*)e.d_prev)[idx]);
          v = e.relu_mask ? (dp > 0.f ? v : 0.f) : v * dp;
        }
        ((T*)e.a_out)[idx] = from_float<T>(v);
      }
    }
  }
}

template <int EPI>
hipError_t simt(hipStream_t s, int elt, int M, int N, int K, const void* A, long sam, long sak, const void* B, long sbk,
                long sbn, const EpiArgs& e) {
  dim3 grid((N + BN - 1) / BN, (M + BM - 1) / BM);
  if (elt == ELT_BF16)
    hipLaunchKernelGGL((gemm_simt_kernel<uint16_t, EPI>), grid, dim3(kThreads), 0, s, M, N, K, (const uint16_t*)A, sam,
                       sak, (const uint16_t*)B, sbk, sbn, e);
  else
    hipLaunchKernelGGL((gemm_simt_kernel<float, EPI>), grid, dim3(kThreads), 0, s, M, N, K, (const float*)A, sam, sak,
                       (const float*)B, sbk, sbn, e);
  return hipGetLastError();
}

// Column sums of dz[M x N] in two fixed-order steps: row chunks -> partials[chunk][N] -> gb[N].
// A lane owns V = 16/sizeof(T) adjacent columns (one 16-byte load per row).  A block covers up
// to 64*V columns; when the matrix is narrower, the spare lanes take other rows, so tall and
// skinny matrices (convolution: rows = all pixels) still use every lane.  The row groups of a
// block are combined through LDS in a fixed order.
struct ColsumShape {
  int lanes_per_row;  // power of two <= 64
  int rows_per_iter;  // kThreads / lanes_per_row
  int col_blocks, chunk_rows, chunks;
};

inline ColsumShape colsum_shape(int M, int N, int V) {
  ColsumShape c;
  const int need = (std::min(N, 64 * V) + V - 1) / V;
  c.lanes_per_row = 1;
  while (c.lanes_per_row < need) c.lanes_per_row *= 2;
  c.rows_per_iter = kThreads / c.lanes_per_row;
  c.col_blocks = (N + c.lanes_per_row * V - 1) / (c.lanes_per_row * V);
  const int target_chunks = std::max(1, 1024 / c.col_blocks);
  c.chunk_rows = std::max(c.rows_per_iter * 2, (M + target_chunks - 1) / target_chunks);
  c.chunks = (M + c.chunk_rows - 1) / c.chunk_rows;
  return c;
}

template <typename T>
__global__ __launch_bounds__(kThreads) void colsum_partial_kernel(int M, int N, ColsumShape cs, const T* __restrict__ dz,
                                                                  float* __restrict__ partials) {
  constexpr int V = 16 / sizeof(T);
  __shared__ float sm[kThreads * V];
  const int lr = threadIdx.x % cs.lanes_per_row, rsub = threadIdx.x / cs.lanes_per_row;
  const int col = (blockIdx.x * cs.lanes_per_row + lr) * V;
  const int r0 = blockIdx.y * cs.chunk_rows;
  const int r1 = min(M, r0 + cs.chunk_rows);
  float s[V];
#pragma unroll
  for (int j = 0; j < V; ++j) s[j] = 0.f;
  if (col + V <= N && (N % V) == 0) {
#pragma unroll 4
    for (int r = r0 + rsub; r < r1; r += cs.rows_per_iter) {
      const uint4 v = *reinterpret_cast<const uint4*>(dz + (size_t)r * N + col);
      const uint32_t w[4] = {v.x, v.y, v.z, v.w};
      if (sizeof(T) == 2) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          s[(2 * j) % V] += __uint_as_float(w[j] << 16);
          s[(2 * j + 1) % V] += __uint_as_float(w[j] & 0xffff0000u);
        }
      } else {
#pragma unroll
        for (int j = 0; j < 4; ++j) s[j % V] += __uint_as_float(w[j]);
      }
    }
  } else {
    for (int r = r0 + rsub; r < r1; r += cs.rows_per_iter)
      for (int j = 0; j < V; ++j)
        if (col + j < N) s[j] += to_float(dz[(size_t)r * N + col + j]);
  }
#pragma unroll
  for (int j = 0; j < V; ++j) sm[(rsub * cs.lanes_per_row + lr) * V + j] = s[j];
  __syncthreads();
  if (rsub == 0) {
    for (int j = 0; j < V; ++j) {
      if (col + j >= N) continue;
      float t = 0.f;
      for (int q = 0; q < cs.rows_per_iter; ++q) t += sm[(q * cs.lanes_per_row + lr) * V + j];
      partials[(size_t)blockIdx.y * N + col + j] = t;
    }
  }
}

// dz = dy (.) d (MASK: d is a ReLU output, the factor is (d > 0)) and, in the same pass, the partial column sums of
// the dz it stores: the first two steps of a backward pass whose last layer has an activation, with the structure --
// and therefore the sums -- of colsum_partial_kernel.  bf16, N % 8 == 0, 16-byte aligned pointers.
template <bool MASK>
__global__ __launch_bounds__(kThreads) void act_backward_colsum_kernel(int M, int N, ColsumShape cs, const uint16_t* __restrict__ dy,
                                                                       const uint16_t* __restrict__ d, uint16_t* __restrict__ dz,
                                                                       float* __restrict__ partials) {
  constexpr int V = 8;
  __shared__ float sm[kThreads * V];
  const int lr = threadIdx.x % cs.lanes_per_row, rsub = threadIdx.x / cs.lanes_per_row;
  const int col = (blockIdx.x * cs.lanes_per_row + lr) * V;
  const int r0 = blockIdx.y * cs.chunk_rows;
  const int r1 = min(M, r0 + cs.chunk_rows);
  float s[V];
#pragma unroll
  for (int j = 0; j < V; ++j) s[j] = 0.f;
  if (col < N) {
#pragma unroll 4
    for (int r = r0 + rsub; r < r1; r += cs.rows_per_iter) {
      const size_t at = (size_t)r * N + col;
      const uint4 a = *reinterpret_cast<const uint4*>(dy + at), b = *reinterpret_cast<const uint4*>(d + at);
      const uint32_t aw[4] = {a.x, a.y, a.z, a.w}, bw[4] = {b.x, b.y, b.z, b.w};
      uint32_t ow[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const float g0 = __uint_as_float(aw[j] << 16), g1 = __uint_as_float(aw[j] & 0xffff0000u);
        const float d0 = __uint_as_float(bw[j] << 16), d1 = __uint_as_float(bw[j] & 0xffff0000u);
        ow[j] = pack_bf16x2(MASK ? (d0 > 0.f ? g0 : 0.f) : g0 * d0, MASK ? (d1 > 0.f ? g1 : 0.f) : g1 * d1);
        s[2 * j] += __uint_as_float(ow[j] << 16);          // what is stored, as the separate pass over dz would read it
        s[2 * j + 1] += __uint_as_float(ow[j] & 0xffff0000u);
      }
      *reinterpret_cast<uint4*>(dz + at) = make_uint4(ow[0], ow[1], ow[2], ow[3]);
    }
  }
#pragma unroll
  for (int j = 0; j < V; ++j) sm[(rsub * cs.lanes_per_row + lr) * V + j] = s[j];
  __syncthreads();
  if (rsub == 0 && col < N) {
    for (int j = 0; j < V; ++j) {
      float t = 0.f;
      for (int q = 0; q < cs.rows_per_iter; ++q) t += sm[(q * cs.lanes_per_row + lr) * V + j];
      partials[(size_t)blockIdx.y * N + col + j] = t;
    }
  }
}

// Sum of partial results.  A block covers IL = 256/ZG consecutive outputs with ZG threads each:
// thread (zg, il) adds partials zg, zg + ZG, ... of output il, the ZG sums are combined through LDS
// in a fixed order.  Large outputs take few threads per output (whole cache lines per partial
// row, enough blocks anyway); small ones take many, so that a thousand partials do not end up
// as one long chain of dependent loads.
constexpr int kSumLds = 64 * (kThreads / 64 + 1);  // floats; the largest of ZG * (256/ZG + 1) for ZG in {4, 16, 64}

template <int ZG>
__device__ __forceinline__ void sum_partials_block(float* sm /* [ZG][IL + 1] */, size_t block, size_t count, int splits,
                                                   size_t stride, const float* __restrict__ partial, float* __restrict__ out) {
  constexpr int IL = kThreads / ZG;
  static_assert(ZG * (IL + 1) <= kSumLds, "LDS of the sum kernels");
  const int il = threadIdx.x % IL, zg = threadIdx.x / IL;
  const size_t i = block * IL + il;
  float s0 = 0.f, s1 = 0.f;
  if (i < count) {
    int z = zg;
    for (; z + ZG < splits; z += 2 * ZG) {  // two independent chains
      s0 += partial[(size_t)z * stride + i];
      s1 += partial[(size_t)(z + ZG) * stride + i];
    }
    if (z < splits) s0 += partial[(size_t)z * stride + i];
  }
  sm[zg * (IL + 1) + il] = s0 + s1;
  __syncthreads();
  if (zg == 0 && i < count) {
    float t = 0.f;
#pragma unroll
    for (int k = 0; k < ZG; ++k) t += sm[k * (IL + 1) + il];
    out[i] = t;
  }
}

template <int ZG>
__global__ __launch_bounds__(kThreads) void sum_partials_kernel(size_t count, int splits, size_t stride,
                                                                const float* __restrict__ partial, float* __restrict__ out) {
  __shared__ float sm[kSumLds];
  sum_partials_block<ZG>(sm, blockIdx.x, count, splits, stride, partial, out);
}

// Few partials of a large output: one thread per four neighbouring outputs, 16-byte loads, the partials added one
// after the other.
__device__ __forceinline__ void sum_partials_block_vec(size_t block, size_t count, int splits, size_t stride,
                                                       const float* __restrict__ partial, float* __restrict__ out) {
  const size_t i = (block * kThreads + threadIdx.x) * 4;
  if (i >= count) return;
  float4 t = *reinterpret_cast<const float4*>(partial + i);
  for (int z = 1; z < splits; ++z) {
    const float4 p = *reinterpret_cast<const float4*>(partial + (size_t)z * stride + i);
    t.x += p.x; t.y += p.y; t.z += p.z; t.w += p.w;
  }
  *reinterpret_cast<float4*>(out + i) = t;
}

__global__ __launch_bounds__(kThreads) void sum_partials_vec_kernel(size_t count, int splits, size_t stride,
                                                                    const float* __restrict__ partial, float* __restrict__ out) {
  sum_partials_block_vec(blockIdx.x, count, splits, stride, partial, out);
}

// Threads per output the sum kernels use for a job of this shape; 0: the 16-byte kernel (four outputs per thread).
inline int sum_zg(size_t count, int splits, size_t stride, const float* partial, const float* out) {
  if (splits <= 8 && count >= 16384 && count % 4 == 0 && stride % 4 == 0 && (((uintptr_t)partial | (uintptr_t)out) & 15) == 0)
    return 0;
  // at least 16 neighbouring outputs per block where there are that many: 64 bytes of every partial row, not 16
  return (count >= 512 * 64 || splits <= 8) ? 4 : count >= 1024 ? 16 : 64;
}
inline int sum_outputs_per_block(int zg) { return zg == 0 ? 4 * kThreads : kThreads / zg; }

// Many sums in one launch.  The table travels as the kernel's argument (no device memory, nothing to upload):
// block b belongs to the job j with first_block[j] <= b < first_block[j + 1] and does there exactly what block
// b - first_block[j] of sum_partials_kernel would do, so both give the same bits.
constexpr int kMaxSumJobs = 96;
struct PackedSumJob {
  const float* partial;
  float* out;
  uint32_t count, stride, splits, zg;
};
struct SumBatch {
  uint32_t njobs;
  uint32_t first_block[kMaxSumJobs + 1];
  PackedSumJob job[kMaxSumJobs];
};
static_assert(sizeof(SumBatch) <= 4096, "kernel arguments are limited to 4 KB");

__global__ __launch_bounds__(kThreads) void sum_jobs_kernel(const SumBatch b) {
  __shared__ float sm[kSumLds];
  int lo = 0, hi = (int)b.njobs;  // first_block[lo] <= blockIdx.x < first_block[hi]
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (b.first_block[mid] <= blockIdx.x) lo = mid; else hi = mid;
  }
  const PackedSumJob& J = b.job[lo];
  const size_t block = blockIdx.x - b.first_block[lo];
  if (J.zg == 0) sum_partials_block_vec(block, J.count, (int)J.splits, J.stride, J.partial, J.out);
  else if (J.zg == 4) sum_partials_block<4>(sm, block, J.count, (int)J.splits, J.stride, J.partial, J.out);
  else if (J.zg == 16) sum_partials_block<16>(sm, block, J.count, (int)J.splits, J.stride, J.partial, J.out);
  else sum_partials_block<64>(sm, block, J.count, (int)J.splits, J.stride, J.partial, J.out);
}

thread_local std::vector<SumJob>* g_sum_sink = nullptr;

}  // namespace

size_t colsum_scratch_floats(int M, int N) {
  // the fp32 shape has the fewer columns per block, hence the more chunks: size for it
  return (size_t)std::max(colsum_shape(M, N, 4).chunks, colsum_shape(M, N, 8).chunks) * (size_t)N;
}

bool fprop_add_supported(int elt, int M, int N, int K) { return elt == ELT_BF16 && mfma_fprop_supported(M, N, K) && N % 8 == 0; }

hipError_t launch_fprop(hipStream_t s, int elt, int M, int N, int K, const void* x, const void* W, const float* bias,
                        int act, void* d_out, void* a_out, void* x_copy, const void* addend) {
  if (addend && (!fprop_add_supported(elt, M, N, K) || ((uintptr_t)addend & 15))) return hipErrorNotSupported;
  const bool aligned = (((uintptr_t)x | (uintptr_t)x_copy) & 15) == 0;
  if (elt == ELT_BF16 && mfma_fprop_supported(M, N, K) && aligned)
    return mfma_fprop(s, M, N, K, (const uint16_t*)x, (const uint16_t*)W, bias, act, (uint16_t*)d_out, (uint16_t*)a_out,
                      (uint16_t*)x_copy, (const uint16_t*)addend);
  if (x_copy) {
    hipError_t err = launch_copy(s, x, x_copy, (size_t)M * K * (elt == ELT_BF16 ? 2 : 4));
    if (err != hipSuccess) return err;
  }
  if (elt == ELT_BF16 && mfma_fprop_supported(M, N, K))
    return mfma_fprop(s, M, N, K, (const uint16_t*)x, (const uint16_t*)W, bias, act, (uint16_t*)d_out, (uint16_t*)a_out,
                      nullptr, (const uint16_t*)addend);
  EpiArgs e{};
  e.bias = bias; e.d_out = d_out; e.a_out = a_out; e.act = act;
  return simt<EPI_FPROP>(s, elt, M, N, K, x, K, 1, W, 1, K, e);
}

hipError_t launch_dgrad(hipStream_t s, int elt, int M, int N, int K, const void* dz, const void* Wb, const void* d_prev,
                        void* out, int relu_mask) {
  if (elt == ELT_BF16 && mfma_dgrad_supported(M, N, K))
    return mfma_dgrad(s, M, N, K, (const uint16_t*)dz, (const uint16_t*)Wb, (const uint16_t*)d_prev, (uint16_t*)out, relu_mask);
  EpiArgs e{};
  e.a_out = out; e.d_prev = d_prev; e.relu_mask = relu_mask;
  // out[M x K] = dz[M x N] . Wb[N x K]: contraction over N
  return simt<EPI_DGRAD>(s, elt, M, K, N, dz, N, 1, Wb, K, 1, e);
}

void set_sum_sink(std::vector<SumJob>* sink) { g_sum_sink = sink; }

hipError_t launch_sum_partials_strided(hipStream_t s, size_t count, int splits, const float* partial, size_t stride,
                                       float* out) {
  if (g_sum_sink && count < (1ull << 32) && stride < (1ull << 32)) {
    g_sum_sink->push_back(SumJob{partial, out, count, stride, splits});
    return hipSuccess;
  }
  auto blocks = [&](int il) { return dim3((unsigned)((count + il - 1) / il)); };
  switch (sum_zg(count, splits, stride, partial, out)) {
    case 0: hipLaunchKernelGGL(sum_partials_vec_kernel, blocks(4 * kThreads), dim3(kThreads), 0, s, count, splits, stride, partial, out); break;
    case 4: hipLaunchKernelGGL(sum_partials_kernel<4>, blocks(64), dim3(kThreads), 0, s, count, splits, stride, partial, out); break;
    case 16: hipLaunchKernelGGL(sum_partials_kernel<16>, blocks(16), dim3(kThreads), 0, s, count, splits, stride, partial, out); break;
    default: hipLaunchKernelGGL(sum_partials_kernel<64>, blocks(4), dim3(kThreads), 0, s, count, splits, stride, partial, out);
  }
  return hipGetLastError();
}

hipError_t launch_sum_jobs(hipStream_t s, const SumJob* jobs, size_t njobs) {
  size_t done = 0;
  while (done < njobs) {
    SumBatch b;
    b.njobs = 0;
    uint64_t blocks = 0;
    while (done < njobs && b.njobs < (uint32_t)kMaxSumJobs) {
      const SumJob& j = jobs[done];
      if (j.count == 0 || j.splits < 1 || j.count >= (1ull << 32) || j.stride >= (1ull << 32)) return hipErrorInvalidValue;
      const int zg = sum_zg(j.count, j.splits, j.stride, j.partial, j.out), il = sum_outputs_per_block(zg);
      const uint64_t nb = (j.count + il - 1) / il;
      if (blocks + nb >= (1ull << 31)) {
        if (b.njobs == 0) return hipErrorInvalidValue;
        break;
      }
      b.first_block[b.njobs] = (uint32_t)blocks;
      b.job[b.njobs] = PackedSumJob{j.partial, j.out, (uint32_t)j.count, (uint32_t)j.stride, (uint32_t)j.splits, (uint32_t)zg};
      blocks += nb;
      ++b.njobs;
      ++done;
    }
    for (uint32_t k = b.njobs; k <= (uint32_t)kMaxSumJobs; ++k) b.first_block[k] = (uint32_t)blocks;
    for (uint32_t k = b.njobs; k < (uint32_t)kMaxSumJobs; ++k) b.job[k] = PackedSumJob{nullptr, nullptr, 0, 0, 0, 4};
    hipLaunchKernelGGL(sum_jobs_kernel, dim3((unsigned)blocks), dim3(kThreads), 0, s, b);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

hipError_t launch_sum_partials(hipStream_t s, size_t count, int splits, const float* partial, float* out) {
  return launch_sum_partials_strided(s, count, splits, partial, count, out);
}

hipError_t launch_colsum(hipStream_t s, int elt, int M, int N, const void* dz, float* gb, float* partials) {
  const ColsumShape cs = colsum_shape(M, N, elt == ELT_BF16 ? 8 : 4);
  dim3 g1(cs.col_blocks, cs.chunks);
  if (elt == ELT_BF16)
    hipLaunchKernelGGL(colsum_partial_kernel<uint16_t>, g1, dim3(kThreads), 0, s, M, N, cs, (const uint16_t*)dz, partials);
  else
    hipLaunchKernelGGL(colsum_partial_kernel<float>, g1, dim3(kThreads), 0, s, M, N, cs, (const float*)dz, partials);
  hipError_t err = hipGetLastError();
  if (err != hipSuccess) return err;
  return launch_sum_partials(s, (size_t)N, cs.chunks, partials, gb);
}

bool act_backward_colsum_supported(int elt, int N) { return elt == ELT_BF16 && N % 8 == 0; }

hipError_t launch_act_backward_colsum(hipStream_t s, int elt, int M, int N, const void* dy, const void* d, void* dz,
                                      int relu_mask, float* gb, float* partials) {
  if (!act_backward_colsum_supported(elt, N) || ((((uintptr_t)dy | (uintptr_t)d | (uintptr_t)dz) & 15) != 0))
    return hipErrorNotSupported;
  const ColsumShape cs = colsum_shape(M, N, 8);
  dim3 g1(cs.col_blocks, cs.chunks);
  if (relu_mask)
    hipLaunchKernelGGL(act_backward_colsum_kernel<true>, g1, dim3(kThreads), 0, s, M, N, cs, (const uint16_t*)dy,
                       (const uint16_t*)d, (uint16_t*)dz, partials);
  else
    hipLaunchKernelGGL(act_backward_colsum_kernel<false>, g1, dim3(kThreads), 0, s, M, N, cs, (const uint16_t*)dy,
                       (const uint16_t*)d, (uint16_t*)dz, partials);
  hipError_t err = hipGetLastError();
  if (err != hipSuccess) return err;
  return launch_sum_partials(s, (size_t)N, cs.chunks, partials, gb);
}

size_t wgrad_scratch_floats(int elt, int M, int N, int K) {
  return elt == ELT_BF16 && mfma_wgrad_supported(M, N, K) ? mfma_wgrad_scratch_floats(M, N, K) : 0;
}

hipError_t launch_wgrad(hipStream_t s, int elt, int M, int N, int K, const void* dz, const void* x, float* gW, float* partial) {
  if (elt == ELT_BF16 && mfma_wgrad_supported(M, N, K))
    return mfma_wgrad(s, M, N, K, (const uint16_t*)dz, (const uint16_t*)x, gW, partial);
  EpiArgs e{};
  e.c_f32 = gW;
  // gW[N x K] = dz^T[N x M] . x[M x K]: contraction over M
  return simt<EPI_STORE_F32>(s, elt, N, K, M, dz, 1, N, x, K, 1, e);
}

}  // namespace tp
