// Elementwise and reduction kernels of the stage library for gfx950 (wave64).
//
//   update_kernel   the fused pass over the parameters: momentum, weight update into the next
//                   ring slot, bf16 compute copy, intermediate weights for the next backward
//                   (Eq. 1-2) and on-the-fly diagnostics.  Pure HBM streaming.
//   blend_kernel    the intermediate weights on their own (when the fused pass did not build them)
//   convert_kernel  fp32 -> bf16 compute copy
//   act_backward    dz = dy (.) d, d = act'(z) saved by the forward pass
//   softmax_ce      loss and its gradient at the last stage
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <mutex>

#include "device_utils.h"
#include "kernels.h"

namespace tp {

namespace {

constexpr int kThreads = 256;
// Launch shape of the update kernel: 8 blocks per CU on 256 CUs, grid-stride beyond that; two 16-byte
// chunks per lane and stream in flight; non-temporal accesses for the streams that are not re-read soon.
constexpr int kUpdateBlocks = 2048;
constexpr int kUnroll = 2;
constexpr bool kNonTemporal = true;

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}

// Sum `NV` values over the block; result valid in thread 0.  Fixed order => deterministic.
template <int NV>
__device__ __forceinline__ void block_sum(float (&v)[NV], float* smem /* [NV][4] */) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    v[i] = wave_sum(v[i]);
    if (lane == 0) smem[i * 4 + wave] = v[i];
  }
  __syncthreads();
  if (threadIdx.x == 0) {
#pragma unroll
    for (int i = 0; i < NV; ++i) v[i] = (smem[i * 4 + 0] + smem[i * 4 + 1]) + (smem[i * 4 + 2] + smem[i * 4 + 3]);
  }
}

template <typename T>
struct Store4;
template <>
struct Store4<float> {
  static __device__ __forceinline__ void st(float* p, float4 v) { *reinterpret_cast<float4*>(p) = v; }
};
template <>
struct Store4<uint16_t> {
  static __device__ __forceinline__ void st(uint16_t* p, float4 v) {
    uint2 o;
    o.x = pack_bf16x2(v.x, v.y);
    o.y = pack_bf16x2(v.z, v.w);
    *reinterpret_cast<uint2*>(p) = o;
  }
};

// Every stream is read or written exactly once.  A block works on contiguous chunks of
// kThreads*kUnroll float4 per stream and issues all its loads (kUnroll per stream per lane, 16
// bytes each) before the first dependent instruction, so that each lane keeps up to 16 loads in
// flight; the fp32 streams that are not re-read soon (momentum, new master weights) bypass the
// caches with non-temporal accesses.

typedef float floatx4 __attribute__((ext_vector_type(4)));

template <typename T, bool BLEND, bool WFWD>
__global__ __launch_bounds__(kThreads) void update_kernel(size_t n4, const floatx4* __restrict__ g,
                                                          floatx4* __restrict__ m, const floatx4* w_old,
                                                          floatx4* w_new, const floatx4* __restrict__ w_stale,
                                                          T* __restrict__ wfwd, T* __restrict__ wb, float lr,
                                                          float mu, float alpha, float beta,
                                                          float* __restrict__ partials) {
  __shared__ float red[4 * 4];
  float acc[4] = {0.f, 0.f, 0.f, 0.f};  // g^2, w^2, drift^2, wb^2
  const size_t chunk = (size_t)kThreads * kUnroll;
  for (size_t base = (size_t)blockIdx.x * chunk; base < n4; base += (size_t)gridDim.x * chunk) {
    floatx4 gv[kUnroll], mv[kUnroll], wv[kUnroll], sv[kUnroll];
    bool ok[kUnroll];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      const size_t i = base + (size_t)u * kThreads + threadIdx.x;
      ok[u] = i < n4;
      if (ok[u]) {
        gv[u] = kNonTemporal ? __builtin_nontemporal_load(g + i) : g[i];
        mv[u] = kNonTemporal ? __builtin_nontemporal_load(m + i) : m[i];
        wv[u] = w_old[i];
        if (BLEND) sv[u] = w_stale[i];
      }
    }
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      if (!ok[u]) continue;
      const size_t i = base + (size_t)u * kThreads + threadIdx.x;
      floatx4 mn, wn;
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        mn[c] = fmaf(mu, mv[u][c], gv[u][c]);
        wn[c] = fmaf(-lr, mn[c], wv[u][c]);
        acc[0] = fmaf(gv[u][c], gv[u][c], acc[0]);
        acc[1] = fmaf(wn[c], wn[c], acc[1]);
      }
      if (kNonTemporal) {
        __builtin_nontemporal_store(mn, m + i);
        __builtin_nontemporal_store(wn, w_new + i);
      } else {
        m[i] = mn;
        w_new[i] = wn;
      }
      if (WFWD) Store4<T>::st(wfwd + 4 * i, make_float4(wn[0], wn[1], wn[2], wn[3]));
      if (BLEND) {
        floatx4 b;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          b[c] = fmaf(alpha, sv[u][c], beta * wn[c]);
          const float dd = wn[c] - sv[u][c];
          acc[2] = fmaf(dd, dd, acc[2]);
          acc[3] = fmaf(b[c], b[c], acc[3]);
        }
        Store4<T>::st(wb + 4 * i, make_float4(b[0], b[1], b[2], b[3]));
      }
    }
  }
  block_sum<4>(acc, red);
  if (threadIdx.x == 0) {
#pragma unroll
    for (int k = 0; k < 4; ++k) partials[k * kUpdateBlocks + blockIdx.x] = acc[k];
  }
}

// Final, fixed-order reduction of the per-block partials into doubles: wave k sums quantity k.
__global__ __launch_bounds__(kThreads) void diag_reduce_kernel(const float* __restrict__ partials, int nblocks,
                                                               double* __restrict__ diag) {
  const int lane = threadIdx.x & 63, k = threadIdx.x >> 6;
  double s = 0.0;
#pragma unroll 8
  for (int i = lane; i < nblocks; i += 64) s += (double)partials[k * kUpdateBlocks + i];
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) s += __shfl_xor(s, off, 64);
  if (lane == 0) diag[k] = s;
}

template <typename T>
__global__ __launch_bounds__(kThreads) void blend_kernel(size_t n4, const float4* __restrict__ ws,
                                                         const float4* __restrict__ wl, float alpha, float beta,
                                                         T* __restrict__ wb) {
  const size_t stride = (size_t)gridDim.x * kThreads;
  for (size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x; i < n4; i += stride) {
    const float4 s = ws[i], l = wl[i];
    float4 b;
    b.x = fmaf(alpha, s.x, beta * l.x); b.y = fmaf(alpha, s.y, beta * l.y);
    b.z = fmaf(alpha, s.z, beta * l.z); b.w = fmaf(alpha, s.w, beta * l.w);
    Store4<T>::st(wb + 4 * i, b);
  }
}

template <typename T>
__global__ __launch_bounds__(kThreads) void convert_kernel(size_t n4, const float4* __restrict__ src,
                                                           T* __restrict__ dst) {
  const size_t stride = (size_t)gridDim.x * kThreads;
  for (size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x; i < n4; i += stride)
    Store4<T>::st(dst + 4 * i, src[i]);
}

// dz = dy (.) d, 16 bytes per lane per step; `count` elements, the tail element-wise.
// dz may be the same buffer as dy (every element is read before it is written by the same lane).
// MASK: d holds a ReLU output instead of its derivative; the factor is (d > 0).
// ADD: the gradient is dy + add (two branches of a residual connection meeting), rounded to T as the separate
// addition would have stored it, before it passes the activation.
template <typename T, bool MASK, bool ADD>
__global__ __launch_bounds__(kThreads) void act_backward_kernel(size_t count, const T* dy, const T* __restrict__ d,
                                                                T* dz, const T* __restrict__ add) {
  constexpr int V = 16 / sizeof(T);
  const size_t nvec = count / V;
  const size_t stride = (size_t)gridDim.x * kThreads;
  const size_t tid = (size_t)blockIdx.x * kThreads + threadIdx.x;
  auto through = [](float g, float dv) { return MASK ? (dv > 0.f ? g : 0.f) : g * dv; };
  auto summed = [](float g, float a) { return ADD ? to_float(from_float<T>(g + a)) : g; };
  for (size_t i = tid; i < nvec; i += stride) {
    const uint4 a = reinterpret_cast<const uint4*>(dy)[i];
    const uint4 b = reinterpret_cast<const uint4*>(d)[i];
    uint4 c = make_uint4(0, 0, 0, 0);
    if constexpr (ADD) c = reinterpret_cast<const uint4*>(add)[i];
    uint4 o;
    if (sizeof(T) == 2) {
      const uint32_t aw[4] = {a.x, a.y, a.z, a.w}, bw[4] = {b.x, b.y, b.z, b.w}, cw[4] = {c.x, c.y, c.z, c.w};
      uint32_t ow[4];
#pragma unroll
      for (int j = 0; j < 4; ++j)
        ow[j] = pack_bf16x2(through(summed(__uint_as_float(aw[j] << 16), __uint_as_float(cw[j] << 16)), __uint_as_float(bw[j] << 16)),
                            through(summed(__uint_as_float(aw[j] & 0xffff0000u), __uint_as_float(cw[j] & 0xffff0000u)),
                                    __uint_as_float(bw[j] & 0xffff0000u)));
      o = make_uint4(ow[0], ow[1], ow[2], ow[3]);
    } else {
      o = make_uint4(__float_as_uint(through(summed(__uint_as_float(a.x), __uint_as_float(c.x)), __uint_as_float(b.x))),
                     __float_as_uint(through(summed(__uint_as_float(a.y), __uint_as_float(c.y)), __uint_as_float(b.y))),
                     __float_as_uint(through(summed(__uint_as_float(a.z), __uint_as_float(c.z)), __uint_as_float(b.z))),
                     __float_as_uint(through(summed(__uint_as_float(a.w), __uint_as_float(c.w)), __uint_as_float(b.w))));
    }
    reinterpret_cast<uint4*>(dz)[i] = o;
  }
  for (size_t i = nvec * V + tid; i < count; i += stride)
    dz[i] = from_float<T>(through(summed(to_float(dy[i]), ADD ? to_float(add[i]) : 0.f), to_float(d[i])));
}

// Plain 16-byte-per-lane copy (activations handed to a stage that are not yet in its workspace).
__global__ __launch_bounds__(kThreads) void copy_kernel(size_t nvec, const uint4* __restrict__ src, uint4* __restrict__ dst,
                                                        size_t tail_bytes, const char* tsrc, char* tdst) {
  const size_t stride = (size_t)gridDim.x * kThreads;
  const size_t tid = (size_t)blockIdx.x * kThreads + threadIdx.x;
  for (size_t i = tid; i < nvec; i += stride) dst[i] = src[i];
  for (size_t i = tid; i < tail_bytes; i += stride) tdst[i] = tsrc[i];
}

// One wave per row.
template <typename T>
__global__ __launch_bounds__(kThreads) void softmax_ce_kernel(int rows, int classes, const T* __restrict__ logits,
                                                              const int32_t* __restrict__ labels,
                                                              T* __restrict__ dlogits, float* __restrict__ row_loss) {
  const int lane = threadIdx.x & 63;
  const int row = blockIdx.x * (kThreads / 64) + (threadIdx.x >> 6);
  if (row >= rows) return;
  const T* lg = logits + (size_t)row * classes;
  float mx = -INFINITY;
  for (int c = lane; c < classes; c += 64) mx = fmaxf(mx, to_float(lg[c]));
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off, 64));
  float sum = 0.f;
  for (int c = lane; c < classes; c += 64) sum += expf(to_float(lg[c]) - mx);
  sum = wave_sum(sum);
  const float lse = logf(sum);
  const int label = labels[row];
  const float inv_rows = 1.0f / (float)rows;
  T* dl = dlogits + (size_t)row * classes;
  for (int c = lane; c < classes; c += 64) {
    const float p = expf(to_float(lg[c]) - mx - lse);
    dl[c] = from_float<T>((p - (c == label ? 1.f : 0.f)) * inv_rows);
  }
  if (lane == 0) row_loss[row] = -(to_float(lg[label]) - mx - lse);
}

__global__ __launch_bounds__(kThreads) void mean_kernel(const float* __restrict__ v, int count, float* __restrict__ out) {
  __shared__ double sm[kThreads];
  double s = 0.0;
  for (int i = threadIdx.x; i < count; i += kThreads) s += (double)v[i];
  sm[threadIdx.x] = s;
  __syncthreads();
  for (int w = kThreads / 2; w > 0; w >>= 1) {
    if (threadIdx.x < w) sm[threadIdx.x] += sm[threadIdx.x + w];
    __syncthreads();
  }
  if (threadIdx.x == 0) *out = (float)(sm[0] / (double)count);
}

inline int stream_blocks(size_t work_items, int max_blocks) {
  size_t b = (work_items + kThreads - 1) / kThreads;
  if (b < 1) b = 1;
  return (int)(b < (size_t)max_blocks ? b : (size_t)max_blocks);
}

template <typename T>
hipError_t update_dispatch(hipStream_t s, const UpdateArgs& a) {
  const size_t n4 = a.count / 4;
  const int blocks = stream_blocks((n4 + kUnroll - 1) / kUnroll, kUpdateBlocks);
  const floatx4* g = (const floatx4*)a.g;
  floatx4* m = (floatx4*)a.m;
  const floatx4* wo = (const floatx4*)a.w_old;
  floatx4* wn = (floatx4*)a.w_new;
  const floatx4* ws = (const floatx4*)a.w_stale;
  T* wf = (T*)a.wfwd;
  T* wb = (T*)a.wb;
  const bool blend = a.w_stale != nullptr && a.wb != nullptr;
  const bool wfwd = a.wfwd != nullptr;
#define TP_LAUNCH_UPDATE(B, F) \
  hipLaunchKernelGGL((update_kernel<T, B, F>), dim3(blocks), dim3(kThreads), 0, s, n4, g, m, wo, wn, ws, wf, wb, a.lr, a.mu, a.alpha, a.beta, a.partials)
  if (blend && wfwd) TP_LAUNCH_UPDATE(true, true);
  else if (blend) TP_LAUNCH_UPDATE(true, false);
  else if (wfwd) TP_LAUNCH_UPDATE(false, true);
  else TP_LAUNCH_UPDATE(false, false);
#undef TP_LAUNCH_UPDATE
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(diag_reduce_kernel, dim3(1), dim3(kThreads), 0, s, a.partials, blocks, a.diag);
  return hipGetLastError();
}

}  // namespace

size_t update_scratch_floats() { return 4 * (size_t)kUpdateBlocks; }

namespace {
// Block partials of the update kernel's diagnostics for the entry point that takes no workspace from the
// caller and allocates nothing: 4 quantities x kUpdateBlocks floats (32 KiB), resident on every GPU the
// library runs on until the process ends.  In host code this name is only a handle for the symbol lookup
// below; kernels and copies get the device address that lookup returns.
static __device__ __align__(256) float scratch[4 * kUpdateBlocks];
constexpr int kMaxDevices = 64;
std::mutex scratch_mutex;
float* scratch_ptr[kMaxDevices] = {};  // per device: each GPU holds its own copy of the array at its own address
}  // namespace

hipError_t update_static_scratch(float** out, size_t* floats) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(scratch_mutex);
  if (!scratch_ptr[dev]) {
    float* p = nullptr;
    e = hipGetSymbolAddress((void**)&p, HIP_SYMBOL(scratch));  // looked up with `dev` current
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    scratch_ptr[dev] = p;
  }
  *out = scratch_ptr[dev];
  if (floats) *floats = 4 * (size_t)kUpdateBlocks;
  return hipSuccess;
}

hipError_t launch_update(hipStream_t s, int elt, const UpdateArgs& a) {
  if (a.count % 4 != 0) return hipErrorInvalidValue;
  return elt == ELT_BF16 ? update_dispatch<uint16_t>(s, a) : update_dispatch<float>(s, a);
}

hipError_t launch_blend(hipStream_t s, int elt, size_t count, const float* w_stale, const float* w_latest,
                        float alpha, float beta, void* wb) {
  if (count % 4 != 0) return hipErrorInvalidValue;
  const size_t n4 = count / 4;
  const int blocks = stream_blocks(n4, kUpdateBlocks);
  if (elt == ELT_BF16)
    hipLaunchKernelGGL(blend_kernel<uint16_t>, dim3(blocks), dim3(kThreads), 0, s, n4, (const float4*)w_stale,
                       (const float4*)w_latest, alpha, beta, (uint16_t*)wb);
  else
    hipLaunchKernelGGL(blend_kernel<float>, dim3(blocks), dim3(kThreads), 0, s, n4, (const float4*)w_stale,
                       (const float4*)w_latest, alpha, beta, (float*)wb);
  return hipGetLastError();
}

hipError_t launch_convert(hipStream_t s, int elt, size_t count, const float* src, void* dst) {
  if (count % 4 != 0) return hipErrorInvalidValue;
  const size_t n4 = count / 4;
  const int blocks = stream_blocks(n4, kUpdateBlocks);
  if (elt == ELT_BF16)
    hipLaunchKernelGGL(convert_kernel<uint16_t>, dim3(blocks), dim3(kThreads), 0, s, n4, (const float4*)src, (uint16_t*)dst);
  else
    hipLaunchKernelGGL(convert_kernel<float>, dim3(blocks), dim3(kThreads), 0, s, n4, (const float4*)src, (float*)dst);
  return hipGetLastError();
}

hipError_t launch_act_backward(hipStream_t s, int elt, size_t count, const void* dy, const void* d, void* dz, int relu_mask,
                               const void* add) {
  if ((((uintptr_t)dy | (uintptr_t)d | (uintptr_t)dz | (uintptr_t)add) & 15) != 0) return hipErrorInvalidValue;
  const int blocks = stream_blocks(count / 8 + 1, 4096);
#define TP_ACT_BWD(T, MASK, ADD)                                                                                        \
  hipLaunchKernelGGL((act_backward_kernel<T, MASK, ADD>), dim3(blocks), dim3(kThreads), 0, s, count, (const T*)dy, (const T*)d, \
                     (T*)dz, (const T*)add)
#define TP_ACT_BWD_T(T)                                   \
  do {                                                    \
    if (relu_mask) {                                      \
      if (add) TP_ACT_BWD(T, true, true); else TP_ACT_BWD(T, true, false);   \
    } else {                                              \
      if (add) TP_ACT_BWD(T, false, true); else TP_ACT_BWD(T, false, false); \
    }                                                     \
  } while (0)
  if (elt == ELT_BF16) TP_ACT_BWD_T(uint16_t); else TP_ACT_BWD_T(float);
#undef TP_ACT_BWD_T
#undef TP_ACT_BWD
  return hipGetLastError();
}

hipError_t launch_copy(hipStream_t s, const void* src, void* dst, size_t bytes) {
  if (((uintptr_t)src | (uintptr_t)dst) & 15) return hipMemcpyAsync(dst, src, bytes, hipMemcpyDeviceToDevice, s);
  const size_t nvec = bytes / 16, tail = bytes % 16;
  const int blocks = stream_blocks(nvec, 2048);
  hipLaunchKernelGGL(copy_kernel, dim3(blocks), dim3(kThreads), 0, s, nvec, (const uint4*)src, (uint4*)dst, tail,
                     (const char*)src + nvec * 16, (char*)dst + nvec * 16);
  return hipGetLastError();
}

hipError_t launch_softmax_ce(hipStream_t s, int elt, int rows, int classes, const void* logits, const int32_t* labels,
                             void* dlogits, float* row_loss, float* loss) {
  const int blocks = (rows + 3) / 4;
  if (elt == ELT_BF16)
    hipLaunchKernelGGL(softmax_ce_kernel<uint16_t>, dim3(blocks), dim3(kThreads), 0, s, rows, classes,
                       (const uint16_t*)logits, labels, (uint16_t*)dlogits, row_loss);
  else
    hipLaunchKernelGGL(softmax_ce_kernel<float>, dim3(blocks), dim3(kThreads), 0, s, rows, classes,
                       (const float*)logits, labels, (float*)dlogits, row_loss);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(mean_kernel, dim3(1), dim3(kThreads), 0, s, row_loss, rows, loss);
  return hipGetLastError();
}

}  // namespace tp
