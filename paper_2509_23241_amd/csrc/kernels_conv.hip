// R x R convolution (R odd, stride 1 or 2, zero padding (R-1)/2) on NHWC activations as implicit GEMMs, 2x2 max
// pooling, 2x subsampling and global average pooling.  Weights are [Cout][R][R][Cin], i.e. a row-major
// [Cout x R*R*Cin] matrix whose k index runs over (tap, input channel), tap = R*kh + kw.
//
//   fprop  z[p][co]  = sum_{tap,ci} x[shift(p,+tap)][ci] * W[co][tap][ci]        rows: output pixels
//   dgrad  dx[p][ci] = sum_{tap,co} dz[shift(p,-tap)][co] * W_b[co][tap][ci]     rows: input pixels
//   wgrad  dW[co][tap][ci] = sum_p dz[p][co] * x[shift(p,+tap)][ci]              contraction: pixels
// shift(p, +tap) moves pixel p = (img, h, w) by (kh-pad, kw-pad); positions outside the image read 0.
// With stride s the output has (H/s) x (W/s) pixels and output pixel (oh, ow) reads the input at
// (s*oh + kh - pad, s*ow + kw - pad); dgrad visits, for an input pixel, the taps whose output position
// (h - kh + pad) / s, (w - kw + pad) / s is whole.
//
// This file holds the shape-generic, bounds-checked SIMT kernel (fp32 FMA, LDS-tiled), used for
// the fp32 mode, for kernel sizes and channel counts the matrix-core kernels do not take and as their reference.  wgrad contracts over all pixels of the mini-batch, so it is
// split over pixel ranges; a second kernel adds the partial results in a fixed order.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <algorithm>

#include "conv.h"
#include "kernels.h"
#include "device_utils.h"

namespace tp {

namespace {

constexpr int BM = 64, BN = 64, BK = 16, kThreads = 256;

struct ConvGeom {
  int imgs, H, W, Cin, Cout;  // H, W: input image
  int S, Ho, Wo;              // stride, output image
  int R, Pd;                  // kernel edge, zero padding on every side
};

__device__ __forceinline__ void pixel_of(int p, int H, int W, int& img, int& h, int& w) {
  w = p % W;
  const int t = p / W;
  h = t % H;
  img = t / H;
}

// PRODUCT: 0 fprop, 1 dgrad, 2 wgrad (partial sums over the pixel range of blockIdx.z)
template <typename T, int PRODUCT>
__global__ __launch_bounds__(kThreads) void conv_simt_kernel(ConvGeom g, const T* __restrict__ act_in,
                                                             const T* __restrict__ wgt_or_dz, const float* __restrict__ bias,
                                                             int act, const T* __restrict__ d_prev, T* __restrict__ d_out,
                                                             T* __restrict__ out, float* __restrict__ partial,
                                                             int pixels_per_split, int relu_mask) {
  __shared__ float As[BK][BM + 4];
  __shared__ float Bs[BK][BN + 4];
  const int Pin = g.imgs * g.H * g.W, Pout = g.imgs * g.Ho * g.Wo;
  const int M = PRODUCT == 0 ? Pout : (PRODUCT == 1 ? Pin : g.Cout);
  const int KK = g.R * g.R;
  const int N = PRODUCT == 0 ? g.Cout : (PRODUCT == 1 ? g.Cin : KK * g.Cin);
  const int Kfull = PRODUCT == 0 ? KK * g.Cin : (PRODUCT == 1 ? KK * g.Cout : Pout);
  const int kbeg = PRODUCT == 2 ? blockIdx.z * pixels_per_split : 0;
  const int kend = PRODUCT == 2 ? min(Pout, kbeg + pixels_per_split) : Kfull;
  const int t = threadIdx.x, tx = t & 15, ty = t >> 4;
  const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;

  // A(m, k) and B(k, n) of the three products
  auto fetch_a = [&](int m, int k) -> float {
    if (m >= M || k >= kend) return 0.f;
    if (PRODUCT == 2) return to_float(wgt_or_dz[(size_t)k * g.Cout + m]);  // dz[p][co]
    const int C = PRODUCT == 0 ? g.Cin : g.Cout;
    const int tap = k / C, c = k % C;
    const int dh = tap / g.R - g.Pd, dw = tap % g.R - g.Pd;
    int img, h, w;
    if (PRODUCT == 0) {  // output pixel m reads the input
      pixel_of(m, g.Ho, g.Wo, img, h, w);
      const int sh = h * g.S + dh, sw = w * g.S + dw;
      if (sh < 0 || sh >= g.H || sw < 0 || sw >= g.W) return 0.f;
      return to_float(act_in[((size_t)(img * g.H + sh) * g.W + sw) * C + c]);
    }
    pixel_of(m, g.H, g.W, img, h, w);  // input pixel m reads dz where the tap lands on a whole output position
    const int nh = h - dh, nw = w - dw;
    if (nh < 0 || nw < 0 || nh % g.S || nw % g.S) return 0.f;
    const int oh = nh / g.S, ow = nw / g.S;
    if (oh >= g.Ho || ow >= g.Wo) return 0.f;
    return to_float(act_in[((size_t)(img * g.Ho + oh) * g.Wo + ow) * C + c]);
  };
  auto fetch_b = [&](int k, int n) -> float {
    if (n >= N || k >= kend) return 0.f;
    if (PRODUCT == 0) return to_float(wgt_or_dz[(size_t)n * (KK * g.Cin) + k]);  // W[co][k]
    if (PRODUCT == 1) {
      const int tap = k / g.Cout, co = k % g.Cout;
      return to_float(wgt_or_dz[(size_t)co * (KK * g.Cin) + tap * g.Cin + n]);  // W_b[co][tap][ci]
    }
    const int tap = n / g.Cin, c = n % g.Cin;
    int img, h, w;
    pixel_of(k, g.Ho, g.Wo, img, h, w);
    const int sh = h * g.S + tap / g.R - g.Pd, sw = w * g.S + tap % g.R - g.Pd;
    if (sh < 0 || sh >= g.H || sw < 0 || sw >= g.W) return 0.f;
    return to_float(act_in[((size_t)(img * g.H + sh) * g.W + sw) * g.Cin + c]);
  };

  float acc[4][4] = {};
  for (int k0 = kbeg; k0 < kend; k0 += BK) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int el = t + i * kThreads;
      // thread -> element so that consecutive threads read consecutive addresses of each operand
      int am, ak, bn, bk;
      if (PRODUCT == 2) { am = el & (BM - 1); ak = el >> 6; } else { ak = el & (BK - 1); am = el >> 4; }
      if (PRODUCT == 0) { bk = el & (BK - 1); bn = el >> 4; } else { bn = el & (BN - 1); bk = el >> 6; }
      As[ak][am] = fetch_a(m0 + am, k0 + ak);
      Bs[bk][bn] = fetch_b(k0 + bk, n0 + bn);
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < BK; ++k) {
      const float4 a = *reinterpret_cast<const float4*>(&As[k][ty * 4]);
      const float4 b = *reinterpret_cast<const float4*>(&Bs[k][tx * 4]);
      const float av[4] = {a.x, a.y, a.z, a.w}, bv[4] = {b.x, b.y, b.z, b.w};
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
      if (PRODUCT == 0) {
        v += bias[n];
        if (d_out) d_out[idx] = from_float<T>(act_derivative(v, act));
        out[idx] = from_float<T>(act_forward(v, act));
      } else if (PRODUCT == 1) {
        if (d_prev) {  // relu_mask: d_prev holds the previous layer's ReLU output, the factor is (output > 0)
          const float dp = to_float(d_prev[idx]);
          v = relu_mask ? (dp > 0.f ? v : 0.f) : v * dp;
        }
        out[idx] = from_float<T>(v);
      } else {
        partial[(size_t)blockIdx.z * M * N + idx] = v;
      }
    }
  }
}

// 2x2 max pooling, stride 2, NHWC; first maximum in row-major window order wins ties.
template <typename T>
__global__ __launch_bounds__(kThreads) void maxpool_fwd_kernel(int imgs, int H, int W, int C, const T* __restrict__ x,
                                                               T* __restrict__ y) {
  const size_t total = (size_t)imgs * (H / 2) * (W / 2) * C;
  for (size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x; i < total; i += (size_t)gridDim.x * kThreads) {
    const int c = i % C;
    size_t t = i / C;
    const int ow = t % (W / 2);
    t /= (W / 2);
    const int oh = t % (H / 2);
    const int img = t / (H / 2);
    const T* p = x + (((size_t)img * H + 2 * oh) * W + 2 * ow) * C + c;
    float m = to_float(p[0]);
    m = fmaxf(m, to_float(p[C]));
    m = fmaxf(m, to_float(p[(size_t)W * C]));
    m = fmaxf(m, to_float(p[(size_t)W * C + C]));
    y[i] = from_float<T>(m);
  }
}

template <typename T>
__global__ __launch_bounds__(kThreads) void maxpool_bwd_kernel(int imgs, int H, int W, int C, const T* __restrict__ x,
                                                               const T* __restrict__ dy, T* __restrict__ dx) {
  const size_t total = (size_t)imgs * (H / 2) * (W / 2) * C;
  for (size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x; i < total; i += (size_t)gridDim.x * kThreads) {
    const int c = i % C;
    size_t t = i / C;
    const int ow = t % (W / 2);
    t /= (W / 2);
    const int oh = t % (H / 2);
    const int img = t / (H / 2);
    const size_t base = (((size_t)img * H + 2 * oh) * W + 2 * ow) * C + c;
    const size_t off[4] = {0, (size_t)C, (size_t)W * C, (size_t)W * C + C};
    float best = to_float(x[base]);
    int arg = 0;
#pragma unroll
    for (int q = 1; q < 4; ++q) {
      const float v = to_float(x[base + off[q]]);
      if (v > best) { best = v; arg = q; }
    }
    const T g = dy[i], zero = from_float<T>(0.f);
#pragma unroll
    for (int q = 0; q < 4; ++q) dx[base + off[q]] = q == arg ? g : zero;
  }
}

// The same for bf16 with C % 8 == 0: a lane takes 8 neighbouring channels (16 bytes) of one window.
__device__ __forceinline__ void unpack_bf16x8(const uint4& u, float (&f)[8]) {
  const uint32_t w[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    f[2 * j] = __uint_as_float(w[j] << 16);
    f[2 * j + 1] = __uint_as_float(w[j] & 0xffff0000u);
  }
}
__device__ __forceinline__ uint4 pack_bf16x8(const float (&f)[8]) {
  return make_uint4(pack_bf16x2(f[0], f[1]), pack_bf16x2(f[2], f[3]), pack_bf16x2(f[4], f[5]), pack_bf16x2(f[6], f[7]));
}

__global__ __launch_bounds__(kThreads) void maxpool_fwd_vec_kernel(int imgs, int H, int W, int CV, const uint4* __restrict__ x,
                                                                   uint4* __restrict__ y) {
  const size_t total = (size_t)imgs * (H / 2) * (W / 2) * CV;
  for (size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x; i < total; i += (size_t)gridDim.x * kThreads) {
    const int c = i % CV;
    size_t t = i / CV;
    const int ow = t % (W / 2);
    t /= (W / 2);
    const int oh = t % (H / 2);
    const size_t img = t / (H / 2);
    const uint4* p = x + ((img * H + 2 * oh) * W + 2 * ow) * CV + c;
    float m[8], v[8];
    unpack_bf16x8(p[0], m);
    const size_t off[3] = {(size_t)CV, (size_t)W * CV, (size_t)W * CV + CV};
#pragma unroll
    for (int q = 0; q < 3; ++q) {
      unpack_bf16x8(p[off[q]], v);
#pragma unroll
      for (int j = 0; j < 8; ++j) m[j] = fmaxf(m[j], v[j]);
    }
    y[i] = pack_bf16x8(m);  // bf16 values: packing is exact
  }
}

// FUSE: the gradient also passes the activation in front of the pooling: dx = (gradient at the maximum) (.) d, with
// d the saved act' tensor at the pooling input's positions, or (MASK) the factor (d > 0) of a saved ReLU output.
template <bool FUSE, bool MASK>
__global__ __launch_bounds__(kThreads) void maxpool_bwd_vec_kernel(int imgs, int H, int W, int CV, const uint4* __restrict__ x,
                                                                   const uint4* __restrict__ dy, const uint4* d,
                                                                   uint4* __restrict__ dx) {
  const size_t total = (size_t)imgs * (H / 2) * (W / 2) * CV;
  for (size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x; i < total; i += (size_t)gridDim.x * kThreads) {
    const int c = i % CV;
    size_t t = i / CV;
    const int ow = t % (W / 2);
    t /= (W / 2);
    const int oh = t % (H / 2);
    const size_t img = t / (H / 2);
    const size_t base = ((img * H + 2 * oh) * W + 2 * ow) * CV + c;
    const size_t off[4] = {0, (size_t)CV, (size_t)W * CV, (size_t)W * CV + CV};
    float xv[4][8], g[8], o[4][8];
#pragma unroll
    for (int q = 0; q < 4; ++q) unpack_bf16x8(x[base + off[q]], xv[q]);
    unpack_bf16x8(dy[i], g);
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      float best = xv[0][j];
      int arg = 0;
#pragma unroll
      for (int q = 1; q < 4; ++q)
        if (xv[q][j] > best) { best = xv[q][j]; arg = q; }
#pragma unroll
      for (int q = 0; q < 4; ++q) o[q][j] = q == arg ? g[j] : 0.f;
    }
    if constexpr (FUSE) {
      const bool same = d == x;  // a ReLU output that is this layer's own saved input
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        float dv[8];
        if (same) {
#pragma unroll
          for (int j = 0; j < 8; ++j) dv[j] = xv[q][j];
        } else {
          unpack_bf16x8(d[base + off[q]], dv);
        }
#pragma unroll
        for (int j = 0; j < 8; ++j) o[q][j] = MASK ? (dv[j] > 0.f ? o[q][j] : 0.f) : o[q][j] * dv[j];
      }
    }
#pragma unroll
    for (int q = 0; q < 4; ++q) dx[base + off[q]] = pack_bf16x8(o[q]);
  }
}

// y[img][oh][ow][:] = x[img][2*oh][2*ow][:] in 16-byte units (CV per pixel); the backward pass writes the
// gradient back to those positions and zero everywhere else.
__global__ __launch_bounds__(kThreads) void subsample_fwd_kernel(int imgs, int H, int W, int CV, const uint4* __restrict__ x,
                                                                 uint4* __restrict__ y) {
  const size_t total = (size_t)imgs * (H / 2) * (W / 2) * CV;
  for (size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x; i < total; i += (size_t)gridDim.x * kThreads) {
    const int c = i % CV;
    size_t t = i / CV;
    const int ow = t % (W / 2);
    t /= (W / 2);
    const int oh = t % (H / 2);
    const size_t img = t / (H / 2);
    y[i] = x[((img * H + 2 * oh) * W + 2 * ow) * CV + c];
  }
}

__global__ __launch_bounds__(kThreads) void subsample_bwd_kernel(int imgs, int H, int W, int CV, const uint4* __restrict__ dy,
                                                                 uint4* __restrict__ dx) {
  const size_t total = (size_t)imgs * H * W * CV;
  for (size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x; i < total; i += (size_t)gridDim.x * kThreads) {
    const int c = i % CV;
    size_t t = i / CV;
    const int w = t % W;
    t /= W;
    const int h = t % H;
    const size_t img = t / H;
    uint4 v = make_uint4(0, 0, 0, 0);
    if (!(h & 1) && !(w & 1)) v = dy[((img * (H / 2) + h / 2) * (W / 2) + w / 2) * CV + c];
    dx[i] = v;
  }
}

// Global average pooling: y[img][c] = mean over the positions of x[img][p][c], summed in position order in fp32;
// backward: every position gets dy[img][c] / positions.
template <typename T>
__global__ __launch_bounds__(kThreads) void avgpool_fwd_kernel(int imgs, int positions, int C, const T* __restrict__ x,
                                                               T* __restrict__ y) {
  const size_t total = (size_t)imgs * C;
  for (size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x; i < total; i += (size_t)gridDim.x * kThreads) {
    const size_t img = i / C;
    const int c = (int)(i - img * C);
    const T* p = x + img * positions * C + c;
    float sum = 0.f;
    for (int q = 0; q < positions; ++q) sum += to_float(p[(size_t)q * C]);
    y[i] = from_float<T>(sum / (float)positions);
  }
}

template <typename T>
__global__ __launch_bounds__(kThreads) void avgpool_bwd_kernel(int imgs, int positions, int C, const T* __restrict__ dy,
                                                               T* __restrict__ dx) {
  const size_t total = (size_t)imgs * positions * C;
  const size_t per_img = (size_t)positions * C;
  for (size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x; i < total; i += (size_t)gridDim.x * kThreads) {
    const size_t img = i / per_img;
    const int c = (int)(i % C);
    dx[i] = from_float<T>(to_float(dy[img * C + c]) / (float)positions);
  }
}

inline int stream_blocks(size_t items, int max_blocks) {
  size_t b = (items + kThreads - 1) / kThreads;
  return (int)(b < 1 ? 1 : (b < (size_t)max_blocks ? b : (size_t)max_blocks));
}

}  // namespace

int conv_wgrad_splits(int pixels, int cin, int cout, int ksize) {
  // enough pixel ranges to put ~1024 workgroups on the chip even when dW has only a handful of
  // tiles (the 3-channel first layer has one), at least 256 pixels each
  const int tiles = ((ksize * ksize * cin + BN - 1) / BN) * ((cout + BM - 1) / BM);
  int s = std::min((1024 + tiles - 1) / tiles, (pixels + 255) / 256);
  return s < 1 ? 1 : (s > 1024 ? 1024 : s);
}

size_t conv_wgrad_scratch_floats(int pixels, int cin, int cout, int ksize) {
  int splits = conv_wgrad_splits(pixels, cin, cout, ksize);
  if (ksize == 3) splits = std::max(splits, conv_mfma_wgrad_max_splits(pixels, cin, cout));
  if (ksize == 7 && cin <= 8 && cout % 64 == 0) splits = std::max(splits, conv_stem_wgrad_splits(pixels, cout));
  return (size_t)splits * cout * ksize * ksize * cin;
}

bool conv_geometry_supported(int ksize, int stride, int pad) {
  return (ksize == 1 || ksize == 3 || ksize == 5 || ksize == 7) && (stride == 1 || stride == 2) && pad == (ksize - 1) / 2;
}

hipError_t launch_conv_fprop(hipStream_t s, int elt, int imgs, int H, int W, int ksize, int stride, int cin, int cout,
                             const void* x, const void* wgt, const float* bias, int act, void* d_out, void* a_out,
                             const void* zeros) {
  if (!conv_geometry_supported(ksize, stride, (ksize - 1) / 2) || (stride == 2 && ((H | W) & 1))) return hipErrorInvalidValue;
  if (ksize == 3 && elt == 1 && zeros && conv_mfma_supported(imgs, H, W, stride, cin, cout))
    return conv_mfma_fprop(s, imgs, H, W, stride, cin, cout, (const uint16_t*)x, (const uint16_t*)wgt, bias, act,
                           (uint16_t*)d_out, (uint16_t*)a_out, (const uint16_t*)zeros);
  const ConvGeom g{imgs, H, W, cin, cout, stride, H / stride, W / stride, ksize, (ksize - 1) / 2};
  const int P = imgs * g.Ho * g.Wo;
  dim3 grid((cout + BN - 1) / BN, (P + BM - 1) / BM);
  if (elt == 1)
    hipLaunchKernelGGL((conv_simt_kernel<uint16_t, 0>), grid, dim3(kThreads), 0, s, g, (const uint16_t*)x, (const uint16_t*)wgt,
                       bias, act, (const uint16_t*)nullptr, (uint16_t*)d_out, (uint16_t*)a_out, (float*)nullptr, 0, 0);
  else
    hipLaunchKernelGGL((conv_simt_kernel<float, 0>), grid, dim3(kThreads), 0, s, g, (const float*)x, (const float*)wgt, bias,
                       act, (const float*)nullptr, (float*)d_out, (float*)a_out, (float*)nullptr, 0, 0);
  return hipGetLastError();
}

hipError_t launch_conv_dgrad(hipStream_t s, int elt, int imgs, int H, int W, int ksize, int stride, int cin, int cout,
                             const void* dz, const void* wb, const void* d_prev, void* out, const void* zeros,
                             int relu_mask) {
  if (!conv_geometry_supported(ksize, stride, (ksize - 1) / 2) || (stride == 2 && ((H | W) & 1))) return hipErrorInvalidValue;
  if (ksize == 3 && elt == 1 && zeros && conv_mfma_supported(imgs, H, W, stride, cin, cout))
    return conv_mfma_dgrad(s, imgs, H, W, stride, cin, cout, (const uint16_t*)dz, (const uint16_t*)wb,
                           (const uint16_t*)d_prev, (uint16_t*)out, (const uint16_t*)zeros, relu_mask);
  const ConvGeom g{imgs, H, W, cin, cout, stride, H / stride, W / stride, ksize, (ksize - 1) / 2};
  const int P = imgs * H * W;
  dim3 grid((cin + BN - 1) / BN, (P + BM - 1) / BM);
  if (elt == 1)
    hipLaunchKernelGGL((conv_simt_kernel<uint16_t, 1>), grid, dim3(kThreads), 0, s, g, (const uint16_t*)dz, (const uint16_t*)wb,
                       (const float*)nullptr, 0, (const uint16_t*)d_prev, (uint16_t*)nullptr, (uint16_t*)out, (float*)nullptr, 0, relu_mask);
  else
    hipLaunchKernelGGL((conv_simt_kernel<float, 1>), grid, dim3(kThreads), 0, s, g, (const float*)dz, (const float*)wb,
                       (const float*)nullptr, 0, (const float*)d_prev, (float*)nullptr, (float*)out, (float*)nullptr, 0, relu_mask);
  return hipGetLastError();
}

hipError_t launch_conv_wgrad(hipStream_t s, int elt, int imgs, int H, int W, int ksize, int stride, int cin, int cout,
                             const void* dz, const void* x, float* gW, float* partial, const void* zeros) {
  if (!conv_geometry_supported(ksize, stride, (ksize - 1) / 2) || (stride == 2 && ((H | W) & 1))) return hipErrorInvalidValue;
  if (ksize == 3 && elt == 1 && zeros && conv_mfma_supported(imgs, H, W, stride, cin, cout))
    return conv_mfma_wgrad(s, imgs, H, W, stride, cin, cout, (const uint16_t*)dz, (const uint16_t*)x, gW, partial,
                           (const uint16_t*)zeros);
  const ConvGeom g{imgs, H, W, cin, cout, stride, H / stride, W / stride, ksize, (ksize - 1) / 2};
  const int P = imgs * g.Ho * g.Wo;  // the contraction runs over output pixels
  const int splits = conv_wgrad_splits(P, cin, cout, ksize);
  const int per = ((P + splits - 1) / splits + BK - 1) / BK * BK;
  dim3 grid((ksize * ksize * cin + BN - 1) / BN, (cout + BM - 1) / BM, splits);
  if (elt == 1)
    hipLaunchKernelGGL((conv_simt_kernel<uint16_t, 2>), grid, dim3(kThreads), 0, s, g, (const uint16_t*)x, (const uint16_t*)dz,
                       (const float*)nullptr, 0, (const uint16_t*)nullptr, (uint16_t*)nullptr, (uint16_t*)nullptr, partial, per, 0);
  else
    hipLaunchKernelGGL((conv_simt_kernel<float, 2>), grid, dim3(kThreads), 0, s, g, (const float*)x, (const float*)dz,
                       (const float*)nullptr, 0, (const float*)nullptr, (float*)nullptr, (float*)nullptr, partial, per, 0);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  const size_t count = (size_t)cout * ksize * ksize * cin;
  return launch_sum_partials(s, count, splits, partial, gW);
}

hipError_t launch_subsample_fwd(hipStream_t s, int elt, int imgs, int H, int W, int C, const void* x, void* y) {
  const int es = elt == 1 ? 2 : 4;
  if ((C * es) % 16 || (H & 1) || (W & 1)) return hipErrorInvalidValue;
  const int CV = C * es / 16;
  const int blocks = stream_blocks((size_t)imgs * (H / 2) * (W / 2) * CV, 8192);
  hipLaunchKernelGGL(subsample_fwd_kernel, dim3(blocks), dim3(kThreads), 0, s, imgs, H, W, CV, (const uint4*)x, (uint4*)y);
  return hipGetLastError();
}

hipError_t launch_subsample_bwd(hipStream_t s, int elt, int imgs, int H, int W, int C, const void* dy, void* dx) {
  const int es = elt == 1 ? 2 : 4;
  if ((C * es) % 16 || (H & 1) || (W & 1)) return hipErrorInvalidValue;
  const int CV = C * es / 16;
  const int blocks = stream_blocks((size_t)imgs * H * W * CV, 8192);
  hipLaunchKernelGGL(subsample_bwd_kernel, dim3(blocks), dim3(kThreads), 0, s, imgs, H, W, CV, (const uint4*)dy, (uint4*)dx);
  return hipGetLastError();
}

hipError_t launch_avgpool_fwd(hipStream_t s, int elt, int imgs, int positions, int C, const void* x, void* y) {
  if (imgs < 1 || positions < 1 || C < 1) return hipErrorInvalidValue;
  const int blocks = stream_blocks((size_t)imgs * C, 8192);
  if (elt == 1)
    hipLaunchKernelGGL(avgpool_fwd_kernel<uint16_t>, dim3(blocks), dim3(kThreads), 0, s, imgs, positions, C, (const uint16_t*)x,
                       (uint16_t*)y);
  else
    hipLaunchKernelGGL(avgpool_fwd_kernel<float>, dim3(blocks), dim3(kThreads), 0, s, imgs, positions, C, (const float*)x, (float*)y);
  return hipGetLastError();
}

hipError_t launch_avgpool_bwd(hipStream_t s, int elt, int imgs, int positions, int C, const void* dy, void* dx) {
  if (imgs < 1 || positions < 1 || C < 1) return hipErrorInvalidValue;
  const int blocks = stream_blocks((size_t)imgs * positions * C, 8192);
  if (elt == 1)
    hipLaunchKernelGGL(avgpool_bwd_kernel<uint16_t>, dim3(blocks), dim3(kThreads), 0, s, imgs, positions, C, (const uint16_t*)dy,
                       (uint16_t*)dx);
  else
    hipLaunchKernelGGL(avgpool_bwd_kernel<float>, dim3(blocks), dim3(kThreads), 0, s, imgs, positions, C, (const float*)dy, (float*)dx);
  return hipGetLastError();
}

inline bool pool_vec_ok(int elt, int C, const void* a, const void* b, const void* c, const void* d) {
  return elt == 1 && C % 8 == 0 && ((((uintptr_t)a | (uintptr_t)b | (uintptr_t)c | (uintptr_t)d) & 15) == 0);
}

hipError_t launch_maxpool_fwd(hipStream_t s, int elt, int imgs, int H, int W, int C, const void* x, void* y) {
  const size_t total = (size_t)imgs * (H / 2) * (W / 2) * C;
  if (pool_vec_ok(elt, C, x, y, nullptr, nullptr)) {
    hipLaunchKernelGGL(maxpool_fwd_vec_kernel, dim3(stream_blocks(total / 8, 8192)), dim3(kThreads), 0, s, imgs, H, W, C / 8,
                       (const uint4*)x, (uint4*)y);
    return hipGetLastError();
  }
  const int blocks = stream_blocks(total, 8192);
  if (elt == 1)
    hipLaunchKernelGGL(maxpool_fwd_kernel<uint16_t>, dim3(blocks), dim3(kThreads), 0, s, imgs, H, W, C, (const uint16_t*)x, (uint16_t*)y);
  else
    hipLaunchKernelGGL(maxpool_fwd_kernel<float>, dim3(blocks), dim3(kThreads), 0, s, imgs, H, W, C, (const float*)x, (float*)y);
  return hipGetLastError();
}

bool maxpool_bwd_fuses_activation(int elt, int C) { return elt == 1 && C % 8 == 0; }

hipError_t launch_maxpool_bwd(hipStream_t s, int elt, int imgs, int H, int W, int C, const void* x, const void* dy,
                              void* dx, const void* d_prev, int relu_mask) {
  const size_t total = (size_t)imgs * (H / 2) * (W / 2) * C;
  if (pool_vec_ok(elt, C, x, dy, dx, d_prev)) {
    const dim3 grid(stream_blocks(total / 8, 8192));
#define TP_POOL_BWD(FUSE, MASK)                                                                                          \
  hipLaunchKernelGGL((maxpool_bwd_vec_kernel<FUSE, MASK>), grid, dim3(kThreads), 0, s, imgs, H, W, C / 8, (const uint4*)x, \
                     (const uint4*)dy, (const uint4*)d_prev, (uint4*)dx)
    if (!d_prev) TP_POOL_BWD(false, false);
    else if (relu_mask) TP_POOL_BWD(true, true);
    else TP_POOL_BWD(true, false);
#undef TP_POOL_BWD
    return hipGetLastError();
  }
  if (d_prev) return hipErrorNotSupported;  // the caller asks maxpool_bwd_fuses_activation first
  const int blocks = stream_blocks(total, 8192);
  if (elt == 1)
    hipLaunchKernelGGL(maxpool_bwd_kernel<uint16_t>, dim3(blocks), dim3(kThreads), 0, s, imgs, H, W, C, (const uint16_t*)x,
                       (const uint16_t*)dy, (uint16_t*)dx);
  else
    hipLaunchKernelGGL(maxpool_bwd_kernel<float>, dim3(blocks), dim3(kThreads), 0, s, imgs, H, W, C, (const float*)x,
                       (const float*)dy, (float*)dx);
  return hipGetLastError();
}

}  // namespace tp
