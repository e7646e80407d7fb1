// Launch interface of the convolution, pooling and subsampling kernels (ksize x ksize with ksize 1, 3, 5 or 7,
// stride 1 or 2, pad (ksize-1)/2; 2x2 max pool; every second pixel; global average).  H, W are the INPUT image
// (even for stride 2); with stride s the output image is (H/s) x (W/s).  elt: 0 = fp32, 1 = bf16.  Activations are
// NHWC, [imgs*H*W x C] row-major; weights [Cout][ksize][ksize][Cin].  The matrix-core kernels take ksize 3 only.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace tp {

// the geometries the kernels take; the launchers return hipErrorInvalidValue for any other
bool conv_geometry_supported(int ksize, int stride, int pad);

// a = act(conv(x, W) + bias), d = act'(.) (d_out may be null).  Outputs [imgs*(H/stride)*(W/stride) x cout].
// zeros: device block of >= 128 zero bytes, 16-byte aligned (what padding positions read); the
// matrix-core kernels need it, null sends everything to the generic kernels.
hipError_t launch_conv_fprop(hipStream_t s, int elt, int imgs, int H, int W, int ksize, int stride, int cin, int cout,
                             const void* x, const void* wgt, const float* bias, int act, void* d_out, void* a_out,
                             const void* zeros);

// out = (transposed convolution of dz with W_b) (.) d_prev;  dz:[imgs*H*W x cout], out:[imgs*H*W x cin].
// relu_mask = 1: d_prev holds the previous layer's ReLU output and the factor is (output > 0).
hipError_t launch_conv_dgrad(hipStream_t s, int elt, int imgs, int H, int W, int ksize, int stride, int cin, int cout,
                             const void* dz, const void* wb, const void* d_prev, void* out, const void* zeros,
                             int relu_mask = 0);

// gW[cout][ksize][ksize][cin] (fp32) = sum over pixels of dz (x) shifted x.
// partial: scratch of conv_wgrad_scratch_floats(output pixels of the mini-batch, cin, cout, ksize) floats.
hipError_t launch_conv_wgrad(hipStream_t s, int elt, int imgs, int H, int W, int ksize, int stride, int cin, int cout,
                             const void* dz, const void* x, float* gW, float* partial, const void* zeros);
size_t conv_wgrad_scratch_floats(int pixels, int cin, int cout, int ksize);

// y[imgs x H/2 x W/2 x C] = 2x2/2 max pooling of x[imgs x H x W x C];  backward recomputes the
// position of the (first) maximum from the saved input x.
hipError_t launch_maxpool_fwd(hipStream_t s, int elt, int imgs, int H, int W, int C, const void* x, void* y);
// d_prev (may be null; only where maxpool_bwd_fuses_activation says so and all pointers are 16-byte aligned): the
// gradient also passes the activation in front of the pooling, dx (.)= d_prev (saved act'), or (relu_mask) the
// factor (d_prev > 0) of a saved ReLU output -- with the bits of the two separate kernels.
hipError_t launch_maxpool_bwd(hipStream_t s, int elt, int imgs, int H, int W, int C, const void* x, const void* dy,
                              void* dx, const void* d_prev = nullptr, int relu_mask = 0);
bool maxpool_bwd_fuses_activation(int elt, int C);

// y[imgs x H/2 x W/2 x C] = x at the even pixel positions; backward: the gradient at those positions, zero elsewhere.
// C * element size must be a multiple of 16 bytes.
hipError_t launch_subsample_fwd(hipStream_t s, int elt, int imgs, int H, int W, int C, const void* x, void* y);
hipError_t launch_subsample_bwd(hipStream_t s, int elt, int imgs, int H, int W, int C, const void* dy, void* dx);

// y[imgs x C] = mean over the positions of x[imgs x positions x C]; backward: dx = dy / positions at every position.
hipError_t launch_avgpool_fwd(hipStream_t s, int elt, int imgs, int positions, int C, const void* x, void* y);
hipError_t launch_avgpool_bwd(hipStream_t s, int elt, int imgs, int positions, int C, const void* dy, void* dx);

// bf16 matrix-core versions (kernels_conv_mfma.hip) and the shapes they take
bool conv_mfma_supported(int imgs, int H, int W, int stride, int cin, int cout);
int conv_mfma_wgrad_splits(int pixels, int cin, int cout);
int conv_mfma_wgrad_max_splits(int pixels, int cin, int cout);
hipError_t conv_mfma_fprop(hipStream_t s, int imgs, int H, int W, int stride, int cin, int cout, const uint16_t* x,
                           const uint16_t* wgt, const float* bias, int act, uint16_t* d_out, uint16_t* a_out,
                           const uint16_t* zeros);
hipError_t conv_mfma_dgrad(hipStream_t s, int imgs, int H, int W, int stride, int cin, int cout, const uint16_t* dz,
                           const uint16_t* wb, const uint16_t* d_prev, uint16_t* out, const uint16_t* zeros, int relu_mask = 0);
hipError_t conv_mfma_wgrad(hipStream_t s, int imgs, int H, int W, int stride, int cin, int cout, const uint16_t* dz,
                           const uint16_t* x, float* gW, float* partial, const uint16_t* zeros);

// First layer of an image net (cin <= 8, bf16) on a zero-padded [pixel][8 channels] copy x8 of its input.
bool conv_c8_supported(int imgs, int H, int W, int cin, int cout);
hipError_t conv_c8_pad(hipStream_t s, size_t pixels, int cin, const uint16_t* x, uint16_t* x8);
hipError_t conv_c8_fprop(hipStream_t s, int imgs, int H, int W, int cin, int cout, const uint16_t* x8, const uint16_t* wgt,
                         const float* bias, int act, uint16_t* d_out, uint16_t* a_out, const uint16_t* zeros);
hipError_t conv_c8_wgrad(hipStream_t s, int imgs, int H, int W, int cin, int cout, const uint16_t* dz, const uint16_t* x8,
                         float* gW, float* partial, const uint16_t* zeros);

// The 7x7 stride-2 pad-3 first layer (cin <= 8, bf16) on the same padded copy; H, W: the input image.
bool conv_stem_supported(int imgs, int H, int W, int cin, int cout);
int conv_stem_wgrad_splits(int out_pixels, int cout);
hipError_t conv_stem_fprop(hipStream_t s, int imgs, int H, int W, int cin, int cout, const uint16_t* x8, const uint16_t* wgt,
                           const float* bias, int act, uint16_t* d_out, uint16_t* a_out, const uint16_t* zeros);
hipError_t conv_stem_wgrad(hipStream_t s, int imgs, int H, int W, int cin, int cout, const uint16_t* dz, const uint16_t* x8,
                           float* gW, float* partial, const uint16_t* zeros);

}  // namespace tp
