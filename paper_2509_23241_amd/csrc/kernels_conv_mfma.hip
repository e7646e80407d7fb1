// 3x3 convolutions (stride 1, pad 1, NHWC) on the gfx950 matrix cores as implicit GEMMs.
//
// The three products use the direct-to-LDS pipeline of the dense GEMMs (global_load_lds_dwordx4
// into XOR-swizzled LDS stages, copies interleaved with the MFMAs, fragments prefetched one k
// step ahead); what changes is where each lane's 16 bytes come from.  A k tile is 64 values of
// the contraction index:
//   fprop  rows = output pixels, k = (tap, 64 input channels):  A gathers x at the pixel shifted by
//          the tap (or a block of zeros outside the image), B = W[Cout][9*Cin] as it lies.
//   dgrad  rows = input pixels,  k = (tap, 64 output channels): A gathers dz at the pixel shifted
//          the other way, B = the [64 co][Cin] block of W_b for that tap (rows 9*Cin apart).
//   wgrad  rows = output channels, columns = input channels of ONE tap, k = 64 pixels: A = dz as it
//          lies, B gathers x at the shifted pixels.  One workgroup handles one tap, one range of
//          pixel tiles and one tile of dW[:, tap, :]; partial sums over the pixel ranges are
//          added by a second kernel in a fixed order.
// Needs: image height and width powers of two (pixel -> (h, w) by shift and mask), channel counts
// that are multiples of 64, pixel count a multiple of 64.  Everything else goes to the generic
// kernels of kernels_conv.hip.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <algorithm>

#include "conv.h"
#include "device_utils.h"
#include "mfma_common.h"

namespace tp {

namespace {

// 16-byte copy global -> LDS with a full 64-bit address per lane
__device__ __forceinline__ void dma16_addr(uint32_t lds_byte_addr, const void* lane_ptr) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off"
               :
               : "s"(lds_byte_addr), "v"(lane_ptr)
               : "memory");
}

struct GatherDesc {
  const uint16_t* base;   // [P][C] activations or gradients
  const uint16_t* zeros;  // >= 128 bytes of zeros, 16-byte aligned
  int P, H, W, lw;        // pixels, image size, log2(W)
  int C;                  // channels of `base`
};

// k-contiguous gathered operand: stage [R pixels][64 channels of one tap].
template <int R, int NW, bool BACKWARD>
struct RowGather {
  using Desc = GatherDesc;
  static constexpr int kPerWave = R / 8 / NW;
  static constexpr int kBytes = R * DBK * 2;
  static_assert((R / 8) % NW == 0, "rows do not divide among the waves");
  Desc d;
  int cblocks;
  uint32_t pix_off[kPerWave];  // byte offset of (pixel, chunk) inside base
  int hw[kPerWave];            // h << 16 | w of the lane's pixel
  uint32_t zoff;

  __device__ __forceinline__ void init(const Desc& desc, int r0, int wave, int lane, int /*batch*/) {
    d = desc;
    cblocks = d.C / DBK;
    zoff = (lane & 7) * 16;
#pragma unroll
    for (int t = 0; t < kPerWave; ++t) {
      const int r = 8 * (wave + NW * t) + (lane >> 3);
      const int c = (lane & 7) ^ ((r >> 1) & 7);
      const int p = min(r0 + r, d.P - 1);  // rows past the end repeat the last pixel: never stored
      hw[t] = (((p >> d.lw) & (d.H - 1)) << 16) | (p & (d.W - 1));
      pix_off[t] = (uint32_t)(((size_t)p * d.C + c * 8) * 2);
    }
  }
  __device__ __forceinline__ void issue_one(int t, uint32_t lds_stage, int tile, int wave) const {
    const int tap = tile / cblocks, c0 = (tile - tap * cblocks) * DBK;  // wave uniform
    int dh = tap / 3 - 1, dw = tap - (tap / 3) * 3 - 1;
    if (BACKWARD) { dh = -dh; dw = -dw; }
    const int sh = (hw[t] >> 16) + dh, sw = (hw[t] & 0xffff) + dw;
    const bool valid = (unsigned)sh < (unsigned)d.H && (unsigned)sw < (unsigned)d.W;
    const long off = (long)pix_off[t] + ((long)(dh * d.W + dw) * d.C + c0) * 2;
    const char* src = valid ? (const char*)d.base + off : (const char*)d.zeros + zoff;
    dma16_addr(lds_stage + (wave + NW * t) * 1024, src);
  }
  static __device__ __forceinline__ bf16x8 frag(const uint16_t* lds, int rbase, int kk, int lane) {
    return RowDma<R, NW>::frag(lds, rbase, kk, lane);
  }
};

// k-strided gathered operand: stage [64 pixels][R channels], one tap per workgroup (batch).
template <int R, int NW>
struct ColGather {
  using Desc = GatherDesc;
  static constexpr int kPerK = R / 8;
  static constexpr int kPerWave = DBK * kPerK / 64 / NW;
  static constexpr int kBytes = R * DBK * 2;
  static_assert((DBK * kPerK / 64) % NW == 0, "rows do not divide among the waves");
  Desc d;
  int dh, dw;
  int krow[kPerWave];
  uint32_t coff[kPerWave];
  uint32_t zoff;

  __device__ __forceinline__ void init(const Desc& desc, int r0, int wave, int lane, int batch) {
    d = desc;
    dh = batch / 3 - 1;
    dw = batch - (batch / 3) * 3 - 1;
    zoff = (lane & 7) * 16;
#pragma unroll
    for (int t = 0; t < kPerWave; ++t) {
      const int flat = 64 * (wave + NW * t) + lane;
      const int k = flat / kPerK;
      const int c = (flat % kPerK) ^ ColDma<R, NW>::swz(k);
      krow[t] = k;
      coff[t] = (uint32_t)(min(r0 + c * 8, d.C - 8) * 2);
    }
  }
  __device__ __forceinline__ void issue_one(int t, uint32_t lds_stage, int tile, int wave) const {
    const int p = tile * DBK + krow[t];
    const int sh = ((p >> d.lw) & (d.H - 1)) + dh, sw = (p & (d.W - 1)) + dw;
    const bool valid = (unsigned)sh < (unsigned)d.H && (unsigned)sw < (unsigned)d.W;
    const long off = ((long)p + dh * d.W + dw) * d.C * 2 + coff[t];
    const char* src = valid ? (const char*)d.base + off : (const char*)d.zeros + zoff;
    dma16_addr(lds_stage + (wave + NW * t) * 1024, src);
  }
  static __device__ __forceinline__ bf16x8 frag(const uint16_t* lds, int rbase, int kk, int lane) {
    return ColDma<R, NW>::frag(lds, rbase, kk, lane);
  }
};

// Operands that lie in memory the way the dense kernels read them; the source of k tile `tile`
// is base + (tile % inner) * step_in + (tile / inner) * step_out elements.
struct PlainDesc {
  const uint16_t* base;
  int ld, rows, inner;
  long step_in, step_out;
};
template <int R, int NW, bool COL>
struct Plain {
  using Desc = PlainDesc;
  using Impl = typename DmaSel<R, NW, COL>::type;
  static constexpr int kPerWave = Impl::kPerWave;
  static constexpr int kBytes = Impl::kBytes;
  Impl impl;
  Desc d;
  __device__ __forceinline__ void init(const Desc& desc, int r0, int wave, int lane, int /*batch*/) {
    d = desc;
    impl.init(d.ld, r0, d.rows, wave, lane);
  }
  __device__ __forceinline__ void issue_one(int t, uint32_t lds_stage, int tile, int wave) const {
    const int q = tile / d.inner;
    impl.issue_one(t, lds_stage, d.base + (tile - q * d.inner) * d.step_in + q * d.step_out, wave);
  }
  static __device__ __forceinline__ bf16x8 frag(const uint16_t* lds, int rbase, int kk, int lane) {
    return Impl::frag(lds, rbase, kk, lane);
  }
};

// fp32 partial tile of dW for one tap and one pixel range
struct EpiWgradConv {
  float* partial;  // [split][Cout][9*Cin]
  int cin, cout;
  static constexpr bool kSwap = false;
  __device__ __forceinline__ EpiWgrad at(int tap, int split) const {
    return EpiWgrad{partial + (size_t)split * cout * 9 * cin + (size_t)tap * cin, 9 * cin};
  }
};
template <class E>
__device__ __forceinline__ const E& epi_at(const E& e, int, int) { return e; }
__device__ __forceinline__ EpiWgrad epi_at(const EpiWgradConv& e, int tap, int split) { return e.at(tap, split); }

// grid = (output tiles, batches, splits); every workgroup runs KT k tiles starting at split*KT.
template <int BM, int BN, int WGM, int WGN, int NS, class AL, class BL, class Epi>
__global__ __launch_bounds__(64 * WGM * WGN) void conv_bf16_dma_kernel(int M, int N, int KT, typename AL::Desc ad,
                                                                        typename BL::Desc bd, Epi epi, TileMap map) {
  constexpr int NW = WGM * WGN;
  constexpr int WM = BM / WGM, WN = BN / WGN;
  constexpr int TM = WM / 32, TN = WN / 32;
  constexpr int kStageBytes = AL::kBytes + BL::kBytes;
  constexpr int kLoads = AL::kPerWave + BL::kPerWave;
  constexpr int NM = (DBK / 16) * TM * TN;
  constexpr bool kSwap = Epi::kSwap;
  static_assert((NS - 2) * kLoads < 64, "too many copies in flight for vmcnt");
  extern __shared__ __attribute__((aligned(16))) uint16_t lds_raw[];

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int wm = (wave / WGN) * WM, wn = (wave % WGN) * WN;
  int tile_m, tile_n;
  map.get(blockIdx.x, tile_m, tile_n);
  const int m0 = tile_m * BM, n0 = tile_n * BN;
  const int batch = blockIdx.y, split = blockIdx.z;
  const int tile0 = split * KT;
  const uint32_t lds_base = lds_addr_of(lds_raw);

  floatx16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  AL ta;
  BL tb;
  ta.init(ad, m0, wave, lane, batch);
  tb.init(bd, n0, wave, lane, batch);

  // tiles past the end re-read the last tile into a stage nobody reads again (constant vmcnt arithmetic)
  auto issue_copy = [&](int t, int tile, int st) {
    const int tc = tile0 + min(tile, KT - 1);
    const uint32_t dst = lds_base + st * kStageBytes;
    if (t < AL::kPerWave) ta.issue_one(t, dst, tc, wave);
    else tb.issue_one(t - AL::kPerWave, dst + AL::kBytes, tc, wave);
  };
#pragma unroll
  for (int st = 0; st < NS - 1; ++st)
#pragma unroll
    for (int t = 0; t < kLoads; ++t) issue_copy(t, st, st);

  int rd = 0, wr = NS - 1;
  for (int kt = 0; kt < KT; ++kt) {
    wait_vmcnt<(NS - 2) * kLoads>();
    lds_barrier();
    const uint16_t* la = lds_raw + rd * (kStageBytes / 2);
    const uint16_t* lb = la + AL::kBytes / 2;
    bf16x8 af[2][TM], bfr[2][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i) af[0][i] = AL::frag(la, wm + i * 32, 0, lane);
#pragma unroll
    for (int j = 0; j < TN; ++j) bfr[0][j] = BL::frag(lb, wn + j * 32, 0, lane);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int kk = 0; kk < DBK / 16; ++kk) {
      const int c = kk & 1, nx = c ^ 1;
      if (kk + 1 < DBK / 16) {
#pragma unroll
        for (int i = 0; i < TM; ++i) af[nx][i] = AL::frag(la, wm + i * 32, kk + 1, lane);
#pragma unroll
        for (int j = 0; j < TN; ++j) bfr[nx][j] = BL::frag(lb, wn + j * 32, kk + 1, lane);
      }
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
          acc[i][j] = mma<kSwap>(af[c][i], bfr[c][j], acc[i][j]);
          const int q = (kk * TM + i) * TN + j;
#pragma unroll
          for (int t = 0; t < kLoads; ++t)
            if ((t * NM) / kLoads == q) {
              __builtin_amdgcn_sched_barrier(0);
              issue_copy(t, kt + NS - 1, wr);
              __builtin_amdgcn_sched_barrier(0);
            }
        }
      __builtin_amdgcn_sched_barrier(0);
    }
    rd = rd + 1 == NS ? 0 : rd + 1;
    wr = wr + 1 == NS ? 0 : wr + 1;
  }
  wait_vmcnt<0>();
  lds_barrier();
  store_tiles<TM, TN>(acc, epi_at(epi, batch, split), m0 + wm, n0 + wn, M, N, lane);
}

template <int BM, int BN, int NS, class AL, class BL, class Epi>
hipError_t launch_conv(hipStream_t s, int M, int N, int KT, int batches, int splits, const typename AL::Desc& ad,
                       const typename BL::Desc& bd, const Epi& epi) {
  constexpr size_t lds_bytes = (size_t)NS * (AL::kBytes + BL::kBytes);
  static_assert(lds_bytes <= 160 * 1024, "stages do not fit the LDS of a CU");
  auto kernel = conv_bf16_dma_kernel<BM, BN, 2, 2, NS, AL, BL, Epi>;
  if (lds_bytes > 32 * 1024) {
    static hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
    if (attr != hipSuccess) return attr;
  }
  const int tiles_m = (M + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
  const TileMap map = make_tile_map(tiles_m, tiles_n);
  hipLaunchKernelGGL(kernel, dim3(tiles_m * tiles_n, batches, splits), dim3(256), lds_bytes, s, M, N, KT, ad, bd, epi, map);
  return hipGetLastError();
}

inline bool pow2(int v) { return v > 0 && (v & (v - 1)) == 0; }
inline int ilog2(int v) { int l = 0; while ((1 << l) < v) ++l; return l; }

__global__ __launch_bounds__(256) void split_sum_mfma_kernel(size_t count, int splits, const float* __restrict__ partial,
                                                             float* __restrict__ out) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= count) return;
  float s = 0.f;
#pragma unroll 8
  for (int z = 0; z < splits; ++z) s += partial[(size_t)z * count + i];
  out[i] = s;
}

}  // namespace

bool conv_mfma_supported(int imgs, int H, int W, int cin, int cout) {
  const long P = (long)imgs * H * W;
  return pow2(H) && pow2(W) && H <= 32768 && W <= 32768 && cin % 64 == 0 && cout % 64 == 0 && P % 64 == 0 &&
         P * std::max(cin, cout) * 2 < (1l << 31);
}

// pixel ranges for wgrad: enough workgroups to fill the chip, at least 4 k tiles each
int conv_mfma_wgrad_splits(int pixels, int cin, int cout) {
  const int tiles = ((cout + 63) / 64) * ((cin + 63) / 64) * 9;
  const int kt = pixels / 64;
  int s = std::max(1, 512 / tiles);
  while (s > 1 && (kt % s != 0 || kt / s < 4)) --s;
  return s;
}

hipError_t conv_mfma_fprop(hipStream_t s, int imgs, int H, int W, int cin, int cout, const uint16_t* x,
                           const uint16_t* wgt, const float* bias, int act, uint16_t* d_out, uint16_t* a_out,
                           const uint16_t* zeros) {
  const int P = imgs * H * W;
  GatherDesc ad{x, zeros, P, H, W, ilog2(W), cin};
  PlainDesc bd{wgt, 9 * cin, cout, 1 << 30, DBK, 0};
  EpiFprop e{bias, d_out, a_out, act, cout};
  const int KT = 9 * cin / DBK;
  if (cout % 128 == 0)
    return launch_conv<128, 128, 3, RowGather<128, 4, false>, Plain<128, 4, false>>(s, P, cout, KT, 1, 1, ad, bd, e);
  return launch_conv<128, 64, 4, RowGather<128, 4, false>, Plain<64, 4, false>>(s, P, cout, KT, 1, 1, ad, bd, e);
}

hipError_t conv_mfma_dgrad(hipStream_t s, int imgs, int H, int W, int cin, int cout, const uint16_t* dz,
                           const uint16_t* wb, const uint16_t* d_prev, uint16_t* out, const uint16_t* zeros) {
  const int P = imgs * H * W;
  GatherDesc ad{dz, zeros, P, H, W, ilog2(W), cout};
  // k tile -> (tap, block of 64 output channels): rows co0.. of W_b, columns tap*Cin..
  PlainDesc bd{wb, 9 * cin, cin, cout / DBK, (long)DBK * 9 * cin, cin};
  EpiDgrad e{d_prev, out, cin};
  const int KT = 9 * cout / DBK;
  if (cin % 128 == 0)
    return launch_conv<128, 128, 3, RowGather<128, 4, true>, Plain<128, 4, true>>(s, P, cin, KT, 1, 1, ad, bd, e);
  return launch_conv<128, 64, 4, RowGather<128, 4, true>, Plain<64, 4, true>>(s, P, cin, KT, 1, 1, ad, bd, e);
}

hipError_t conv_mfma_wgrad(hipStream_t s, int imgs, int H, int W, int cin, int cout, const uint16_t* dz,
                           const uint16_t* x, float* gW, float* partial, const uint16_t* zeros) {
  const int P = imgs * H * W;
  const int splits = conv_mfma_wgrad_splits(P, cin, cout);
  const int KT = P / DBK / splits;
  PlainDesc ad{dz, cout, cout, 1 << 30, (long)DBK * cout, 0};
  GatherDesc bd{x, zeros, P, H, W, ilog2(W), cin};
  EpiWgradConv e{splits > 1 ? partial : gW, cin, cout};
  hipError_t err;
  if (cout % 128 == 0 && cin % 128 == 0)
    err = launch_conv<128, 128, 3, Plain<128, 4, true>, ColGather<128, 4>>(s, cout, cin, KT, 9, splits, ad, bd, e);
  else
    err = launch_conv<64, 64, 4, Plain<64, 4, true>, ColGather<64, 4>>(s, cout, cin, KT, 9, splits, ad, bd, e);
  if (err != hipSuccess || splits == 1) return err;
  const size_t count = (size_t)cout * 9 * cin;
  hipLaunchKernelGGL(split_sum_mfma_kernel, dim3((unsigned)((count + 255) / 256)), dim3(256), 0, s, count, splits, partial, gW);
  return hipGetLastError();
}

}  // namespace tp
