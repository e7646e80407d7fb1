// 3x3 convolutions (stride 1 or 2, pad 1, NHWC) on the gfx950 matrix cores as implicit GEMMs.
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
// kernels of kernels_conv.hip.  Stride 2 runs on the gather kernels only: the rows (fprop, wgrad:
// output pixels; dgrad: input pixels, one parity class at a time) and the pixels they read live on grids of
// different size.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <algorithm>

#include "conv.h"
#include "kernels.h"
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
  const uint16_t* base;   // [pixels of the source grid][C] activations or gradients
  const uint16_t* zeros;  // >= 128 bytes of zeros, 16-byte aligned
  int P, H, W, lw;        // the grid the rows (or the contraction index) run over: pixels, image size, log2(W)
  int C;                  // channels of `base`
  int SH, SW;             // image size of the source grid (= H, W at stride 1)
};

// Source pixel of output position (h, w) for tap offset (dh, dw) at stride S (fprop, wgrad): the input at
// S*(h, w) + (dh, dw).  (The input gradient at stride 2 goes by parity class of the input pixels: RowGatherS2.)
template <int S>
__device__ __forceinline__ bool source_pixel(int h, int w, int dh, int dw, int SH, int SW, int& sh, int& sw) {
  sh = h * S + dh;
  sw = w * S + dw;
  return (unsigned)sh < (unsigned)SH && (unsigned)sw < (unsigned)SW;
}

// k-contiguous gathered operand: stage [R pixels][64 channels of one tap].
template <int R, int NW, bool BACKWARD, int S = 1>
struct RowGather {
  using Desc = GatherDesc;
  static constexpr int kPerWave = R / 8 / NW;
  static constexpr int kBytes = R * DBK * 2;
  static_assert((R / 8) % NW == 0, "rows do not divide among the waves");
  Desc d;
  int cblocks;
  uint32_t pix_off[kPerWave];  // S == 1: byte offset of (pixel, chunk) inside base; else of (image, chunk)
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
      if (S == 1) {
        pix_off[t] = (uint32_t)(((size_t)p * d.C + c * 8) * 2);
      } else {
        const int img = p / (d.H * d.W);
        pix_off[t] = (uint32_t)(((size_t)img * d.SH * d.SW * d.C + c * 8) * 2);
      }
    }
  }
  __device__ __forceinline__ void issue_one(int t, uint32_t lds_stage, int tile, int wave) const {
    const int tap = tile / cblocks, c0 = (tile - tap * cblocks) * DBK;  // wave uniform
    int dh = tap / 3 - 1, dw = tap - (tap / 3) * 3 - 1;
    if (BACKWARD) { dh = -dh; dw = -dw; }
    bool valid;
    long off;
    if (S == 1) {
      const int sh = (hw[t] >> 16) + dh, sw = (hw[t] & 0xffff) + dw;
      valid = (unsigned)sh < (unsigned)d.H && (unsigned)sw < (unsigned)d.W;
      off = (long)pix_off[t] + ((long)(dh * d.W + dw) * d.C + c0) * 2;
    } else {
      int sh, sw;
      static_assert(!BACKWARD || S == 1, "the stride-2 input gradient runs on RowGatherS2");
      valid = source_pixel<S>(hw[t] >> 16, hw[t] & 0xffff, dh, dw, d.SH, d.SW, sh, sw);
      off = (long)pix_off[t] + ((long)(sh * d.SW + sw) * d.C + c0) * 2;
    }
    const char* src = valid ? (const char*)d.base + off : (const char*)d.zeros + zoff;
    dma16_addr(lds_stage + (wave + NW * t) * 1024, src);
  }
  static __device__ __forceinline__ bf16x8 frag(const uint16_t* lds, int rbase, int kk, int lane) {
    return RowDma<R, NW>::frag(lds, rbase, kk, lane);
  }
  static __device__ __forceinline__ int tiles_of(const Desc&, int /*batch*/, int KT) { return KT; }
};

// The 3x3 input gradient at stride 2, one parity class of input pixels per batch.  An input pixel (h, w) gets a
// contribution from tap (kh, kw) only where h - kh + 1 and w - kw + 1 are even: for even h that is kh = 1, for odd
// h kh = 0 and 2, likewise along w, so the four classes (h & 1, w & 1) have 1, 2, 2 and 4 taps -- 9 tap-products in
// all where rows running over every input pixel and all nine taps multiply zeros three times out of four.
// Class of a batch: the one with the most taps first (its workgroups run longest).
__host__ __device__ __forceinline__ int s2_class(int batch) { return 3 - batch; }                  // 2*(h&1) + (w&1)
__host__ __device__ __forceinline__ int s2_class_taps(int cls) { return (1 + (cls >> 1)) * (1 + (cls & 1)); }
__device__ __forceinline__ int s2_class_tap(int cls, int ti) {  // ti-th tap of the class, as 3*kh + kw
  const int ph = cls >> 1, pw = cls & 1;
  const int kh = ph ? 2 * (ti >> pw) : 1, kw = pw ? 2 * (ti & 1) : 1;
  return 3 * kh + kw;
}

// Rows: the pixels (img, h2, w2) of one class on the (H/2) x (W/2) grid, i.e. input pixel (2 h2 + ph, 2 w2 + pw);
// the source is dz on that same grid at (h2 + (ph - kh + 1)/2, w2 + (pw - kw + 1)/2), zero past its edge.
template <int R, int NW>
struct RowGatherS2 {
  using Desc = GatherDesc;  // P, H, W, lw: rows and grid of one class; SH, SW: the dz grid (the same size)
  static constexpr int kPerWave = R / 8 / NW;
  static constexpr int kBytes = R * DBK * 2;
  static_assert((R / 8) % NW == 0, "rows do not divide among the waves");
  Desc d;
  int cblocks, cls;
  uint32_t img_off[kPerWave];  // byte offset of (image, chunk) inside base
  int hw[kPerWave];            // h2 << 16 | w2 of the lane's pixel
  uint32_t zoff;

  __device__ __forceinline__ void init(const Desc& desc, int r0, int wave, int lane, int batch) {
    d = desc;
    cblocks = d.C / DBK;
    cls = s2_class(batch);
    zoff = (lane & 7) * 16;
#pragma unroll
    for (int t = 0; t < kPerWave; ++t) {
      const int r = 8 * (wave + NW * t) + (lane >> 3);
      const int c = (lane & 7) ^ ((r >> 1) & 7);
      const int p = min(r0 + r, d.P - 1);  // rows past the end repeat the last pixel: never stored
      hw[t] = (((p >> d.lw) & (d.H - 1)) << 16) | (p & (d.W - 1));
      const int img = p / (d.H * d.W);
      img_off[t] = (uint32_t)(((size_t)img * d.SH * d.SW * d.C + c * 8) * 2);
    }
  }
  __device__ __forceinline__ void issue_one(int t, uint32_t lds_stage, int tile, int wave) const {
    const int ti = tile / cblocks, c0 = (tile - ti * cblocks) * DBK;  // wave uniform
    const int tap = s2_class_tap(cls, ti);
    const int kh = tap / 3, kw = tap - 3 * kh;
    const int sh = (hw[t] >> 16) + (((cls >> 1) - kh + 1) >> 1), sw = (hw[t] & 0xffff) + (((cls & 1) - kw + 1) >> 1);
    const bool valid = sh < d.SH && sw < d.SW;
    const long off = (long)img_off[t] + ((long)(sh * d.SW + sw) * d.C + c0) * 2;
    const char* src = valid ? (const char*)d.base + off : (const char*)d.zeros + zoff;
    dma16_addr(lds_stage + (wave + NW * t) * 1024, src);
  }
  static __device__ __forceinline__ bf16x8 frag(const uint16_t* lds, int rbase, int kk, int lane) {
    return RowDma<R, NW>::frag(lds, rbase, kk, lane);
  }
  static __device__ __forceinline__ int tiles_of(const Desc& desc, int batch, int /*KT*/) {
    return s2_class_taps(s2_class(batch)) * (desc.C / DBK);
  }
};

// k-strided gathered operand: stage [64 pixels][R channels], one tap per workgroup (batch).
template <int R, int NW, int S = 1>
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
    bool valid;
    long off;
    if (S == 1) {
      const int sh = ((p >> d.lw) & (d.H - 1)) + dh, sw = (p & (d.W - 1)) + dw;
      valid = (unsigned)sh < (unsigned)d.H && (unsigned)sw < (unsigned)d.W;
      off = ((long)p + dh * d.W + dw) * d.C * 2 + coff[t];
    } else {
      int sh, sw;
      valid = source_pixel<S>((p >> d.lw) & (d.H - 1), p & (d.W - 1), dh, dw, d.SH, d.SW, sh, sw);
      const int img = p / (d.H * d.W);
      off = (((long)img * d.SH + sh) * d.SW + sw) * d.C * 2 + coff[t];
    }
    const char* src = valid ? (const char*)d.base + off : (const char*)d.zeros + zoff;
    dma16_addr(lds_stage + (wave + NW * t) * 1024, src);
  }
  static __device__ __forceinline__ bf16x8 frag(const uint16_t* lds, int rbase, int kk, int lane) {
    return ColDma<R, NW>::frag(lds, rbase, kk, lane);
  }
  static __device__ __forceinline__ int tiles_of(const Desc&, int /*batch*/, int KT) { return KT; }
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
  static __device__ __forceinline__ int tiles_of(const Desc&, int /*batch*/, int KT) { return KT; }
};

// The weights of the stride-2 input gradient by parity class: k tile -> (ti-th tap of the batch's class, block of 64
// output channels); the source of tile `tile` is base + (tile % inner) * step_in + tap * step_out.
template <int R, int NW>
struct PlainS2 {
  using Desc = PlainDesc;
  using Impl = ColDma<R, NW>;
  static constexpr int kPerWave = Impl::kPerWave;
  static constexpr int kBytes = Impl::kBytes;
  Impl impl;
  Desc d;
  int cls;
  __device__ __forceinline__ void init(const Desc& desc, int r0, int wave, int lane, int batch) {
    d = desc;
    cls = s2_class(batch);
    impl.init(d.ld, r0, d.rows, wave, lane);
  }
  __device__ __forceinline__ void issue_one(int t, uint32_t lds_stage, int tile, int wave) const {
    const int ti = tile / d.inner;
    impl.issue_one(t, lds_stage, d.base + (tile - ti * d.inner) * d.step_in + s2_class_tap(cls, ti) * d.step_out, wave);
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
// The input gradient of one parity class: row m of the class is input pixel (img, 2 h2 + ph, 2 w2 + pw)
struct EpiDgradClass {
  EpiDgrad e;
  int H, W, lw2, lh2, ph, pw;  // input image, log2 of its half sizes
  static constexpr bool kSwap = true;
  __device__ __forceinline__ int pixel(int m) const {
    const int w2 = m & ((W >> 1) - 1), h2 = (m >> lw2) & ((H >> 1) - 1), img = m >> (lw2 + lh2);
    return (img * H + 2 * h2 + ph) * W + 2 * w2 + pw;
  }
  __device__ __forceinline__ void row8(int m, int n, float (&v)[8]) const { e.row8(pixel(m), n, v); }
  __device__ __forceinline__ void quad(int m, int n, int count, float v0, float v1, float v2, float v3) const {
    e.quad(pixel(m), n, count, v0, v1, v2, v3);
  }
};
struct EpiDgradS2 {
  EpiDgrad e;
  int H, W, lw2, lh2;
  static constexpr bool kSwap = true;
  __device__ __forceinline__ EpiDgradClass at(int batch) const {
    const int cls = s2_class(batch);
    return EpiDgradClass{e, H, W, lw2, lh2, cls >> 1, cls & 1};
  }
};
template <class E>
__device__ __forceinline__ const E& epi_at(const E& e, int, int) { return e; }
__device__ __forceinline__ EpiDgradClass epi_at(const EpiDgradS2& e, int batch, int) { return e.at(batch); }
__device__ __forceinline__ EpiWgrad epi_at(const EpiWgradConv& e, int tap, int split) { return e.at(tap, split); }

// grid = (output tiles, batches, splits); every workgroup runs KT k tiles starting at split*KT.
// KG = 2: two groups of WGM x WGN waves share the output tile and take every other k tile each (group g the tiles
// g, g + 2, ...; KT even), with stage buffers and copies of their own; both groups meet at the same barriers.  At
// the end the second group hands its accumulators over through LDS and the first one stores the tile.  For products
// with few output tiles and a long contraction (3x3 convolutions on 4x4 maps: 128 workgroups, 36 k tiles, one MFMA
// per wave and k step) this halves the chain of barrier -> fragment reads -> MFMAs: 17.3 -> 15.4 us.  What remains is
// the 576 KB every workgroup gathers through its CU's L1 (each input pixel nine times), 7.5 us at the rate one CU
// fetches from L2.
template <int BM, int BN, int WGM, int WGN, int NS, class AL, class BL, class Epi, int KG = 1>
__global__ __launch_bounds__(64 * WGM * WGN * KG) void conv_bf16_dma_kernel(int M, int N, int KT, typename AL::Desc ad,
                                                                             typename BL::Desc bd, Epi epi, TileMap map) {
  constexpr int NW = WGM * WGN;  // waves of one group
  constexpr int WM = BM / WGM, WN = BN / WGN;
  constexpr int TM = WM / 32, TN = WN / 32;
  constexpr int kStageBytes = AL::kBytes + BL::kBytes;
  constexpr int kLoads = AL::kPerWave + BL::kPerWave;
  constexpr int NM = (DBK / 16) * TM * TN;
  constexpr bool kSwap = Epi::kSwap;
  static_assert((NS - 2) * kLoads < 64, "too many copies in flight for vmcnt");
  static_assert(KG == 1 || KG == 2, "one or two groups of waves along the contraction");
  extern __shared__ __attribute__((aligned(16))) uint16_t lds_raw[];

  const int lane = threadIdx.x & 63;
  const int wave_all = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int kg = KG == 1 ? 0 : wave_all / NW;  // group along the contraction
  const int wave = KG == 1 ? wave_all : wave_all % NW;
  const int wm = (wave / WGN) * WM, wn = (wave % WGN) * WN;
  int tile_m, tile_n;
  map.get(blockIdx.x, tile_m, tile_n);
  const int m0 = tile_m * BM, n0 = tile_n * BN;
  const int batch = blockIdx.y, split = blockIdx.z;
  KT = AL::tiles_of(ad, batch, KT);  // the same for every batch but where batches differ in their taps
  const int tile0 = split * KT;
  const int KTg = KT / KG;  // k tiles of this group: tile0 + kg, tile0 + kg + KG, ...
  const uint32_t lds_base = lds_addr_of(lds_raw) + kg * (NS * kStageBytes);
  const uint16_t* lds_group = lds_raw + kg * (NS * kStageBytes / 2);

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
    const int tc = tile0 + min(tile, KTg - 1) * KG + kg;
    const uint32_t dst = lds_base + st * kStageBytes;
    if (t < AL::kPerWave) ta.issue_one(t, dst, tc, wave);
    else tb.issue_one(t - AL::kPerWave, dst + AL::kBytes, tc, wave);
  };
#pragma unroll
  for (int st = 0; st < NS - 1; ++st)
#pragma unroll
    for (int t = 0; t < kLoads; ++t) issue_copy(t, st, st);

  int rd = 0, wr = NS - 1;
  for (int kt = 0; kt < KTg; ++kt) {
    wait_vmcnt<(NS - 2) * kLoads>();
    lds_barrier();
    const uint16_t* la = lds_group + rd * (kStageBytes / 2);
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
  lds_barrier();  // all waves of both groups are done with the stages
  if constexpr (KG == 2) {
    // the second group's accumulators go through LDS, behind the regions the first group's epilogue turns its tiles
    // through: [wave][accumulator register][lane]
    float* handover = reinterpret_cast<float*>(lds_raw) + NW * (wave_epilogue_bytes<TM, TN>() / 4) + wave * (TM * TN * 16 * 64);
    if (kg == 1) {
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
          for (int r = 0; r < 16; ++r) handover[((i * TN + j) * 16 + r) * 64 + lane] = acc[i][j][r];
    }
    lds_barrier();  // the last barrier of the workgroup: every wave of both groups reaches it
    if (kg == 1) return;
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][j][r] += handover[((i * TN + j) * 16 + r) * 64 + lane];
  }
  if constexpr (Epi::kSwap) {
    if (m0 + wm + WM <= M && n0 + wn + WN <= N && (N & 7) == 0) {
      float* wave_lds = reinterpret_cast<float*>(lds_raw) + wave * (wave_epilogue_bytes<TM, TN>() / 4);
      store_tiles_coalesced<TM, TN>(acc, epi_at(epi, batch, split), m0 + wm, n0 + wn, lane, wave_lds);
      return;
    }
  }
  store_tiles<TM, TN>(acc, epi_at(epi, batch, split), m0 + wm, n0 + wn, M, N, lane);
}

template <int BM, int BN, int NS, class AL, class BL, class Epi, int KG = 1>
hipError_t launch_conv(hipStream_t s, int M, int N, int KT, int batches, int splits, const typename AL::Desc& ad,
                       const typename BL::Desc& bd, const Epi& epi) {
  constexpr size_t stage_bytes = (size_t)KG * NS * (AL::kBytes + BL::kBytes);
  // epilogue: the four wave tiles turned through LDS, and behind them (KG = 2) the second group's accumulators
  constexpr size_t epi_bytes = (size_t)4 * wave_epilogue_bytes<BM / 64, BN / 64>() + (KG == 2 ? (size_t)BM * BN * 4 : 0);
  constexpr size_t lds_bytes = stage_bytes > epi_bytes ? stage_bytes : epi_bytes;
  static_assert(lds_bytes <= 160 * 1024, "stages do not fit the LDS of a CU");
  if (KG == 2 && (KT % 2 != 0 || KT < 4)) return hipErrorInvalidValue;
  auto kernel = conv_bf16_dma_kernel<BM, BN, 2, 2, NS, AL, BL, Epi, KG>;
  if (lds_bytes > 32 * 1024) {
    static hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
    if (attr != hipSuccess) return attr;
  }
  const int tiles_m = (M + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
  const TileMap map = make_tile_map(tiles_m, tiles_n);
  hipLaunchKernelGGL(kernel, dim3(tiles_m * tiles_n, batches, splits), dim3(256 * KG), lds_bytes, s, M, N, KT, ad, bd, epi, map);
  return hipGetLastError();
}

// ================================================================================================
// Patch kernels: the input tile lives in LDS once, with its halo
// ================================================================================================
// A tile of BM output pixels = BM/W whole image rows.  The (BM/W + 2) x (W + 2) input pixels it
// needs (zero outside the image) are copied to LDS once, [patch pixel][channel]; the nine taps
// then read the same LDS data at shifted pixel positions.  Compared with gathering every
// (tap, channel block) k tile from L2 this cuts the activation traffic into the CU ninefold.

struct PatchDesc {
  const uint16_t* base;   // [P][C]
  const uint16_t* zeros;  // >= 128 zero bytes
  int H, W, lw;           // image size, log2(W)
  int C;                  // channels of `base` (pixel pitch in elements)
  int c0;                 // first channel staged
  int CB;                 // 16-byte chunks staged per pixel (channels staged / 8)
  int tr;                 // 1: layout for transposed reads (pixels are the contraction index)
};

// chunk c of patch pixel pp is stored in slot c ^ patch_swz(pp)
__device__ __forceinline__ int patch_swz(int pp, int CB, int tr) {
  if (tr) return 4 * ((pp >> 1) & 1);             // as the [k][64] stages of the dense kernels
  return (CB & 15) ? ((pp >> 1) & 7) : (pp & 15);  // 128-byte pixels: 8 slots over same-parity pixels; wider: 16
}

// All waves of the workgroup copy the patch of the tile whose first pixel is p0 (a multiple of BM)
template <int BM, int NW>
__device__ __forceinline__ void issue_patch(const PatchDesc& d, uint32_t lds_patch, int p0, int wave, int lane) {
  const int PC = d.W + 2, NPIX = (BM / d.W + 2) * PC;
  const int img_px = d.H * d.W;
  const int img = p0 / img_px, h0 = (p0 - img * img_px) >> d.lw;
  const int px_bytes = d.CB * 16;
  const int instrs = (NPIX * px_bytes + 1023) / 1024;
  for (int i = wave; i < instrs; i += NW) {
    const int off = i * 1024 + lane * 16;
    const int pp = off / px_bytes, slot = (off - pp * px_bytes) >> 4;
    const int chunk = slot ^ patch_swz(pp, d.CB, d.tr);
    const int pr = pp / PC, pc = pp - pr * PC;
    const int h = h0 + pr - 1, w = pc - 1;
    const bool valid = pp < NPIX && (unsigned)h < (unsigned)d.H && (unsigned)w < (unsigned)d.W;
    const long src = (((long)img * d.H + h) * d.W + w) * d.C + d.c0 + chunk * 8;
    const uint16_t* ptr = valid ? d.base + src : d.zeros + (lane & 7) * 8;
    dma16_addr(lds_patch + i * 1024, ptr);
  }
}
__host__ __device__ inline int patch_bytes(int BM, int W, int CB) {
  return (((BM / W + 2) * (W + 2) * CB * 16 + 1023) / 1024) * 1024;
}

// fprop (BWD = false) and dgrad (BWD = true): out[p][n] = sum_{tap, c} in[p shifted by tap][c] * B[(tap, c)][n]
template <int BM, int BN, int WGM, int WGN, int NS, bool BWD, class BL, class Epi>
__global__ __launch_bounds__(64 * WGM * WGN) void conv_patch_kernel(int P, int N, PatchDesc pd, typename BL::Desc bd, Epi epi,
                                                                     int tiles_n) {
  constexpr int NW = WGM * WGN;
  constexpr int WM = BM / WGM, WN = BN / WGN;
  constexpr int TM = WM / 32, TN = WN / 32;
  constexpr int kLoads = BL::kPerWave;
  constexpr int NM = (DBK / 16) * TM * TN;
  static_assert((NS - 2) * kLoads < 64, "too many copies in flight for vmcnt");
  extern __shared__ __attribute__((aligned(16))) uint16_t lds_raw[];

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int wm = (wave / WGN) * WM, wn = (wave % WGN) * WN;
  const int tile_p = blockIdx.x / tiles_n, tile_n = blockIdx.x - tile_p * tiles_n;
  const int m0 = tile_p * BM, n0 = tile_n * BN;
  const uint32_t lds_base = lds_addr_of(lds_raw);
  const int pbytes = patch_bytes(BM, pd.W, pd.CB);
  const uint32_t lds_stage0 = lds_base + pbytes;
  const uint16_t* stage0 = lds_raw + pbytes / 2;

  floatx16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  issue_patch<BM, NW>(pd, lds_base, m0, wave, lane);
  BL tb;
  tb.init(bd, n0, wave, lane, 0);
  const int cbs = pd.C / DBK;  // 64-channel blocks per tap
  const int KT = 9 * cbs;
  auto issue_copy = [&](int t, int tile, int st) {
    tb.issue_one(t, lds_stage0 + st * BL::kBytes, min(tile, KT - 1), wave);
  };
#pragma unroll
  for (int st = 0; st < NS - 1; ++st)
#pragma unroll
    for (int t = 0; t < kLoads; ++t) issue_copy(t, st, st);

  // centre patch pixel of the lane's row in each of its MFMA row tiles
  const int PC = pd.W + 2;
  int ppc[TM];
#pragma unroll
  for (int i = 0; i < TM; ++i) {
    const int q = wm + i * 32 + (lane & 31);
    ppc[i] = ((q >> pd.lw) + 1) * PC + (q & (pd.W - 1)) + 1;
  }
  const int khalf = lane >> 5;

  int rd = 0, wr = NS - 1;
  int tap = 0, cb = 0;
  for (int kt = 0; kt < KT; ++kt) {
    wait_vmcnt<(NS - 2) * kLoads>();  // the patch copies are older than any stage: they have landed too
    lds_barrier();
    const uint16_t* lb = stage0 + rd * (BL::kBytes / 2);
    int dh = tap / 3 - 1, dw = tap - (tap / 3) * 3 - 1;
    if (BWD) { dh = -dh; dw = -dw; }
    const int tapoff = dh * PC + dw;
    uint32_t prow[TM];  // element offset of the lane's shifted pixel
    int psw[TM];
#pragma unroll
    for (int i = 0; i < TM; ++i) {
      const int ppt = ppc[i] + tapoff;
      prow[i] = (uint32_t)ppt * pd.CB * 8;
      psw[i] = patch_swz(ppt, pd.CB, 0);
    }
    auto afrag = [&](int i, int kk) {
      const int chunk = cb * 8 + kk * 2 + khalf;
      const uint4 v = *reinterpret_cast<const uint4*>(lds_raw + prow[i] + ((chunk ^ psw[i]) << 3));
      return __builtin_bit_cast(bf16x8, v);
    };
    bf16x8 af[2][TM], bfr[2][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i) af[0][i] = afrag(i, 0);
#pragma unroll
    for (int j = 0; j < TN; ++j) bfr[0][j] = BL::frag(lb, wn + j * 32, 0, lane);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int kk = 0; kk < DBK / 16; ++kk) {
      const int c = kk & 1, nx = c ^ 1;
      if (kk + 1 < DBK / 16) {
#pragma unroll
        for (int i = 0; i < TM; ++i) af[nx][i] = afrag(i, kk + 1);
#pragma unroll
        for (int j = 0; j < TN; ++j) bfr[nx][j] = BL::frag(lb, wn + j * 32, kk + 1, lane);
      }
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
          acc[i][j] = mma<Epi::kSwap>(af[c][i], bfr[c][j], acc[i][j]);
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
    if (++cb == cbs) { cb = 0; ++tap; }
  }
  wait_vmcnt<0>();
  lds_barrier();
  if (n0 + wn + WN <= N && (N & 7) == 0) {  // pixel tiles are always whole
    float* wave_lds = reinterpret_cast<float*>(lds_raw) + wave * (wave_epilogue_bytes<TM, TN>() / 4);
    store_tiles_coalesced<TM, TN>(acc, epi, m0 + wm, n0 + wn, lane, wave_lds);
  } else {
    store_tiles<TM, TN>(acc, epi, m0 + wm, n0 + wn, P, N, lane);
  }
}

// wgrad: dW[co][tap][ci] = sum_p dz[p][co] * x[p shifted by tap][ci] for one block of 64 output and 64
// input channels and all nine taps; the workgroup walks over pixel tiles split, split + splits, ...,
// double buffered: the copies of the next tile fly while the current one is multiplied.
template <int BM>
__global__ __launch_bounds__(256) void conv_wgrad_patch_kernel(PatchDesc xd, const uint16_t* __restrict__ dz, int cout,
                                                               int px_tiles, int ci_blocks, float* __restrict__ out) {
  constexpr int NW = 4;
  using DZ = ColDma<64, NW>;  // stage [pixel][64 output channels]; k index = pixel
  constexpr int kDzInstr = BM * 8 / 64 / NW;
  extern __shared__ __attribute__((aligned(16))) uint16_t lds_raw[];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int cob = blockIdx.x / ci_blocks, cib = blockIdx.x - cob * ci_blocks;
  const int split = blockIdx.y, splits = gridDim.y;
  const int cin = xd.C;
  xd.c0 = cib * 64;
  const int pbytes = patch_bytes(BM, xd.W, 8);
  const int buf_bytes = pbytes + BM * 128;
  const uint32_t lds_base = lds_addr_of(lds_raw);
  const int rb_co = (wave >> 1) * 32, rb_ci = (wave & 1) * 32;
  const int PC = xd.W + 2;

  floatx16 acc[9];
#pragma unroll
  for (int t = 0; t < 9; ++t)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[t][r] = 0.f;

  // per-lane source offsets of the dz tile (the same in every tile, relative to its first pixel)
  uint32_t dzoff[kDzInstr];
#pragma unroll
  for (int i = 0; i < kDzInstr; ++i) {
    const int flat = 64 * (wave + NW * i) + lane;
    const int k = flat >> 3, c = (flat & 7) ^ DZ::swz(k);
    dzoff[i] = (uint32_t)(((size_t)k * cout + cob * 64 + c * 8) * 2);
  }
  auto issue_tile = [&](int tile, int buf) {
    const uint32_t dst = lds_base + buf * buf_bytes;
    issue_patch<BM, NW>(xd, dst, tile * BM, wave, lane);
    const uint16_t* src = dz + (size_t)tile * BM * cout;
#pragma unroll
    for (int i = 0; i < kDzInstr; ++i) dma16(dst + pbytes + (wave + NW * i) * 1024, src, dzoff[i]);
  };

  if (split < px_tiles) issue_tile(split, 0);
  int buf = 0;
  for (int tile = split; tile < px_tiles; tile += splits) {
    wait_vmcnt<0>();  // this tile has landed (nothing else is in flight)
    lds_barrier();    // ... for every wave, and every wave is done with the other buffer
    if (tile + splits < px_tiles) issue_tile(tile + splits, buf ^ 1);
    const uint16_t* lp = lds_raw + buf * (buf_bytes / 2);
    const uint16_t* ldz = lp + pbytes / 2;
    const int g = lane >> 4, s = lane & 15;
    const int col = rb_ci + 16 * (g & 1) + 4 * (s & 3);
#pragma unroll 2
    for (int kk = 0; kk < BM / 16; ++kk) {
      const bf16x8 a = DZ::frag(ldz, rb_co, kk, lane);
      const int kq = kk * 16 + 8 * (g >> 1) + (s >> 2);
      const int ppc = ((kq >> xd.lw) + 1) * PC + (kq & (xd.W - 1)) + 1;
#pragma unroll
      for (int t = 0; t < 9; ++t) {
        const int ppt = ppc + (t / 3 - 1) * PC + (t % 3 - 1);
        const int slot = (col >> 3) ^ patch_swz(ppt, 8, 1);
        typedef __attribute__((address_space(3))) shortx4* lds_ptr;
        const uint16_t* p = lp + ppt * 64 + slot * 8 + (col & 7);
        const shortx4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(p));
        const shortx4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(p + 4 * 64));
        const shortx8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        acc[t] = mma<false>(a, __builtin_bit_cast(bf16x8, v), acc[t]);
      }
    }
    buf ^= 1;
  }
  float* o = out + (size_t)split * cout * 9 * cin;
#pragma unroll
  for (int t = 0; t < 9; ++t) {
    floatx16 one[1][1];
    one[0][0] = acc[t];
    store_tiles<1, 1>(one, EpiWgrad{o + (size_t)t * cin, 9 * cin}, cob * 64 + rb_co, cib * 64 + rb_ci, cout, cin, lane);
  }
}

// ================================================================================================
// First layer of an image net: a handful of input channels (3), padded to 8
// ================================================================================================
// With the input stored [pixel][8 channels] (16 bytes per pixel, channels >= Cin zero), one k step
// of the MFMA (16 values) is two taps x 8 channels: the lane half that holds k 0..7 reads tap
// 2*kk, the other tap 2*kk + 1, each one 16-byte LDS read of the patch at its shifted pixel.
// Nine taps fill 4.5 steps; a tenth tap reads a zero pixel.  The whole contraction is 5 steps, so
// the weights of 64 output channels sit in registers and nothing is streamed: the kernels are
// bound by writing the outputs (fprop) and by reading dz (wgrad).

constexpr int kC8 = 8;

// patch of [pixel][8] plus one zero pixel behind it; returns its size in bytes (multiple of 1 KB)
template <int BM, int NW>
__device__ __forceinline__ int issue_patch_c8(const uint16_t* x8, const uint16_t* zeros, int H, int W, int lw, uint32_t lds_patch,
                                              int p0, int wave, int lane) {
  const int PC = W + 2, NPIX = (BM / W + 2) * PC;
  const int img_px = H * W;
  const int img = p0 / img_px, h0 = (p0 - img * img_px) >> lw;
  const int instrs = ((NPIX + 1) * 16 + 1023) / 1024;
  for (int i = wave; i < instrs; i += NW) {
    const int pp = i * 64 + lane;
    const int pr = pp / PC, pc = pp - pr * PC;
    const int h = h0 + pr - 1, w = pc - 1;
    const bool valid = pp < NPIX && (unsigned)h < (unsigned)H && (unsigned)w < (unsigned)W;
    const uint16_t* ptr = valid ? x8 + ((((long)img * H + h) * W + w) << 3) : zeros;
    dma16_addr(lds_patch + i * 1024, ptr);
  }
  return instrs * 1024;
}
__host__ __device__ inline int patch_c8_bytes(int BM, int W) { return ((((BM / W + 2) * (W + 2) + 1) * 16 + 1023) / 1024) * 1024; }

// out[p][co0 .. co0+63]: 256 pixels per workgroup, 4 waves x (64 pixels x 64 channels)
__global__ __launch_bounds__(256) void conv_c8_fprop_kernel(int P, int H, int W, int lw, int cin, int cout,
                                                           const uint16_t* __restrict__ x8, const uint16_t* __restrict__ zeros,
                                                           const uint16_t* __restrict__ wgt, EpiFprop epi) {
  constexpr int BM = 256;
  extern __shared__ __attribute__((aligned(16))) uint16_t lds_raw[];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int m0 = blockIdx.x * BM, n0 = blockIdx.y * 64;
  issue_patch_c8<BM, 4>(x8, zeros, H, W, lw, lds_addr_of(lds_raw), m0, wave, lane);

  // weights: fragment (kk, j) = channels n0 + 32*j + lane%32, tap 2*kk + lane/32, 8 channel slots
  bf16x8 bfr[5][2];
  const int khalf = lane >> 5;
#pragma unroll
  for (int kk = 0; kk < 5; ++kk)
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int co = n0 + 32 * j + (lane & 31), tap = 2 * kk + khalf;
      shortx8 v = {0, 0, 0, 0, 0, 0, 0, 0};
      if (tap < 9 && co < cout) {
        const uint16_t* wp = wgt + ((size_t)co * 9 + tap) * cin;
#pragma unroll
        for (int c = 0; c < kC8; ++c)
          if (c < cin) v[c] = (short)wp[c];
      }
      bfr[kk][j] = __builtin_bit_cast(bf16x8, v);
    }

  const int PC = W + 2, NPIX = (BM / W + 2) * PC;
  floatx16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
  int ppc[2];
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int q = wave * 64 + i * 32 + (lane & 31);
    ppc[i] = ((q >> lw) + 1) * PC + (q & (W - 1)) + 1;
  }
  wait_vmcnt<0>();
  __syncthreads();
#pragma unroll
  for (int kk = 0; kk < 5; ++kk) {
    const int tap = 2 * kk + khalf;
    const int tapoff = (tap / 3 - 1) * PC + (tap % 3 - 1);
    bf16x8 af[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int pp = tap < 9 ? ppc[i] + tapoff : NPIX;  // the zero pixel behind the patch
      af[i] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(lds_raw + pp * 8));
    }
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j) acc[i][j] = mma<true>(af[i], bfr[kk][j], acc[i][j]);
  }
  __syncthreads();  // the patch is dead: its LDS is reused for the output tiles
  if (n0 + 64 <= cout && (cout & 7) == 0) {
    float* wave_lds = reinterpret_cast<float*>(lds_raw) + wave * (wave_epilogue_bytes<2, 2>() / 4);
    store_tiles_coalesced<2, 2>(acc, epi, m0 + wave * 64, n0, lane, wave_lds);
  } else {
    store_tiles<2, 2>(acc, epi, m0 + wave * 64, n0, P, cout, lane);
  }
}

// partial dW[co0..co0+63][tap][c] over the pixel tiles split, split + splits, ...; 128 pixels per tile.
// Wave w: output channels 32*(w&1).., columns (tap, c) 0..63 (w < 2) or 64..95 (w >= 2; taps 8..11,
// of which only tap 8 exists).
__global__ __launch_bounds__(256) void conv_c8_wgrad_kernel(int H, int W, int lw, int cin, int cout, int px_tiles,
                                                           const uint16_t* __restrict__ x8, const uint16_t* __restrict__ zeros,
                                                           const uint16_t* __restrict__ dz, float* __restrict__ out) {
  constexpr int BM = 128, NW = 4;
  using DZ = ColDma<64, NW>;
  constexpr int kDzInstr = BM * 8 / 64 / NW;
  extern __shared__ __attribute__((aligned(16))) uint16_t lds_raw[];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int cob = blockIdx.x, split = blockIdx.y, splits = gridDim.y;
  const int pbytes = patch_c8_bytes(BM, W);
  const int buf_bytes = pbytes + BM * 128;
  const uint32_t lds_base = lds_addr_of(lds_raw);
  const int PC = W + 2, NPIX = (BM / W + 2) * PC;
  const int rb_co = (wave & 1) * 32;
  const int ntile0 = wave < 2 ? 0 : 2, ntiles = wave < 2 ? 2 : 1;

  floatx16 acc[2];
#pragma unroll
  for (int t = 0; t < 2; ++t)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[t][r] = 0.f;
  uint32_t dzoff[kDzInstr];
#pragma unroll
  for (int i = 0; i < kDzInstr; ++i) {
    const int flat = 64 * (wave + NW * i) + lane;
    const int k = flat >> 3, c = (flat & 7) ^ DZ::swz(k);
    dzoff[i] = (uint32_t)(((size_t)k * cout + cob * 64 + c * 8) * 2);
  }
  auto issue_tile = [&](int tile, int buf) {
    const uint32_t dst = lds_base + buf * buf_bytes;
    issue_patch_c8<BM, NW>(x8, zeros, H, W, lw, dst, tile * BM, wave, lane);
    const uint16_t* src = dz + (size_t)tile * BM * cout;
#pragma unroll
    for (int i = 0; i < kDzInstr; ++i) dma16(dst + pbytes + (wave + NW * i) * 1024, src, dzoff[i]);
  };
  if (split < px_tiles) issue_tile(split, 0);
  int buf = 0;
  const int g = lane >> 4, s = lane & 15;
  for (int tile = split; tile < px_tiles; tile += splits) {
    wait_vmcnt<0>();
    lds_barrier();
    if (tile + splits < px_tiles) issue_tile(tile + splits, buf ^ 1);
    const uint16_t* lp = lds_raw + buf * (buf_bytes / 2);
    const uint16_t* ldz = lp + pbytes / 2;
#pragma unroll 2
    for (int kk = 0; kk < BM / 16; ++kk) {
      const bf16x8 a = DZ::frag(ldz, rb_co, kk, lane);
      const int kq = kk * 16 + 8 * (g >> 1) + (s >> 2);
      const int ppc = ((kq >> lw) + 1) * PC + (kq & (W - 1)) + 1;
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        if (t < ntiles) {
          const int col = (ntile0 + t) * 32 + 16 * (g & 1) + 4 * (s & 3);
          const int tap = col >> 3;
          const int tapoff = (tap / 3 - 1) * PC + (tap % 3 - 1);
          typedef __attribute__((address_space(3))) shortx4* lds_ptr;
          // rows kq and kq + 4 of the lane's 4 columns; taps past the ninth read the zero pixel
          const uint16_t* p0 = lp + (tap < 9 ? ppc + tapoff : NPIX) * 8 + (col & 4);
          const uint16_t* p1 = lp + (tap < 9 ? ppc + 4 + tapoff : NPIX) * 8 + (col & 4);
          const shortx4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(p0));
          const shortx4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(p1));
          const shortx8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
          acc[t] = mma<false>(a, __builtin_bit_cast(bf16x8, v), acc[t]);
        }
      }
    }
    buf ^= 1;
  }
  // accumulator element r: row co = rb_co + 8*(r/4) + 4*(lane/32) + r%4, column lane%32 of the tile
  float* o = out + (size_t)split * cout * 9 * cin;
#pragma unroll
  for (int t = 0; t < 2; ++t) {
    if (t >= ntiles) continue;
    const int col = (ntile0 + t) * 32 + (lane & 31);
    const int tap = col >> 3, c = col & 7;
    if (tap >= 9 || c >= cin) continue;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int co = cob * 64 + rb_co + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
      if (co < cout) o[((size_t)co * 9 + tap) * cin + c] = acc[t][r];
    }
  }
}

// ------------------------------------------------------------------------------------------------
// The same for an R x R kernel at stride S (the 7x7 stride-2 stem of a ResNet-style net), pad (R-1)/2
// ------------------------------------------------------------------------------------------------
// H, W: input image; the output is (H/S) x (W/S).  A tile of BM output pixels is BM/Wo whole output rows of one
// image; its patch holds the S*(BM/Wo - 1) + R input rows they read, W + R - 1 pixels each (pad included), as
// [pixel][8 channel slots], plus one zero pixel.  R*R taps are (R*R + 1)/2 k steps of two taps; the weights of 64
// output channels, laid out [tap][channel][8 slots], are too many for registers (25 steps x 2 fragments) and sit
// in LDS behind the patch.
template <int R, int S>
struct C8S {
  static constexpr int kTaps = R * R, kSteps = (kTaps + 1) / 2, kPad = (R - 1) / 2;
  static constexpr int kWeightBytes = 2 * kSteps * 64 * 16;
  __host__ __device__ static int patch_cols(int W) { return W + R - 1; }
  __host__ __device__ static int patch_rows(int BM, int Wo) { return S * (BM / Wo - 1) + R; }
  __host__ __device__ static int patch_bytes(int BM, int W) {
    return (((patch_rows(BM, W / S) * patch_cols(W) + 1) * 16 + 1023) / 1024) * 1024;
  }
};

// p0: first output pixel of the tile (a multiple of the output row length, inside one image)
template <int R, int S, int BM, int NW>
__device__ __forceinline__ void issue_patch_c8s(const uint16_t* x8, const uint16_t* zeros, int H, int W, int lwo, uint32_t lds_patch,
                                                int p0, int wave, int lane) {
  using G = C8S<R, S>;
  const int Wo = W / S, Ho = H / S;
  const int PC = G::patch_cols(W), NPIX = G::patch_rows(BM, Wo) * PC;
  const int img = p0 / (Ho * Wo), orow0 = (p0 - img * Ho * Wo) >> lwo;
  const int instrs = G::patch_bytes(BM, W) / 1024;
  for (int i = wave; i < instrs; i += NW) {
    const int pp = i * 64 + lane;
    const int pr = pp / PC, pc = pp - pr * PC;
    const int h = S * orow0 - G::kPad + pr, w = pc - G::kPad;
    const bool valid = pp < NPIX && (unsigned)h < (unsigned)H && (unsigned)w < (unsigned)W;
    const uint16_t* ptr = valid ? x8 + ((((long)img * H + h) * W + w) << 3) : zeros;
    dma16_addr(lds_patch + i * 1024, ptr);
  }
}

// out[p][co0 .. co0+63]: 256 output pixels per workgroup, 4 waves x (64 pixels x 64 channels)
template <int R, int S>
__global__ __launch_bounds__(256) void conv_c8s_fprop_kernel(int P, int H, int W, int lwo, int cin, int cout,
                                                            const uint16_t* __restrict__ x8, const uint16_t* __restrict__ zeros,
                                                            const uint16_t* __restrict__ wgt, EpiFprop epi) {
  using G = C8S<R, S>;
  constexpr int BM = 256, KT = G::kTaps, KS = G::kSteps;
  extern __shared__ __attribute__((aligned(16))) uint16_t lds_raw[];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int m0 = blockIdx.x * BM, n0 = blockIdx.y * 64;
  const int Wo = W / S;
  const int PC = G::patch_cols(W), NPIX = G::patch_rows(BM, Wo) * PC;
  const int pbytes = G::patch_bytes(BM, W);
  issue_patch_c8s<R, S, BM, 4>(x8, zeros, H, W, lwo, lds_addr_of(lds_raw), m0, wave, lane);

  // weights -> LDS: entry (tap, channel) = 8 slots, channels >= cin and taps >= R*R zero.  Lanes 8 apart take
  // neighbouring taps of one channel (consecutive in memory), lanes 1 apart neighbouring channels (consecutive in LDS).
  uint16_t* wl = lds_raw + pbytes / 2;
  for (int e = threadIdx.x; e < 64 * 8 * ((2 * KS + 7) / 8); e += 256) {
    const int c = (e & 7) + 8 * ((e >> 6) & 7), tap = ((e >> 3) & 7) + 8 * (e >> 9);
    if (tap >= 2 * KS) continue;
    shortx8 v = {0, 0, 0, 0, 0, 0, 0, 0};
    if (tap < KT && n0 + c < cout) {
      const uint16_t* wp = wgt + ((size_t)(n0 + c) * KT + tap) * cin;
#pragma unroll
      for (int ch = 0; ch < kC8; ++ch)
        if (ch < cin) v[ch] = (short)wp[ch];
    }
    *reinterpret_cast<shortx8*>(wl + (tap * 64 + c) * 8) = v;
  }

  floatx16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
  const int khalf = lane >> 5;
  int ppc[2];  // patch position of tap (0, 0) of the lane's output pixel
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int q = wave * 64 + i * 32 + (lane & 31);
    ppc[i] = S * (q >> lwo) * PC + S * (q & (Wo - 1));
  }
  wait_vmcnt<0>();
  __syncthreads();
#pragma unroll
  for (int kk = 0; kk < KS; ++kk) {
    const int tap = 2 * kk + khalf;
    const int tapoff = (tap / R) * PC + tap % R;
    bf16x8 af[2], bfr[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int pp = tap < KT ? ppc[i] + tapoff : NPIX;  // the zero pixel behind the patch
      af[i] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(lds_raw + pp * 8));
    }
#pragma unroll
    for (int j = 0; j < 2; ++j)
      bfr[j] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(wl + (tap * 64 + j * 32 + (lane & 31)) * 8));
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j) acc[i][j] = mma<true>(af[i], bfr[j], acc[i][j]);
  }
  __syncthreads();  // patch and weights are dead: their LDS is reused for the output tiles
  if (n0 + 64 <= cout && (cout & 7) == 0) {
    float* wave_lds = reinterpret_cast<float*>(lds_raw) + wave * (wave_epilogue_bytes<2, 2>() / 4);
    store_tiles_coalesced<2, 2>(acc, epi, m0 + wave * 64, n0, lane, wave_lds);
  } else {
    store_tiles<2, 2>(acc, epi, m0 + wave * 64, n0, P, cout, lane);
  }
}

// partial dW[co0..co0+63][tap][c] over the output-pixel tiles split, split + splits, ...; 128 output pixels per tile.
// The columns (tap, channel slot) are NT = ceil(R*R*8 / 32) tiles of 32 (4 taps each); waves 0, 1 (output channels
// 0..31, 32..63) take the first half of them, waves 2, 3 the rest.
template <int R, int S>
__global__ __launch_bounds__(256) void conv_c8s_wgrad_kernel(int H, int W, int lwo, int cin, int cout, int px_tiles,
                                                            const uint16_t* __restrict__ x8, const uint16_t* __restrict__ zeros,
                                                            const uint16_t* __restrict__ dz, float* __restrict__ out) {
  using G = C8S<R, S>;
  constexpr int BM = 128, NW = 4, KT = G::kTaps;
  constexpr int NT = (KT * 8 + 31) / 32, TPW = (NT + 1) / 2;
  using DZ = ColDma<64, NW>;
  constexpr int kDzInstr = BM * 8 / 64 / NW;
  extern __shared__ __attribute__((aligned(16))) uint16_t lds_raw[];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int cob = blockIdx.x, split = blockIdx.y, splits = gridDim.y;
  const int Wo = W / S;
  const int pbytes = G::patch_bytes(BM, W);
  const int buf_bytes = pbytes + BM * 128;
  const uint32_t lds_base = lds_addr_of(lds_raw);
  const int PC = G::patch_cols(W), NPIX = G::patch_rows(BM, Wo) * PC;
  const int rb_co = (wave & 1) * 32;
  const int ntile0 = (wave >> 1) * TPW, ntiles = min(TPW, NT - ntile0);

  floatx16 acc[TPW];
#pragma unroll
  for (int t = 0; t < TPW; ++t)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[t][r] = 0.f;
  uint32_t dzoff[kDzInstr];
#pragma unroll
  for (int i = 0; i < kDzInstr; ++i) {
    const int flat = 64 * (wave + NW * i) + lane;
    const int k = flat >> 3, c = (flat & 7) ^ DZ::swz(k);
    dzoff[i] = (uint32_t)(((size_t)k * cout + cob * 64 + c * 8) * 2);
  }
  auto issue_tile = [&](int tile, int buf) {
    const uint32_t dst = lds_base + buf * buf_bytes;
    issue_patch_c8s<R, S, BM, NW>(x8, zeros, H, W, lwo, dst, tile * BM, wave, lane);
    const uint16_t* src = dz + (size_t)tile * BM * cout;
#pragma unroll
    for (int i = 0; i < kDzInstr; ++i) dma16(dst + pbytes + (wave + NW * i) * 1024, src, dzoff[i]);
  };
  if (split < px_tiles) issue_tile(split, 0);
  int buf = 0;
  const int g = lane >> 4, s = lane & 15;
  // the lane's 4 columns (tap, slots 0..3 or 4..7) in each of its column tiles: patch offset of the tap, or -1
  int tapoff[TPW], slot4[TPW];
#pragma unroll
  for (int t = 0; t < TPW; ++t) {
    const int col = (ntile0 + t) * 32 + 16 * (g & 1) + 4 * (s & 3);
    const int tap = col >> 3;
    tapoff[t] = tap < KT ? (tap / R) * PC + tap % R : -1;
    slot4[t] = col & 4;
  }
  for (int tile = split; tile < px_tiles; tile += splits) {
    wait_vmcnt<0>();
    lds_barrier();
    if (tile + splits < px_tiles) issue_tile(tile + splits, buf ^ 1);
    const uint16_t* lp = lds_raw + buf * (buf_bytes / 2);
    const uint16_t* ldz = lp + pbytes / 2;
#pragma unroll 2
    for (int kk = 0; kk < BM / 16; ++kk) {
      const bf16x8 a = DZ::frag(ldz, rb_co, kk, lane);
      const int kq = kk * 16 + 8 * (g >> 1) + (s >> 2);              // output pixel of the tile; kq + 4 lies S*4 input
      const int ppc = S * (kq >> lwo) * PC + S * (kq & (Wo - 1));    // pixels to the right in the same row (Wo >= 8)
#pragma unroll
      for (int t = 0; t < TPW; ++t) {
        if (t < ntiles) {
          typedef __attribute__((address_space(3))) shortx4* lds_ptr;
          const uint16_t* p0 = lp + (tapoff[t] >= 0 ? ppc + tapoff[t] : NPIX) * 8 + slot4[t];
          const uint16_t* p1 = lp + (tapoff[t] >= 0 ? ppc + 4 * S + tapoff[t] : NPIX) * 8 + slot4[t];
          const shortx4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(p0));
          const shortx4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(p1));
          const shortx8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
          acc[t] = mma<false>(a, __builtin_bit_cast(bf16x8, v), acc[t]);
        }
      }
    }
    buf ^= 1;
  }
  // accumulator element r: row co = rb_co + 8*(r/4) + 4*(lane/32) + r%4, column lane%32 of the tile
  float* o = out + (size_t)split * cout * KT * cin;
#pragma unroll
  for (int t = 0; t < TPW; ++t) {
    if (t >= ntiles) continue;
    const int col = (ntile0 + t) * 32 + (lane & 31);
    const int tap = col >> 3, c = col & 7;
    if (tap >= KT || c >= cin) continue;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int co = cob * 64 + rb_co + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
      if (co < cout) o[((size_t)co * KT + tap) * cin + c] = acc[t][r];
    }
  }
}

// x[P][cin] -> x8[P][8], channels >= cin zero
__global__ __launch_bounds__(256) void pad_channels_kernel(size_t pixels, int cin, const uint16_t* __restrict__ x,
                                                           uint16_t* __restrict__ x8) {
  for (size_t p = (size_t)blockIdx.x * 256 + threadIdx.x; p < pixels; p += (size_t)gridDim.x * 256) {
    shortx8 v = {0, 0, 0, 0, 0, 0, 0, 0};
    for (int c = 0; c < kC8; ++c)
      if (c < cin) v[c] = (short)x[p * cin + c];
    *reinterpret_cast<shortx8*>(x8 + p * 8) = v;
  }
}

inline bool pow2(int v) { return v > 0 && (v & (v - 1)) == 0; }
inline int ilog2(int v) { int l = 0; while ((1 << l) < v) ++l; return l; }

}  // namespace

constexpr int kMaxLds = 160 * 1024;

inline bool patch_shape_ok(int H, int W, int BM) {
  return pow2(H) && pow2(W) && W >= 8 && BM % W == 0 && (H * W) % BM == 0;
}

template <int BM, int BN, int WGM, int WGN, int NS, bool BWD, class Epi>
struct PatchCfg {
  using BL = Plain<BN, WGM * WGN, BWD>;
  static size_t lds(int W, int CB) {
    const size_t loop = (size_t)patch_bytes(BM, W, CB) + (size_t)NS * BL::kBytes;
    const size_t epi = (size_t)WGM * WGN * wave_epilogue_bytes<BM / WGM / 32, BN / WGN / 32>();
    return std::max(loop, epi);
  }
  static bool ok(int H, int W, int C) { return patch_shape_ok(H, W, BM) && lds(W, C / 8) <= kMaxLds; }
  static long tiles(long P, int N) { return (P / BM) * ((N + BN - 1) / BN); }
  static hipError_t launch(hipStream_t s, int P, int N, const PatchDesc& pd, const PlainDesc& bd, const Epi& e) {
    auto kernel = conv_patch_kernel<BM, BN, WGM, WGN, NS, BWD, BL, Epi>;
    static hipError_t attr =
        hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, kMaxLds);
    if (attr != hipSuccess) return attr;
    const int tiles_n = (N + BN - 1) / BN;
    hipLaunchKernelGGL(kernel, dim3((unsigned)(P / BM * tiles_n)), dim3(64 * WGM * WGN), lds(pd.W, pd.CB), s, P, N, pd, bd, e,
                       tiles_n);
    return hipGetLastError();
  }
};

// The largest tile that still gives every CU a workgroup; failing that, the one with the most
// workgroups.  Returns hipErrorNotSupported when no patch tile fits the shape.
template <bool BWD, class Epi>
hipError_t launch_patch_conv(hipStream_t s, int P, int H, int W, int C, int N, const PatchDesc& pd, const PlainDesc& bd,
                             const Epi& e) {
  using A = PatchCfg<256, 128, 4, 2, 3, BWD, Epi>;
  using B = PatchCfg<256, 64, 4, 2, 3, BWD, Epi>;
  using Cc = PatchCfg<128, 128, 2, 2, 3, BWD, Epi>;
  using D = PatchCfg<128, 64, 2, 2, 4, BWD, Epi>;
  const bool wide = N % 128 == 0;
  const bool ok[4] = {wide && A::ok(H, W, C), B::ok(H, W, C), wide && Cc::ok(H, W, C), D::ok(H, W, C)};
  const long tiles[4] = {A::tiles(P, N), B::tiles(P, N), Cc::tiles(P, N), D::tiles(P, N)};
  int pick = -1;
  for (int i = 0; i < 4 && pick < 0; ++i)
    if (ok[i] && tiles[i] >= 256) pick = i;
  if (pick < 0)
    for (int i = 0; i < 4; ++i)
      if (ok[i] && (pick < 0 || tiles[i] > tiles[pick])) pick = i;
  switch (pick) {
    case 0: return A::launch(s, P, N, pd, bd, e);
    case 1: return B::launch(s, P, N, pd, bd, e);
    case 2: return Cc::launch(s, P, N, pd, bd, e);
    case 3: return D::launch(s, P, N, pd, bd, e);
    default: return hipErrorNotSupported;
  }
}

constexpr int kWgradBM = 128;
inline size_t wgrad_patch_lds(int W) { return 2 * ((size_t)patch_bytes(kWgradBM, W, 8) + kWgradBM * 128); }
inline bool wgrad_patch_ok(int H, int W) { return patch_shape_ok(H, W, kWgradBM) && wgrad_patch_lds(W) <= kMaxLds; }
inline int wgrad_patch_splits(long px_tiles, int cin, int cout) {
  const long blocks = std::max(1l, (long)(cin / 64) * (cout / 64));
  return (int)std::max(1l, std::min(px_tiles, 256 / blocks));
}

bool conv_mfma_supported(int imgs, int H, int W, int stride, int cin, int cout) {
  const long P = (long)imgs * H * W, Pout = P / (stride * stride);
  if (stride != 1 && !(stride == 2 && H >= 2 && W >= 2)) return false;
  return pow2(H) && pow2(W) && H <= 32768 && W <= 32768 && cin % 64 == 0 && cout % 64 == 0 && Pout % 64 == 0 &&
         P * std::max(cin, cout) * 2 < (1l << 31);
}

// most partial sums either matrix-core wgrad kernel may write for this layer
int conv_mfma_wgrad_max_splits(int pixels, int cin, int cout) {
  const int c8 = cin <= 8 && cout % 64 == 0 ? std::max(1, std::min(pixels / 128, 512 / (cout / 64))) : 1;
  return std::max({conv_mfma_wgrad_splits(pixels, cin, cout), wgrad_patch_splits(pixels / kWgradBM, cin, cout), c8});
}

// pixel ranges for wgrad: enough workgroups to fill the chip, at least 4 k tiles each
int conv_mfma_wgrad_splits(int pixels, int cin, int cout) {
  const int tiles = ((cout + 63) / 64) * ((cin + 63) / 64) * 9;
  const int kt = pixels / 64;
  int s = std::max(1, 512 / tiles);
  while (s > 1 && (kt % s != 0 || kt / s < 4)) --s;
  return s;
}

// Gathered fprop / dgrad: the largest tile that still gives every CU a workgroup, else the smallest.
template <bool BWD, int S, class Epi>
hipError_t launch_gather_rows(hipStream_t s, int P, int N, int KT, const GatherDesc& ad, const PlainDesc& bd, const Epi& e) {
  const long rows128 = (P + 127) / 128;
  if (N % 128 == 0 && rows128 * (N / 128) >= 256)
    return launch_conv<128, 128, 3, RowGather<128, 4, BWD, S>, Plain<128, 4, BWD>>(s, P, N, KT, 1, 1, ad, bd, e);
  if (rows128 * ((N + 63) / 64) >= 256)
    return launch_conv<128, 64, 4, RowGather<128, 4, BWD, S>, Plain<64, 4, BWD>>(s, P, N, KT, 1, 1, ad, bd, e);
  // no more than half the CUs get a 64 x 64 tile and the contraction is long: two groups of waves share it
  const long tiles64 = (long)((P + 63) / 64) * ((N + 63) / 64);
  if (tiles64 <= 128 && KT % 2 == 0 && KT >= 8)
    return launch_conv<64, 64, 4, RowGather<64, 4, BWD, S>, Plain<64, 4, BWD>, Epi, 2>(s, P, N, KT, 1, 1, ad, bd, e);
  return launch_conv<64, 64, 4, RowGather<64, 4, BWD, S>, Plain<64, 4, BWD>>(s, P, N, KT, 1, 1, ad, bd, e);
}

hipError_t conv_mfma_fprop(hipStream_t s, int imgs, int H, int W, int stride, int cin, int cout, const uint16_t* x,
                           const uint16_t* wgt, const float* bias, int act, uint16_t* d_out, uint16_t* a_out,
                           const uint16_t* zeros) {
  PlainDesc bd{wgt, 9 * cin, cout, 1 << 30, DBK, 0};
  EpiFprop e{bias, d_out, a_out, act, cout};
  const int KT = 9 * cin / DBK;
  if (stride == 2) {  // rows: output pixels on the (H/2) x (W/2) grid, source: the input
    const int Ho = H / 2, Wo = W / 2, P = imgs * Ho * Wo;
    GatherDesc ad{x, zeros, P, Ho, Wo, ilog2(Wo), cin, H, W};
    return launch_gather_rows<false, 2>(s, P, cout, KT, ad, bd, e);
  }
  const int P = imgs * H * W;
  {
    const PatchDesc pd{x, zeros, H, W, ilog2(W), cin, 0, cin / 8, 0};
    const hipError_t err = launch_patch_conv<false>(s, P, H, W, cin, cout, pd, bd, e);
    if (err != hipErrorNotSupported) return err;
  }
  GatherDesc ad{x, zeros, P, H, W, ilog2(W), cin, H, W};
  return launch_gather_rows<false, 1>(s, P, cout, KT, ad, bd, e);
}

hipError_t conv_mfma_dgrad(hipStream_t s, int imgs, int H, int W, int stride, int cin, int cout, const uint16_t* dz,
                           const uint16_t* wb, const uint16_t* d_prev, uint16_t* out, const uint16_t* zeros, int relu_mask) {
  const int P = imgs * H * W;
  // k tile -> (tap, block of 64 output channels): rows co0.. of W_b, columns tap*Cin..
  PlainDesc bd{wb, 9 * cin, cin, cout / DBK, (long)DBK * 9 * cin, cin};
  EpiDgrad e{d_prev, out, cin, relu_mask};
  if (stride == 2) {  // one batch of workgroups per parity class of input pixels, each with its own taps
    const int H2 = H / 2, W2 = W / 2, Pc = imgs * H2 * W2;
    GatherDesc ad{dz, zeros, Pc, H2, W2, ilog2(W2), cout, H2, W2};
    EpiDgradS2 e2{e, H, W, ilog2(W2), ilog2(H2)};
    const int KT = 4 * cout / DBK;  // of the class with four taps; the kernel takes every class's own count
    const long rows128 = (Pc + 127) / 128;
    if (cin % 128 == 0 && 4 * rows128 * (cin / 128) >= 256)
      return launch_conv<128, 128, 3, RowGatherS2<128, 4>, PlainS2<128, 4>>(s, Pc, cin, KT, 4, 1, ad, bd, e2);
    if (4 * rows128 * ((cin + 63) / 64) >= 256)
      return launch_conv<128, 64, 4, RowGatherS2<128, 4>, PlainS2<64, 4>>(s, Pc, cin, KT, 4, 1, ad, bd, e2);
    return launch_conv<64, 64, 4, RowGatherS2<64, 4>, PlainS2<64, 4>>(s, Pc, cin, KT, 4, 1, ad, bd, e2);
  }
  {
    const PatchDesc pd{dz, zeros, H, W, ilog2(W), cout, 0, cout / 8, 0};
    const hipError_t err = launch_patch_conv<true>(s, P, H, W, cout, cin, pd, bd, e);
    if (err != hipErrorNotSupported) return err;
  }
  GatherDesc ad{dz, zeros, P, H, W, ilog2(W), cout, H, W};
  return launch_gather_rows<true, 1>(s, P, cin, 9 * cout / DBK, ad, bd, e);
}

hipError_t conv_mfma_wgrad(hipStream_t s, int imgs, int H, int W, int stride, int cin, int cout, const uint16_t* dz,
                           const uint16_t* x, float* gW, float* partial, const uint16_t* zeros) {
  const size_t count = (size_t)cout * 9 * cin;
  if (stride == 2) {  // contraction over the output pixels; x is gathered at 2*(oh, ow) + tap
    const int Ho = H / 2, Wo = W / 2, P = imgs * Ho * Wo;
    const int splits = conv_mfma_wgrad_splits(P, cin, cout);
    const int KT = P / DBK / splits;
    PlainDesc ad{dz, cout, cout, 1 << 30, (long)DBK * cout, 0};
    GatherDesc bd{x, zeros, P, Ho, Wo, ilog2(Wo), cin, H, W};
    EpiWgradConv e{splits > 1 ? partial : gW, cin, cout};
    hipError_t err;
    if (cout % 128 == 0 && cin % 128 == 0 && (long)(cout / 128) * (cin / 128) * 9 * splits >= 256)
      err = launch_conv<128, 128, 3, Plain<128, 4, true>, ColGather<128, 4, 2>>(s, cout, cin, KT, 9, splits, ad, bd, e);
    else
      err = launch_conv<64, 64, 4, Plain<64, 4, true>, ColGather<64, 4, 2>>(s, cout, cin, KT, 9, splits, ad, bd, e);
    if (err != hipSuccess || splits == 1) return err;
    return launch_sum_partials(s, count, splits, partial, gW);
  }
  const int P = imgs * H * W;
  if (wgrad_patch_ok(H, W)) {
    const int px_tiles = P / kWgradBM;
    const int splits = wgrad_patch_splits(px_tiles, cin, cout);
    const PatchDesc xd{x, zeros, H, W, ilog2(W), cin, 0, 8, 1};
    auto kernel = conv_wgrad_patch_kernel<kWgradBM>;
    static hipError_t attr =
        hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, kMaxLds);
    if (attr != hipSuccess) return attr;
    hipLaunchKernelGGL(kernel, dim3((cin / 64) * (cout / 64), splits), dim3(256), wgrad_patch_lds(W), s, xd, dz, cout, px_tiles,
                       cin / 64, splits > 1 ? partial : gW);
    hipError_t err = hipGetLastError();
    if (err != hipSuccess || splits == 1) return err;
    return launch_sum_partials(s, count, splits, partial, gW);
  }
  const int splits = conv_mfma_wgrad_splits(P, cin, cout);
  const int KT = P / DBK / splits;
  PlainDesc ad{dz, cout, cout, 1 << 30, (long)DBK * cout, 0};
  GatherDesc bd{x, zeros, P, H, W, ilog2(W), cin, H, W};
  EpiWgradConv e{splits > 1 ? partial : gW, cin, cout};
  hipError_t err;
  if (cout % 128 == 0 && cin % 128 == 0 && (long)(cout / 128) * (cin / 128) * 9 * splits >= 256)
    err = launch_conv<128, 128, 3, Plain<128, 4, true>, ColGather<128, 4>>(s, cout, cin, KT, 9, splits, ad, bd, e);
  else
    err = launch_conv<64, 64, 4, Plain<64, 4, true>, ColGather<64, 4>>(s, cout, cin, KT, 9, splits, ad, bd, e);
  if (err != hipSuccess || splits == 1) return err;
  return launch_sum_partials(s, count, splits, partial, gW);
}

// ---- first layer (cin <= 8) on a padded [pixel][8] copy of the input -------------------------
bool conv_c8_supported(int imgs, int H, int W, int cin, int cout) {
  const long P = (long)imgs * H * W;
  return cin >= 1 && cin <= kC8 && cout % 64 == 0 && patch_shape_ok(H, W, 256) && patch_shape_ok(H, W, 128) &&
         P * 16 < (1l << 31) &&
         P * cout * 2 < (1l << 31);
}

hipError_t conv_c8_pad(hipStream_t s, size_t pixels, int cin, const uint16_t* x, uint16_t* x8) {
  const unsigned blocks = (unsigned)std::min<size_t>((pixels + 255) / 256, 4096);
  hipLaunchKernelGGL(pad_channels_kernel, dim3(blocks), dim3(256), 0, s, pixels, cin, x, x8);
  return hipGetLastError();
}

hipError_t conv_c8_fprop(hipStream_t s, int imgs, int H, int W, int cin, int cout, const uint16_t* x8, const uint16_t* wgt,
                         const float* bias, int act, uint16_t* d_out, uint16_t* a_out, const uint16_t* zeros) {
  const int P = imgs * H * W;
  const size_t lds = std::max<size_t>(patch_c8_bytes(256, W), 4 * wave_epilogue_bytes<2, 2>());
  static hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(conv_c8_fprop_kernel),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, kMaxLds);
  if (attr != hipSuccess) return attr;
  if (lds > (size_t)kMaxLds) return hipErrorInvalidValue;
  hipLaunchKernelGGL(conv_c8_fprop_kernel, dim3(P / 256, cout / 64), dim3(256), lds, s, P, H, W, ilog2(W), cin, cout, x8, zeros,
                     wgt, EpiFprop{bias, d_out, a_out, act, cout});
  return hipGetLastError();
}

int conv_c8_wgrad_splits(int pixels, int cout) { return std::max(1, std::min(pixels / 128, 512 / (cout / 64))); }

hipError_t conv_c8_wgrad(hipStream_t s, int imgs, int H, int W, int cin, int cout, const uint16_t* dz, const uint16_t* x8,
                         float* gW, float* partial, const uint16_t* zeros) {
  const int P = imgs * H * W;
  const int px_tiles = P / 128;
  const int splits = conv_c8_wgrad_splits(P, cout);
  const size_t lds = 2 * ((size_t)patch_c8_bytes(128, W) + 128 * 128);
  static hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(conv_c8_wgrad_kernel),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, kMaxLds);
  if (attr != hipSuccess) return attr;
  if (lds > (size_t)kMaxLds) return hipErrorInvalidValue;
  hipLaunchKernelGGL(conv_c8_wgrad_kernel, dim3(cout / 64, splits), dim3(256), lds, s, H, W, ilog2(W), cin, cout, px_tiles, x8,
                     zeros, dz, splits > 1 ? partial : gW);
  hipError_t err = hipGetLastError();
  if (err != hipSuccess || splits == 1) return err;
  return launch_sum_partials(s, (size_t)cout * 9 * cin, splits, partial, gW);
}

// ---- the same for the 7x7 stride-2 stem ---------------------------------------------------------
namespace {
using Stem = C8S<7, 2>;
inline size_t stem_fprop_lds(int W) {
  return std::max<size_t>((size_t)Stem::patch_bytes(256, W) + Stem::kWeightBytes, 4 * wave_epilogue_bytes<2, 2>());
}
inline size_t stem_wgrad_lds(int W) { return 2 * ((size_t)Stem::patch_bytes(128, W) + 128 * 128); }
}  // namespace

bool conv_stem_supported(int imgs, int H, int W, int cin, int cout) {
  if (!(pow2(H) && pow2(W) && H >= 2 && W >= 16)) return false;
  const int Ho = H / 2, Wo = W / 2;
  const long P = (long)imgs * H * W;
  return cin >= 1 && cin <= kC8 && cout % 64 == 0 && 128 % Wo == 0 && (Ho * Wo) % 256 == 0 &&
         stem_fprop_lds(W) <= (size_t)kMaxLds && stem_wgrad_lds(W) <= (size_t)kMaxLds && P * 16 < (1l << 31) &&
         (P / 4) * cout * 2 < (1l << 31);
}

hipError_t conv_stem_fprop(hipStream_t s, int imgs, int H, int W, int cin, int cout, const uint16_t* x8, const uint16_t* wgt,
                           const float* bias, int act, uint16_t* d_out, uint16_t* a_out, const uint16_t* zeros) {
  if (!conv_stem_supported(imgs, H, W, cin, cout)) return hipErrorInvalidValue;
  const int P = imgs * (H / 2) * (W / 2);
  auto kernel = conv_c8s_fprop_kernel<7, 2>;
  static hipError_t attr =
      hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, kMaxLds);
  if (attr != hipSuccess) return attr;
  hipLaunchKernelGGL(kernel, dim3(P / 256, cout / 64), dim3(256), stem_fprop_lds(W), s, P, H, W, ilog2(W / 2), cin, cout, x8,
                     zeros, wgt, EpiFprop{bias, d_out, a_out, act, cout});
  return hipGetLastError();
}

int conv_stem_wgrad_splits(int out_pixels, int cout) { return std::max(1, std::min(out_pixels / 128, 512 / (cout / 64))); }

hipError_t conv_stem_wgrad(hipStream_t s, int imgs, int H, int W, int cin, int cout, const uint16_t* dz, const uint16_t* x8,
                           float* gW, float* partial, const uint16_t* zeros) {
  if (!conv_stem_supported(imgs, H, W, cin, cout)) return hipErrorInvalidValue;
  const int P = imgs * (H / 2) * (W / 2);
  const int px_tiles = P / 128;
  const int splits = conv_stem_wgrad_splits(P, cout);
  auto kernel = conv_c8s_wgrad_kernel<7, 2>;
  static hipError_t attr =
      hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, kMaxLds);
  if (attr != hipSuccess) return attr;
  hipLaunchKernelGGL(kernel, dim3(cout / 64, splits), dim3(256), stem_wgrad_lds(W), s, H, W, ilog2(W / 2), cin, cout, px_tiles, x8,
                     zeros, dz, splits > 1 ? partial : gW);
  hipError_t err = hipGetLastError();
  if (err != hipSuccess || splits == 1) return err;
  return launch_sum_partials(s, (size_t)cout * 49 * cin, splits, partial, gW);
}

}  // namespace tp
