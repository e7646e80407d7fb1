// bf16 GEMMs on the gfx950 matrix cores (v_mfma_f32_32x32x16_bf16, fp32 accumulate).
//
// One kernel template covers the three products of a dense layer.  With C[M x N] = A . B:
//   fprop  z  = x W^T      A = x  [M][K] (k contiguous)   B = W   [N][K] (k contiguous)
//   dgrad  dx = dz W_b     A = dz [M][K] (k contiguous)   B = W_b [K][N] (n contiguous)
//   wgrad  dW = dz^T x     A = dz [K][M] (m contiguous)   B = x   [K][N] (n contiguous)
// An operand whose contraction index is the contiguous one is staged in LDS row by row and
// each lane reads its 8 consecutive k values with one 128-bit LDS read.  An operand whose
// contraction index is the strided one is staged as it lies in memory ([k][row]) and each
// lane gets its 8 k values through two LDS transpose reads.
//
// Block: 256 threads = 4 waves in a 2 x 2 grid, block tile BM x BN, k tile 64, LDS double
// buffered with one barrier per k tile; global loads of tile t+1 are in flight while the
// matrix cores work on tile t.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "device_utils.h"
#include "gemm_mfma.h"

namespace tp {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int BK = 64;        // k extent of one LDS tile
constexpr int kThreads = 256;
constexpr int ROW_LD = BK + 8;  // bf16 per LDS row of a k-contiguous tile (144 B: conflict-free b128 reads)

// ---- staging of one operand tile -------------------------------------------------------------
// k-contiguous operand: tile [R rows][64 k]; memory element (r, k) at base[r*ld + k].
template <int R>
struct RowTile {
  static constexpr int kChunks = R * (BK / 8) / kThreads;  // 16-byte chunks per thread
  static constexpr int kLdsElems = R * ROW_LD;
  uint4 regs[kChunks];

  __device__ __forceinline__ void load(const uint16_t* __restrict__ base, int ld, int r0, int rows, int k0, int K) {
    const int c = threadIdx.x & 7;
#pragma unroll
    for (int i = 0; i < kChunks; ++i) {
      const int r = (threadIdx.x >> 3) + 32 * i;
      const int gr = min(r0 + r, rows - 1);           // clamp: rows past the edge are never stored
      const int k = k0 + c * 8;
      regs[i] = k < K ? *reinterpret_cast<const uint4*>(base + (size_t)gr * ld + k) : make_uint4(0, 0, 0, 0);
    }
  }
  __device__ __forceinline__ void store(uint16_t* lds) const {
    const int c = threadIdx.x & 7;
#pragma unroll
    for (int i = 0; i < kChunks; ++i) {
      const int r = (threadIdx.x >> 3) + 32 * i;
      *reinterpret_cast<uint4*>(lds + r * ROW_LD + c * 8) = regs[i];
    }
  }
  // operand rows rbase..rbase+31: lane reads the 8 consecutive k = kk*16 + 8*(lane/32).. of row rbase + lane%32
  static __device__ __forceinline__ bf16x8 frag(const uint16_t* lds, int rbase, int kk, int lane) {
    const uint4 v = *reinterpret_cast<const uint4*>(lds + (rbase + (lane & 31)) * ROW_LD + kk * 16 + (lane >> 5) * 8);
    return __builtin_bit_cast(bf16x8, v);
  }
};

// k-strided operand: tile [64 k][R rows]; memory element (r, k) at base[k*ld + r].
// Fragments come from the LDS transpose read (ds_read_b64_tr_b16): within each group of 16
// lanes, lane s supplies the address of 4 consecutive bf16 and receives element s%4 of the
// four lanes 4*j + s/4 (j = 0..3).  With lane s pointing at row k0 + s/4, columns
// c0 + 4*(s%4) .. +3, lane i of the group ends up with rows k0..k0+3 of column c0 + i: four
// consecutive k of its own row/column of the MFMA operand.  Two such reads give the 8 k values.
typedef short shortx4 __attribute__((ext_vector_type(4)));
typedef short shortx8 __attribute__((ext_vector_type(8)));

template <int R>
struct ColTile {
  static constexpr int LD = R + 32;  // row stride = 64 B (mod 256 B): the 4 rows of a transpose read hit distinct banks
  static constexpr int kChunks = BK * (R / 8) / kThreads;
  static constexpr int kLdsElems = BK * LD;
  static constexpr int kChunksPerK = R / 8;
  uint4 regs[kChunks];

  __device__ __forceinline__ void load(const uint16_t* __restrict__ base, int ld, int r0, int rows, int k0, int K) {
#pragma unroll
    for (int i = 0; i < kChunks; ++i) {
      const int id = threadIdx.x + kThreads * i;
      const int c = id % kChunksPerK, k = id / kChunksPerK;
      const int r = r0 + c * 8;
      const bool ok = (k0 + k < K) && (r + 8 <= rows);
      regs[i] = ok ? *reinterpret_cast<const uint4*>(base + (size_t)(k0 + k) * ld + r) : make_uint4(0, 0, 0, 0);
    }
  }
  __device__ __forceinline__ void store(uint16_t* lds) const {
#pragma unroll
    for (int i = 0; i < kChunks; ++i) {
      const int id = threadIdx.x + kThreads * i;
      const int c = id % kChunksPerK, k = id / kChunksPerK;
      *reinterpret_cast<uint4*>(lds + k * LD + c * 8) = regs[i];
    }
  }
  // operand rows rbase..rbase+31, k = kk*16 + 8*(lane/32) .. +7 for row rbase + lane%32
  static __device__ __forceinline__ bf16x8 frag(const uint16_t* lds, int rbase, int kk, int lane) {
    const int g = lane >> 4, s = lane & 15;
    const int k = kk * 16 + 8 * (g >> 1) + (s >> 2);
    const int c = rbase + 16 * (g & 1) + 4 * (s & 3);
    typedef __attribute__((address_space(3))) shortx4* lds_ptr;
    const uint16_t* p = lds + k * LD + c;
    const shortx4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(p));
    const shortx4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(p + 4 * LD));
    const shortx8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, v);
  }
};

template <int R, bool COL>
struct TileSel { using type = RowTile<R>; };
template <int R>
struct TileSel<R, true> { using type = ColTile<R>; };

// ---- epilogues: called once per accumulator element with its (m, n) ---------------------------
struct EpiFprop {
  const float* bias; uint16_t* z_out; uint16_t* a_out; int act; int ldc;
  __device__ __forceinline__ void operator()(int m, int n, float v) const {
    v += bias[n];
    const size_t i = (size_t)m * ldc + n;
    if (z_out) z_out[i] = float_to_bf16(v);
    a_out[i] = float_to_bf16(act_forward(v, act));
  }
};
struct EpiDgrad {
  const uint16_t* z_prev; uint16_t* out; int act; int ldc;
  __device__ __forceinline__ void operator()(int m, int n, float v) const {
    const size_t i = (size_t)m * ldc + n;
    if (z_prev) v *= act_derivative(bf16_to_float(z_prev[i]), act);
    out[i] = float_to_bf16(v);
  }
};
struct EpiWgrad {
  float* out; int ldc;
  __device__ __forceinline__ void operator()(int m, int n, float v) const { out[(size_t)m * ldc + n] = v; }
};

template <int BM, int BN, bool A_COL, bool B_COL, class Epi>
__global__ __launch_bounds__(kThreads) void gemm_bf16_mfma_kernel(int M, int N, int K, const uint16_t* __restrict__ A,
                                                                  int lda, const uint16_t* __restrict__ B, int ldb,
                                                                  Epi epi) {
  using ATile = typename TileSel<BM, A_COL>::type;
  using BTile = typename TileSel<BN, B_COL>::type;
  constexpr int WM = BM / 2, WN = BN / 2;  // wave tile
  constexpr int TM = WM / 32, TN = WN / 32;
  extern __shared__ __attribute__((aligned(16))) uint16_t lds_raw[];
  auto lds_a = [&](int buf) { return lds_raw + buf * ATile::kLdsElems; };
  auto lds_b = [&](int buf) { return lds_raw + 2 * ATile::kLdsElems + buf * BTile::kLdsElems; };

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm = (wave >> 1) * WM, wn = (wave & 1) * WN;
  const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;

  floatx16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  ATile ta;
  BTile tb;
  const int KT = (K + BK - 1) / BK;
  ta.load(A, lda, m0, M, 0, K);
  tb.load(B, ldb, n0, N, 0, K);
  ta.store(lds_a(0));
  tb.store(lds_b(0));
  __syncthreads();
  for (int kt = 0; kt < KT; ++kt) {
    const int cur = kt & 1;
    if (kt + 1 < KT) {
      ta.load(A, lda, m0, M, (kt + 1) * BK, K);
      tb.load(B, ldb, n0, N, (kt + 1) * BK, K);
    }
#pragma unroll
    for (int kk = 0; kk < BK / 16; ++kk) {
      bf16x8 af[TM], bfr[TN];
#pragma unroll
      for (int i = 0; i < TM; ++i) af[i] = ATile::frag(lds_a(cur), wm + i * 32, kk, lane);
#pragma unroll
      for (int j = 0; j < TN; ++j) bfr[j] = BTile::frag(lds_b(cur), wn + j * 32, kk, lane);
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
    }
    if (kt + 1 < KT) {
      ta.store(lds_a(cur ^ 1));
      tb.store(lds_b(cur ^ 1));
    }
    __syncthreads();
  }
  // accumulator element r of a lane: row 8*(r/4) + 4*(lane/32) + r%4, column lane%32
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const int n = n0 + wn + j * 32 + (lane & 31);
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int m = m0 + wm + i * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
        if (m < M && n < N) epi(m, n, acc[i][j][r]);
      }
    }
}

template <int BM, int BN, bool A_COL, bool B_COL, class Epi>
hipError_t launch(hipStream_t s, int M, int N, int K, const uint16_t* A, int lda, const uint16_t* B, int ldb,
                  const Epi& epi) {
  using ATile = typename TileSel<BM, A_COL>::type;
  using BTile = typename TileSel<BN, B_COL>::type;
  constexpr size_t lds_bytes = 2 * (ATile::kLdsElems + BTile::kLdsElems) * sizeof(uint16_t);
  auto kernel = gemm_bf16_mfma_kernel<BM, BN, A_COL, B_COL, Epi>;
  if (lds_bytes > 64 * 1024) {
    static hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
    if (attr != hipSuccess) return attr;
  }
  dim3 grid((N + BN - 1) / BN, (M + BM - 1) / BM);
  hipLaunchKernelGGL(kernel, grid, dim3(kThreads), lds_bytes, s, M, N, K, A, lda, B, ldb, epi);
  return hipGetLastError();
}

}  // namespace

// Contraction extents must be a multiple of 8 (16-byte chunks along k); operands that are staged
// [k][row] also need their row extent to be a multiple of 8.
bool mfma_fprop_supported(int M, int N, int K) { return M >= 1 && N >= 1 && K % 8 == 0; }
bool mfma_dgrad_supported(int M, int N, int K) { return M >= 1 && N % 8 == 0 && K % 8 == 0; }
bool mfma_wgrad_supported(int M, int N, int K) { return M >= 1 && N % 8 == 0 && K % 8 == 0; }

hipError_t mfma_fprop(hipStream_t s, int M, int N, int K, const uint16_t* x, const uint16_t* W, const float* bias,
                      int act, uint16_t* z_out, uint16_t* a_out) {
  EpiFprop e{bias, z_out, a_out, act, N};
  if (M <= 64) return launch<64, 64, false, false>(s, M, N, K, x, K, W, K, e);
  return launch<128, 128, false, false>(s, M, N, K, x, K, W, K, e);
}

hipError_t mfma_dgrad(hipStream_t s, int M, int N, int K, const uint16_t* dz, const uint16_t* Wb,
                      const uint16_t* z_prev, int act_prev, uint16_t* out) {
  // out[M x K] = dz[M x N] . Wb[N x K]: GEMM (M, K, contraction N)
  EpiDgrad e{z_prev, out, act_prev, K};
  if (M <= 64) return launch<64, 64, false, true>(s, M, K, N, dz, N, Wb, K, e);
  return launch<128, 128, false, true>(s, M, K, N, dz, N, Wb, K, e);
}

hipError_t mfma_wgrad(hipStream_t s, int M, int N, int K, const uint16_t* dz, const uint16_t* x, float* gW) {
  // gW[N x K] = dz^T[N x M] . x[M x K]: GEMM (N, K, contraction M)
  EpiWgrad e{gW, K};
  if (N <= 64 || K <= 64) return launch<64, 64, true, true>(s, N, K, M, dz, N, x, K, e);
  return launch<128, 128, true, true>(s, N, K, M, dz, N, x, K, e);
}

}  // namespace tp
