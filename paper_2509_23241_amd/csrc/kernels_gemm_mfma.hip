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
// Two kernels share the tile and epilogue code:
//   gemm_bf16_mfma_kernel  any shape whose extents are multiples of 8: global loads go through
//                          registers, one k tile ahead, LDS double buffered and padded.
//   gemm_bf16_dma_kernel   contraction extent a multiple of 64: global loads write LDS directly
//                          (global_load_lds_dwordx4), NS stages deep, no staging registers; LDS is
//                          unpadded, bank conflicts are avoided by an XOR swizzle of the 16-byte
//                          chunks, applied on the global side of the copy.
// Workgroup ids are remapped so that the workgroups of one XCD (ids equal mod 8) cover a
// compact 2-D patch of output tiles and share their operand panels in that XCD's L2.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <stdint.h>

#include "device_utils.h"
#include "gemm_mfma.h"
#include "mfma_common.h"
#include "kernels.h"

namespace tp {

namespace {


// ---- staging of one operand tile -------------------------------------------------------------
// k-contiguous operand: tile [R rows][BKT k]; memory element (r, k) at base[r*ld + k].
template <int R, int BKT, int NT>
struct RowTile {
  static constexpr int LD = BKT + 8;             // +16 B per row: conflict-free 128-bit reads
  static constexpr int kPerRow = BKT / 8;        // 16-byte chunks per row
  static constexpr int kChunks = R * kPerRow / NT;
  static constexpr int kRowStep = NT / kPerRow;
  static constexpr int kLdsElems = R * LD;
  static_assert(R * kPerRow % NT == 0, "tile does not divide among the threads");

  static __device__ __forceinline__ void load(uint4 (&regs)[kChunks], const uint16_t* __restrict__ base, int ld, int r0,
                                              int rows, int k0, int K) {
    const int c = threadIdx.x % kPerRow;
    const int k = k0 + c * 8;
#pragma unroll
    for (int i = 0; i < kChunks; ++i) {
      const int r = threadIdx.x / kPerRow + kRowStep * i;
      const int gr = min(r0 + r, rows - 1);  // clamp: rows past the edge are computed but never stored
      regs[i] = k < K ? *reinterpret_cast<const uint4*>(base + (size_t)gr * ld + k) : make_uint4(0, 0, 0, 0);
    }
  }
  static __device__ __forceinline__ void store(const uint4 (&regs)[kChunks], uint16_t* lds) {
    const int c = threadIdx.x % kPerRow;
#pragma unroll
    for (int i = 0; i < kChunks; ++i) {
      const int r = threadIdx.x / kPerRow + kRowStep * i;
      *reinterpret_cast<uint4*>(lds + r * LD + c * 8) = regs[i];
    }
  }
  // operand rows rbase..rbase+31: the lane reads k = kk*16 + 8*(lane/32) .. +7 of row rbase + lane%32
  static __device__ __forceinline__ bf16x8 frag(const uint16_t* lds, int rbase, int kk, int lane) {
    const uint4 v = *reinterpret_cast<const uint4*>(lds + (rbase + (lane & 31)) * LD + kk * 16 + (lane >> 5) * 8);
    return __builtin_bit_cast(bf16x8, v);
  }
};

// k-strided operand: tile [BKT k][R rows]; memory element (r, k) at base[k*ld + r].
// Fragments come from the LDS transpose read (ds_read_b64_tr_b16): within each group of 16
// lanes, lane s supplies the address of 4 consecutive bf16 and receives element s%4 of the
// four lanes 4*j + s/4 (j = 0..3).  With lane s pointing at row k0 + s/4, columns
// c0 + 4*(s%4) .. +3, lane i of the group ends up with rows k0..k0+3 of column c0 + i: four
// consecutive k of its own row/column of the MFMA operand.  Two such reads give the 8 k values.
template <int R, int BKT, int NT>
struct ColTile {
  static constexpr int LD = R + 32;  // row stride = 64 B (mod 256 B): the 4 rows of a transpose read hit distinct banks
  static constexpr int kPerK = R / 8;
  static constexpr int kChunks = BKT * kPerK / NT;
  static constexpr int kLdsElems = BKT * LD;
  static_assert(BKT * kPerK % NT == 0, "tile does not divide among the threads");

  static __device__ __forceinline__ void load(uint4 (&regs)[kChunks], const uint16_t* __restrict__ base, int ld, int r0,
                                              int rows, int k0, int K) {
#pragma unroll
    for (int i = 0; i < kChunks; ++i) {
      const int id = threadIdx.x + NT * i;
      const int c = id % kPerK, k = id / kPerK;
      const int r = r0 + c * 8;
      const bool ok = (k0 + k < K) && (r + 8 <= rows);
      regs[i] = ok ? *reinterpret_cast<const uint4*>(base + (size_t)(k0 + k) * ld + r) : make_uint4(0, 0, 0, 0);
    }
  }
  static __device__ __forceinline__ void store(const uint4 (&regs)[kChunks], uint16_t* lds) {
#pragma unroll
    for (int i = 0; i < kChunks; ++i) {
      const int id = threadIdx.x + NT * i;
      const int c = id % kPerK, k = id / kPerK;
      *reinterpret_cast<uint4*>(lds + k * LD + c * 8) = regs[i];
    }
  }
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

template <int R, int BKT, int NT, bool COL>
struct TileSel { using type = RowTile<R, BKT, NT>; };
template <int R, int BKT, int NT>
struct TileSel<R, BKT, NT, true> { using type = ColTile<R, BKT, NT>; };


// ---- the kernel --------------------------------------------------------------------------------
template <int BM, int BN, int WGM, int WGN, int BKT, bool A_COL, bool B_COL, class Epi>
__global__ __launch_bounds__(64 * WGM * WGN) void gemm_bf16_mfma_kernel(int M, int N, int K,
                                                                         const uint16_t* __restrict__ A, int lda,
                                                                         const uint16_t* __restrict__ B, int ldb,
                                                                         Epi epi, TileMap map) {
  constexpr int NT = 64 * WGM * WGN;
  using ATile = typename TileSel<BM, BKT, NT, A_COL>::type;
  using BTile = typename TileSel<BN, BKT, NT, B_COL>::type;
  constexpr int WM = BM / WGM, WN = BN / WGN;  // wave tile
  constexpr int TM = WM / 32, TN = WN / 32;
  extern __shared__ __attribute__((aligned(16))) uint16_t lds_raw[];
  auto lds_a = [&](int buf) { return lds_raw + buf * ATile::kLdsElems; };
  auto lds_b = [&](int buf) { return lds_raw + 2 * ATile::kLdsElems + buf * BTile::kLdsElems; };

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm = (wave / WGN) * WM, wn = (wave % WGN) * WN;
  int tile_m, tile_n;
  map.get(blockIdx.x, tile_m, tile_n);
  const int m0 = tile_m * BM, n0 = tile_n * BN;

  floatx16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  auto compute = [&](int buf) {
    const uint16_t* la = lds_a(buf);
    const uint16_t* lb = lds_b(buf);
#pragma unroll
    for (int kk = 0; kk < BKT / 16; ++kk) {
      bf16x8 af[TM], bfr[TN];
#pragma unroll
      for (int i = 0; i < TM; ++i) af[i] = ATile::frag(la, wm + i * 32, kk, lane);
#pragma unroll
      for (int j = 0; j < TN; ++j) bfr[j] = BTile::frag(lb, wn + j * 32, kk, lane);
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[i][j] = mma<Epi::kSwap>(af[i], bfr[j], acc[i][j]);
    }
  };

  uint4 ra[ATile::kChunks], rb[BTile::kChunks];
  const int KT = (K + BKT - 1) / BKT;
  ATile::load(ra, A, lda, m0, M, 0, K);
  BTile::load(rb, B, ldb, n0, N, 0, K);
  ATile::store(ra, lds_a(0));
  BTile::store(rb, lds_b(0));
  __syncthreads();
  for (int kt = 0; kt < KT; ++kt) {
    const int cur = kt & 1;
    if (kt + 1 < KT) {
      ATile::load(ra, A, lda, m0, M, (kt + 1) * BKT, K);
      BTile::load(rb, B, ldb, n0, N, (kt + 1) * BKT, K);
    }
    compute(cur);
    if (kt + 1 < KT) {
      ATile::store(ra, lds_a(cur ^ 1));
      BTile::store(rb, lds_b(cur ^ 1));
    }
    __syncthreads();
  }

  store_tiles<TM, TN>(acc, epi, m0 + wm, n0 + wn, M, N, lane);
}

template <int BM, int BN, int WGM, int WGN, int BKT, bool A_COL, bool B_COL, class Epi>
hipError_t launch(hipStream_t s, int M, int N, int K, const uint16_t* A, int lda, const uint16_t* B, int ldb,
                  const Epi& epi, SideCopy side = SideCopy{nullptr, nullptr, 0}) {
  if (side.nvec) {  // this kernel has no side job: a plain copy first
    hipError_t e = hipMemcpyAsync(side.dst, side.src, side.nvec * 16, hipMemcpyDeviceToDevice, s);
    if (e != hipSuccess) return e;
  }
  constexpr int NT = 64 * WGM * WGN;
  using ATile = typename TileSel<BM, BKT, NT, A_COL>::type;
  using BTile = typename TileSel<BN, BKT, NT, B_COL>::type;
  constexpr size_t lds_bytes = 2 * (ATile::kLdsElems + BTile::kLdsElems) * sizeof(uint16_t);
  static_assert(lds_bytes <= 160 * 1024, "tile does not fit the LDS of a CU");
  auto kernel = gemm_bf16_mfma_kernel<BM, BN, WGM, WGN, BKT, A_COL, B_COL, Epi>;
  if (lds_bytes > 64 * 1024) {
    static hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
    if (attr != hipSuccess) return attr;
  }
  const int tiles_m = (M + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
  const TileMap map = make_tile_map(tiles_m, tiles_n);
  hipLaunchKernelGGL(kernel, dim3(tiles_m * tiles_n), dim3(NT), lds_bytes, s, M, N, K, A, lda, B, ldb, epi, map);
  return hipGetLastError();
}


// output of contraction range `split`: only the fp32 weight-gradient product is ever split
template <class E>
__device__ __forceinline__ const E& epi_of_split(const E& e, int) { return e; }
struct EpiWgradSplit {
  float* out; int ldc; size_t split_stride;
  static constexpr bool kSwap = false;
};
__device__ __forceinline__ EpiWgrad epi_of_split(const EpiWgradSplit& e, int split) {
  return EpiWgrad{e.out + (size_t)split * e.split_stride, e.ldc};
}

// LEAN: small wave tiles (one or two 32x32 blocks) have so few MFMAs per k tile that the address and stage
// bookkeeping is a third of the instructions of the loop.  The k loop is then unrolled over the NS stage buffers,
// so that every LDS address is a loop-invariant register plus an immediate and the stage indices are constants;
// the source pointers of the copies advance instead of being recomputed.  The last tiles (no copies left to issue
// in step with them) run through the generic loop.  Worth about 5 % on the 64x64 and 128x64 tiles.
// ROT: the barrier that makes a k tile visible sits one k step early, before the last MFMA group of the tile
// before it, so that the first fragment reads of the new tile run under that group instead of stalling the wave
// (with one wave per SIMD nothing else would cover them).
template <int BM, int BN, int WGM, int WGN, int NS, bool A_COL, bool B_COL, class Epi, bool LEAN = false,
          bool ROT = false>
__global__ __launch_bounds__(64 * WGM * WGN) void gemm_bf16_dma_kernel(int M, int N, int K,
                                                                        const uint16_t* __restrict__ A, int lda,
                                                                        const uint16_t* __restrict__ B, int ldb,
                                                                        Epi epi, TileMap map, SideCopy side) {
  constexpr int NW = WGM * WGN;
  using AT = typename DmaSel<BM, NW, A_COL>::type;
  using BT = typename DmaSel<BN, NW, B_COL>::type;
  constexpr int WM = BM / WGM, WN = BN / WGN;
  constexpr int TM = WM / 32, TN = WN / 32;
  constexpr int kStageBytes = AT::kBytes + BT::kBytes;
  constexpr int kLoads = AT::kPerWave + BT::kPerWave;  // copies one wave issues per stage
  static_assert((NS - 2) * kLoads < 64, "too many copies in flight for vmcnt");
  extern __shared__ __attribute__((aligned(16))) uint16_t lds_raw[];

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int wm = (wave / WGN) * WM, wn = (wave % WGN) * WN;
  int tile_m, tile_n;
  map.get(blockIdx.x, tile_m, tile_n);
  const int m0 = tile_m * BM, n0 = tile_n * BN;
  const uint32_t lds_base = lds_addr_of(lds_raw);
  // blockIdx.y: range of the contraction this workgroup sums over (K is the length of one range); each range
  // writes its own output (fp32 partial results that a second kernel adds in a fixed order)
  const int split = blockIdx.y;
  A += (size_t)split * K * (A_COL ? lda : 1);
  B += (size_t)split * K * (B_COL ? ldb : 1);

  floatx16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  for (size_t i = (size_t)blockIdx.x * (64 * NW) + threadIdx.x; i < side.nvec; i += (size_t)gridDim.x * (64 * NW))
    side.dst[i] = side.src[i];

  AT ta;
  BT tb;
  ta.init(lda, m0, M, wave, lane);
  tb.init(ldb, n0, N, wave, lane);
  const int KT = K / DBK;
  const size_t step_a = AT::tile_step(lda), step_b = BT::tile_step(ldb);
  constexpr int NM = (DBK / 16) * TM * TN;  // MFMAs of one wave per k tile
  // MFMA after which copy t of the next tile is issued.  With three or more stages a copy has a whole tile of slack
  // and the copies are spread evenly; with two stages the tile they fill is waited for at the next barrier, so
  // they all go out during the first MFMAs and the rest of the tile's arithmetic covers their latency.
  auto copy_slot = [](int t) constexpr { return NS == 2 && kLoads <= NM ? t : (t * NM) / kLoads; };

  // copy number t (0 .. kLoads-1) of k tile `tile` into stage `st`.  Tiles past the end re-read
  // the last tile into a stage nobody reads again, which keeps the number of copies per
  // iteration -- and with it the vmcnt arithmetic -- the same from the first tile to the last.
  auto issue_copy = [&](int t, int tile, int st) {
    const int tc = min(tile, KT - 1);
    const uint32_t dst = lds_base + st * kStageBytes;
    if (t < AT::kPerWave) ta.issue_one(t, dst, A + tc * step_a, wave);
    else tb.issue_one(t - AT::kPerWave, dst + AT::kBytes, B + tc * step_b, wave);
  };

  // prologue: stages 0 .. NS-2
#pragma unroll
  for (int st = 0; st < NS - 1; ++st)
#pragma unroll
    for (int t = 0; t < kLoads; ++t) issue_copy(t, st, st);

  int kt0 = 0;
  if constexpr (LEAN) {
    const uint16_t* pa = A + (size_t)(NS - 1) * step_a;  // source of the next tile to copy
    const uint16_t* pb = B + (size_t)(NS - 1) * step_b;
    for (; kt0 + NS <= KT - (NS - 1); kt0 += NS) {
#pragma unroll
      for (int u = 0; u < NS; ++u) {  // tile kt0 + u lives in buffer u, tile kt0 + u + NS - 1 goes to buffer (u + NS - 1) % NS
        wait_vmcnt<(NS - 2) * kLoads>();
        lds_barrier();
        const uint16_t* la = lds_raw + u * (kStageBytes / 2);
        const uint16_t* lb = la + AT::kBytes / 2;
        const uint32_t dst = lds_base + ((u + NS - 1) % NS) * kStageBytes;
        bf16x8 af[2][TM], bfr[2][TN];
#pragma unroll
        for (int i = 0; i < TM; ++i) af[0][i] = AT::frag(la, wm + i * 32, 0, lane);
#pragma unroll
        for (int j = 0; j < TN; ++j) bfr[0][j] = BT::frag(lb, wn + j * 32, 0, lane);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int kk = 0; kk < DBK / 16; ++kk) {
          const int c = kk & 1, nx = c ^ 1;
          if (kk + 1 < DBK / 16) {
#pragma unroll
            for (int i = 0; i < TM; ++i) af[nx][i] = AT::frag(la, wm + i * 32, kk + 1, lane);
#pragma unroll
            for (int j = 0; j < TN; ++j) bfr[nx][j] = BT::frag(lb, wn + j * 32, kk + 1, lane);
          }
          __builtin_amdgcn_sched_barrier(0);
#pragma unroll
          for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) {
              acc[i][j] = mma<Epi::kSwap>(af[c][i], bfr[c][j], acc[i][j]);
              const int q = (kk * TM + i) * TN + j;  // compile-time after unrolling
#pragma unroll
              for (int t = 0; t < kLoads; ++t)
                if (copy_slot(t) == q) {
                  __builtin_amdgcn_sched_barrier(0);
                  if (t < AT::kPerWave) ta.issue_one(t, dst, pa, wave);
                  else tb.issue_one(t - AT::kPerWave, dst + AT::kBytes, pb, wave);
                  __builtin_amdgcn_sched_barrier(0);
                }
            }
          __builtin_amdgcn_sched_barrier(0);
        }
        pa += step_a;
        pb += step_b;
      }
    }
  }
  int rd = 0;        // stage holding tile kt (kt0 is a multiple of NS)
  int wr = NS - 1;   // stage that receives tile kt + NS - 1
  if constexpr (ROT) {
    static_assert(!LEAN, "the rotated loop has no unrolled form");
    constexpr int KS = DBK / 16;
    static_assert(KS % 2 == 0, "fragment buffers alternate with the k steps");
    // Step s of iteration kt reads the fragments of (tile kt, k step s) and multiplies those of the step before:
    // step 0 multiplies the last k step of tile kt-1 (zeros in the first iteration).
    bf16x8 af[2][TM], bfr[2][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int e = 0; e < 8; ++e) af[1][i][e] = 0;
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int e = 0; e < 8; ++e) bfr[1][j][e] = 0;
    for (int kt = 0; kt < KT; ++kt) {
      wait_vmcnt<(NS - 2) * kLoads>();
      lds_barrier();  // tile kt visible; every wave holds its last fragments of tile kt-1 in registers
      const uint16_t* la = lds_raw + rd * (kStageBytes / 2);
      const uint16_t* lb = la + AT::kBytes / 2;
#pragma unroll
      for (int st = 0; st < KS; ++st) {
        const int nx = st & 1, c = nx ^ 1;
#pragma unroll
        for (int i = 0; i < TM; ++i) af[nx][i] = AT::frag(la, wm + i * 32, st, lane);
#pragma unroll
        for (int j = 0; j < TN; ++j) bfr[nx][j] = BT::frag(lb, wn + j * 32, st, lane);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
          for (int j = 0; j < TN; ++j) {
            acc[i][j] = mma<Epi::kSwap>(af[c][i], bfr[c][j], acc[i][j]);
            const int q = (st * TM + i) * TN + j;
#pragma unroll
            for (int t = 0; t < kLoads; ++t)
              if (copy_slot(t) == q) {
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
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j) acc[i][j] = mma<Epi::kSwap>(af[1][i], bfr[1][j], acc[i][j]);
    kt0 = KT;
  }
  for (int kt = kt0; kt < KT; ++kt) {
    // tile kt has landed once at most the NS-2 newer tiles are still in flight
    wait_vmcnt<(NS - 2) * kLoads>();
    lds_barrier();  // tile kt visible to all waves; everybody is done reading stage `wr`
    const uint16_t* la = lds_raw + rd * (kStageBytes / 2);
    const uint16_t* lb = la + AT::kBytes / 2;
    {
      // Fixed schedule per k step: the LDS reads of step kk+1 go out first, then the MFMAs of
      // step kk with the global->LDS copies of tile kt+NS-1 spread evenly between them, so that
      // the wave never sits in the memory-instruction queue while its matrix core idles.
      bf16x8 af[2][TM], bfr[2][TN];
#pragma unroll
      for (int i = 0; i < TM; ++i) af[0][i] = AT::frag(la, wm + i * 32, 0, lane);
#pragma unroll
      for (int j = 0; j < TN; ++j) bfr[0][j] = BT::frag(lb, wn + j * 32, 0, lane);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int kk = 0; kk < DBK / 16; ++kk) {
        const int c = kk & 1, nx = c ^ 1;
        if (kk + 1 < DBK / 16) {
#pragma unroll
          for (int i = 0; i < TM; ++i) af[nx][i] = AT::frag(la, wm + i * 32, kk + 1, lane);
#pragma unroll
          for (int j = 0; j < TN; ++j) bfr[nx][j] = BT::frag(lb, wn + j * 32, kk + 1, lane);
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
          for (int j = 0; j < TN; ++j) {
            acc[i][j] = mma<Epi::kSwap>(af[c][i], bfr[c][j], acc[i][j]);
            const int q = (kk * TM + i) * TN + j;  // compile-time after unrolling
#pragma unroll
            for (int t = 0; t < kLoads; ++t)
              if (copy_slot(t) == q) {
                __builtin_amdgcn_sched_barrier(0);
                issue_copy(t, kt + NS - 1, wr);
                __builtin_amdgcn_sched_barrier(0);
              }
          }
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    rd = rd + 1 == NS ? 0 : rd + 1;
    wr = wr + 1 == NS ? 0 : wr + 1;
  }
  wait_vmcnt<0>();  // the trailing dummy copies must have landed before LDS is reused
  lds_barrier();    // all waves are done with the last stage
  if constexpr (Epi::kSwap && 64 % (4 * TN) == 0) {  // a row of the wave tile is stored by 4 * TN lanes
    if (m0 + wm + WM <= M && n0 + wn + WN <= N && (N & 7) == 0) {
      if constexpr (NW * wave_epilogue_bytes<TM, TN>() <= 160 * 1024) {
        float* wave_lds = reinterpret_cast<float*>(lds_raw) + wave * (wave_epilogue_bytes<TM, TN>() / 4);
        store_tiles_coalesced<TM, TN>(acc, epi, m0 + wm, n0 + wn, lane, wave_lds);
      } else {
        // the whole wave tiles do not fit the LDS together (256x256): one 32-row block of every wave at a time
        float* wave_lds = reinterpret_cast<float*>(lds_raw) + wave * (wave_epilogue_bytes<1, TN>() / 4);
#pragma unroll
        for (int i = 0; i < TM; ++i)
          store_tiles_coalesced<1, TN>(reinterpret_cast<const floatx16(&)[1][TN]>(acc[i]), epi, m0 + wm + 32 * i, n0 + wn,
                                       lane, wave_lds);
      }
      return;
    }
  }
  store_tiles<TM, TN>(acc, epi_of_split(epi, split), m0 + wm, n0 + wn, M, N, lane);
}

// Shapes the direct-to-LDS kernel takes: whole 64-wide k tiles, 32-bit byte offsets inside each
// operand, and at least one 8-wide chunk along the rows of an operand staged [k][row].
inline bool dma_ok(int M, int N, int K, int lda, int ldb, bool a_col, bool b_col) {
  if (K < DBK || K % DBK) return false;
  const size_t a_bytes = (size_t)(a_col ? K : M) * lda * 2, b_bytes = (size_t)(b_col ? K : N) * ldb * 2;
  if (a_bytes >= (1ull << 31) || b_bytes >= (1ull << 31)) return false;
  if ((a_col && M < 8) || (b_col && N < 8)) return false;
  return true;
}

template <int BM, int BN, int WGM, int WGN, int NS, bool A_COL, bool B_COL, class Epi, bool LEAN = false,
          bool ROT = false>
hipError_t launch_dma(hipStream_t s, int M, int N, int K, const uint16_t* A, int lda, const uint16_t* B, int ldb,
                      const Epi& epi, SideCopy side = SideCopy{nullptr, nullptr, 0}, int splits = 1) {
  constexpr int NW = WGM * WGN;
  using AT = typename DmaSel<BM, NW, A_COL>::type;
  using BT = typename DmaSel<BN, NW, B_COL>::type;
  constexpr size_t stage_bytes = (size_t)NS * (AT::kBytes + BT::kBytes);
  constexpr size_t epi_whole = (size_t)NW * wave_epilogue_bytes<BM / WGM / 32, BN / WGN / 32>();
  constexpr size_t epi_rows = (size_t)NW * wave_epilogue_bytes<1, BN / WGN / 32>();  // one 32-row block per wave
  constexpr bool epi_lds = Epi::kSwap && 64 % (4 * (BN / WGN / 32)) == 0;
  constexpr size_t epi_bytes = !epi_lds ? 0 : epi_whole <= 160 * 1024 ? epi_whole : epi_rows;  // tiles turned through LDS
  constexpr size_t lds_bytes = stage_bytes > epi_bytes ? stage_bytes : epi_bytes;
  static_assert(lds_bytes <= 160 * 1024, "stages do not fit the LDS of a CU");
  auto kernel = gemm_bf16_dma_kernel<BM, BN, WGM, WGN, NS, A_COL, B_COL, Epi, LEAN, ROT>;
  if (lds_bytes > 64 * 1024) {
    static hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
    if (attr != hipSuccess) return attr;
  }
  const int tiles_m = (M + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
  const TileMap map = make_tile_map(tiles_m, tiles_n);
  hipLaunchKernelGGL(kernel, dim3(tiles_m * tiles_n, splits), dim3(64 * NW), lds_bytes, s, M, N, K / splits, A, lda, B, ldb,
                     epi, map, side);
  return hipGetLastError();
}

int g_cfg[3] = {-1, -1, -1};  // tuning override per product (fprop, dgrad, wgrad); -1 = heuristic

// Tile choice.  The direct-to-LDS kernel is taken whenever the shape allows it: the largest of
// its tiles that still gives every CU a workgroup (large tiles cut the L2->LDS traffic, which
// together with the LDS reads is what bounds these kernels).  Ragged shapes go to the
// register-staged kernel.
int pick(int rows, int cols, int contraction, int lda, int ldb, bool a_col, bool b_col, int override_cfg) {
  const bool dma = dma_ok(rows, cols, contraction, lda, ldb, a_col, b_col);
  if (override_cfg >= 0 && (override_cfg < 10 || dma)) return override_cfg;  // a direct-to-LDS tile only where it is valid
  auto blocks = [&](int bm, int bn) { return (long)((rows + bm - 1) / bm) * ((cols + bn - 1) / bn); };
  if (dma) {
    // The tile that needs the least time on 256 CUs, taken as (rounds of 256 workgroups) x (tile area) / (rate the
    // tile sustains relative to the largest one): large tiles move less data per flop, but a last round that fills
    // a fraction of the chip costs a whole round -- the 6144 x 2048 weight gradient of a fused QKV projection is 1.5
    // rounds of 256x128 tiles, 192 tiles of 256x256 and exactly 256 tiles of 384x128 (51 us against 65 us and 57 us
    // at 2048 rows).  The 384-wide tiles serve the fp32-output product only (three 32-wide blocks per wave row do
    // not fit the 16-byte row stores of the bf16 epilogues) and only shapes they divide.
    struct Tile { int cfg, bm, bn, rate; bool wgrad_only; };  // rate in per cent of the 256x256 tile's
    static const Tile tiles[] = {{18, 256, 256, 100, false}, {25, 384, 128, 88, true}, {24, 128, 384, 88, true},
                                 {19, 256, 128, 88, false},  {12, 128, 128, 78, false}, {11, 128, 64, 62, false},
                                 {10, 64, 64, 45, false}};
    int best = 10;
    long best_cost = -1;
    for (const Tile& t : tiles) {
      if (t.wgrad_only && !(a_col && b_col && rows % t.bm == 0 && cols % t.bn == 0)) continue;
      const long cost = ((blocks(t.bm, t.bn) + 255) / 256) * t.bm * t.bn * 100 / t.rate;
      if (best_cost < 0 || cost < best_cost) { best_cost = cost; best = t.cfg; }
    }
    return best;
  }
  if (blocks(128, 128) >= 256) return 2;
  if (blocks(128, 64) >= 128) return 1;
  return 0;
}

}  // namespace

void mfma_set_config(int product, int cfg) {
  if (product >= 0 && product < 3) g_cfg[product] = cfg;
}

// Contraction extents must be a multiple of 8 (16-byte chunks along k); operands that are staged
// [k][row] also need their row extent to be a multiple of 8.
bool mfma_fprop_supported(int M, int N, int K) { return M >= 1 && N >= 1 && K % 8 == 0; }
bool mfma_dgrad_supported(int M, int N, int K) { return M >= 1 && N % 8 == 0 && K % 8 == 0; }
bool mfma_wgrad_supported(int M, int N, int K) { return M >= 1 && N % 8 == 0 && K % 8 == 0; }

#define TP_GEMM_DISPATCH(cfg, ACOL, BCOL, ...)                                  \
  switch (cfg) {                                                                \
    case 10: return launch_dma<64, 64, 2, 2, 4, ACOL, BCOL, decltype(e), true>(__VA_ARGS__);  \
    case 11: return launch_dma<128, 64, 2, 2, 4, ACOL, BCOL, decltype(e), true>(__VA_ARGS__); \
    case 30: return launch_dma<64, 64, 2, 2, 8, ACOL, BCOL, decltype(e), true>(__VA_ARGS__);  \
    case 31: return launch_dma<64, 64, 2, 2, 6, ACOL, BCOL, decltype(e), true>(__VA_ARGS__);  \
    case 12: return launch_dma<128, 128, 2, 2, 3, ACOL, BCOL, decltype(e), false, true>(__VA_ARGS__); \
    case 18: return launch_dma<256, 256, 2, 4, 2, ACOL, BCOL, decltype(e), false, true>(__VA_ARGS__); \
    case 19: return launch_dma<256, 128, 2, 4, 3, ACOL, BCOL, decltype(e), false, true>(__VA_ARGS__); \
    case 24: return launch_dma<128, 384, 2, 4, 2, ACOL, BCOL, decltype(e), false, true>(__VA_ARGS__); \
    case 25: return launch_dma<384, 128, 4, 2, 2, ACOL, BCOL, decltype(e), false, true>(__VA_ARGS__); \
    case 2: return launch<128, 128, 2, 2, 64, ACOL, BCOL>(__VA_ARGS__);         \
    case 1: return launch<128, 64, 2, 2, 64, ACOL, BCOL>(__VA_ARGS__);          \
    default: return launch<64, 64, 2, 2, 64, ACOL, BCOL>(__VA_ARGS__);          \
  }

hipError_t mfma_fprop(hipStream_t s, int M, int N, int K, const uint16_t* x, const uint16_t* W, const float* bias,
                      int act, uint16_t* d_out, uint16_t* a_out, uint16_t* x_copy, const uint16_t* addend) {
  // x is [M x K] with K % 8 == 0 and 16-byte aligned rows, so it is a whole number of 16-byte units
  SideCopy side{(const uint4*)x, (uint4*)x_copy, x_copy ? (size_t)M * K / 8 : 0};
  if (addend) {
    EpiFpropAdd e{bias, d_out, a_out, act, N, addend};
    TP_GEMM_DISPATCH(pick(M, N, K, K, K, false, false, g_cfg[0]), false, false, s, M, N, K, x, K, W, K, e, side)
  }
  EpiFprop e{bias, d_out, a_out, act, N};
  TP_GEMM_DISPATCH(pick(M, N, K, K, K, false, false, g_cfg[0]), false, false, s, M, N, K, x, K, W, K, e, side)
}

hipError_t mfma_dgrad(hipStream_t s, int M, int N, int K, const uint16_t* dz, const uint16_t* Wb,
                      const uint16_t* d_prev, uint16_t* out, int relu_mask) {
  // out[M x K] = dz[M x N] . Wb[N x K]: GEMM (M, K, contraction N)
  EpiDgrad e{d_prev, out, K, relu_mask};
  TP_GEMM_DISPATCH(pick(M, K, N, N, K, false, true, g_cfg[1]), false, true, s, M, K, N, dz, N, Wb, K, e)
}

// Ranges of the contraction (the rows of the mini-batch) a weight gradient is split into when its output has too
// few tiles to fill the chip: whole 64-row k tiles, at least 8 per range, as many ranges as give every CU a
// workgroup (a 64 x 64 gradient over the 131072 pixels of 16x16 maps is one tile and 2048 k tiles).
int mfma_wgrad_splits(int M, int N, int K) {
  if (!dma_ok(N, K, M, N, K, true, true)) return 1;
  const int cfg = pick(N, K, M, N, K, true, true, g_cfg[2]);
  if (cfg != 10) return 1;  // larger tiles are only chosen when they already give 256 workgroups
  const long blocks = (long)((N + 63) / 64) * ((K + 63) / 64);
  int s = (int)std::min<long>(256, 256 / std::max<long>(blocks, 1));
  while (s > 1 && (M % (DBK * s) != 0 || M / (DBK * s) < 8)) --s;
  return std::max(s, 1);
}

size_t mfma_wgrad_scratch_floats(int M, int N, int K) {
  const int s = mfma_wgrad_splits(M, N, K);
  return s > 1 ? (size_t)s * N * K : 0;
}

hipError_t mfma_wgrad(hipStream_t s, int M, int N, int K, const uint16_t* dz, const uint16_t* x, float* gW, float* partial) {
  // gW[N x K] = dz^T[N x M] . x[M x K]: GEMM (N, K, contraction M)
  const int splits = partial ? mfma_wgrad_splits(M, N, K) : 1;
  if (splits > 1) {
    EpiWgradSplit e{partial, K, (size_t)N * K};
    const hipError_t err = launch_dma<64, 64, 2, 2, 4, true, true>(s, N, K, M, dz, N, x, K, e, SideCopy{nullptr, nullptr, 0}, splits);
    if (err != hipSuccess) return err;
    return launch_sum_partials(s, (size_t)N * K, splits, partial, gW);
  }
  EpiWgrad e{gW, K};
  TP_GEMM_DISPATCH(pick(N, K, M, N, K, true, true, g_cfg[2]), true, true, s, N, K, M, dz, N, x, K, e)
}

}  // namespace tp
