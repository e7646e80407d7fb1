// Causal multi-head attention on the matrix cores (bf16), as batched GEMMs around row-wise softmax
// kernels.  One workgroup row (blockIdx.y) per (sequence, head); the GEMM kernel is the direct-to-LDS
// pipeline of the dense layers with per-batch operand offsets and three causal shortcuts:
//   skip    output tiles that lie entirely above the diagonal are not computed (Q K^T, dO V^T);
//   limit   the contraction over keys stops at the last query row of the tile (P V, dS K);
//   start   the contraction over queries starts at the first key row of the tile (P^T dO, dS^T Q).
// forward   head widths 64 and 128: one fused kernel (online softmax, no score matrix in memory), see below;
//           otherwise S = Q K^T (fp32)  ->  P = softmax(scale S) (bf16, zeros above the diagonal), lse  ->  O = P V
// backward  S = Q K^T, dP = dO V^T (fp32)  ->  P, dS = scale P (dP - rowsum(P dP)) (bf16)
//           ->  dQ = dS K, dK = dS^T Q, dV = P^T dO
// The score matrices are transient: a call works through the sequences in chunks that fit the
// scratch the caller provides.  Needs tokens % 64 == 0 and head width % 64 == 0; other shapes
// stay on the wavefront kernels of kernels_transformer.hip.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <algorithm>

#include "device_utils.h"
#include "mfma_common.h"
#include "transformer.h"

namespace tp {

namespace {

struct BatchOffsets {
  int heads;
  long a_b, a_h, b_b, b_h, c_b, c_h;  // element offsets per sequence / per head of the three operands
};
enum Causal : int { kSkipTiles = 1, kLimitK = 2, kStartK = 3 };

__device__ __forceinline__ EpiWgrad epi_at(const EpiWgrad& e, long off) { return EpiWgrad{e.out + off, e.ldc}; }
__device__ __forceinline__ EpiDgrad epi_at(const EpiDgrad& e, long off) { return EpiDgrad{nullptr, e.out + off, e.ldc}; }

template <int BM, int BN, int WGM, int WGN, int NS, bool A_COL, bool B_COL, class Epi>
__global__ __launch_bounds__(64 * WGM * WGN) void attn_gemm_kernel(int M, int N, int K, const uint16_t* __restrict__ A, int lda,
                                                                    const uint16_t* __restrict__ B, int ldb, Epi epi,
                                                                    BatchOffsets bo, int causal, int tiles_n) {
  constexpr int NW = WGM * WGN;
  using AT = typename DmaSel<BM, NW, A_COL>::type;
  using BT = typename DmaSel<BN, NW, B_COL>::type;
  constexpr int WM = BM / WGM, WN = BN / WGN;
  constexpr int TM = WM / 32, TN = WN / 32;
  constexpr int kStageBytes = AT::kBytes + BT::kBytes;
  constexpr int kLoads = AT::kPerWave + BT::kPerWave;
  constexpr int NM = (DBK / 16) * TM * TN;
  static_assert((NS - 2) * kLoads < 64, "too many copies in flight for vmcnt");
  extern __shared__ __attribute__((aligned(16))) uint16_t lds_raw[];

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int wm = (wave / WGN) * WM, wn = (wave % WGN) * WN;
  const int tile_m = blockIdx.x / tiles_n, tile_n = blockIdx.x - tile_m * tiles_n;
  const int m0 = tile_m * BM, n0 = tile_n * BN;
  if (causal == kSkipTiles && n0 > m0 + BM - 1) return;  // every column of the tile lies beyond every row
  const int zb = blockIdx.y / bo.heads, zh = blockIdx.y - zb * bo.heads;
  A += zb * bo.a_b + zh * bo.a_h;
  B += zb * bo.b_b + zh * bo.b_h;
  const uint32_t lds_base = lds_addr_of(lds_raw);

  floatx16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  AT ta;
  BT tb;
  ta.init(lda, m0, M, wave, lane);
  tb.init(ldb, n0, N, wave, lane);
  // k tiles kt0 .. kt0 + KT - 1 of the contraction
  int kt0 = 0, KT = K / DBK;
  if (causal == kLimitK) KT = min(KT, (m0 + BM + DBK - 1) / DBK);
  if (causal == kStartK) {
    kt0 = m0 / DBK;
    KT -= kt0;
  }
  const size_t step_a = AT::tile_step(lda), step_b = BT::tile_step(ldb);
  auto issue_copy = [&](int t, int tile, int st) {
    const int tc = kt0 + min(tile, KT - 1);
    const uint32_t dst = lds_base + st * kStageBytes;
    if (t < AT::kPerWave) ta.issue_one(t, dst, A + tc * step_a, wave);
    else tb.issue_one(t - AT::kPerWave, dst + AT::kBytes, B + tc * step_b, wave);
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
    const uint16_t* lb = la + AT::kBytes / 2;
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
  const Epi e = epi_at(epi, zb * bo.c_b + zh * bo.c_h);
  if constexpr (Epi::kSwap) {
    if (m0 + wm + WM <= M && n0 + wn + WN <= N && (N & 7) == 0) {
      float* wave_lds = reinterpret_cast<float*>(lds_raw) + wave * (wave_epilogue_bytes<TM, TN>() / 4);
      store_tiles_coalesced<TM, TN>(acc, e, m0 + wm, n0 + wn, lane, wave_lds);
      return;
    }
  }
  store_tiles<TM, TN>(acc, e, m0 + wm, n0 + wn, M, N, lane);
}

// 128 x BN tiles, 4 waves, 3 stages
template <int BN, bool A_COL, bool B_COL, class Epi>
hipError_t launch_attn_gemm(hipStream_t s, int Z, int M, int N, int K, const uint16_t* A, int lda, const uint16_t* B, int ldb,
                            const Epi& epi, const BatchOffsets& bo, int causal) {
  constexpr int BM = 128, NS = 3, NW = 4;
  using AT = typename DmaSel<BM, NW, A_COL>::type;
  using BT = typename DmaSel<BN, NW, B_COL>::type;
  constexpr size_t stage_bytes = (size_t)NS * (AT::kBytes + BT::kBytes);
  constexpr size_t epi_bytes = Epi::kSwap ? (size_t)NW * wave_epilogue_bytes<BM / 64, BN / 64>() : 0;
  constexpr size_t lds_bytes = stage_bytes > epi_bytes ? stage_bytes : epi_bytes;
  auto kernel = attn_gemm_kernel<BM, BN, 2, 2, NS, A_COL, B_COL, Epi>;
  static hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
  if (attr != hipSuccess) return attr;
  const int tiles_m = (M + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
  hipLaunchKernelGGL(kernel, dim3(tiles_m * tiles_n, Z), dim3(64 * NW), lds_bytes, s, M, N, K, A, lda, B, ldb, epi, bo, causal,
                     tiles_n);
  return hipGetLastError();
}

__device__ __forceinline__ float wsum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ float wmax(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}

// one wave per query row: P[i][j] = softmax over j <= i of scale * S[i][j], zeros for j > i; lse[i]
__global__ __launch_bounds__(256) void attn_softmax_fwd_kernel(int S, size_t rows, float scale, const float* __restrict__ scores,
                                                               uint16_t* __restrict__ P, float* __restrict__ lse) {
  const int lane = threadIdx.x & 63;
  const size_t r = (size_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (r >= rows) return;
  const int i = (int)(r % S);
  const float* sr = scores + r * S;
  float m = -INFINITY;
  for (int j = lane; j <= i; j += 64) m = fmaxf(m, sr[j] * scale);
  m = wmax(m);
  float l = 0.f;
  for (int j = lane; j <= i; j += 64) l += __expf(sr[j] * scale - m);
  l = wsum(l);
  const float inv = 1.f / l;
  for (int j = lane; j < S; j += 64) P[r * S + j] = j <= i ? float_to_bf16(__expf(sr[j] * scale - m) * inv) : (uint16_t)0;
  if (lane == 0) lse[r] = m + __logf(l);
}

// P = exp(scale S - lse), dS = scale * P * (dP - rowsum(P dP)); both bf16 with zeros above the diagonal
__global__ __launch_bounds__(256) void attn_softmax_bwd_kernel(int S, size_t rows, float scale, const float* __restrict__ scores,
                                                               const float* __restrict__ dP, const float* __restrict__ lse,
                                                               uint16_t* __restrict__ P, uint16_t* __restrict__ dS) {
  const int lane = threadIdx.x & 63;
  const size_t r = (size_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (r >= rows) return;
  const int i = (int)(r % S);
  const float* sr = scores + r * S;
  const float* dr = dP + r * S;
  const float li = lse[r];
  float delta = 0.f;
  for (int j = lane; j <= i; j += 64) delta += __expf(sr[j] * scale - li) * dr[j];
  delta = wsum(delta);
  for (int j = lane; j < S; j += 64) {
    float p = 0.f, ds = 0.f;
    if (j <= i) {
      p = __expf(sr[j] * scale - li);
      ds = scale * p * (dr[j] - delta);
    }
    P[r * S + j] = float_to_bf16(p);
    dS[r * S + j] = float_to_bf16(ds);
  }
}

// ---- fused forward --------------------------------------------------------------------------------
// One workgroup = 256 queries of one (sequence, head): 8 waves x 32 queries.  It walks over the keys
// in blocks of 64; K [64 keys][dh] and V [64 keys][dh] of a block are copied global -> LDS (three
// stages in flight) and shared by the eight waves.  Per wave and block:
//   S^T = K Q^T     the transposed score tile: MFMA rows = keys, columns = the wave's queries.  Every
//                   lane then holds ONE query (lane % 32) and 16 of the 32 keys of a tile, so the
//                   running maximum / sum of the online softmax are per-lane scalars and one exchange
//                   with lane ^ 32 per block completes them.  Q fragments stay in registers.
//   O^T += V^T P^T  P = exp(S - max) never leaves the registers: accumulator element r of a lane is
//                   key 8*(r/4) + 4*(lane/32) + r%4, so packing elements 8g..8g+7 to bf16 gives the B
//                   fragment of a 16-key MFMA step in which lanes 0-31 carry keys {0-3, 8-11} and lanes
//                   32-63 keys {4-7, 12-15}; the V fragment is read from LDS (transposing reads) with
//                   its keys in the same order.
// Key blocks above the diagonal are skipped per wave; the diagonal ones are masked.  The output tile is
// divided by the row sums and turned through LDS for 16-byte row stores; lse = max + log(sum) (natural
// logarithm of the scaled scores) is what the backward pass recomputes the probabilities from.
// No score matrix reaches memory.
constexpr int kFlashWaves = 8, kFlashStages = 3, kFlashQ = 32 * kFlashWaves;

template <int DH>
__device__ __forceinline__ bf16x8 flash_v_frag(const uint16_t* lds, int dbase, int g16, int lane) {
  using VT = ColDma<DH, kFlashWaves>;  // only its chunk swizzle is used, which does not depend on the wave count
  const int g = lane >> 4, s = lane & 15;
  const int k = g16 * 16 + 4 * (g >> 1) + (s >> 2);       // keys {0-3} / {4-7} of the group, +8 below
  const int col = dbase + 16 * (g & 1) + 4 * (s & 3);
  const int slot = (col >> 3) ^ VT::swz(k);
  typedef __attribute__((address_space(3))) shortx4* lds_ptr;
  const uint16_t* p = lds + k * DH + slot * 8 + (col & 7);
  const shortx4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(p));
  const shortx4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(p + 8 * DH));  // k+8: same swizzle
  const shortx8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
  return __builtin_bit_cast(bf16x8, v);
}

template <int DH>
__global__ __launch_bounds__(64 * kFlashWaves) void attn_flash_fwd_kernel(int S, int heads, const uint16_t* __restrict__ qkv,
                                                                          uint16_t* __restrict__ out, float* __restrict__ lse,
                                                                          float scale_log2) {
  constexpr int NW = kFlashWaves, NS = kFlashStages;
  constexpr int HALVES = DH / 64, TN = DH / 32;
  using KT = RowDma<64, NW>;   // 64 keys x one 64-wide chunk of the head dimension
  using VT = ColDma<DH, NW>;   // [64 keys][DH]
  constexpr int kKBytes = HALVES * KT::kBytes;
  constexpr int kStageBytes = kKBytes + VT::kBytes;
  constexpr int kLoads = HALVES * KT::kPerWave + VT::kPerWave;
  static_assert((NS - 2) * kLoads < 64, "too many copies in flight for vmcnt");
  extern __shared__ __attribute__((aligned(16))) uint16_t lds_raw[];

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int half = lane >> 5;
  // grid: x = (sequence, head), y = query block.  Workgroups are handed out x first, so all the longest rows of
  // the triangle (the last query block of every head) start before any shorter one
  const int zb = blockIdx.x / heads, zh = blockIdx.x - zb * heads;
  const int D = heads * DH, ld = 3 * D;
  const int q0 = (gridDim.y - 1 - blockIdx.y) * kFlashQ;
  const int qw = q0 + wave * 32;                           // first query of this wave
  const bool active = qw < S;                              // S is a multiple of 64: a wave is whole or absent
  const uint16_t* qbase = qkv + (size_t)zb * S * ld + zh * DH;
  const uint16_t* kbase = qbase + D;
  const uint16_t* vbase = qbase + 2 * D;
  const uint32_t lds_base = lds_addr_of(lds_raw);

  // Q fragments (B operand: column = query lane % 32, 8 consecutive head-dimension values)
  bf16x8 qf[DH / 16];
  {
    const uint16_t* qrow = qbase + (size_t)(active ? qw + (lane & 31) : 0) * ld + 8 * half;
#pragma unroll
    for (int kk = 0; kk < DH / 16; ++kk) qf[kk] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(qrow + kk * 16));
  }
  wait_vmcnt<0>();  // nothing but the copies below is in flight from here on
#pragma unroll
  for (int kk = 0; kk < DH / 16; ++kk) asm volatile("" : "+v"(qf[kk]));  // the compiler's own wait for these loads lands here

  KT kt;
  VT vt;
  kt.init(ld, 0, 64, wave, lane);
  vt.init(ld, 0, DH, wave, lane);
  const int nkb = min(S, q0 + kFlashQ) / 64;  // key blocks any query of the workgroup can see
  auto issue_block = [&](int blk, int st) {
    const int kb = min(blk, nkb - 1);  // blocks past the end re-read the last one into a stage nobody reads again
    const uint32_t dst = lds_base + st * kStageBytes;
    const uint16_t* ksrc = kbase + (size_t)kb * 64 * ld;
    const uint16_t* vsrc = vbase + (size_t)kb * 64 * ld;
#pragma unroll
    for (int c = 0; c < HALVES; ++c)
#pragma unroll
      for (int t = 0; t < KT::kPerWave; ++t) kt.issue_one(t, dst + c * KT::kBytes, ksrc + c * 64, wave);
#pragma unroll
    for (int t = 0; t < VT::kPerWave; ++t) vt.issue_one(t, dst + kKBytes, vsrc, wave);
  };
#pragma unroll
  for (int st = 0; st < NS - 1; ++st) issue_block(st, st);

  floatx16 oacc[1][TN];
#pragma unroll
  for (int j = 0; j < TN; ++j)
#pragma unroll
    for (int r = 0; r < 16; ++r) oacc[0][j][r] = 0.f;
  float mrun = -INFINITY, lsum = 0.f;  // running maximum (log2 domain) and this lane's share of the row sum
  const int query = qw + (lane & 31);

  int rd = 0, wr = NS - 1;
  for (int kb = 0; kb < nkb; ++kb) {
    wait_vmcnt<(NS - 2) * kLoads>();
    lds_barrier();  // block kb visible to all waves; everybody is done reading stage `wr`
    issue_block(kb + NS - 1, wr);
    if (active && kb * 64 <= qw + 31) {  // wave-uniform: some key of the block is visible to some query of the wave
      const uint16_t* lk = lds_raw + rd * (kStageBytes / 2);
      const uint16_t* lv = lk + kKBytes / 2;
      floatx16 sacc[2];
#pragma unroll
      for (int j = 0; j < 2; ++j) {
#pragma unroll
        for (int r = 0; r < 16; ++r) sacc[j][r] = 0.f;
#pragma unroll
        for (int c = 0; c < HALVES; ++c)
#pragma unroll
          for (int kk = 0; kk < 4; ++kk)
            sacc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(KT::frag(lk + c * (KT::kBytes / 2), 32 * j, kk, lane),
                                                              qf[c * 4 + kk], sacc[j], 0, 0, 0);
      }
      const bool diagonal = kb * 64 + 63 > qw;  // some (query, key) pair of this wave and block is masked
      float mloc = -INFINITY;
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          float v = sacc[j][r] * scale_log2;
          if (diagonal) {
            const int key = kb * 64 + 32 * j + 8 * (r >> 2) + 4 * half + (r & 3);
            if (key > query) v = -INFINITY;
          }
          sacc[j][r] = v;
          mloc = fmaxf(mloc, v);
        }
      mloc = fmaxf(mloc, __shfl_xor(mloc, 32, 64));
      const float mnew = fmaxf(mrun, mloc);  // finite: block 0 shows key 0 to every query
      const float alpha = __builtin_amdgcn_exp2f(mrun - mnew);
      mrun = mnew;
      float psum = 0.f;
      bf16x8 pf[4];
#pragma unroll
      for (int g16 = 0; g16 < 4; ++g16) {
        float e[8];
#pragma unroll
        for (int t = 0; t < 8; ++t) {
          e[t] = __builtin_amdgcn_exp2f(sacc[g16 >> 1][8 * (g16 & 1) + t] - mnew);
          psum += e[t];
        }
        const uint4 u = make_uint4(pack_bf16x2(e[0], e[1]), pack_bf16x2(e[2], e[3]), pack_bf16x2(e[4], e[5]), pack_bf16x2(e[6], e[7]));
        pf[g16] = __builtin_bit_cast(bf16x8, u);
      }
      lsum = fmaf(lsum, alpha, psum);
      if (__builtin_amdgcn_ballot_w64(alpha != 1.f) != 0) {  // some row's maximum moved: rescale what is accumulated
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
          for (int r = 0; r < 16; ++r) oacc[0][j][r] *= alpha;
      }
#pragma unroll
      for (int g16 = 0; g16 < 4; ++g16)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          oacc[0][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(flash_v_frag<DH>(lv, 32 * j, g16, lane), pf[g16], oacc[0][j], 0, 0, 0);
    }
    rd = rd + 1 == NS ? 0 : rd + 1;
    wr = wr + 1 == NS ? 0 : wr + 1;
  }
  wait_vmcnt<0>();  // the trailing dummy copies must have landed before LDS is reused
  lds_barrier();
  if (!active) return;
  const float ltot = lsum + __shfl_xor(lsum, 32, 64);
  const float inv = 1.f / ltot;
#pragma unroll
  for (int j = 0; j < TN; ++j)
#pragma unroll
    for (int r = 0; r < 16; ++r) oacc[0][j][r] *= inv;
  if (half == 0) lse[(size_t)blockIdx.x * S + query] = (mrun + __builtin_amdgcn_logf(ltot)) * 0.6931471805599453f;
  float* wave_lds = reinterpret_cast<float*>(lds_raw) + wave * (wave_epilogue_bytes<1, TN>() / 4);
  store_tiles_coalesced<1, TN>(oacc, EpiDgrad{nullptr, out, D}, zb * S + qw, zh * DH, lane, wave_lds);
}

template <int DH>
hipError_t launch_flash_fwd(hipStream_t s, int seqs, int S, int heads, const uint16_t* qkv, uint16_t* out, float* lse) {
  constexpr size_t stage_bytes = (size_t)kFlashStages * ((DH / 64) * RowDma<64, kFlashWaves>::kBytes + ColDma<DH, kFlashWaves>::kBytes);
  constexpr size_t epi_bytes = (size_t)kFlashWaves * wave_epilogue_bytes<1, DH / 32>();
  constexpr size_t lds_bytes = stage_bytes > epi_bytes ? stage_bytes : epi_bytes;
  static_assert(lds_bytes <= 160 * 1024, "stages do not fit the LDS of a CU");
  auto kernel = attn_flash_fwd_kernel<DH>;
  static hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
  if (attr != hipSuccess) return attr;
  // scores are scaled by 1/sqrt(dh) and exponentiated in base 2
  const float scale_log2 = 1.4426950408889634f / sqrtf((float)DH);
  hipLaunchKernelGGL(kernel, dim3(seqs * heads, (S + kFlashQ - 1) / kFlashQ), dim3(64 * kFlashWaves), lds_bytes, s, S, heads, qkv,
                     out, lse, scale_log2);
  return hipGetLastError();
}

// ---- fused backward -------------------------------------------------------------------------------
// Two launches of one kernel template, both in the register layout of the fused forward:
//   dQ      a workgroup owns 256 queries (8 waves x 32) and walks over the key blocks up to its diagonal:
//           S^T = K Q^T and dP^T = V dO^T with Q, dO fragments in registers, K and V streamed through LDS;
//           lse and delta = dO . O are per-lane scalars; dQ^T += K^T dS^T.
//   dK, dV  a workgroup owns 256 keys and walks over the query blocks from its diagonal to the end:
//           S = Q K^T and dP = dO V^T with K, V fragments in registers, Q and dO streamed; lse, delta of the 64
//           streamed queries come through LDS with the block; dV^T += dO^T P, dK^T += Q^T dS.
// P = exp(scale S - lse) and dS = scale P (dP - delta) are formed in registers and packed to bf16 as the B
// fragments of the second products, exactly like P in the forward kernel; the streamed operand is staged twice,
// once in the row layout the first products read and once in the layout the transposing reads of the second
// products want.  The scores are recomputed in both launches (7 matrix products instead of 5), no score-sized
// tensor reaches memory, nothing is accumulated with atomics: every output element has one owner.
// 8 waves per workgroup, two per SIMD: the second wave covers the first one's LDS and barrier stalls (25 % faster than
// 4 waves in both launches).  The dK/dV launch fits the 256 registers that leaves because only one half of a streamed
// block has its score tiles alive at a time.
constexpr int kBwdWaves = 8;
constexpr float kLog2e = 1.4426950408889634f;

// stat[(z*S + i)*2] = lse_i * log2(e), stat[(z*S + i)*2 + 1] = delta_i = sum_d dO[i][d] * O[i][d];  z = sequence*heads + head.
// One wave per token row; a lane takes 8 consecutive columns per step, the dh/8 lanes of a head are added.
__global__ __launch_bounds__(256) void attn_stat_kernel(int S, int heads, int dh, size_t rows, const uint16_t* __restrict__ dout,
                                                        const uint16_t* __restrict__ out, const float* __restrict__ lse,
                                                        float* __restrict__ stat) {
  const int lane = threadIdx.x & 63;
  const size_t row = (size_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= rows) return;
  const int D = heads * dh, group = dh / 8;
  const size_t b = row / S, i = row - b * S;
  for (int c0 = 0; c0 < D; c0 += 512) {
    const int col = c0 + lane * 8;
    float acc = 0.f;
    if (col < D) {
      const uint4 a = *reinterpret_cast<const uint4*>(dout + row * D + col), o = *reinterpret_cast<const uint4*>(out + row * D + col);
      const uint32_t aw[4] = {a.x, a.y, a.z, a.w}, ow[4] = {o.x, o.y, o.z, o.w};
#pragma unroll
      for (int j = 0; j < 4; ++j)
        acc += __uint_as_float(aw[j] << 16) * __uint_as_float(ow[j] << 16) +
               __uint_as_float(aw[j] & 0xffff0000u) * __uint_as_float(ow[j] & 0xffff0000u);
    }
    for (int off = 1; off < group; off <<= 1) acc += __shfl_xor(acc, off, 64);
    if (col < D && (lane % group) == 0) {
      const size_t zi = (b * heads + col / dh) * S + i;
      stat[zi * 2] = lse[zi] * kLog2e;
      stat[zi * 2 + 1] = acc;
    }
  }
}

template <int DH, bool OWN_KEYS>
__global__ __launch_bounds__(64 * kBwdWaves) void attn_flash_bwd_kernel(int S, int heads, const uint16_t* __restrict__ qkv,
                                                                        const uint16_t* __restrict__ dout,
                                                                        const float* __restrict__ stat, uint16_t* __restrict__ dqkv,
                                                                        float scale, float scale_log2) {
  constexpr int NW = kBwdWaves, kBwdOwn = 32 * NW;
  constexpr int HALVES = DH / 64, TN = DH / 32;
  using RT = RowDma<64, NW>;   // 64 streamed rows x one 64-wide chunk of the head dimension
  using CT = ColDma<DH, NW>;   // [64 streamed rows][DH], read transposed
  constexpr int kRowBytes = HALVES * RT::kBytes;
  constexpr int kStatBytes = OWN_KEYS ? 1024 : 0;
  constexpr int kCols = OWN_KEYS ? 2 : 1;
  constexpr int kStageBytes = 2 * kRowBytes + kCols * CT::kBytes + kStatBytes;
  extern __shared__ __attribute__((aligned(16))) uint16_t lds_raw[];

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int half = lane >> 5;
  const int z = blockIdx.x, zb = z / heads, zh = z - zb * heads;  // grid: x = (sequence, head), y = block of own rows
  const int D = heads * DH, ld3 = 3 * D;
  const uint16_t* qp = qkv + (size_t)zb * S * ld3 + zh * DH;
  const uint16_t* dop = dout + (size_t)zb * S * D + zh * DH;
  // own rows (fragments in registers) and streamed rows (through LDS)
  const uint16_t* own1 = OWN_KEYS ? qp + D : qp;          // K | Q
  const uint16_t* own2 = OWN_KEYS ? qp + 2 * D : dop;     // V | dO
  const int ld_own2 = OWN_KEYS ? ld3 : D;
  const uint16_t* str1 = OWN_KEYS ? qp : qp + D;          // Q | K
  const uint16_t* str2 = OWN_KEYS ? dop : qp + 2 * D;     // dO | V
  const int ld_str2 = OWN_KEYS ? D : ld3;
  // the workgroups with the most blocks to walk start first: low keys, high queries
  const int o0 = (OWN_KEYS ? (int)blockIdx.y : (int)(gridDim.y - 1 - blockIdx.y)) * kBwdOwn;
  const int ow = o0 + wave * 32;
  const bool active = ow < S;
  const int oi = ow + (lane & 31);  // this lane's own row
  const uint32_t lds_base = lds_addr_of(lds_raw);

  bf16x8 f1[DH / 16], f2[DH / 16];
  float own_l2 = 0.f, own_delta = 0.f;
  {
    const size_t r = active ? oi : 0;
    const uint16_t* p1 = own1 + r * ld3 + 8 * half;
    const uint16_t* p2 = own2 + r * ld_own2 + 8 * half;
#pragma unroll
    for (int kk = 0; kk < DH / 16; ++kk) {
      f1[kk] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(p1 + kk * 16));
      f2[kk] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(p2 + kk * 16));
    }
    if (!OWN_KEYS) {
      const float2 st = *reinterpret_cast<const float2*>(stat + ((size_t)z * S + r) * 2);
      own_l2 = st.x;
      own_delta = st.y;
    }
  }
  wait_vmcnt<0>();  // nothing but the copies below is in flight from here on
#pragma unroll
  for (int kk = 0; kk < DH / 16; ++kk) asm volatile("" : "+v"(f1[kk]), "+v"(f2[kk]));
  asm volatile("" : "+v"(own_l2), "+v"(own_delta));

  RT rt1, rt2;
  CT ct1, ct2;
  rt1.init(ld3, 0, 64, wave, lane);
  rt2.init(ld_str2, 0, 64, wave, lane);
  ct1.init(ld3, 0, DH, wave, lane);
  ct2.init(ld_str2, 0, DH, wave, lane);
  // streamed blocks of 64 rows: keys 0 .. diagonal of the workgroup | queries diagonal .. end
  const int sb_begin = OWN_KEYS ? o0 / 64 : 0;
  const int sb_end = OWN_KEYS ? S / 64 : min(S, o0 + kBwdOwn) / 64;
  auto issue_block = [&](int blk, int st) {
    const int sb = min(blk, sb_end - 1);  // past the end: re-read the last block into a stage nobody reads again
    const uint32_t dst = lds_base + st * kStageBytes;
    const uint16_t* s1 = str1 + (size_t)sb * 64 * ld3;
    const uint16_t* s2 = str2 + (size_t)sb * 64 * ld_str2;
#pragma unroll
    for (int c = 0; c < HALVES; ++c)
#pragma unroll
      for (int t = 0; t < RT::kPerWave; ++t) {
        rt1.issue_one(t, dst + c * RT::kBytes, s1 + c * 64, wave);
        rt2.issue_one(t, dst + kRowBytes + c * RT::kBytes, s2 + c * 64, wave);
      }
#pragma unroll
    for (int t = 0; t < CT::kPerWave; ++t) {
      ct1.issue_one(t, dst + 2 * kRowBytes, s1, wave);
      if (OWN_KEYS) ct2.issue_one(t, dst + 2 * kRowBytes + CT::kBytes, s2, wave);
    }
    // (lse*log2e, delta) of the 64 streamed queries: 512 bytes, lanes 32-63 repeat lanes 0-31 into the spare half
    if (OWN_KEYS) dma16(dst + 2 * kRowBytes + 2 * CT::kBytes, stat + ((size_t)z * S + (size_t)sb * 64) * 2, (uint32_t)(lane & 31) * 16);
  };
  issue_block(sb_begin, 0);

  floatx16 acc1[1][TN], acc2[1][TN];  // dQ | dK, and dV
#pragma unroll
  for (int j = 0; j < TN; ++j)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc1[0][j][r] = acc2[0][j][r] = 0.f;

  int st = 0;
  for (int sb = sb_begin; sb < sb_end; ++sb) {
    wait_vmcnt<0>();
    lds_barrier();  // block sb visible to all waves; everybody is done reading the other stage
    issue_block(sb + 1, st ^ 1);
    // wave-uniform: does any (query, key <= query) pair of this wave fall into the block?
    const bool some = OWN_KEYS ? sb * 64 + 63 >= ow : sb * 64 <= ow + 31;
    if (active && some) {
      const uint16_t* lr1 = lds_raw + st * (kStageBytes / 2);
      const uint16_t* lr2 = lr1 + kRowBytes / 2;
      const uint16_t* lc1 = lr2 + kRowBytes / 2;
      const uint16_t* lc2 = lc1 + CT::kBytes / 2;
      const float* lstat = reinterpret_cast<const float*>(lc1 + kCols * (CT::kBytes / 2));
      // some pair of this wave and block lies above the diagonal
      const bool diagonal = OWN_KEYS ? sb * 64 < ow + 31 : sb * 64 + 63 > ow;
      // one half of the block (32 streamed rows) at a time, first products to second products: the score tiles of
      // one half only are alive at any time, which is what lets two waves share a SIMD's registers
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        floatx16 sacc, pacc;
#pragma unroll
        for (int r = 0; r < 16; ++r) sacc[r] = pacc[r] = 0.f;
#pragma unroll
        for (int c = 0; c < HALVES; ++c)
#pragma unroll
          for (int kk = 0; kk < 4; ++kk) {
            sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(RT::frag(lr1 + c * (RT::kBytes / 2), 32 * j, kk, lane),
                                                           f1[c * 4 + kk], sacc, 0, 0, 0);
            pacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(RT::frag(lr2 + c * (RT::kBytes / 2), 32 * j, kk, lane),
                                                           f2[c * 4 + kk], pacc, 0, 0, 0);
          }
        bf16x8 pf[2], dsf[2];
#pragma unroll
        for (int h = 0; h < 2; ++h) {
          float pe[8], de[8];
          // (lse, delta) of the streamed rows of this lane's elements: two runs of four consecutive rows, 32 bytes each
#pragma unroll
          for (int q = 0; q < 2; ++q) {
            float l2v[4] = {own_l2, own_l2, own_l2, own_l2}, dlv[4] = {own_delta, own_delta, own_delta, own_delta};
            if (OWN_KEYS) {
              const float4* sp = reinterpret_cast<const float4*>(lstat + 2 * (32 * j + 8 * (2 * h + q) + 4 * half));
              const float4 s0 = sp[0], s1 = sp[1];
              l2v[0] = s0.x; dlv[0] = s0.y; l2v[1] = s0.z; dlv[1] = s0.w;
              l2v[2] = s1.x; dlv[2] = s1.y; l2v[3] = s1.z; dlv[3] = s1.w;
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
              const int t = 4 * q + u, r = 8 * h + t;
              const int srow = 32 * j + 8 * (r >> 2) + 4 * half + (r & 3);  // streamed row inside the block
              float p = __builtin_amdgcn_exp2f(sacc[r] * scale_log2 - l2v[u]);
              if (diagonal) {
                const int si = sb * 64 + srow;
                const int key = OWN_KEYS ? oi : si, query = OWN_KEYS ? si : oi;
                if (key > query) p = 0.f;
              }
              pe[t] = p;
              de[t] = p * (pacc[r] - dlv[u]) * scale;
            }
          }
          pf[h] = __builtin_bit_cast(bf16x8, make_uint4(pack_bf16x2(pe[0], pe[1]), pack_bf16x2(pe[2], pe[3]),
                                                         pack_bf16x2(pe[4], pe[5]), pack_bf16x2(pe[6], pe[7])));
          dsf[h] = __builtin_bit_cast(bf16x8, make_uint4(pack_bf16x2(de[0], de[1]), pack_bf16x2(de[2], de[3]),
                                                          pack_bf16x2(de[4], de[5]), pack_bf16x2(de[6], de[7])));
        }
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
          for (int jj = 0; jj < TN; ++jj) {
            acc1[0][jj] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(flash_v_frag<DH>(lc1, 32 * jj, 2 * j + h, lane), dsf[h],
                                                                  acc1[0][jj], 0, 0, 0);
            if (OWN_KEYS)
              acc2[0][jj] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(flash_v_frag<DH>(lc2, 32 * jj, 2 * j + h, lane), pf[h],
                                                                    acc2[0][jj], 0, 0, 0);
          }
        if (OWN_KEYS) __builtin_amdgcn_sched_barrier(0);
      }
    }
    st ^= 1;
  }
  wait_vmcnt<0>();  // the trailing dummy copies must have landed before LDS is reused
  lds_barrier();
  if (!active) return;
  float* wave_lds = reinterpret_cast<float*>(lds_raw) + wave * (wave_epilogue_bytes<1, TN>() / 4);
  store_tiles_coalesced<1, TN>(acc1, EpiDgrad{nullptr, dqkv + (OWN_KEYS ? D : 0), ld3}, zb * S + ow, zh * DH, lane, wave_lds);
  if (OWN_KEYS) store_tiles_coalesced<1, TN>(acc2, EpiDgrad{nullptr, dqkv + 2 * D, ld3}, zb * S + ow, zh * DH, lane, wave_lds);
}

template <int DH, bool OWN_KEYS>
hipError_t launch_flash_bwd(hipStream_t s, int seqs, int S, int heads, const uint16_t* qkv, const uint16_t* dout, const float* stat,
                            uint16_t* dqkv) {
  constexpr int kBwdOwn = 32 * kBwdWaves;
  constexpr size_t row_bytes = (size_t)(DH / 64) * RowDma<64, kBwdWaves>::kBytes, col_bytes = ColDma<DH, kBwdWaves>::kBytes;
  constexpr size_t stage_bytes = 2 * (2 * row_bytes + (OWN_KEYS ? 2 : 1) * col_bytes + (OWN_KEYS ? 1024 : 0));
  constexpr size_t epi_bytes = (size_t)kBwdWaves * wave_epilogue_bytes<1, DH / 32>();
  constexpr size_t lds_bytes = stage_bytes > epi_bytes ? stage_bytes : epi_bytes;
  static_assert(lds_bytes <= 160 * 1024, "stages do not fit the LDS of a CU");
  auto kernel = attn_flash_bwd_kernel<DH, OWN_KEYS>;
  static hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
  if (attr != hipSuccess) return attr;
  const float scale = 1.0f / sqrtf((float)DH);
  hipLaunchKernelGGL(kernel, dim3(seqs * heads, (S + kBwdOwn - 1) / kBwdOwn), dim3(64 * kBwdWaves), lds_bytes, s, S, heads, qkv, dout,
                     stat, dqkv, scale, scale * kLog2e);
  return hipGetLastError();
}

// bytes of scratch per sequence: scores and dP in fp32, P and dS in bf16
inline size_t per_seq_bytes(int S, int heads) { return (size_t)heads * S * S * 12; }

}  // namespace

bool attention_mfma_supported(int S, int heads, int dh) {
  return S >= 128 && S % 64 == 0 && dh % 64 == 0 && dh <= 256 && heads >= 1 && (size_t)heads * S * S * 4 < (1ull << 31) &&
         3ull * heads * dh * S * 2 < (1ull << 31);
}

size_t attention_mfma_scratch_bytes(int seqs, int S, int heads) {
  // as many sequences at a time as fit 2 GiB, at least one
  const size_t per = per_seq_bytes(S, heads);
  const size_t chunk = std::max<size_t>(1, std::min<size_t>(seqs, (2ull << 30) / per));
  return chunk * per;
}

bool attention_flash_fwd_supported(int seqs, int S, int heads, int dh) {
  return (dh == 64 || dh == 128) && S >= 64 && S % 64 == 0 && heads >= 1 && seqs >= 1 && (long)seqs * heads <= 65535 &&
         64ull * 3 * heads * dh * 2 < (1ull << 31);  // 32-bit byte offsets inside one 64-key block
}

hipError_t attention_flash_fwd(hipStream_t s, int seqs, int S, int heads, int dh, const uint16_t* qkv, uint16_t* out, float* lse) {
  if (!attention_flash_fwd_supported(seqs, S, heads, dh)) return hipErrorNotSupported;
  return dh == 64 ? launch_flash_fwd<64>(s, seqs, S, heads, qkv, out, lse) : launch_flash_fwd<128>(s, seqs, S, heads, qkv, out, lse);
}

size_t attention_flash_bwd_scratch_bytes(int seqs, int S, int heads) { return (size_t)seqs * heads * S * 2 * sizeof(float); }

hipError_t attention_flash_bwd(hipStream_t s, int seqs, int S, int heads, int dh, const uint16_t* qkv, const uint16_t* out,
                               const uint16_t* dout, const float* lse, uint16_t* dqkv, void* scratch, size_t scratch_bytes) {
  if (!attention_flash_fwd_supported(seqs, S, heads, dh) || !scratch || scratch_bytes < attention_flash_bwd_scratch_bytes(seqs, S, heads))
    return hipErrorNotSupported;
  float* stat = (float*)scratch;
  const size_t rows = (size_t)seqs * S;
  hipLaunchKernelGGL(attn_stat_kernel, dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, s, S, heads, dh, rows, dout, out, lse, stat);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  e = dh == 64 ? launch_flash_bwd<64, false>(s, seqs, S, heads, qkv, dout, stat, dqkv)
               : launch_flash_bwd<128, false>(s, seqs, S, heads, qkv, dout, stat, dqkv);
  if (e != hipSuccess) return e;
  return dh == 64 ? launch_flash_bwd<64, true>(s, seqs, S, heads, qkv, dout, stat, dqkv)
                  : launch_flash_bwd<128, true>(s, seqs, S, heads, qkv, dout, stat, dqkv);
}

hipError_t attention_mfma_fwd(hipStream_t s, int seqs, int S, int heads, int dh, const uint16_t* qkv, uint16_t* out, float* lse,
                              void* scratch, size_t scratch_bytes) {
  const int D = heads * dh;
  const size_t per = per_seq_bytes(S, heads);
  const int chunk = (int)std::min<size_t>(seqs, scratch_bytes / per);
  if (chunk < 1) return hipErrorInvalidValue;
  const float scale = 1.0f / sqrtf((float)dh);
  const long SS = (long)S * S;
  for (int b0 = 0; b0 < seqs; b0 += chunk) {
    const int nb = std::min(chunk, seqs - b0);
    const int Z = nb * heads;
    float* scores = (float*)scratch;
    uint16_t* P = (uint16_t*)((char*)scratch + (size_t)chunk * heads * SS * 8);
    const uint16_t* q = qkv + (size_t)b0 * S * 3 * D;
    hipError_t e = launch_attn_gemm<128, false, false>(s, Z, S, S, dh, q, 3 * D, q + D, 3 * D, EpiWgrad{scores, S},
                                                       BatchOffsets{heads, (long)S * 3 * D, dh, (long)S * 3 * D, dh, heads * SS, SS},
                                                       kSkipTiles);
    if (e != hipSuccess) return e;
    const size_t rows = (size_t)Z * S;
    hipLaunchKernelGGL(attn_softmax_fwd_kernel, dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, s, S, rows, scale, scores, P,
                       lse + (size_t)b0 * heads * S);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    e = launch_attn_gemm<128, false, true>(s, Z, S, dh, S, P, S, q + 2 * D, 3 * D, EpiDgrad{nullptr, out + (size_t)b0 * S * D, D},
                                           BatchOffsets{heads, heads * SS, SS, (long)S * 3 * D, dh, (long)S * D, dh}, kLimitK);
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

hipError_t attention_mfma_bwd(hipStream_t s, int seqs, int S, int heads, int dh, const uint16_t* qkv, const uint16_t* dout,
                              const float* lse, uint16_t* dqkv, void* scratch, size_t scratch_bytes) {
  const int D = heads * dh;
  const size_t per = per_seq_bytes(S, heads);
  const int chunk = (int)std::min<size_t>(seqs, scratch_bytes / per);
  if (chunk < 1) return hipErrorInvalidValue;
  const float scale = 1.0f / sqrtf((float)dh);
  const long SS = (long)S * S, row3 = (long)S * 3 * D, rowd = (long)S * D;
  for (int b0 = 0; b0 < seqs; b0 += chunk) {
    const int nb = std::min(chunk, seqs - b0);
    const int Z = nb * heads;
    const size_t zss = (size_t)chunk * heads * SS;
    float* scores = (float*)scratch;
    float* dP = scores + zss;
    uint16_t* P = (uint16_t*)(dP + zss);
    uint16_t* dS = P + zss;
    const uint16_t* q = qkv + (size_t)b0 * row3;
    const uint16_t* dob = dout + (size_t)b0 * rowd;
    uint16_t* dq = dqkv + (size_t)b0 * row3;
    const BatchOffsets to_scores{heads, row3, dh, row3, dh, heads * SS, SS};
    hipError_t e = launch_attn_gemm<128, false, false>(s, Z, S, S, dh, q, 3 * D, q + D, 3 * D, EpiWgrad{scores, S}, to_scores,
                                                       kSkipTiles);
    if (e != hipSuccess) return e;
    e = launch_attn_gemm<128, false, false>(s, Z, S, S, dh, dob, D, q + 2 * D, 3 * D, EpiWgrad{dP, S},
                                            BatchOffsets{heads, rowd, dh, row3, dh, heads * SS, SS}, kSkipTiles);
    if (e != hipSuccess) return e;
    const size_t rows = (size_t)Z * S;
    hipLaunchKernelGGL(attn_softmax_bwd_kernel, dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, s, S, rows, scale, scores, dP,
                       lse + (size_t)b0 * heads * S, P, dS);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    // dQ = dS K        (rows: queries, contraction over keys <= the tile's last query)
    e = launch_attn_gemm<128, false, true>(s, Z, S, dh, S, dS, S, q + D, 3 * D, EpiDgrad{nullptr, dq, 3 * D},
                                           BatchOffsets{heads, heads * SS, SS, row3, dh, row3, dh}, kLimitK);
    if (e != hipSuccess) return e;
    // dK = dS^T Q      (rows: keys, contraction over queries >= the tile's first key)
    e = launch_attn_gemm<128, true, true>(s, Z, S, dh, S, dS, S, q, 3 * D, EpiDgrad{nullptr, dq + D, 3 * D},
                                          BatchOffsets{heads, heads * SS, SS, row3, dh, row3, dh}, kStartK);
    if (e != hipSuccess) return e;
    // dV = P^T dO
    e = launch_attn_gemm<128, true, true>(s, Z, S, dh, S, P, S, dob, D, EpiDgrad{nullptr, dq + 2 * D, 3 * D},
                                          BatchOffsets{heads, heads * SS, SS, rowd, dh, row3, dh}, kStartK);
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

}  // namespace tp
