// Causal multi-head attention on the matrix cores (bf16), as batched GEMMs around row-wise softmax
// kernels.  One workgroup row (blockIdx.y) per (sequence, head); the GEMM kernel is the direct-to-LDS
// pipeline of the dense layers with per-batch operand offsets and three causal shortcuts:
//   skip    output tiles that lie entirely above the diagonal are not computed (Q K^T, dO V^T);
//   limit   the contraction over keys stops at the last query row of the tile (P V, dS K);
//   start   the contraction over queries starts at the first key row of the tile (P^T dO, dS^T Q).
// forward   S = Q K^T (fp32)  ->  P = softmax(scale S) (bf16, zeros above the diagonal), lse  ->  O = P V
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
