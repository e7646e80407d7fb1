// Device code shared by the bf16 matrix-core kernels (dense GEMMs and implicit-GEMM convolutions):
// MFMA fragment types, the epilogues, the workgroup-id -> tile mapping, and the direct-to-LDS copy
// machinery with its two LDS stage layouts.  Everything lives in an unnamed namespace: each
// translation unit that includes this header gets its own copy.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "device_utils.h"

namespace tp {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef short shortx4 __attribute__((ext_vector_type(4)));
typedef short shortx8 __attribute__((ext_vector_type(8)));

// ---- epilogues ---------------------------------------------------------------------------------
// bf16 outputs: the MFMA operands are swapped (the kernel accumulates the transposed tile), so
// that each lane ends up with 4 consecutive COLUMNS n..n+3 of one output row m and can load and
// store 8 contiguous bytes without a trip through LDS.  fp32 output (wgrad) keeps the plain
// orientation, where the 32 lanes of a half wave already cover 128 contiguous bytes.
// ADD: the epilogue also adds `addend` (an [M x ldc] tensor: the residual add that follows the layer) to the rounded
// activation; a type of its own so that the plain forward GEMM carries none of it.
template <bool ADD>
struct EpiFpropT {
  const float* bias; uint16_t* d_out; uint16_t* a_out; int act; int ldc;  // d_out: act'(z) for the backward, or null
  const uint16_t* addend = nullptr;
  static constexpr bool kSwap = true;
  // 8 consecutive columns n..n+7 of row m (n and ldc multiples of 8)
  __device__ __forceinline__ void row8(int m, int n, float (&v)[8]) const {
    const size_t i = (size_t)m * ldc + n;
    const float4 b0 = *reinterpret_cast<const float4*>(bias + n), b1 = *reinterpret_cast<const float4*>(bias + n + 4);
    const float b[8] = {b0.x, b0.y, b0.z, b0.w, b1.x, b1.y, b1.z, b1.w};
    float a[8], d[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const ActPair p = act_pair_fast(v[j] + b[j], act);
      a[j] = p.a;
      d[j] = p.d;
    }
    if constexpr (ADD) {
      const uint4 u = *reinterpret_cast<const uint4*>(addend + i);
      const uint32_t w[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        a[2 * j] = bf16_to_float(float_to_bf16(a[2 * j])) + __uint_as_float(w[j] << 16);
        a[2 * j + 1] = bf16_to_float(float_to_bf16(a[2 * j + 1])) + __uint_as_float(w[j] & 0xffff0000u);
      }
    }
    if (d_out)
      *reinterpret_cast<uint4*>(d_out + i) =
          make_uint4(pack_bf16x2(d[0], d[1]), pack_bf16x2(d[2], d[3]), pack_bf16x2(d[4], d[5]), pack_bf16x2(d[6], d[7]));
    *reinterpret_cast<uint4*>(a_out + i) =
        make_uint4(pack_bf16x2(a[0], a[1]), pack_bf16x2(a[2], a[3]), pack_bf16x2(a[4], a[5]), pack_bf16x2(a[6], a[7]));
  }
  __device__ __forceinline__ void quad(int m, int n, int count, float v0, float v1, float v2, float v3) const {
    const size_t i = (size_t)m * ldc + n;
    if (count == 4 && (ldc & 3) == 0 && !ADD) {
      const float4 b = *reinterpret_cast<const float4*>(bias + n);
      const ActPair p0 = act_pair_fast(v0 + b.x, act), p1 = act_pair_fast(v1 + b.y, act);
      const ActPair p2 = act_pair_fast(v2 + b.z, act), p3 = act_pair_fast(v3 + b.w, act);
      if (d_out) *reinterpret_cast<uint2*>(d_out + i) = make_uint2(pack_bf16x2(p0.d, p1.d), pack_bf16x2(p2.d, p3.d));
      *reinterpret_cast<uint2*>(a_out + i) = make_uint2(pack_bf16x2(p0.a, p1.a), pack_bf16x2(p2.a, p3.a));
    } else {
      const float v[4] = {v0, v1, v2, v3};
      for (int j = 0; j < count; ++j) {
        const ActPair p = act_pair_fast(v[j] + bias[n + j], act);
        if (d_out) d_out[i + j] = float_to_bf16(p.d);
        a_out[i + j] = ADD ? float_to_bf16(bf16_to_float(float_to_bf16(p.a)) + bf16_to_float(addend[i + j])) : float_to_bf16(p.a);
      }
    }
  }
};
using EpiFprop = EpiFpropT<false>;
using EpiFpropAdd = EpiFpropT<true>;
struct EpiDgrad {
  const uint16_t* d_prev; uint16_t* out; int ldc;  // d_prev: saved act'(z) of the previous layer, or null
  int relu_mask = 0;  // 1: d_prev holds the previous layer's ReLU OUTPUT instead; its derivative is (output > 0)
  static constexpr bool kSwap = true;
  __device__ __forceinline__ float through(float v, float d) const { return relu_mask ? (d > 0.f ? v : 0.f) : v * d; }
  // 8 consecutive columns n..n+7 of row m (n and ldc multiples of 8)
  __device__ __forceinline__ void row8(int m, int n, float (&v)[8]) const {
    const size_t i = (size_t)m * ldc + n;
    if (d_prev) {
      const uint4 d = *reinterpret_cast<const uint4*>(d_prev + i);
      const uint32_t w[4] = {d.x, d.y, d.z, d.w};
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        v[2 * j] = through(v[2 * j], __uint_as_float(w[j] << 16));
        v[2 * j + 1] = through(v[2 * j + 1], __uint_as_float(w[j] & 0xffff0000u));
      }
    }
    *reinterpret_cast<uint4*>(out + i) =
        make_uint4(pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]), pack_bf16x2(v[4], v[5]), pack_bf16x2(v[6], v[7]));
  }
  __device__ __forceinline__ void quad(int m, int n, int count, float v0, float v1, float v2, float v3) const {
    const size_t i = (size_t)m * ldc + n;
    if (count == 4 && (ldc & 3) == 0) {
      if (d_prev) {
        const uint2 d = *reinterpret_cast<const uint2*>(d_prev + i);
        v0 = through(v0, __uint_as_float(d.x << 16));
        v1 = through(v1, __uint_as_float(d.x & 0xffff0000u));
        v2 = through(v2, __uint_as_float(d.y << 16));
        v3 = through(v3, __uint_as_float(d.y & 0xffff0000u));
      }
      *reinterpret_cast<uint2*>(out + i) = make_uint2(pack_bf16x2(v0, v1), pack_bf16x2(v2, v3));
    } else {
      const float v[4] = {v0, v1, v2, v3};
      for (int j = 0; j < count; ++j) {
        float d = v[j];
        if (d_prev) d = through(d, bf16_to_float(d_prev[i + j]));
        out[i + j] = float_to_bf16(d);
      }
    }
  }
};
struct EpiWgrad {
  float* out; int ldc;
  static constexpr bool kSwap = false;
  __device__ __forceinline__ void elem(int m, int n, float v) const { out[(size_t)m * ldc + n] = v; }
};

// Accumulator element r of a lane sits at tile row 8*(r/4) + 4*(lane/32) + r%4, tile column
// lane%32 of what the MFMA computed; with swapped operands that is the transposed output tile.
template <int TM, int TN, class Epi>
__device__ __forceinline__ void store_tiles(const floatx16 (&acc)[TM][TN], const Epi& epi, int mbase, int nbase, int M,
                                            int N, int lane) {
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      if constexpr (Epi::kSwap) {
        const int m = mbase + i * 32 + (lane & 31);
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const int n = nbase + j * 32 + 8 * g + 4 * (lane >> 5);
          if (m < M && n < N)
            epi.quad(m, n, min(4, N - n), acc[i][j][4 * g], acc[i][j][4 * g + 1], acc[i][j][4 * g + 2],
                     acc[i][j][4 * g + 3]);
        }
      } else {
        const int n = nbase + j * 32 + (lane & 31);
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int m = mbase + i * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
          if (m < M && n < N) epi.elem(m, n, acc[i][j][r]);
        }
      }
    }
}

// bf16 outputs, coalesced.  Straight from the accumulators a lane owns 4 columns of one row, so
// a store instruction would touch 32 rows with 16 bytes each, and the memory pipeline takes one
// partial cache line per row: at 64 k tiles per workgroup that is tolerable, for short
// contractions (convolutions) it costs more than the multiplications.  Here each wave turns its
// (32*TM) x (32*TN) fp32 tile through a private LDS region (row pitch 32*TN + 4 floats: writes
// and reads are bank-conflict free) and then walks it row-wise: a lane takes 8 consecutive
// columns, applies the epilogue and stores 16 bytes, 4*TN lanes per row.  Needs the whole wave
// tile inside the matrix and N a multiple of 8; the caller falls back to store_tiles otherwise.
template <int TM, int TN>
constexpr int wave_epilogue_bytes() { return 32 * TM * (32 * TN + 4) * 4; }

template <int TM, int TN, class Epi>
__device__ __forceinline__ void store_tiles_coalesced(const floatx16 (&acc)[TM][TN], const Epi& epi, int mbase, int nbase,
                                                      int lane, float* wave_lds) {
  constexpr int PITCH = 32 * TN + 4;
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        float* p = wave_lds + (i * 32 + (lane & 31)) * PITCH + j * 32 + 8 * g + 4 * (lane >> 5);
        *reinterpret_cast<float4*>(p) =
            make_float4(acc[i][j][4 * g], acc[i][j][4 * g + 1], acc[i][j][4 * g + 2], acc[i][j][4 * g + 3]);
      }
  // same wave on both sides: LDS operations of a wave complete in order
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
  constexpr int kLanesPerRow = 4 * TN;            // 8 columns each
  constexpr int kRowsPerPass = 64 / kLanesPerRow;
  const int rsub = lane / kLanesPerRow, c8 = (lane % kLanesPerRow) * 8;
#pragma unroll
  for (int r0 = 0; r0 < 32 * TM; r0 += kRowsPerPass) {
    const int r = r0 + rsub;
    const float* p = wave_lds + r * PITCH + c8;
    const float4 lo = *reinterpret_cast<const float4*>(p), hi = *reinterpret_cast<const float4*>(p + 4);
    float v[8] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
    epi.row8(mbase + r, nbase + c8, v);
  }
}

// acc += A_frag . B_frag, or its transpose when the epilogue wants columns along the registers
template <bool SWAP>
__device__ __forceinline__ floatx16 mma(bf16x8 a, bf16x8 b, floatx16 c) {
  return SWAP ? __builtin_amdgcn_mfma_f32_32x32x16_bf16(b, a, c, 0, 0, 0)
              : __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// ---- workgroup id -> output tile, XCD aware ---------------------------------------------------
// Hardware hands workgroup b to XCD b % 8.  The 8 XCDs are laid out as an xm x xn grid over the
// tile space; XCD (xi, xj) owns the (tiles_m/xm) x (tiles_n/xn) patch at that position.
struct TileMap {
  int tiles_m, tiles_n, xm, xn;  // xm*xn == 8, or xm == 0 for the plain row-major mapping
  __device__ __forceinline__ void get(int b, int& tm, int& tn) const {
    if (xm == 0) { tm = b / tiles_n; tn = b % tiles_n; return; }
    const int xcd = b & 7, i = b >> 3;
    const int cm = tiles_m / xm, cn = tiles_n / xn;
    tm = (xcd / xn) * cm + i / cn;
    tn = (xcd % xn) * cn + i % cn;
  }
};

// Optional side job of a forward GEMM: keep a copy of its input (the stage saves the activations a
// micro-batch arrives with).  The workgroups share the copy evenly, 16 bytes per lane per step.
struct SideCopy {
  const uint4* src;
  uint4* dst;
  size_t nvec;  // 16-byte units; 0 = nothing to do
};

inline TileMap make_tile_map(int tiles_m, int tiles_n) {
  static const int cand[4][2] = {{2, 4}, {4, 2}, {1, 8}, {8, 1}};
  TileMap best{tiles_m, tiles_n, 0, 0};
  long best_cost = -1;
  for (auto& c : cand) {
    if (tiles_m % c[0] || tiles_n % c[1]) continue;
    const long cost = tiles_m / c[0] + tiles_n / c[1];  // operand panels one XCD touches
    if (best_cost < 0 || cost < best_cost) { best_cost = cost; best = TileMap{tiles_m, tiles_n, c[0], c[1]}; }
  }
  return best;
}

// ================================================================================================
// Direct-to-LDS variant
// ================================================================================================
// global_load_lds_dwordx4 copies 16 bytes per lane from global memory to LDS address
// M0 + 16*lane: one wave instruction fills 1 KB of contiguous LDS, so tiles lie unpadded and
// bank conflicts are removed by storing chunk c of a row in slot c ^ f(row); the XOR is applied
// when each lane picks the global chunk it fetches for its (fixed) LDS slot, and again when
// fragments are read.  The copies do not touch the register file and complete out of band;
// s_waitcnt vmcnt(n) keeps the NS-1 newest tiles in flight while the oldest is consumed.

constexpr int DBK = 64;  // k extent of one stage

__device__ __forceinline__ void dma16(uint32_t lds_byte_addr, const void* sbase, uint32_t voff_bytes) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
               :
               : "s"(lds_byte_addr), "v"(voff_bytes), "s"(sbase)
               : "memory");
}

template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// Barrier without the global-memory fence of __syncthreads(): only LDS traffic of this wave is
// drained, outstanding global->LDS copies of later stages stay in flight.
__device__ __forceinline__ void lds_barrier() {
  asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
}

__device__ __forceinline__ uint32_t lds_addr_of(const void* p) {
  return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const char*)p;
}

// k-contiguous operand, stage = [R rows][64 k] = 128 B per row, 8 chunks; slot = chunk ^ ((row/2)%8).
template <int R, int NW>
struct RowDma {
  static constexpr int kInstr = R / 8;          // wave instructions per stage (8 rows each)
  static constexpr int kPerWave = kInstr / NW;
  static constexpr int kBytes = R * DBK * 2;
  static_assert(kInstr % NW == 0, "rows do not divide among the waves");
  uint32_t voff[kPerWave];

  __device__ __forceinline__ void init(int ld, int r0, int rows, int wave, int lane) {
#pragma unroll
    for (int t = 0; t < kPerWave; ++t) {
      const int r = 8 * (wave + NW * t) + (lane >> 3);
      const int c = (lane & 7) ^ ((r >> 1) & 7);
      voff[t] = (uint32_t)(((size_t)min(r0 + r, rows - 1) * ld + c * 8) * 2);
    }
  }
  // base: operand pointer advanced to the stage's first k
  __device__ __forceinline__ void issue_one(int t, uint32_t lds_stage, const uint16_t* base, int wave) const {
    dma16(lds_stage + (wave + NW * t) * 1024, base, voff[t]);
  }
  static __device__ __forceinline__ size_t tile_step(int) { return DBK; }  // elements between k tiles
  static __device__ __forceinline__ bf16x8 frag(const uint16_t* lds, int rbase, int kk, int lane) {
    const int r = rbase + (lane & 31);
    const int c = (kk * 2 + (lane >> 5)) ^ ((r >> 1) & 7);
    const uint4 v = *reinterpret_cast<const uint4*>(lds + r * DBK + c * 8);
    return __builtin_bit_cast(bf16x8, v);
  }
};

// k-strided operand, stage = [64 k][R rows]; R/8 chunks per k row; slot = chunk ^ f(k) so that the
// four k rows of one transpose read fall into four different 64-byte bank groups.
template <int R, int NW>
struct ColDma {
  static constexpr int kPerK = R / 8;
  static constexpr int kInstr = DBK * kPerK / 64;
  static constexpr int kPerWave = kInstr / NW;
  static constexpr int kBytes = R * DBK * 2;
  static_assert(kInstr % NW == 0, "rows do not divide among the waves");
  static_assert(R >= 64, "stage rows shorter than 128 bytes are not laid out");
  uint32_t voff[kPerWave];

  static __device__ __forceinline__ int swz(int k) { return R >= 128 ? 4 * (k & 3) : 4 * ((k >> 1) & 1); }

  __device__ __forceinline__ void init(int ld, int r0, int rows, int wave, int lane) {
#pragma unroll
    for (int t = 0; t < kPerWave; ++t) {
      const int flat = 64 * (wave + NW * t) + lane;
      const int k = flat / kPerK;
      const int c = (flat % kPerK) ^ swz(k);
      // chunks past the edge re-read the last valid chunk: those columns are never stored
      voff[t] = (uint32_t)(((size_t)k * ld + min(r0 + c * 8, rows - 8)) * 2);
    }
  }
  __device__ __forceinline__ void issue_one(int t, uint32_t lds_stage, const uint16_t* base, int wave) const {
    dma16(lds_stage + (wave + NW * t) * 1024, base, voff[t]);
  }
  static __device__ __forceinline__ size_t tile_step(int ld) { return (size_t)DBK * ld; }
  static __device__ __forceinline__ bf16x8 frag(const uint16_t* lds, int rbase, int kk, int lane) {
    const int g = lane >> 4, s = lane & 15;
    const int k = kk * 16 + 8 * (g >> 1) + (s >> 2);
    const int col = rbase + 16 * (g & 1) + 4 * (s & 3);
    const int slot = (col >> 3) ^ swz(k);
    typedef __attribute__((address_space(3))) shortx4* lds_ptr;
    const uint16_t* p = lds + k * R + slot * 8 + (col & 7);
    const shortx4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(p));
    const shortx4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(p + 4 * R));  // k+4: same swizzle
    const shortx8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, v);
  }
};

template <int R, int NW, bool COL>
struct DmaSel { using type = RowDma<R, NW>; };
template <int R, int NW>
struct DmaSel<R, NW, true> { using type = ColDma<R, NW>; };

}  // namespace

}  // namespace tp
