// Layer normalisation, residual add and causal multi-head self-attention (forward and backward).
//
// These are plain wavefront kernels in fp32 arithmetic: correct at every shape the stage accepts,
// not yet tuned (the attention in particular does its dot products on the vector ALUs; the GEMMs
// around it are where a transformer stage spends its time).
//
// Attention works one query row per wave at a time.  For each tile of 64 keys: lane j forms the
// score of key j (a dot product over the head dimension against the query held in LDS), the wave
// reduces max and sum for the running softmax, then lane d accumulates output column d with the 64
// probabilities broadcast from the lanes that hold them.  K/V tiles are staged in LDS once per
// workgroup and shared by its query rows.  The backward pass recomputes the probabilities from the
// saved log-sum-exp: one kernel walks over the keys of each query (dQ), a second one over the
// queries of each key (dK, dV); rowsum(dP . P) comes from dO . O.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <algorithm>

#include "device_utils.h"
#include "kernels.h"
#include "transformer.h"

namespace tp {

namespace {

constexpr int kThreads = 256;
constexpr float kLnEps = 1e-5f;

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
// value of lane `src` (wave uniform) for every lane, whatever the execution mask
__device__ __forceinline__ float lane_value(float v, int src) {
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), src));
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}

// ---- layer normalisation: one wave per row ------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(kThreads) void layernorm_fwd_kernel(size_t rows, int D, const T* __restrict__ x,
                                                                 const float* __restrict__ gamma, const float* __restrict__ beta,
                                                                 T* __restrict__ y, float* __restrict__ stats) {
  const int lane = threadIdx.x & 63;
  const size_t r = (size_t)blockIdx.x * (kThreads / 64) + (threadIdx.x >> 6);
  if (r >= rows) return;
  const T* xr = x + r * D;
  float s = 0.f;
  for (int d = lane; d < D; d += 64) s += to_float(xr[d]);
  const float mean = wave_sum(s) / D;
  float v = 0.f;
  for (int d = lane; d < D; d += 64) {
    const float c = to_float(xr[d]) - mean;
    v += c * c;
  }
  const float rstd = rsqrtf(wave_sum(v) / D + kLnEps);
  for (int d = lane; d < D; d += 64) y[r * D + d] = from_float<T>(fmaf((to_float(xr[d]) - mean) * rstd, gamma[d], beta[d]));
  if (lane == 0) {
    stats[2 * r] = mean;
    stats[2 * r + 1] = rstd;
  }
}

// dx per row (one wave per row); each workgroup also adds dgamma / dbeta over its rows into
// partial[block][2*D] (fixed order: the wave's rows in sequence, then the four waves through LDS)
template <typename T>
__global__ __launch_bounds__(kThreads) void layernorm_bwd_kernel(size_t rows, int D, int rows_per_block, const T* __restrict__ dy,
                                                                 const T* __restrict__ x, const float* __restrict__ stats,
                                                                 const float* __restrict__ gamma_s, const float* __restrict__ gamma_l,
                                                                 float alpha, float beta_c, T* __restrict__ dx,
                                                                 float* __restrict__ partial) {
  extern __shared__ float sm[];  // [4 waves][2*D]
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  float* mine = sm + (size_t)wave * 2 * D;
  for (int d = lane; d < 2 * D; d += 64) mine[d] = 0.f;
  const size_t r0 = (size_t)blockIdx.x * rows_per_block;
  const size_t r1 = std::min(rows, r0 + rows_per_block);
  for (size_t r = r0 + wave; r < r1; r += kThreads / 64) {
    const float mean = stats[2 * r], rstd = stats[2 * r + 1];
    const T* xr = x + r * D;
    const T* gr = dy + r * D;
    float s1 = 0.f, s2 = 0.f;
    for (int d = lane; d < D; d += 64) {
      const float g = fmaf(alpha, gamma_s[d], beta_c * gamma_l[d]);
      const float xh = (to_float(xr[d]) - mean) * rstd, dyv = to_float(gr[d]);
      const float dxh = dyv * g;
      s1 += dxh;
      s2 += dxh * xh;
      mine[d] += dyv * xh;   // same lane touches the same d every row: no race
      mine[D + d] += dyv;
    }
    s1 = wave_sum(s1) / D;
    s2 = wave_sum(s2) / D;
    for (int d = lane; d < D; d += 64) {
      const float g = fmaf(alpha, gamma_s[d], beta_c * gamma_l[d]);
      const float xh = (to_float(xr[d]) - mean) * rstd;
      dx[r * D + d] = from_float<T>(rstd * (to_float(gr[d]) * g - s1 - xh * s2));
    }
  }
  __syncthreads();
  for (int d = threadIdx.x; d < 2 * D; d += kThreads)
    partial[(size_t)blockIdx.x * 2 * D + d] = sm[d] + sm[2 * D + d] + sm[4 * D + d] + sm[6 * D + d];
}

// bf16 rows whose width is NG * 512 (NG <= 8): every lane owns NG groups of 8 consecutive features,
// reads them with 16-byte loads, keeps the row in registers between the two passes, and carries its
// share of dgamma / dbeta in registers across the rows of the workgroup.
__device__ __forceinline__ void unpack8(const uint4& v, float (&f)[8]) {
  const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    f[2 * j] = __uint_as_float(w[j] << 16);
    f[2 * j + 1] = __uint_as_float(w[j] & 0xffff0000u);
  }
}
__device__ __forceinline__ uint4 pack8(const float (&f)[8]) {
  return make_uint4(pack_bf16x2(f[0], f[1]), pack_bf16x2(f[2], f[3]), pack_bf16x2(f[4], f[5]), pack_bf16x2(f[6], f[7]));
}

template <int NG>
__global__ __launch_bounds__(kThreads) void layernorm_fwd_bf16_kernel(size_t rows, const uint16_t* __restrict__ x,
                                                                      const float* __restrict__ gamma, const float* __restrict__ beta,
                                                                      uint16_t* __restrict__ y, float* __restrict__ stats) {
  constexpr int D = NG * 512;
  const int lane = threadIdx.x & 63;
  const size_t r = (size_t)blockIdx.x * (kThreads / 64) + (threadIdx.x >> 6);
  if (r >= rows) return;
  float v[NG][8];
  float s = 0.f;
#pragma unroll
  for (int k = 0; k < NG; ++k) {
    unpack8(*reinterpret_cast<const uint4*>(x + r * D + (lane + 64 * k) * 8), v[k]);
#pragma unroll
    for (int j = 0; j < 8; ++j) s += v[k][j];
  }
  const float mean = wave_sum(s) / D;
  float q = 0.f;
#pragma unroll
  for (int k = 0; k < NG; ++k)
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      v[k][j] -= mean;
      q += v[k][j] * v[k][j];
    }
  const float rstd = rsqrtf(wave_sum(q) / D + kLnEps);
#pragma unroll
  for (int k = 0; k < NG; ++k) {
    const int d0 = (lane + 64 * k) * 8;
    const float4 g0 = *reinterpret_cast<const float4*>(gamma + d0), g1 = *reinterpret_cast<const float4*>(gamma + d0 + 4);
    const float4 b0 = *reinterpret_cast<const float4*>(beta + d0), b1 = *reinterpret_cast<const float4*>(beta + d0 + 4);
    const float g[8] = {g0.x, g0.y, g0.z, g0.w, g1.x, g1.y, g1.z, g1.w}, b[8] = {b0.x, b0.y, b0.z, b0.w, b1.x, b1.y, b1.z, b1.w};
    float o[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) o[j] = fmaf(v[k][j] * rstd, g[j], b[j]);
    *reinterpret_cast<uint4*>(y + r * D + d0) = pack8(o);
  }
  if (lane == 0) {
    stats[2 * r] = mean;
    stats[2 * r + 1] = rstd;
  }
}

template <int NG>
__global__ __launch_bounds__(kThreads) void layernorm_bwd_bf16_kernel(size_t rows, int rows_per_block, const uint16_t* __restrict__ dy,
                                                                      const uint16_t* __restrict__ x, const float* __restrict__ stats,
                                                                      const float* __restrict__ gamma_s, const float* __restrict__ gamma_l,
                                                                      float alpha, float beta_c, const uint16_t* __restrict__ addend,
                                                                      uint16_t* __restrict__ dx, float* __restrict__ partial) {
  constexpr int D = NG * 512;
  extern __shared__ float sm[];  // [4 waves][2*D]
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  float g[NG][8], dg[NG][8], db[NG][8];
#pragma unroll
  for (int k = 0; k < NG; ++k) {
    const int d0 = (lane + 64 * k) * 8;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      g[k][j] = fmaf(alpha, gamma_s[d0 + j], beta_c * gamma_l[d0 + j]);
      dg[k][j] = db[k][j] = 0.f;
    }
  }
  const size_t r0 = (size_t)blockIdx.x * rows_per_block;
  const size_t r1 = std::min(rows, r0 + rows_per_block);
  for (size_t r = r0 + wave; r < r1; r += kThreads / 64) {
    const float mean = stats[2 * r], rstd = stats[2 * r + 1];
    float xh[NG][8], dyv[NG][8];
    float s1 = 0.f, s2 = 0.f;
#pragma unroll
    for (int k = 0; k < NG; ++k) {
      const size_t at = r * D + (lane + 64 * k) * 8;
      unpack8(*reinterpret_cast<const uint4*>(x + at), xh[k]);
      unpack8(*reinterpret_cast<const uint4*>(dy + at), dyv[k]);
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        xh[k][j] = (xh[k][j] - mean) * rstd;
        const float dxh = dyv[k][j] * g[k][j];
        s1 += dxh;
        s2 += dxh * xh[k][j];
        dg[k][j] += dyv[k][j] * xh[k][j];
        db[k][j] += dyv[k][j];
      }
    }
    s1 = wave_sum(s1) / D;
    s2 = wave_sum(s2) / D;
#pragma unroll
    for (int k = 0; k < NG; ++k) {
      float o[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) o[j] = rstd * (dyv[k][j] * g[k][j] - s1 - xh[k][j] * s2);
      if (addend) {  // the gradient that went around the residual branch: added to the rounded result, as a separate add would
        float sk[8];
        unpack8(*reinterpret_cast<const uint4*>(addend + r * D + (lane + 64 * k) * 8), sk);
#pragma unroll
        for (int j = 0; j < 8; ++j) o[j] = bf16_to_float(float_to_bf16(o[j])) + sk[j];
      }
      *reinterpret_cast<uint4*>(dx + r * D + (lane + 64 * k) * 8) = pack8(o);
    }
  }
  float* mine = sm + (size_t)wave * 2 * D;
#pragma unroll
  for (int k = 0; k < NG; ++k)
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      mine[(lane + 64 * k) * 8 + j] = dg[k][j];
      mine[D + (lane + 64 * k) * 8 + j] = db[k][j];
    }
  __syncthreads();
  for (int d = threadIdx.x; d < 2 * D; d += kThreads)
    partial[(size_t)blockIdx.x * 2 * D + d] = sm[d] + sm[2 * D + d] + sm[4 * D + d] + sm[6 * D + d];
}

template <typename T>
__global__ __launch_bounds__(kThreads) void add_kernel(size_t count, const T* a, const T* b, T* out) {
  const size_t stride = (size_t)gridDim.x * kThreads;
  for (size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x; i < count; i += stride)
    out[i] = from_float<T>(to_float(a[i]) + to_float(b[i]));
}

// bf16, 16 bytes per lane; `tail` elements behind the last whole unit go one by one
__global__ __launch_bounds__(kThreads) void add_bf16_vec_kernel(size_t nvec, size_t tail, const uint4* a, const uint4* b, uint4* out) {
  const size_t stride = (size_t)gridDim.x * kThreads;
  const size_t tid = (size_t)blockIdx.x * kThreads + threadIdx.x;
  for (size_t i = tid; i < nvec; i += stride) {
    const uint4 u = a[i], v = b[i];
    const uint32_t uw[4] = {u.x, u.y, u.z, u.w}, vw[4] = {v.x, v.y, v.z, v.w};
    uint32_t ow[4];
#pragma unroll
    for (int j = 0; j < 4; ++j)
      ow[j] = pack_bf16x2(__uint_as_float(uw[j] << 16) + __uint_as_float(vw[j] << 16),
                          __uint_as_float(uw[j] & 0xffff0000u) + __uint_as_float(vw[j] & 0xffff0000u));
    out[i] = make_uint4(ow[0], ow[1], ow[2], ow[3]);
  }
  const uint16_t* ta = reinterpret_cast<const uint16_t*>(a + nvec);
  const uint16_t* tb = reinterpret_cast<const uint16_t*>(b + nvec);
  uint16_t* to = reinterpret_cast<uint16_t*>(out + nvec);
  for (size_t i = tid; i < tail; i += stride) to[i] = float_to_bf16(bf16_to_float(ta[i]) + bf16_to_float(tb[i]));
}

// ---- attention ------------------------------------------------------------------------------------
constexpr int kTile = 64;   // keys (or queries) per LDS tile
constexpr int kRows = 16;   // rows of the walking side per workgroup (4 per wave)
constexpr int kMaxDh = 256;

// stage `count` rows of width dh (row stride ld elements, starting at base) in LDS as fp32, row pitch dh + 1
template <typename T>
__device__ __forceinline__ void stage_rows(float* dst, const T* base, size_t ld, int count, int dh) {
  for (int i = threadIdx.x; i < count * dh; i += kThreads) {
    const int r = i / dh, d = i - r * dh;
    dst[r * (dh + 1) + d] = to_float(base[(size_t)r * ld + d]);
  }
}

// out[i] = softmax_j<=i(q_i . k_j * scale) v_j ; lse[i] = log sum_j exp(q_i . k_j * scale)
template <typename T>
__global__ __launch_bounds__(kThreads) void attention_fwd_kernel(int S, int heads, int dh, float scale, const T* __restrict__ qkv,
                                                                 T* __restrict__ out, float* __restrict__ lse) {
  extern __shared__ float sm[];
  const int D = heads * dh;
  const size_t ld = 3 * (size_t)D;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int h = blockIdx.y, b = blockIdx.z;
  const int q0 = blockIdx.x * kRows;
  const T* base = qkv + (size_t)b * S * ld + (size_t)h * dh;
  float* qs = sm;                              // [kRows][dh + 1]
  float* ks = qs + kRows * (dh + 1);           // [kTile][dh + 1]
  float* vs = ks + kTile * (dh + 1);           // [kTile][dh + 1]
  const int nq = min(kRows, S - q0);
  stage_rows(qs, base + (size_t)q0 * ld, ld, nq, dh);
  constexpr int RW = kRows / 4;                // query rows per wave
  constexpr int ND = kMaxDh / 64;              // output columns per lane
  float m[RW], l[RW], o[RW][ND];
#pragma unroll
  for (int r = 0; r < RW; ++r) {
    m[r] = -INFINITY;
    l[r] = 0.f;
#pragma unroll
    for (int c = 0; c < ND; ++c) o[r][c] = 0.f;
  }
  const int last_key = min(S, q0 + kRows) - 1;  // causal: nothing beyond the last query of the block
  for (int k0 = 0; k0 <= last_key; k0 += kTile) {
    const int nk = min(kTile, S - k0);
    __syncthreads();
    stage_rows(ks, base + D + (size_t)k0 * ld, ld, nk, dh);
    stage_rows(vs, base + 2 * D + (size_t)k0 * ld, ld, nk, dh);
    __syncthreads();
#pragma unroll
    for (int r = 0; r < RW; ++r) {
      const int qi = wave * RW + r;            // row inside the block (wave uniform)
      const int i = q0 + qi;
      if (qi >= nq || k0 > i) continue;
      const int j = k0 + lane;
      float sc = -INFINITY;
      if (lane < nk && j <= i) {
        float acc = 0.f;
        for (int d = 0; d < dh; ++d) acc = fmaf(qs[qi * (dh + 1) + d], ks[lane * (dh + 1) + d], acc);
        sc = acc * scale;
      }
      const float mn = fmaxf(m[r], wave_max(sc));
      const float p = sc == -INFINITY ? 0.f : __expf(sc - mn);
      const float corr = __expf(m[r] - mn);    // exp(-inf) = 0 on the first tile
      l[r] = l[r] * corr + wave_sum(p);
      m[r] = mn;
      const int jmax = min(nk, i - k0 + 1);
#pragma unroll
      for (int c = 0; c < ND; ++c) {
        const int d = lane + 64 * c;
        float acc = o[r][c] * corr;
        if (64 * c < dh)  // wave uniform
          for (int jj = 0; jj < jmax; ++jj) {
            const float pj = lane_value(p, jj);
            if (d < dh) acc = fmaf(pj, vs[jj * (dh + 1) + d], acc);
          }
        o[r][c] = acc;
      }
    }
  }
#pragma unroll
  for (int r = 0; r < RW; ++r) {
    const int qi = wave * RW + r, i = q0 + qi;
    if (qi >= nq) continue;
    const float inv = 1.f / l[r];
#pragma unroll
    for (int c = 0; c < ND; ++c) {
      const int d = lane + 64 * c;
      if (d < dh) out[((size_t)b * S + i) * D + h * dh + d] = from_float<T>(o[r][c] * inv);
    }
    if (lane == 0) lse[((size_t)b * heads + h) * S + i] = m[r] + __logf(l[r]);
  }
}

// dq_i = scale * sum_{j<=i} ds_ij k_j,  ds_ij = p_ij (dO_i . v_j - delta_i),  p_ij = exp(q_i.k_j*scale - lse_i)
template <typename T>
__global__ __launch_bounds__(kThreads) void attention_bwd_q_kernel(int S, int heads, int dh, float scale, const T* __restrict__ qkv,
                                                                   const T* __restrict__ out, const T* __restrict__ dout,
                                                                   const float* __restrict__ lse, T* __restrict__ dqkv) {
  extern __shared__ float sm[];
  const int D = heads * dh;
  const size_t ld = 3 * (size_t)D;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int h = blockIdx.y, b = blockIdx.z;
  const int q0 = blockIdx.x * kRows;
  const T* base = qkv + (size_t)b * S * ld + (size_t)h * dh;
  const T* obase = out + (size_t)b * S * D + (size_t)h * dh;
  const T* dobase = dout + (size_t)b * S * D + (size_t)h * dh;
  float* qs = sm;                               // [kRows][dh + 1]
  float* dos = qs + kRows * (dh + 1);           // [kRows][dh + 1]
  float* ks = dos + kRows * (dh + 1);           // [kTile][dh + 1]
  float* vs = ks + kTile * (dh + 1);
  const int nq = min(kRows, S - q0);
  stage_rows(qs, base + (size_t)q0 * ld, ld, nq, dh);
  stage_rows(dos, dobase + (size_t)q0 * D, (size_t)D, nq, dh);
  __syncthreads();
  constexpr int RW = kRows / 4, ND = kMaxDh / 64;
  float delta[RW], li[RW], dq[RW][ND];
#pragma unroll
  for (int r = 0; r < RW; ++r) {
    const int qi = wave * RW + r, i = q0 + qi;
    float s = 0.f;
    if (qi < nq)
      for (int d = lane; d < dh; d += 64) s += dos[qi * (dh + 1) + d] * to_float(obase[(size_t)i * D + d]);
    delta[r] = wave_sum(s);
    li[r] = qi < nq ? lse[((size_t)b * heads + h) * S + i] : 0.f;
#pragma unroll
    for (int c = 0; c < ND; ++c) dq[r][c] = 0.f;
  }
  const int last_key = min(S, q0 + kRows) - 1;
  for (int k0 = 0; k0 <= last_key; k0 += kTile) {
    const int nk = min(kTile, S - k0);
    __syncthreads();
    stage_rows(ks, base + D + (size_t)k0 * ld, ld, nk, dh);
    stage_rows(vs, base + 2 * D + (size_t)k0 * ld, ld, nk, dh);
    __syncthreads();
#pragma unroll
    for (int r = 0; r < RW; ++r) {
      const int qi = wave * RW + r, i = q0 + qi;
      if (qi >= nq || k0 > i) continue;
      const int j = k0 + lane;
      float ds = 0.f;
      if (lane < nk && j <= i) {
        float sc = 0.f, dp = 0.f;
        for (int d = 0; d < dh; ++d) {
          sc = fmaf(qs[qi * (dh + 1) + d], ks[lane * (dh + 1) + d], sc);
          dp = fmaf(dos[qi * (dh + 1) + d], vs[lane * (dh + 1) + d], dp);
        }
        ds = __expf(sc * scale - li[r]) * (dp - delta[r]);
      }
      const int jmax = min(nk, i - k0 + 1);
#pragma unroll
      for (int c = 0; c < ND; ++c) {
        const int d = lane + 64 * c;
        if (64 * c < dh) {  // wave uniform
          float acc = dq[r][c];
          for (int jj = 0; jj < jmax; ++jj) {
            const float dsj = lane_value(ds, jj);
            if (d < dh) acc = fmaf(dsj, ks[jj * (dh + 1) + d], acc);
          }
          dq[r][c] = acc;
        }
      }
    }
  }
#pragma unroll
  for (int r = 0; r < RW; ++r) {
    const int qi = wave * RW + r, i = q0 + qi;
    if (qi >= nq) continue;
#pragma unroll
    for (int c = 0; c < ND; ++c) {
      const int d = lane + 64 * c;
      if (d < dh) dqkv[((size_t)b * S + i) * ld + h * dh + d] = from_float<T>(dq[r][c] * scale);
    }
  }
}

// dk_j = scale * sum_{i>=j} ds_ij q_i,  dv_j = sum_{i>=j} p_ij dO_i : rows are keys, the walk is over queries
template <typename T>
__global__ __launch_bounds__(kThreads) void attention_bwd_kv_kernel(int S, int heads, int dh, float scale, const T* __restrict__ qkv,
                                                                    const T* __restrict__ out, const T* __restrict__ dout,
                                                                    const float* __restrict__ lse, T* __restrict__ dqkv) {
  extern __shared__ float sm[];
  const int D = heads * dh;
  const size_t ld = 3 * (size_t)D;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int h = blockIdx.y, b = blockIdx.z;
  const int j0 = blockIdx.x * kRows;
  const T* base = qkv + (size_t)b * S * ld + (size_t)h * dh;
  const T* obase = out + (size_t)b * S * D + (size_t)h * dh;
  const T* dobase = dout + (size_t)b * S * D + (size_t)h * dh;
  float* ks = sm;                               // [kRows][dh + 1]  keys of this block
  float* vs = ks + kRows * (dh + 1);            // [kRows][dh + 1]
  float* qs = vs + kRows * (dh + 1);            // [kTile][dh + 1]  queries of the tile
  float* dos = qs + kTile * (dh + 1);           // [kTile][dh + 1]
  float* dl = dos + kTile * (dh + 1);           // [kTile] delta_i
  float* ls = dl + kTile;                       // [kTile] lse_i
  const int nkeys = min(kRows, S - j0);
  stage_rows(ks, base + D + (size_t)j0 * ld, ld, nkeys, dh);
  stage_rows(vs, base + 2 * D + (size_t)j0 * ld, ld, nkeys, dh);
  constexpr int RW = kRows / 4, ND = kMaxDh / 64;
  float dk[RW][ND], dv[RW][ND];
#pragma unroll
  for (int r = 0; r < RW; ++r)
#pragma unroll
    for (int c = 0; c < ND; ++c) dk[r][c] = dv[r][c] = 0.f;
  const int first_tile = (j0 / kTile) * kTile;  // queries before the first key of the block see none of its keys
  for (int i0 = first_tile; i0 < S; i0 += kTile) {
    const int ni = min(kTile, S - i0);
    __syncthreads();
    stage_rows(qs, base + (size_t)i0 * ld, ld, ni, dh);
    stage_rows(dos, dobase + (size_t)i0 * D, (size_t)D, ni, dh);
    __syncthreads();
    // delta_i = dO_i . O_i and lse_i of the tile's queries: one wave per 16 queries
    for (int q = wave; q < ni; q += 4) {
      float s = 0.f;
      for (int d = lane; d < dh; d += 64) s += dos[q * (dh + 1) + d] * to_float(obase[(size_t)(i0 + q) * D + d]);
      s = wave_sum(s);
      if (lane == 0) {
        dl[q] = s;
        ls[q] = lse[((size_t)b * heads + h) * S + i0 + q];
      }
    }
    __syncthreads();
#pragma unroll
    for (int r = 0; r < RW; ++r) {
      const int kj = wave * RW + r, j = j0 + kj;
      if (kj >= nkeys || i0 + ni - 1 < j) continue;
      const int i = i0 + lane;                  // lane = query of the tile
      float p = 0.f, ds = 0.f;
      if (lane < ni && i >= j) {
        float sc = 0.f, dp = 0.f;
        for (int d = 0; d < dh; ++d) {
          sc = fmaf(qs[lane * (dh + 1) + d], ks[kj * (dh + 1) + d], sc);
          dp = fmaf(dos[lane * (dh + 1) + d], vs[kj * (dh + 1) + d], dp);
        }
        p = __expf(sc * scale - ls[lane]);
        ds = p * (dp - dl[lane]);
      }
      const int ifirst = max(0, j - i0);        // first query of the tile that sees key j
#pragma unroll
      for (int c = 0; c < ND; ++c) {
        const int d = lane + 64 * c;
        if (64 * c >= dh) continue;  // wave uniform
        float ak = dk[r][c], av = dv[r][c];
        for (int ii = ifirst; ii < ni; ++ii) {
          const float pb = lane_value(p, ii), dsb = lane_value(ds, ii);
          if (d < dh) {
            ak = fmaf(dsb, qs[ii * (dh + 1) + d], ak);
            av = fmaf(pb, dos[ii * (dh + 1) + d], av);
          }
        }
        dk[r][c] = ak;
        dv[r][c] = av;
      }
    }
  }
#pragma unroll
  for (int r = 0; r < RW; ++r) {
    const int kj = wave * RW + r, j = j0 + kj;
    if (kj >= nkeys) continue;
#pragma unroll
    for (int c = 0; c < ND; ++c) {
      const int d = lane + 64 * c;
      if (d < dh) {
        dqkv[((size_t)b * S + j) * ld + D + h * dh + d] = from_float<T>(dk[r][c] * scale);
        dqkv[((size_t)b * S + j) * ld + 2 * D + h * dh + d] = from_float<T>(dv[r][c]);
      }
    }
  }
}

inline int blocks_for(size_t work, int cap) { return (int)std::min<size_t>(std::max<size_t>(work, 1), (size_t)cap); }
inline int ln_rows_per_block(size_t rows) { return (int)std::max<size_t>(4, (rows + 1023) / 1024); }

}  // namespace

hipError_t launch_layernorm_fwd(hipStream_t s, int elt, size_t rows, int D, const void* x, const float* gamma,
                                const float* beta, void* y, float* stats) {
  const unsigned blocks = (unsigned)((rows + 3) / 4);
  if (elt == ELT_BF16 && D % 512 == 0 && D <= 4096 && !(((uintptr_t)x | (uintptr_t)y) & 15)) {
    switch (D / 512) {
#define TP_LN_FWD(NG) \
  case NG: hipLaunchKernelGGL(layernorm_fwd_bf16_kernel<NG>, dim3(blocks), dim3(kThreads), 0, s, rows, (const uint16_t*)x, gamma, \
                              beta, (uint16_t*)y, stats); break;
      TP_LN_FWD(1) TP_LN_FWD(2) TP_LN_FWD(3) TP_LN_FWD(4) TP_LN_FWD(5) TP_LN_FWD(6) TP_LN_FWD(7) TP_LN_FWD(8)
#undef TP_LN_FWD
    }
    return hipGetLastError();
  }
  if (elt == ELT_BF16)
    hipLaunchKernelGGL(layernorm_fwd_kernel<uint16_t>, dim3(blocks), dim3(kThreads), 0, s, rows, D, (const uint16_t*)x, gamma,
                       beta, (uint16_t*)y, stats);
  else
    hipLaunchKernelGGL(layernorm_fwd_kernel<float>, dim3(blocks), dim3(kThreads), 0, s, rows, D, (const float*)x, gamma, beta,
                       (float*)y, stats);
  return hipGetLastError();
}

size_t layernorm_scratch_floats(size_t rows, int D) {
  const int rpb = ln_rows_per_block(rows);
  return ((rows + rpb - 1) / rpb) * 2 * (size_t)D;
}

bool layernorm_bwd_add_supported(int elt, int D) { return elt == ELT_BF16 && D % 512 == 0 && D <= 2048; }

hipError_t launch_layernorm_bwd(hipStream_t s, int elt, size_t rows, int D, const void* dy, const void* x,
                                const float* stats, const float* gamma_s, const float* gamma_l, float alpha, float beta_c,
                                void* dx, float* dgamma, float* dbeta, float* partials, const void* addend) {
  if (addend && (!layernorm_bwd_add_supported(elt, D) || (((uintptr_t)x | (uintptr_t)dy | (uintptr_t)dx | (uintptr_t)addend) & 15)))
    return hipErrorNotSupported;
  const int rpb = ln_rows_per_block(rows);
  const unsigned blocks = (unsigned)((rows + rpb - 1) / rpb);
  const size_t lds = (size_t)4 * 2 * D * sizeof(float);
  if (lds > 160 * 1024) return hipErrorInvalidValue;
  static hipError_t attr_h = hipFuncSetAttribute(reinterpret_cast<const void*>(layernorm_bwd_kernel<uint16_t>),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
  static hipError_t attr_f = hipFuncSetAttribute(reinterpret_cast<const void*>(layernorm_bwd_kernel<float>),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
  if (attr_h != hipSuccess) return attr_h;
  if (attr_f != hipSuccess) return attr_f;
  if (elt == ELT_BF16 && D % 512 == 0 && D <= 2048 && !(((uintptr_t)x | (uintptr_t)dy | (uintptr_t)dx) & 15)) {
    switch (D / 512) {
#define TP_LN_BWD(NG)                                                                                                         \
  case NG: {                                                                                                                  \
    static hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(layernorm_bwd_bf16_kernel<NG>),                \
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);                    \
    if (attr != hipSuccess) return attr;                                                                                      \
    hipLaunchKernelGGL(layernorm_bwd_bf16_kernel<NG>, dim3(blocks), dim3(kThreads), lds, s, rows, rpb, (const uint16_t*)dy,   \
                       (const uint16_t*)x, stats, gamma_s, gamma_l, alpha, beta_c, (const uint16_t*)addend, (uint16_t*)dx,  \
                       partials);                                                                                              \
  } break;
      TP_LN_BWD(1) TP_LN_BWD(2) TP_LN_BWD(3) TP_LN_BWD(4)
#undef TP_LN_BWD
    }
  } else if (elt == ELT_BF16)
    hipLaunchKernelGGL(layernorm_bwd_kernel<uint16_t>, dim3(blocks), dim3(kThreads), lds, s, rows, D, rpb, (const uint16_t*)dy,
                       (const uint16_t*)x, stats, gamma_s, gamma_l, alpha, beta_c, (uint16_t*)dx, partials);
  else
    hipLaunchKernelGGL(layernorm_bwd_kernel<float>, dim3(blocks), dim3(kThreads), lds, s, rows, D, rpb, (const float*)dy,
                       (const float*)x, stats, gamma_s, gamma_l, alpha, beta_c, (float*)dx, partials);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  // partial[block][0..D) = dgamma, [D..2D) = dbeta: strided sums over the blocks, one launch when the two
  // gradients lie side by side
  if (dbeta == dgamma + D) return launch_sum_partials_strided(s, 2 * (size_t)D, (int)blocks, partials, 2 * (size_t)D, dgamma);
  e = launch_sum_partials_strided(s, (size_t)D, (int)blocks, partials, 2 * (size_t)D, dgamma);
  if (e != hipSuccess) return e;
  return launch_sum_partials_strided(s, (size_t)D, (int)blocks, partials + D, 2 * (size_t)D, dbeta);
}

hipError_t launch_add(hipStream_t s, int elt, size_t count, const void* a, const void* b, void* out) {
  if (elt == ELT_BF16 && ((((uintptr_t)a | (uintptr_t)b | (uintptr_t)out) & 15) == 0)) {
    const size_t nvec = count / 8;
    hipLaunchKernelGGL(add_bf16_vec_kernel, dim3(blocks_for((nvec + kThreads - 1) / kThreads + 1, 4096)), dim3(kThreads), 0, s, nvec,
                       count % 8, (const uint4*)a, (const uint4*)b, (uint4*)out);
    return hipGetLastError();
  }
  const int blocks = blocks_for((count + kThreads - 1) / kThreads, 8192);
  if (elt == ELT_BF16)
    hipLaunchKernelGGL(add_kernel<uint16_t>, dim3(blocks), dim3(kThreads), 0, s, count, (const uint16_t*)a, (const uint16_t*)b,
                       (uint16_t*)out);
  else
    hipLaunchKernelGGL(add_kernel<float>, dim3(blocks), dim3(kThreads), 0, s, count, (const float*)a, (const float*)b,
                       (float*)out);
  return hipGetLastError();
}

bool attention_supported(int S, int heads, int dh) {
  return S >= 1 && heads >= 1 && heads <= 65535 && dh >= 1 && dh <= kMaxDh;
}

size_t attention_scratch_bytes(int elt, int seqs, int S, int heads, int dh) {
  if (elt != ELT_BF16) return 0;
  if (attention_flash_fwd_supported(seqs, S, heads, dh)) return attention_flash_bwd_scratch_bytes(seqs, S, heads);
  return attention_mfma_supported(S, heads, dh) ? attention_mfma_scratch_bytes(seqs, S, heads) : 0;
}

hipError_t launch_attention_fwd(hipStream_t s, int elt, int seqs, int S, int heads, int dh, const void* qkv, void* out,
                                float* lse, void* scratch, size_t scratch_bytes) {
  if (!attention_supported(S, heads, dh) || seqs > 65535) return hipErrorInvalidValue;
  if (elt == ELT_BF16 && attention_flash_fwd_supported(seqs, S, heads, dh))
    return attention_flash_fwd(s, seqs, S, heads, dh, (const uint16_t*)qkv, (uint16_t*)out, lse);
  if (elt == ELT_BF16 && scratch && attention_mfma_supported(S, heads, dh) &&
      scratch_bytes >= attention_mfma_scratch_bytes(1, S, heads))
    return attention_mfma_fwd(s, seqs, S, heads, dh, (const uint16_t*)qkv, (uint16_t*)out, lse, scratch, scratch_bytes);
  const float scale = 1.0f / sqrtf((float)dh);
  const dim3 grid((S + kRows - 1) / kRows, heads, seqs);
  const size_t lds = (size_t)(kRows + 2 * kTile) * (dh + 1) * sizeof(float);
  if (elt == ELT_BF16) {
    static hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(attention_fwd_kernel<uint16_t>),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    if (attr != hipSuccess) return attr;
    hipLaunchKernelGGL(attention_fwd_kernel<uint16_t>, grid, dim3(kThreads), lds, s, S, heads, dh, scale, (const uint16_t*)qkv,
                       (uint16_t*)out, lse);
  } else {
    static hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(attention_fwd_kernel<float>),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    if (attr != hipSuccess) return attr;
    hipLaunchKernelGGL(attention_fwd_kernel<float>, grid, dim3(kThreads), lds, s, S, heads, dh, scale, (const float*)qkv,
                       (float*)out, lse);
  }
  return hipGetLastError();
}

template <typename T>
static hipError_t attention_bwd_typed(hipStream_t s, int seqs, int S, int heads, int dh, const T* qkv, const T* out, const T* dout,
                                      const float* lse, T* dqkv) {
  const float scale = 1.0f / sqrtf((float)dh);
  const dim3 grid((S + kRows - 1) / kRows, heads, seqs);
  const size_t lds_q = (size_t)(2 * kRows + 2 * kTile) * (dh + 1) * sizeof(float);
  const size_t lds_kv = lds_q + 2 * kTile * sizeof(float);
  static hipError_t attr_q = hipFuncSetAttribute(reinterpret_cast<const void*>(attention_bwd_q_kernel<T>),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
  static hipError_t attr_kv = hipFuncSetAttribute(reinterpret_cast<const void*>(attention_bwd_kv_kernel<T>),
                                                  hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
  if (attr_q != hipSuccess) return attr_q;
  if (attr_kv != hipSuccess) return attr_kv;
  hipLaunchKernelGGL(attention_bwd_q_kernel<T>, grid, dim3(kThreads), lds_q, s, S, heads, dh, scale, qkv, out, dout, lse, dqkv);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(attention_bwd_kv_kernel<T>, grid, dim3(kThreads), lds_kv, s, S, heads, dh, scale, qkv, out, dout, lse, dqkv);
  return hipGetLastError();
}

hipError_t launch_attention_bwd(hipStream_t s, int elt, int seqs, int S, int heads, int dh, const void* qkv, const void* out,
                                const void* dout, const float* lse, void* dqkv, void* scratch, size_t scratch_bytes) {
  if (!attention_supported(S, heads, dh) || seqs > 65535) return hipErrorInvalidValue;
  if (elt == ELT_BF16 && scratch && attention_flash_fwd_supported(seqs, S, heads, dh) &&
      scratch_bytes >= attention_flash_bwd_scratch_bytes(seqs, S, heads))
    return attention_flash_bwd(s, seqs, S, heads, dh, (const uint16_t*)qkv, (const uint16_t*)out, (const uint16_t*)dout, lse,
                               (uint16_t*)dqkv, scratch, scratch_bytes);
  if (elt == ELT_BF16 && scratch && attention_mfma_supported(S, heads, dh) &&
      scratch_bytes >= attention_mfma_scratch_bytes(1, S, heads))
    return attention_mfma_bwd(s, seqs, S, heads, dh, (const uint16_t*)qkv, (const uint16_t*)dout, lse, (uint16_t*)dqkv, scratch,
                              scratch_bytes);
  if (elt == ELT_BF16)
    return attention_bwd_typed<uint16_t>(s, seqs, S, heads, dh, (const uint16_t*)qkv, (const uint16_t*)out, (const uint16_t*)dout,
                                         lse, (uint16_t*)dqkv);
  return attention_bwd_typed<float>(s, seqs, S, heads, dh, (const float*)qkv, (const float*)out, (const float*)dout, lse,
                                    (float*)dqkv);
}

}  // namespace tp
