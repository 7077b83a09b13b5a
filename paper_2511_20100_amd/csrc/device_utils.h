// Device-side helpers: wavefront/block reductions, the counter-based generator, Gumbel noise.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "common.h"

namespace mtmc {

constexpr int kWave = 64;

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, kWave));
  return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
  return v;
}

// Sum over a block of up to 1024 threads; every thread gets the result.  `red` holds >= 16 floats.
__device__ __forceinline__ float block_sum(float v, float* red) {
  v = wave_sum(v);
  const int lane = threadIdx.x & 63, wid = threadIdx.x >> 6, nw = (blockDim.x + 63) >> 6;
  __syncthreads();
  if (lane == 0) red[wid] = v;
  __syncthreads();
  float t = 0.f;
  for (int i = 0; i < nw; ++i) t += red[i];
  return t;
}
__device__ __forceinline__ float block_max(float v, float* red) {
  v = wave_max(v);
  const int lane = threadIdx.x & 63, wid = threadIdx.x >> 6, nw = (blockDim.x + 63) >> 6;
  __syncthreads();
  if (lane == 0) red[wid] = v;
  __syncthreads();
  float t = red[0];
  for (int i = 1; i < nw; ++i) t = fmaxf(t, red[i]);
  return t;
}

// ---- Philox4x32-10 (Salmon et al., SC'11): ten rounds, key bumped by the Weyl constants ----
__device__ __forceinline__ uint4 philox4x32_10(uint4 c, uint32_t k0, uint32_t k1) {
  constexpr uint32_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u, W0 = 0x9E3779B9u, W1 = 0xBB67AE85u;
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    // one 32 x 32 -> 64 bit product per multiplier (a single multiply instruction gives both halves)
    const uint64_t p0 = (uint64_t)M0 * c.x, p1 = (uint64_t)M1 * c.z;
    c = make_uint4((uint32_t)(p1 >> 32) ^ c.y ^ k0, (uint32_t)p1, (uint32_t)(p0 >> 32) ^ c.w ^ k1, (uint32_t)p0);
    k0 += W0;
    k1 += W1;
  }
  return c;
}

// u = ((r >> 9) + 1/2) 2^-23 lies strictly inside (0, 1) and is exact in fp32; g = -ln(-ln u).
// Both logarithms are the hardware's base-2 logarithm (1 ulp) times ln 2: u and -ln u (6e-8 .. 16.7) are normal
// numbers, so none of the library routine's range fix-ups is needed; g is within about 2e-6 of the exact value.
__device__ __forceinline__ float gumbel_from_bits(uint32_t r) {
  constexpr float kLn2 = 0.6931471805599453f;
  const float u = ((float)(r >> 9) + 0.5f) * 1.1920928955078125e-07f;
  const float l = -kLn2 * __builtin_amdgcn_logf(u);
  return -kLn2 * __builtin_amdgcn_logf(l);
}

// Online log-sum-exp state (m = running max, s = sum of exp(x - m)).
struct Lse {
  float m, s;
};
__device__ __forceinline__ Lse lse_empty() { return {-INFINITY, 0.f}; }
__device__ __forceinline__ void lse_push(Lse& a, float x) {
  if (x > a.m) {
    a.s = a.s * expf(a.m - x) + 1.f;
    a.m = x;
  } else {
    a.s += expf(x - a.m);
  }
}
// The same for four values at once, without branches: the new maximum first, then the old sum and the four terms
// rescaled to it with the hardware's 2^x (relative error about 1e-7 per term; every argument is <= 0).  An empty
// state (m = -inf, s = 0) and values of -inf contribute exp2(-inf) = 0; the four values must not all be -inf while
// the state is empty.
__device__ __forceinline__ void lse_push4(Lse& a, float x0, float x1, float x2, float x3) {
  constexpr float kLog2e = 1.4426950408889634f;
  const float m = fmaxf(fmaxf(a.m, fmaxf(x0, x1)), fmaxf(x2, x3));
  const float mk = m * kLog2e;
  float s = a.s * __builtin_amdgcn_exp2f(fmaf(a.m, kLog2e, -mk));
  s += __builtin_amdgcn_exp2f(fmaf(x0, kLog2e, -mk));
  s += __builtin_amdgcn_exp2f(fmaf(x1, kLog2e, -mk));
  s += __builtin_amdgcn_exp2f(fmaf(x2, kLog2e, -mk));
  s += __builtin_amdgcn_exp2f(fmaf(x3, kLog2e, -mk));
  a.m = m;
  a.s = s;
}
__device__ __forceinline__ Lse lse_merge(Lse a, Lse b) {
  if (b.s == 0.f) return a;
  if (a.s == 0.f) return b;
  const float m = fmaxf(a.m, b.m);
  return {m, a.s * expf(a.m - m) + b.s * expf(b.m - m)};
}

// Arg-max with "lowest index wins ties".
struct Best {
  float y;
  int idx;
};
__device__ __forceinline__ Best best_empty() { return {-INFINITY, 0x7fffffff}; }
__device__ __forceinline__ Best best_merge(Best a, Best b) {
  return (b.y > a.y || (b.y == a.y && b.idx < a.idx)) ? b : a;
}

// Largest and second largest value (with the index of the largest; lowest index on ties).
struct Top2 {
  float v1;
  int i1;
  float v2;
};
__device__ __forceinline__ Top2 top2_empty() { return {-INFINITY, 0x7fffffff, -INFINITY}; }
__device__ __forceinline__ void top2_push(Top2& t, float v, int i) {
  if (v > t.v1 || (v == t.v1 && i < t.i1)) {
    t.v2 = t.v1;
    t.v1 = v;
    t.i1 = i;
  } else if (v > t.v2) {
    t.v2 = v;
  }
}
__device__ __forceinline__ Top2 top2_merge(Top2 a, Top2 b) {
  const bool b_wins = (b.v1 > a.v1 || (b.v1 == a.v1 && b.i1 < a.i1));
  Top2 r;
  if (b_wins) {
    r.v1 = b.v1; r.i1 = b.i1; r.v2 = fmaxf(a.v1, fmaxf(a.v2, b.v2));
  } else {
    r.v1 = a.v1; r.i1 = a.i1; r.v2 = fmaxf(b.v1, fmaxf(a.v2, b.v2));
  }
  return r;
}

__device__ __forceinline__ int tok_seq(const TokMap& m, int t) { return t / m.S; }
__device__ __forceinline__ int tok_pos(const TokMap& m, int t) {
  return (m.row_pos ? m.row_pos[t / m.S] : m.pos_base) + (m.d_step ? *m.d_step : 0) + t % m.S;
}

}  // namespace mtmc
