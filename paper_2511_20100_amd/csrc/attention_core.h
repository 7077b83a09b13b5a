// The MFMA inner step of the decode attention kernel: two KV pages against blocks of 16 query columns
// of grouped-query attention over the paged fp16 KV cache (head_dim 128).
//
// Page layouts (16 tokens x 128 dims = 4 KiB per (layer, K or V, kv head, page)):
//   K page: [dim / 8][token][dim % 8]   -> the four 16x32 "A" operands of S^T = K Q^T are the
//                                          four consecutive 1 KiB quarters of the page;
//   V page: [dim][token]                -> a lane's "A" operand of O^T = V^T P^T is 4 consecutive
//                                          tokens of one dim from each of two pages (2 x 8 bytes).
// Scores are produced transposed (S^T[token][query]), so a lane owns one query column: the
// softmax reductions run over its 8 registers plus two cross-lane steps, and exp(S^T) is
// already in the "B" operand layout of the second product -- no transpose through LDS.
// The k index of that product maps (lane / 16, e) to token 4 (lane / 16) + e % 4 of page e / 4,
// the same permutation on both operands.
#pragma once

#include "common.h"
#include "frag.h"

namespace mtmc {
namespace bf16 {

template <int NQB>
struct AttnState {
  float m[NQB];      // running maximum of the column (same in the 4 lanes that share a column)
  float l[NQB];      // this lane's share of the running sum
  v4f o[NQB][8];     // O^T[dim = 16 cb + 4 (lane / 16) + r][column]
};

template <int NQB>
__device__ __forceinline__ void attn_init(AttnState<NQB>& st) {
#pragma unroll
  for (int i = 0; i < NQB; ++i) {
    st.m[i] = -INFINITY;
    st.l[i] = 0.f;
#pragma unroll
    for (int cb = 0; cb < 8; ++cb) st.o[i][cb] = v4f{0.f, 0.f, 0.f, 0.f};
  }
}

// One step over two pages (32 tokens starting at tok0) for up to NQB blocks of 16 query columns.
// qpos[i] is the position of this lane's column in block i (-1: padding column, fully masked).
template <int NQB>
__device__ __forceinline__ void attn_pair(const h16_t* __restrict__ K0, const h16_t* __restrict__ K1,
                                          const h16_t* __restrict__ V0, const h16_t* __restrict__ V1,
                                          int tok0, const v8bf (&qf)[NQB][4], const int (&qpos)[NQB],
                                          int nqb, float scale, AttnState<NQB>& st, int lane) {
  const int lg = lane >> 4;
  v8bf kf[2][4];
#pragma unroll
  for (int kb = 0; kb < 4; ++kb) {
    kf[0][kb] = load_frag(K0 + kb * 512, lane);
    kf[1][kb] = load_frag(K1 + kb * 512, lane);
  }
  v8bf pf[NQB];
#pragma unroll
  for (int i = 0; i < NQB; ++i) {
    if (i >= nqb) continue;
    v4f s0 = v4f{0.f, 0.f, 0.f, 0.f}, s1 = s0;
#pragma unroll
    for (int kb = 0; kb < 4; ++kb) {
      s0 = mfma16(kf[0][kb], qf[i][kb], s0);
      s1 = mfma16(kf[1][kb], qf[i][kb], s1);
    }
    float sv[8];
    float tmax = -INFINITY;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int t0 = tok0 + 4 * lg + r, t1 = t0 + 16;
      sv[r] = (t0 <= qpos[i]) ? s0[r] * scale : -INFINITY;
      sv[4 + r] = (t1 <= qpos[i]) ? s1[r] * scale : -INFINITY;
      tmax = fmaxf(tmax, fmaxf(sv[r], sv[4 + r]));
    }
    tmax = fmaxf(tmax, __shfl_xor(tmax, 16, 64));
    tmax = fmaxf(tmax, __shfl_xor(tmax, 32, 64));
    const float m_new = fmaxf(st.m[i], tmax);
    const float m_safe = (m_new == -INFINITY) ? 0.f : m_new;
    const float corr = expf(st.m[i] - m_safe);
    float p[8], psum = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      p[e] = expf(sv[e] - m_safe);
      psum += p[e];
    }
    st.l[i] = st.l[i] * corr + psum;
    st.m[i] = m_new;
    v4u pk;
    pk[0] = pack_h16x2(p[0], p[1]);
    pk[1] = pack_h16x2(p[2], p[3]);
    pk[2] = pack_h16x2(p[4], p[5]);
    pk[3] = pack_h16x2(p[6], p[7]);
    pf[i] = __builtin_bit_cast(v8bf, pk);
#pragma unroll
    for (int cb = 0; cb < 8; ++cb) st.o[i][cb] = st.o[i][cb] * corr;
  }
  const int voff = (lane & 15) * kPageTokens + 4 * lg;
#pragma unroll
  for (int cb = 0; cb < 8; ++cb) {
    const uint2 a = *reinterpret_cast<const uint2*>(V0 + cb * 256 + voff);
    const uint2 b = *reinterpret_cast<const uint2*>(V1 + cb * 256 + voff);
    const v4u raw = {a.x, a.y, b.x, b.y};
    const v8bf vf = __builtin_bit_cast(v8bf, raw);
#pragma unroll
    for (int i = 0; i < NQB; ++i) {
      if (i >= nqb) continue;
      st.o[i][cb] = mfma16(vf, pf[i], st.o[i][cb]);
    }
  }
}

}  // namespace bf16
}  // namespace mtmc
