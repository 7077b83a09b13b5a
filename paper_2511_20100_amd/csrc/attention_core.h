// Layout of the paged fp16 KV cache and the softmax state of the decode attention kernel
// (grouped-query attention, head_dim hd = 128 or 64).
//
// Page layouts (16 tokens x hd dims = 4 or 2 KiB per (layer, K or V, kv head, page)):
//   K page: [dim / 8][token][dim % 8]   -> the hd / 32 16x32 "A" operands of S^T = K Q^T are the
//                                          consecutive 1 KiB pieces of the page;
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

// Running softmax state of one block of 16 query columns over CB blocks of 16 head dims.
template <int CB>
struct AttnState {
  float m;       // running maximum of the column (same in the 4 lanes that share a column)
  float l;       // this lane's share of the running sum
  v4f o[CB];     // O^T[dim = 16 cb + 4 (lane / 16) + r][column]
};

template <int CB>
__device__ __forceinline__ void attn_init(AttnState<CB>& st) {
  st.m = -INFINITY;
  st.l = 0.f;
#pragma unroll
  for (int cb = 0; cb < CB; ++cb) st.o[cb] = v4f{0.f, 0.f, 0.f, 0.f};
}

}  // namespace bf16
}  // namespace mtmc
