// Grouped-query attention over the paged bf16 KV cache (head_dim 128), on MFMA.
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
#include "attention_core.h"
#include "bf16_kernels.h"
#include "device_utils.h"
#include "frag.h"

namespace mtmc {
namespace bf16 {

constexpr int HD = 128;
constexpr int PAGE_ELEMS = kPageTokens * HD;

__device__ __forceinline__ const h16_t* kv_page(const KvPool& pool, int layer, int which, int page, int g) {
  return (const h16_t*)pool.base +
         ((((size_t)layer * 2 + which) * pool.n_pages + page) * pool.n_kv_heads + g) * (size_t)PAGE_ELEMS;
}

// ======================================================================================
// decode: one workgroup per (sequence, kv head, context chunk); the G query heads of the kv
// head are the (padded to 16) columns; four wavefronts share the chunk's page pairs.
// ======================================================================================
size_t attn_part_floats(int B, int Hkv, int G, int n_chunks) {
  return (size_t)B * Hkv * n_chunks * G * (HD + 2);
}

__global__ __launch_bounds__(256) void k_attn_decode(float* part, const h16_t* q, int Hq, int Hkv,
                                                     TokMap map, KvPool pool, int layer,
                                                     int chunk_pages, int n_chunks) {
  __shared__ float s_o[4][16][HD + 1];
  __shared__ float s_m[4][16], s_l[4][16];
  const int b = blockIdx.x, g = blockIdx.y, chunk = blockIdx.z;
  const int G = Hq / Hkv;
  const int pos = tok_pos(map, b);
  const int n_ctx_pages = pos / kPageTokens + 1;
  const int p_lo = chunk * chunk_pages, p_hi = min(n_ctx_pages, p_lo + chunk_pages);
  if (p_lo >= p_hi) return;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int col = lane & 15, lg = lane >> 4;
  const int* table = pool.page_table + (size_t)tok_seq(map, b) * map.row_stride * pool.max_pages;

  v8bf qf[1][4];
  int qpos[1];
  qpos[0] = (col < G) ? pos : -1;
#pragma unroll
  for (int kb = 0; kb < 4; ++kb) {
    v4u raw = {0u, 0u, 0u, 0u};
    if (col < G)
      raw = *reinterpret_cast<const v4u*>(q + (size_t)b * Hq * HD + (size_t)(g * G + col) * HD + kb * 32 + 8 * lg);
    qf[0][kb] = __builtin_bit_cast(v8bf, raw);
  }
  AttnState<1> st;
  attn_init(st);
  const float scale = 0.08838834764831845f;  // 1 / sqrt(128)
  for (int pg = p_lo + 2 * wave; pg < p_hi; pg += 8) {
    const int id0 = table[pg], id1 = table[min(pg + 1, n_ctx_pages - 1)];
    attn_pair<1>(kv_page(pool, layer, 0, id0, g), kv_page(pool, layer, 0, id1, g),
                 kv_page(pool, layer, 1, id0, g), kv_page(pool, layer, 1, id1, g), pg * kPageTokens, qf,
                 qpos, 1, scale, st, lane);
  }
  float l = st.l[0];
  l += __shfl_xor(l, 16, 64);
  l += __shfl_xor(l, 32, 64);
#pragma unroll
  for (int cb = 0; cb < 8; ++cb)
#pragma unroll
    for (int r = 0; r < 4; ++r) s_o[wave][col][cb * 16 + 4 * lg + r] = st.o[0][cb][r];
  if (lg == 0) {
    s_m[wave][col] = st.m[0];
    s_l[wave][col] = l;
  }
  __syncthreads();
  float* out = part + (((size_t)b * Hkv + g) * n_chunks + chunk) * (size_t)(G * (HD + 2));
  for (int idx = threadIdx.x; idx < G * HD; idx += blockDim.x) {
    const int c = idx / HD, d = idx % HD;
    const float mm = fmaxf(fmaxf(s_m[0][c], s_m[1][c]), fmaxf(s_m[2][c], s_m[3][c]));
    float acc = 0.f;
#pragma unroll
    for (int w = 0; w < 4; ++w) acc += expf(s_m[w][c] - mm) * s_o[w][c][d];
    out[idx] = acc;
  }
  if (threadIdx.x < G) {
    const int c = threadIdx.x;
    const float mm = fmaxf(fmaxf(s_m[0][c], s_m[1][c]), fmaxf(s_m[2][c], s_m[3][c]));
    float acc = 0.f;
#pragma unroll
    for (int w = 0; w < 4; ++w) acc += expf(s_m[w][c] - mm) * s_l[w][c];
    out[G * HD + c] = mm;
    out[G * HD + G + c] = acc;
  }
}

void attention_decode(float* part, const h16_t* q, int B, int Hq, int Hkv, TokMap map, KvPool pool,
                      int layer, int chunk_pages, int n_chunks, hipStream_t st) {
  k_attn_decode<<<dim3(B, Hkv, n_chunks), 256, 0, st>>>(part, q, Hq, Hkv, map, pool, layer, chunk_pages,
                                                       n_chunks);
}

// Merge of the chunk partials -> o (bf16, tiled activation layout with k = head * 128 + dim).
__global__ __launch_bounds__(256) void k_attn_decode_merge(h16_t* o, const float* part, int Mpad, int Hq,
                                                           int Hkv, TokMap map, int chunk_pages,
                                                           int n_chunks) {
  const int b = blockIdx.x, g = blockIdx.y;
  const int G = Hq / Hkv;
  const int pos = tok_pos(map, b);
  const int n_act = (pos / kPageTokens + 1 + chunk_pages - 1) / chunk_pages;
  const int t = threadIdx.x;  // one thread per (column, 8 consecutive dims)
  if (t >= G * (HD / 8)) return;
  const int c = t / (HD / 8), d0 = (t % (HD / 8)) * 8;
  const size_t stride = (size_t)G * (HD + 2);
  const float* base = part + ((size_t)b * Hkv + g) * n_chunks * stride;
  float mm = -INFINITY;
  for (int k = 0; k < n_act; ++k) mm = fmaxf(mm, base[k * stride + G * HD + c]);
  float l = 0.f, acc[8] = {};
  for (int k = 0; k < n_act; ++k) {
    const float w = expf(base[k * stride + G * HD + c] - mm);
    l += w * base[k * stride + G * HD + G + c];
    const float* src = base + k * stride + (size_t)c * HD + d0;
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] += w * src[e];
  }
  const float inv = 1.0f / l;
  v4u pk;
#pragma unroll
  for (int e = 0; e < 4; ++e) pk[e] = pack_h16x2(acc[2 * e] * inv, acc[2 * e + 1] * inv);
  *reinterpret_cast<v4u*>(o + act_off(b, (g * G + c) * HD + d0, Mpad)) = pk;
}

void attention_decode_merge(h16_t* o, const float* part, int B, int m_tiles, int Hq, int Hkv,
                            TokMap map, int chunk_pages, int n_chunks, hipStream_t st) {
  k_attn_decode_merge<<<dim3(B, Hkv), 256, 0, st>>>(o, part, m_tiles * 16, Hq, Hkv, map, chunk_pages,
                                                   n_chunks);
}

}  // namespace bf16
}  // namespace mtmc
