// Causal grouped-query attention of the prefill / scoring pass (head_dim 128 or 64) on the 32x32x16 MFMA.
//
// One workgroup per (128 query columns, kv head, sequence).  The columns of a kv head are the
// (query head of its group, position) pairs, position fastest: with S a multiple of 128 a workgroup holds 128
// consecutive positions of one query head; with short sequences (the candidate rows of action scoring, small
// prompts) the G query heads of the group sit side by side in one workgroup and share every K/V step.
// Four column blocks of 32, one per wavefront, and three workgroups per CU: a wavefront's chain
// (K Q^T -> softmax -> V^T P^T) is serial, so the matrix products of one wavefront run under the softmax
// arithmetic of the others on its SIMD (with two blocks per wavefront and one workgroup per CU the kernel took
// 1.9 times as long).  The workgroup walks the keys in steps of 32 tokens (two 16-token pages): the four
// wavefronts copy the two K pages and two V pages of a step (16 KiB at head_dim 128) into a ring of three LDS
// buffers with LDS-direct loads, two steps ahead, and every wavefront reads them from there; a wavefront skips
// the arithmetic of steps that lie wholly behind its own columns.  Query j of a sequence sits at position
// pos_base + j and sees keys 0 .. pos_base + j.
//
// Per step and column block:  S^T[token][column] = K Q^T  (8 MFMAs over the 128 dims), online softmax
// down each column (a column's 32 tokens sit in 16 registers of lanes l and l + 32), then
// O^T[dim][column] += V^T P^T (4 blocks of 32 dims x 2 MFMAs over 16 tokens).  exp(S^T) is already in
// the B-operand layout of the second product: with the K rows permuted on their way into LDS (see the copy
// code), slot e of lane (column, half h) in token group jj holds token 16 jj + 8 h + e, and the V^T operand
// of a lane is one 16-byte piece of a V page row.  Page layouts: see attention_core.h.
#include "bf16_kernels.h"
#include "device_utils.h"
#include "frag.h"

namespace mtmc {
namespace bf16 {

namespace {

constexpr int kAStages = 3;

typedef __attribute__((ext_vector_type(16))) float v16f;
typedef __attribute__((address_space(3))) void* lds_ptr_t;
typedef const __attribute__((address_space(1))) void* glb_ptr_t;

__device__ __forceinline__ const uint8_t* page_ptr(const KvPool& pool, int layer, int which, int page, int g,
                                                   int page_bytes) {
  return (const uint8_t*)pool.base +
         ((((size_t)layer * 2 + which) * pool.n_pages + page) * pool.n_kv_heads + g) * (size_t)page_bytes;
}

template <int N>
__device__ __forceinline__ void wait_vm() {
  __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | (7 << 4) | (15 << 8));
}

constexpr int NCB = 1;    // column blocks per wavefront
constexpr int QB = 128;   // query columns per workgroup

template <int PHD>
__global__ __launch_bounds__(256, 3) void k_attn_prefill32(h16_t* o, const h16_t* q, int S, int Mpad, int Hq, int Hkv,
                                                           int row_stride, int pos_base, KvPool pool, int layer,
                                                           int* err_flag, const int* seq_start) {
  constexpr int kPageBytes = kPageTokens * PHD * 2;  // 4 or 2 KiB
  constexpr int kAStageBytes = 4 * kPageBytes;       // K page 0, K page 1, V page 0, V page 1
  constexpr int kPageKiB = kPageBytes / 1024;
  constexpr int kCopies = kAStageBytes / 1024 / 4;   // 1 KiB copies per wavefront and step
  extern __shared__ __attribute__((aligned(1024))) uint8_t lds[];
  const int qblk = gridDim.x - 1 - blockIdx.x;  // longest columns first
  const int c0 = qblk * QB, g = blockIdx.y, seq = blockIdx.z;
  // sequences of different lengths packed back to back: this one holds the tokens tok0 .. tok0 + S - 1 (the grid
  // is sized for the longest; a workgroup whose columns lie beyond this sequence's has nothing to do)
  int tok0 = seq * S;
  if (seq_start) {
    tok0 = seq_start[seq];
    S = seq_start[seq + 1] - tok0;
  }
  const int G = Hq / Hkv, n_cols = G * S;
  if (c0 >= n_cols) return;  // whole workgroup, before any barrier
  // positions covered by the workgroup's columns: exact when they belong to one query head, else all
  const int c_last = min(c0 + QB, n_cols) - 1;
  const bool one_head = c0 / S == c_last / S;
  const int min_pos = one_head ? c0 % S : 0, max_pos = one_head ? c_last % S : S - 1;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int uwave = __builtin_amdgcn_readfirstlane(wave);
  const int col = lane & 31, hh = lane >> 5;
  const int* table = pool.page_table + (size_t)seq * row_stride * pool.max_pages;
  // query j of the sequence sits at position pos_base + j and sees the keys at positions 0 .. pos_base + j
  const int seq_pages = (pos_base + S + kPageTokens - 1) / kPageTokens;
  const int n_steps = (pos_base + max_pos + 32) / 32;  // key blocks 0 .. n_steps - 1 (causal)

  // ---- page ids of the steps, staged in LDS behind the ring (a global load inside the loop would be a
  // vector load, and waiting for it would drain the ring of copies in flight)
  int* s_ids = reinterpret_cast<int*>(lds + kAStages * kAStageBytes);
  for (int i = threadIdx.x; i < 2 * n_steps; i += 256) s_ids[i] = table[min(i, seq_pages - 1)];
  __syncthreads();
  // ---- copies of one step: the stage is 4 * kPageKiB pieces of 1 KiB (pages K0, K1, V0, V1 in this order);
  // wavefront w moves pieces w, w + 4, ... (at head_dim 128: KiB w of each of the four pages).  A copy puts
  // the 16 bytes of lane s at offset 16 s of its piece, and the lane may fetch them from anywhere: the pieces
  // are permuted on the way in, so that every later LDS read is one 16-byte access at offset 16 * lane.
  //   K piece (4 dim groups x 16 tokens): slot (dim group, i) <- token i with bits 2 and 3 swapped.  Operand
  //     row r of the K MFMA operand then stands for token tau(r) = r with bits 2 and 3 swapped, which makes
  //     the 8 scores a lane holds per token group, and hence its 8 k-slots of the second product, the 8
  //     CONSECUTIVE tokens 16 jj + 8 hh .. + 7;
  //   V piece (32 dims x 2 halves of 8 tokens): slot 32 hh + c <- (dim c, tokens 8 hh .. 8 hh + 7), which is
  //     exactly the V^T operand of lane (c, hh).
  // (Two 8-byte reads per lane from the unpermuted V page cost four-way bank conflicts: 64 % of the LDS cycles.)
  const int src_k = ((lane & 0x30) | ((lane & 4) << 1) | ((lane & 8) >> 1) | (lane & 3)) * 16;
  const int src_v = ((lane & 31) * 2 + (lane >> 5)) * 16;
  auto issue = [&](int step, int buf) {
    const int st = min(step, n_steps - 1);
    const int id0 = __builtin_amdgcn_readfirstlane(s_ids[2 * st]);
    const int id1 = __builtin_amdgcn_readfirstlane(s_ids[2 * st + 1]);
#pragma unroll
    for (int c = 0; c < kCopies; ++c) {
      const int piece = 4 * c + uwave;
      const int page = piece / kPageKiB, kib = piece % kPageKiB;  // page: 0 = K0, 1 = K1, 2 = V0, 3 = V1
      const uint8_t* src = page_ptr(pool, layer, page >> 1, (page & 1) ? id1 : id0, g, kPageBytes) + kib * 1024 +
                           ((page >> 1) ? src_v : src_k);
      __builtin_amdgcn_global_load_lds((glb_ptr_t)src, (lds_ptr_t)(lds + buf * kAStageBytes + piece * 1024), 16, 0, 0);
    }
  };
#pragma unroll
  for (int s = 0; s < kAStages - 1; ++s) issue(s, s);

  // ---- this wavefront's column blocks (columns c0 + 32 b + col, b = wave and 7 - wave).
  // Q fragments (B operand: column col, dims 16 j + 8 hh + 0..7).
  v8h qf[NCB][PHD / 16];
  int qpos[NCB], qabs[NCB], qhd[NCB];  // index in the sequence / position among the keys (-1: padding), head
#pragma unroll
  for (int i = 0; i < NCB; ++i) {
    const int b = (NCB == 1) ? uwave : (i == 0) ? uwave : 7 - uwave;
    const int c = c0 + 32 * b + col;
    const bool live = c < n_cols;
    const int jh = live ? c / S : 0, pos = c - jh * S;
    qpos[i] = live ? pos : -1;
    qabs[i] = live ? pos_base + pos : -1;
    qhd[i] = g * G + jh;
    const h16_t* qrow = q + ((size_t)tok0 + max(qpos[i], 0)) * Hq * PHD + (size_t)qhd[i] * PHD + 8 * hh;
#pragma unroll
    for (int j = 0; j < PHD / 16; ++j) {
      v4u raw = {0u, 0u, 0u, 0u};
      if (qpos[i] >= 0) raw = *reinterpret_cast<const v4u*>(qrow + 16 * j);
      qf[i][j] = __builtin_bit_cast(v8h, raw);
    }
  }
  // last key step that holds a key some column of this wavefront's block may see (-1: the block is all padding)
  int my_last = -1;
  {
    static_assert(NCB == 1, "one column block per wavefront");
    const int b0 = c0 + 32 * uwave, b1 = min(b0 + 31, n_cols - 1);
    if (b0 < n_cols) my_last = (pos_base + ((b0 / S == b1 / S) ? b1 % S : S - 1)) / 32;
  }
  v16f oacc[NCB][PHD / 32];
  float mrun[NCB], lrun[NCB];
#pragma unroll
  for (int i = 0; i < NCB; ++i) {
    mrun[i] = -INFINITY;
    lrun[i] = 0.f;
#pragma unroll
    for (int d = 0; d < PHD / 32; ++d)
#pragma unroll
      for (int e = 0; e < 16; ++e) oacc[i][d][e] = 0.f;
  }
  // exp(x / sqrt(head_dim)) = exp2(x c)
  const float c2 = (PHD == 128 ? 0.08838834764831845f : 0.125f) * 1.4426950408889634f;
  // lane offsets inside a stage: K operand (operand row col, dim group 2 j + hh) and V operand
  // (dim row 32 d + col, tokens 8 hh .. 8 hh + 7 of page jj)
  const int koff = (col >> 4) * kPageBytes + (hh * 16 + (col & 15)) * 16;
  const int voff = 2 * kPageBytes + lane * 16;

  // One key step for both column blocks.
  auto step = [&](int t, const uint8_t* sb) {
    // ---- S^T = K Q^T: K fragments read from LDS once, used by every active block
    v16f sacc[NCB];
#pragma unroll
    for (int i = 0; i < NCB; ++i)
#pragma unroll
      for (int e = 0; e < 16; ++e) sacc[i][e] = 0.f;
#pragma unroll
    for (int j = 0; j < PHD / 16; ++j) {
      const v8h kf = *reinterpret_cast<const v8h*>(sb + koff + j * 512);
#pragma unroll
      for (int i = 0; i < NCB; ++i)
        sacc[i] = __builtin_amdgcn_mfma_f32_32x32x16_f16(kf, qf[i][j], sacc[i], 0, 0, 0);
    }
    // ---- online softmax down each column; P^T fragments for the two token groups
    v8h pf[NCB][2];
    const bool diag = 32 * t + 31 > pos_base + min_pos;  // some column of the workgroup may not see all 32 tokens
#pragma unroll
    for (int i = 0; i < NCB; ++i) {
      float sv[16];
#pragma unroll
      for (int e = 0; e < 16; ++e) sv[e] = sacc[i][e];
      if (diag || qpos[i] < 0) {
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const int tok = 32 * t + 16 * (e >> 3) + 8 * hh + (e & 7);  // operand row 8 (e / 4) + 4 hh + e % 4 -> tau
          if (tok > qabs[i]) sv[e] = -INFINITY;
        }
      }
      float bm = sv[0];
#pragma unroll
      for (int e = 1; e < 16; ++e) bm = fmaxf(bm, sv[e]);
      bm = fmaxf(bm, __shfl_xor(bm, 32, 64));
      const float m_new = fmaxf(mrun[i], bm);
      const float m_safe = (m_new == -INFINITY) ? 0.f : m_new;
      const float corr = __builtin_amdgcn_exp2f((mrun[i] - m_safe) * c2);  // exp2(-inf) = 0 on the first step
      const float mc = m_safe * c2;
      float psum = 0.f;
      float p[16];
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        p[e] = __builtin_amdgcn_exp2f(sv[e] * c2 - mc);
        psum += p[e];
      }
      lrun[i] = lrun[i] * corr + psum;
      // rescale O only when some column's maximum moved (rare after the first steps)
      if (__builtin_expect(__builtin_amdgcn_ballot_w64(m_new > mrun[i]) != 0, 0)) {
#pragma unroll
        for (int d = 0; d < PHD / 32; ++d) oacc[i][d] = oacc[i][d] * corr;
      }
      mrun[i] = m_new;
#pragma unroll
      for (int jj = 0; jj < 2; ++jj) {
        v4u pk;
        pk[0] = pack_h16x2_inrange(p[8 * jj + 0], p[8 * jj + 1]);  // exp(s - max) lies in [0, 1]
        pk[1] = pack_h16x2_inrange(p[8 * jj + 2], p[8 * jj + 3]);
        pk[2] = pack_h16x2_inrange(p[8 * jj + 4], p[8 * jj + 5]);
        pk[3] = pack_h16x2_inrange(p[8 * jj + 6], p[8 * jj + 7]);
        pf[i][jj] = __builtin_bit_cast(v8h, pk);
      }
    }
    // ---- O^T += V^T P^T: V fragments read from LDS once, used by every active block
#pragma unroll
    for (int jj = 0; jj < 2; ++jj)
#pragma unroll
      for (int d = 0; d < PHD / 32; ++d) {
        const v8h vf = *reinterpret_cast<const v8h*>(sb + voff + jj * kPageBytes + d * 1024);
#pragma unroll
        for (int i = 0; i < NCB; ++i)
          oacc[i][d] = __builtin_amdgcn_mfma_f32_32x32x16_f16(vf, pf[i][jj], oacc[i][d], 0, 0, 0);
      }
  };
  for (int t = 0; t < n_steps; ++t) {
    wait_vm<(kAStages - 2) * kCopies>();  // step t landed; the later ones may be in flight
    __builtin_amdgcn_s_barrier();
    issue(t + kAStages - 1, (t + kAStages - 1) % kAStages);
    const uint8_t* sb = lds + (t % kAStages) * kAStageBytes;
    if (t <= my_last) step(t, sb);  // wavefront-uniform: later steps hold only keys behind this block
  }
  wait_vm<0>();  // the clamped copies past the last step still target this workgroup's LDS

  // ---- normalise and store: lane holds dims 32 d + 8 qq + 4 hh + 0..3 of its column in registers 4 qq ..
#pragma unroll
  for (int i = 0; i < NCB; ++i) {
    float l = lrun[i];
    l += __shfl_xor(l, 32, 64);
    if (qpos[i] < 0) continue;
    const float inv = 1.0f / l;
    const int tok = tok0 + qpos[i];
#pragma unroll
    for (int d = 0; d < PHD / 32; ++d)
#pragma unroll
      for (int qq = 0; qq < 4; ++qq) {
        uint2 pk;
        pk.x = pack_h16x2_flag(oacc[i][d][4 * qq] * inv, oacc[i][d][4 * qq + 1] * inv, err_flag);
        pk.y = pack_h16x2_flag(oacc[i][d][4 * qq + 2] * inv, oacc[i][d][4 * qq + 3] * inv, err_flag);
        *reinterpret_cast<uint2*>(o + act_off(tok, qhd[i] * PHD + 32 * d + 8 * qq + 4 * hh, Mpad)) = pk;
      }
  }
}

}  // namespace

void attention_prefill(h16_t* o, const h16_t* q, int n_seqs, int S, int m_tiles, int Hq, int Hkv,
                       TokMap map, KvPool pool, int layer, int* err_flag, hipStream_t st, const int* seq_start) {
  static bool configured = false;
  constexpr int kLdsMax = 160 * 1024;
  if (!configured) {
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&k_attn_prefill32<128>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, kLdsMax);
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&k_attn_prefill32<64>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, kLdsMax);
    configured = true;
  }
  // ring of K/V steps + page ids of one sequence (2 per step of 32 tokens)
  const int hd = pool.head_dim;
  const int lds_bytes = kAStages * 4 * kPageTokens * hd * 2 + 2 * ((map.pos_base + S + 31) / 32) * (int)sizeof(int);
  const int n_cols = Hq / Hkv * S;
  const dim3 grid((n_cols + QB - 1) / QB, Hkv, n_seqs);
  if (hd == 64)
    k_attn_prefill32<64><<<grid, 256, lds_bytes, st>>>(o, q, S, m_tiles * 16, Hq, Hkv, map.row_stride, map.pos_base, pool,
                                                       layer, err_flag, seq_start);
  else
    k_attn_prefill32<128><<<grid, 256, lds_bytes, st>>>(o, q, S, m_tiles * 16, Hq, Hkv, map.row_stride, map.pos_base,
                                                        pool, layer, err_flag, seq_start);
}

}  // namespace bf16
}  // namespace mtmc
