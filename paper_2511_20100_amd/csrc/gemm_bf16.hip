// bf16 MFMA GEMMs of the bf16 path.  Both operands are read in the fragment-tiled layouts of
// frag.h straight into MFMA operand registers: weights stream from HBM as contiguous 1 KiB
// blocks, activations (small, cache resident) come from L2 in the same block format.
//
// Orientation: the weight tile is the MFMA "A" operand (rows = output features n) and the
// activation tile the "B" operand (columns = tokens m), so a lane ends up holding 4 consecutive
// output features of one token: D[n = 4 (lane / 16) + r][m = lane % 16].
#include <algorithm>

#include "bf16_kernels.h"
#include "device_utils.h"
#include "frag.h"

namespace mtmc {
namespace bf16 {

// acc[nb][mb] += W[n tiles nt0 + nb] . X[m tiles mt0 + mb] over k tiles [k0, k1).
// Tile indices past the end are clamped (their results are never stored).  Operands live in a
// ring of PF k-steps of registers: the loads of step k + PF are issued as soon as step k has
// been consumed, so PF * (NB + MB) KiB per wavefront are always in flight.
template <int NB, int MB, int PF>
__device__ __forceinline__ void wave_gemm(const h16_t* __restrict__ Wt, int k_tiles, int n_tiles,
                                          int nt0, const h16_t* __restrict__ Xt, int m_tiles,
                                          int mt0, int k0, int k1, int lane, v4f (&acc)[NB][MB]) {
  if (k0 >= k1) return;
  const h16_t* wp[NB];
  const h16_t* xp[MB];
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) wp[nb] = Wt + (size_t)min(nt0 + nb, n_tiles - 1) * k_tiles * 512 + lane * 8;
#pragma unroll
  for (int mb = 0; mb < MB; ++mb) xp[mb] = Xt + (size_t)min(mt0 + mb, m_tiles - 1) * 512 + lane * 8;
  const size_t xstep = (size_t)m_tiles * 512;
  v8h wr[PF][NB], xr[PF][MB];
#pragma unroll
  for (int s = 0; s < PF; ++s) {
    const int kk = min(k0 + s, k1 - 1);
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) wr[s][nb] = load_frag(wp[nb] + (size_t)kk * 512, 0);
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) xr[s][mb] = load_frag(xp[mb] + (size_t)kk * xstep, 0);
  }
  int ks = k0;
  // Steady state: every slot that is multiplied is refilled, unconditionally, and before the next slot is
  // multiplied.  (Behind a branch the refill makes the compiler wait at the join for every outstanding load, the
  // other slot's included; unpinned, it sinks all loads of a trip behind all its products.)
  for (; ks + 2 * PF <= k1; ks += PF) {
#pragma unroll
    for (int s = 0; s < PF; ++s) {
#pragma unroll
      for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) acc[nb][mb] = mfma16(wr[s][nb], xr[s][mb], acc[nb][mb]);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) wr[s][nb] = load_frag(wp[nb] + (size_t)(ks + s + PF) * 512, 0);
#pragma unroll
      for (int mb = 0; mb < MB; ++mb) xr[s][mb] = load_frag(xp[mb] + (size_t)(ks + s + PF) * xstep, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
  }
  for (; ks < k1; ks += PF) {  // the last PF .. 2 PF - 1 steps: refills only while the range lasts
#pragma unroll
    for (int s = 0; s < PF; ++s) {
      if (ks + s < k1) {
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
          for (int mb = 0; mb < MB; ++mb) acc[nb][mb] = mfma16(wr[s][nb], xr[s][mb], acc[nb][mb]);
        const int kn = ks + s + PF;
        if (kn < k1) {
#pragma unroll
          for (int nb = 0; nb < NB; ++nb) wr[s][nb] = load_frag(wp[nb] + (size_t)kn * 512, 0);
#pragma unroll
          for (int mb = 0; mb < MB; ++mb) xr[s][mb] = load_frag(xp[mb] + (size_t)kn * xstep, 0);
        }
      }
    }
  }
}

__device__ __forceinline__ float silu_f(float g) { return g / (1.0f + expf(-g)); }

// ======================================================================================
// Large GEMM (prefill / scoring): workgroup tile 128 features x 128 tokens, four wavefronts
// in a 2 x 2 arrangement of 64 x 64 sub-tiles, full K per workgroup.
// ======================================================================================
enum { LEPI_STORE = 0, LEPI_ADD = 1, LEPI_SWIGLU = 2 };

// Workgroup -> output block.  Launch index L runs on XCD L % 8 (round-robin hand-out), and each XCD
// has its own L2.  Every XCD therefore owns whole rows of token blocks (token block = xcd + 8 i) and
// walks them in bands of LGM token blocks x all feature blocks, feature index slowest, so that the
// ~32-64 workgroups resident on an XCD at one time share LGM activation panels and a few weight
// panels through that L2.
// With fewer token blocks than XCDs (a prompt or two) the XCDs share out the feature blocks instead, or most of them
// would have nothing to do.
constexpr int LGM = 4;
struct LargeBlock { int nb, mb; bool valid; };
__device__ __forceinline__ LargeBlock large_block(int L, int nb_n, int nb_m) {
  const bool by_feature = nb_m < 8 && nb_n > nb_m;
  const int n_walk = by_feature ? nb_m : nb_n, n_own = by_feature ? nb_n : nb_m;
  const int xcd = L & 7, j = L >> 3;
  const int band = j / (LGM * n_walk), r = j - band * (LGM * n_walk);
  const int wb = r / LGM, oi = band * LGM + (r - wb * LGM);
  const int ob = xcd + 8 * oi;
  return by_feature ? LargeBlock{ob, wb, ob < n_own} : LargeBlock{wb, ob, ob < n_own};
}
static int large_grid(int nb_n, int nb_m) {
  const bool by_feature = nb_m < 8 && nb_n > nb_m;
  const int n_walk = by_feature ? nb_m : nb_n, n_own = by_feature ? nb_n : nb_m;
  const int per_xcd = (n_own + 7) / 8, bands = (per_xcd + LGM - 1) / LGM;
  return 8 * bands * LGM * n_walk;
}

template <int EPI>
__global__ __launch_bounds__(256) void k_gemm_large(LargeArgs a) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const LargeBlock blk = large_block(blockIdx.x, (a.n_tiles + 7) / 8, (a.m_tiles + 7) / 8);
  if (!blk.valid) return;
  const int nt0 = blk.nb * 8 + (wave & 1) * 4;
  const int mt0 = blk.mb * 8 + (wave >> 1) * 4;
  if (nt0 >= a.n_tiles || mt0 >= a.m_tiles) return;
  if (a.d_rows && mt0 * 16 >= *a.d_rows) return;  // rows packed on the device: no token in these rows
  v4f acc[4][4];
#pragma unroll
  for (int nb = 0; nb < 4; ++nb)
#pragma unroll
    for (int mb = 0; mb < 4; ++mb) acc[nb][mb] = v4f{0.f, 0.f, 0.f, 0.f};
  wave_gemm<4, 4, 2>(a.Wt, a.k_tiles, a.n_tiles, nt0, a.Xt, a.m_tiles, mt0, 0, a.k_tiles, lane, acc);
  const int col = lane & 15, rq = (lane >> 4) * 4;
  const int Mpad = a.m_tiles * 16;
#pragma unroll
  for (int nb = 0; nb < 4; ++nb) {
    if (nt0 + nb >= a.n_tiles) continue;
    if (EPI == LEPI_SWIGLU && (nb & 1)) continue;
#pragma unroll
    for (int mb = 0; mb < 4; ++mb) {
      const int m = (mt0 + mb) * 16 + col;
      if (m >= a.M) continue;
      if (EPI == LEPI_SWIGLU) {
        const int f = ((nt0 + nb) >> 1) * 16 + rq;
        const v4f g = acc[nb][mb], u = acc[nb + 1][mb];
        uint2 pk;
        pk.x = pack_h16x2_flag(silu_f(g[0]) * u[0], silu_f(g[1]) * u[1], a.err_flag);
        pk.y = pack_h16x2_flag(silu_f(g[2]) * u[2], silu_f(g[3]) * u[3], a.err_flag);
        *reinterpret_cast<uint2*>(a.out_bf16 + act_off(m, f, Mpad)) = pk;
      } else {
        const int n = (nt0 + nb) * 16 + rq;
        if (n >= a.N) continue;
        v4f* c = reinterpret_cast<v4f*>(a.out_f32 + (size_t)m * a.ld_out + n);
        if (EPI == LEPI_ADD) *c = *c + acc[nb][mb];
        else *c = acc[nb][mb];
      }
    }
  }
}

static void launch_large(const LargeArgs& a, int epi, hipStream_t st) {
  const dim3 grid(large_grid((a.n_tiles + 7) / 8, (a.m_tiles + 7) / 8));
  if (epi == LEPI_STORE) k_gemm_large<LEPI_STORE><<<grid, 256, 0, st>>>(a);
  else if (epi == LEPI_ADD) k_gemm_large<LEPI_ADD><<<grid, 256, 0, st>>>(a);
  else k_gemm_large<LEPI_SWIGLU><<<grid, 256, 0, st>>>(a);
}

// The LDS-staged kernel (256 x 256 blocks, one workgroup per CU) takes over once the output has
// at least `lds_min_blocks` such blocks; smaller problems keep the 128 x 128 direct kernel, which
// spreads them over more workgroups.
static bool use_lds_kernel(int n_tiles, int k_tiles, int m_tiles, int lds_min_blocks) {
  // the LDS pipeline streams k-steps in pairs through a ring of four buffers
  return k_tiles >= 4 && k_tiles % 2 == 0 && ((n_tiles + 15) / 16) * ((m_tiles + 15) / 16) >= lds_min_blocks;
}
void gemm_large_f32(float* C, int ldc, int N, bool accumulate, const h16_t* Wt, int n_tiles,
                    int k_tiles, const h16_t* Xt, int M, int m_tiles, int lds_min_blocks, const int* d_rows,
                    hipStream_t st, float* part, size_t part_floats) {
  LargeArgs a{};
  a.Wt = Wt; a.Xt = Xt; a.n_tiles = n_tiles; a.k_tiles = k_tiles; a.m_tiles = m_tiles; a.M = M; a.N = N;
  a.out_f32 = C; a.ld_out = ldc; a.d_rows = d_rows;
  const int epi = accumulate ? LEPI_ADD : LEPI_STORE;
  if (part && gemm_lds_split(a, accumulate, part, part_floats, st)) return;
  if (use_lds_kernel(n_tiles, k_tiles, m_tiles, lds_min_blocks)) gemm_lds(a, epi, st);
  else launch_large(a, epi, st);
}
void gemm_large_swiglu(h16_t* act, const h16_t* Wt, int n_tiles, int k_tiles, const h16_t* Xt,
                       int M, int m_tiles, int lds_min_blocks, int* err_flag, const int* d_rows, hipStream_t st) {
  LargeArgs a{};
  a.Wt = Wt; a.Xt = Xt; a.n_tiles = n_tiles; a.k_tiles = k_tiles; a.m_tiles = m_tiles; a.M = M;
  a.out_bf16 = act; a.err_flag = err_flag; a.d_rows = d_rows;
  if (use_lds_kernel(n_tiles, k_tiles, m_tiles, lds_min_blocks)) gemm_lds(a, LEPI_SWIGLU, st);
  else launch_large(a, LEPI_SWIGLU, st);
}

// ======================================================================================
// Scoring LM head: logits are never stored.  A workgroup owns 128 rows and a range of
// vocabulary tiles; every lane keeps running (log-sum-exp, top-2, target logit) for its rows.
// ======================================================================================
__global__ __launch_bounds__(256) void k_lmhead_score(ScoreHeadArgs a) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wn = wave & 1;
  const int mt0 = blockIdx.y * 8 + (wave >> 1) * 4;
  if (mt0 >= a.m_tiles) return;
  if (a.d_rows && mt0 * 16 >= *a.d_rows) return;  // rows packed on the device: no token in these rows
  const int col = lane & 15, rq = (lane >> 4) * 4;
  Lse lse[4];
  Top2 top[4];
  float zt[4];
  int target[4];
#pragma unroll
  for (int mb = 0; mb < 4; ++mb) {
    lse[mb] = lse_empty();
    top[mb] = top2_empty();
    zt[mb] = -INFINITY;
    const int m = (mt0 + mb) * 16 + col;
    target[mb] = (m < a.M) ? a.targets[m] : -1;
  }
  const int g_lo = blockIdx.x * a.groups_per_block, g_hi = min(a.n_groups, g_lo + a.groups_per_block);
  for (int g = g_lo; g < g_hi; ++g) {
    const int nt0 = g * 8 + wn * 4;
    if (nt0 >= a.n_tiles) break;
    v4f acc[4][4];
#pragma unroll
    for (int nb = 0; nb < 4; ++nb)
#pragma unroll
      for (int mb = 0; mb < 4; ++mb) acc[nb][mb] = v4f{0.f, 0.f, 0.f, 0.f};
    wave_gemm<4, 4, 2>(a.Wt, a.k_tiles, a.n_tiles, nt0, a.Xt, a.m_tiles, mt0, 0, a.k_tiles, lane, acc);
#pragma unroll
    for (int nb = 0; nb < 4; ++nb) {
      if (nt0 + nb >= a.n_tiles) continue;
      const int v0 = (nt0 + nb) * 16 + rq;
#pragma unroll
      for (int mb = 0; mb < 4; ++mb)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const float z = acc[nb][mb][r];
          lse_push(lse[mb], z);
          top2_push(top[mb], z, v0 + r);
          if (v0 + r == target[mb]) zt[mb] = z;
        }
    }
  }
#pragma unroll
  for (int mb = 0; mb < 4; ++mb) {
#pragma unroll
    for (int o = 16; o <= 32; o <<= 1) {
      const Lse ol = {__shfl_xor(lse[mb].m, o, 64), __shfl_xor(lse[mb].s, o, 64)};
      const Top2 ot = {__shfl_xor(top[mb].v1, o, 64), __shfl_xor(top[mb].i1, o, 64),
                       __shfl_xor(top[mb].v2, o, 64)};
      lse[mb] = lse_merge(lse[mb], ol);
      top[mb] = top2_merge(top[mb], ot);
      zt[mb] = fmaxf(zt[mb], __shfl_xor(zt[mb], o, 64));
    }
    const int m = (mt0 + mb) * 16 + col;
    if (lane < 16 && m < a.M) {
      ScorePartial* p = reinterpret_cast<ScorePartial*>(a.part) + ((size_t)(blockIdx.x * 2 + wn)) * a.M + m;
      p->m = lse[mb].m; p->s = lse[mb].s; p->v1 = top[mb].v1; p->i1 = top[mb].i1; p->v2 = top[mb].v2;
      p->zt = zt[mb];
    }
  }
}

int score_head_blocks(int n_tiles, int* groups_per_block) {
  const int n_groups = (n_tiles + 7) / 8;           // 128 vocabulary entries per group
  const int gpb = std::max(1, std::min(n_groups, 16));
  *groups_per_block = gpb;
  return (n_groups + gpb - 1) / gpb;
}

void lmhead_score(float* part, const h16_t* Wt, int n_tiles, int k_tiles, const h16_t* Xt, int M,
                  int m_tiles, const int* targets, bool want_top, int lds_min_blocks, const int* d_rows,
                  hipStream_t st) {
  ScoreHeadArgs a{};
  a.want_top = want_top ? 1 : 0;
  a.d_rows = d_rows;
  a.Wt = Wt; a.Xt = Xt; a.n_tiles = n_tiles; a.k_tiles = k_tiles; a.m_tiles = m_tiles; a.M = M;
  a.targets = targets; a.part = part;
  a.n_groups = (n_tiles + 7) / 8;
  const int blocks = score_head_blocks(n_tiles, &a.groups_per_block);
  // same vocabulary slices (and partial results) in both kernels: 128 row tiles per slice
  if (use_lds_kernel(n_tiles, k_tiles, m_tiles, lds_min_blocks)) lmhead_score_lds(a, blocks, st);
  else k_lmhead_score<<<dim3(blocks, (m_tiles + 7) / 8), 256, 0, st>>>(a);
}

// Row r of the chunk is position i = first + (row0 + r) % n_scored of sequence
// n = seq0 + (row0 + r) / n_scored; targets[r] = seqs[n, i + 1] (clamped, flagging bad ids).
__global__ void k_score_targets(int* targets, const int* seqs, int R, int S, int first, int n_scored,
                                int seq0, int row0, int vocab, int* err_flag) {
  const int r = blockIdx.x * blockDim.x + threadIdx.x;
  if (r >= R) return;
  const int n = seq0 + (row0 + r) / n_scored, i = first + (row0 + r) % n_scored;
  int t = seqs[(size_t)n * S + i + 1];
  if (t < 0 || t >= vocab) {
    atomicOr(err_flag, 1);
    t = t < 0 ? 0 : vocab - 1;
  }
  targets[r] = t;
}
void score_targets(int* targets, const int* seqs, int R, int S, int first, int n_scored, int seq0,
                   int row0, int vocab, int* err_flag, hipStream_t st) {
  k_score_targets<<<(R + 255) / 256, 256, 0, st>>>(targets, seqs, R, S, first, n_scored, seq0, row0,
                                                  vocab, err_flag);
}

__global__ __launch_bounds__(64) void k_score_reduce(const ScorePartial* part, int n_parts, int R, int S,
                                                     int first, int n_scored, int seq0, int row0,
                                                     float* out_logprobs, int* out_top1,
                                                     float* out_margin) {
  const int r = blockIdx.x;
  const int lane = threadIdx.x;
  Lse lse = lse_empty();
  Top2 top = top2_empty();
  float zt = -INFINITY;
  for (int g = lane; g < n_parts; g += 64) {
    const ScorePartial p = part[(size_t)g * R + r];
    lse = lse_merge(lse, Lse{p.m, p.s});
    top = top2_merge(top, Top2{p.v1, p.i1, p.v2});
    zt = fmaxf(zt, p.zt);
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    const Lse ol = {__shfl_xor(lse.m, o, 64), __shfl_xor(lse.s, o, 64)};
    const Top2 ot = {__shfl_xor(top.v1, o, 64), __shfl_xor(top.i1, o, 64), __shfl_xor(top.v2, o, 64)};
    lse = lse_merge(lse, ol);
    top = top2_merge(top, ot);
    zt = fmaxf(zt, __shfl_xor(zt, o, 64));
  }
  if (lane == 0) {
    const int n = seq0 + (row0 + r) / n_scored, i = first + (row0 + r) % n_scored;
    const size_t slot = (size_t)n * (S - 1) + i;
    out_logprobs[slot] = zt - (lse.m + logf(lse.s));
    if (out_top1) out_top1[slot] = top.i1;
    if (out_margin) out_margin[slot] = top.v1 - top.v2;
  }
}
void score_reduce(const float* part, int n_parts, int R, int S, int first, int n_scored, int seq0,
                  int row0, float* out_logprobs, int* out_top1, float* out_margin, hipStream_t st) {
  k_score_reduce<<<R, 64, 0, st>>>(reinterpret_cast<const ScorePartial*>(part), n_parts, R, S, first,
                                   n_scored, seq0, row0, out_logprobs, out_top1, out_margin);
}

__global__ __launch_bounds__(64) void k_score_reduce_scatter(const ScorePartial* part, int n_parts, int R,
                                                             const int* d_rows, const int* out_index,
                                                             float* out_logprobs) {
  const int r = blockIdx.x;
  if (r >= *d_rows) return;
  const int lane = threadIdx.x;
  Lse lse = lse_empty();
  float zt = -INFINITY;
  for (int g = lane; g < n_parts; g += 64) {
    const ScorePartial p = part[(size_t)g * R + r];
    lse = lse_merge(lse, Lse{p.m, p.s});
    zt = fmaxf(zt, p.zt);
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    const Lse ol = {__shfl_xor(lse.m, o, 64), __shfl_xor(lse.s, o, 64)};
    lse = lse_merge(lse, ol);
    zt = fmaxf(zt, __shfl_xor(zt, o, 64));
  }
  if (lane == 0) out_logprobs[out_index[r]] = zt - (lse.m + logf(lse.s));
}
void score_reduce_scatter(const float* part, int n_parts, int R, const int* d_rows, const int* out_index,
                          float* out_logprobs, hipStream_t st) {
  if (R == 0) return;
  k_score_reduce_scatter<<<R, 64, 0, st>>>(reinterpret_cast<const ScorePartial*>(part), n_parts, R, d_rows, out_index,
                                           out_logprobs);
}

// One workgroup of 1024 threads: thread t owns the candidates t, t + 1024, ... in blocks of consecutive
// candidates, sums their lengths, the 1024 sums are scanned in LDS, then every thread writes its candidates.
__global__ __launch_bounds__(1024) void k_build_packed_actions(int* seq_start, int* d_rows, int* ids, int* targets,
                                                               int* out_index, const int* states, const int* actions,
                                                               const int* action_len, int P, int K, int A, int r0,
                                                               int nr, int vocab, int* err_flag) {
  __shared__ int s_sum[1024];
  const int tid = threadIdx.x;
  const int per = (nr + 1023) / 1024;            // consecutive candidates per thread
  const int c0 = min(tid * per, nr), c1 = min(c0 + per, nr);
  auto len_of = [&](int c) {
    const int raw = action_len[r0 + c];
    if (raw < 0 || raw > A) atomicOr(err_flag, 4);
    return min(max(raw, 0), A);
  };
  int mine = 0;
  for (int c = c0; c < c1; ++c) mine += len_of(c);
  s_sum[tid] = mine;
  __syncthreads();
  // inclusive scan (Hillis-Steele, 10 rounds)
  for (int off = 1; off < 1024; off <<= 1) {
    const int v = tid >= off ? s_sum[tid - off] : 0;
    __syncthreads();
    s_sum[tid] += v;
    __syncthreads();
  }
  int at = s_sum[tid] - mine;                      // first packed token of this thread's candidates
  if (tid == 1023) d_rows[0] = s_sum[1023];
  for (int c = c0; c < c1; ++c) {
    const int b = r0 + c, len = min(max(action_len[b], 0), A);
    seq_start[c] = at;
    const int* act = actions + (size_t)b * A;
    for (int i = 0; i < len; ++i) {
      int in = i == 0 ? states[(size_t)(b / K) * P + P - 1] : act[i - 1];
      int tg = act[i];
      if (tg < 0 || tg >= vocab) {
        atomicOr(err_flag, 1);
        tg = tg < 0 ? 0 : vocab - 1;
      }
      if (in < 0 || in >= vocab) {
        atomicOr(err_flag, 1);
        in = in < 0 ? 0 : vocab - 1;
      }
      ids[at + i] = in;
      targets[at + i] = tg;
      out_index[at + i] = b * A + i;
    }
    at += len;
  }
  if (tid == 1023) seq_start[nr] = s_sum[1023];
}
void build_packed_actions(int* seq_start, int* d_rows, int* ids, int* targets, int* out_index, const int* states,
                          const int* actions, const int* action_len, int P, int K, int A, int r0, int nr, int vocab,
                          int* err_flag, hipStream_t st) {
  k_build_packed_actions<<<1, 1024, 0, st>>>(seq_start, d_rows, ids, targets, out_index, states, actions, action_len,
                                             P, K, A, r0, nr, vocab, err_flag);
}

}  // namespace bf16
}  // namespace mtmc
