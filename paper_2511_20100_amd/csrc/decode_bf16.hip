// Decode-step kernels of the bf16 path: six launches per residual block.
//
//   qkv   = W_qkv x'                      k_gemm_dec<STORE>
//   o     = attention(rope(q), cache)     k_attn_dec   (also rotates/writes the new K, V; output per context chunk)
//   h    += W_o o;   x' for the FFN       k_gemm_dec<RESID>   (combines the context chunks)
//   a     = silu(W_g x') * (W_u x')       k_gemm_dec<SWIGLU>
//   P_s   = W_d[:, k range s] a           k_gemm_dec<PARTIAL> (split-K: the matrix has too few rows to fill the chip)
//   h    += sum_s P_s; x' for the next block   k_resid_reduce
//
// Apart from the down projection every GEMM workgroup owns whole output columns (all of K), so its results are
// complete when the workgroup ends.  Nothing is accumulated with atomics: every sum has a fixed order.
//
// Deferred RMSNorm.  A producer (RESID) cannot know the new row norm (other workgroups hold the
// other columns), so it writes x' = fp16(h_new * gain * r_old), r_old = 1/rms of the row *before*
// its update (a well-scaled fp16 value), together with the sum of squares of its 16 new columns.
// The consumer sums those per-tile squares in a fixed order to get r_new and multiplies its
// fp32 accumulators by r_new / r_old: W (h g r_new) = (W (h g r_old)) r_new / r_old.
#include "attention_core.h"
#include "bf16_kernels.h"
#include "device_utils.h"
#include "frag.h"

namespace mtmc {
namespace bf16 {

// acc[nb][mb] += W[n tile nt0 + nb] . X[m tile mb] over k tiles [k0, k1).  Weight fragments (HBM,
// long latency) are kept PFW k-steps ahead in registers, activation fragments (L2) PFX ahead.
// The operand streams of one wavefront: weight tiles nt0 .. nt0 + NB - 1 and all MB token tiles over k tiles
// [k0, k1), through register rings PFW / PFX k-steps deep.  start() issues the first loads (so that they are
// in flight while the kernel does other things), run() multiplies.
template <int NB, int MB, int PFW, int PFX>
struct DecStream {
  static_assert(PFW % PFX == 0, "the weight ring must be a multiple of the activation ring");
  const h16_t* wp[NB];
  const h16_t* xp[MB];
  size_t xstep;
  int k0, k1;
  v8h wr[PFW][NB], xr[PFX][MB];

  __device__ __forceinline__ void start(const h16_t* __restrict__ Wt, int k_tiles, int n_tiles, int nt0,
                                        const h16_t* __restrict__ Xt, int m_tiles, int mt0, int k0_, int k1_,
                                        int lane) {
    k0 = k0_;
    k1 = k1_;
    if (k0 >= k1) return;
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) wp[nb] = Wt + (size_t)min(nt0 + nb, n_tiles - 1) * k_tiles * 512 + lane * 8;
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) xp[mb] = Xt + (size_t)min(mt0 + mb, m_tiles - 1) * 512 + lane * 8;
    xstep = (size_t)m_tiles * 512;
#pragma unroll
    for (int s = 0; s < PFW; ++s) {
      const int kk = min(k0 + s, k1 - 1);
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) wr[s][nb] = load_frag(wp[nb] + (size_t)kk * 512, 0);
    }
#pragma unroll
    for (int s = 0; s < PFX; ++s) {
      const int kk = min(k0 + s, k1 - 1);
#pragma unroll
      for (int mb = 0; mb < MB; ++mb) xr[s][mb] = load_frag(xp[mb] + (size_t)kk * xstep, 0);
    }
  }

  __device__ __forceinline__ void run(v4f (&acc)[NB][MB]) {
    if (k0 >= k1) return;
    int ks = k0;
    // Steady state: every slot that is multiplied is refilled, unconditionally.  (A refill behind a branch makes the
    // compiler wait, at the join, for every outstanding load -- the other slots' refills included -- so the ring
    // would never hold more than one slot in flight.)
    for (; ks + 2 * PFW <= k1; ks += PFW) {
#pragma unroll
      for (int s = 0; s < PFW; ++s) {
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
          for (int mb = 0; mb < MB; ++mb) acc[nb][mb] = mfma16(wr[s][nb], xr[s % PFX][mb], acc[nb][mb]);
        // the slot's refill goes out before the next slot is multiplied (the scheduler would otherwise sink every
        // load to the end of the trip, behind all the products)
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) wr[s][nb] = load_frag(wp[nb] + (size_t)(ks + s + PFW) * 512, 0);
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) xr[s % PFX][mb] = load_frag(xp[mb] + (size_t)(ks + s + PFX) * xstep, 0);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    // the last PFW .. 2 PFW - 1 steps: refills only while the range lasts
    for (; ks < k1; ks += PFW) {
#pragma unroll
      for (int s = 0; s < PFW; ++s) {
        if (ks + s < k1) {
#pragma unroll
          for (int nb = 0; nb < NB; ++nb)
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) acc[nb][mb] = mfma16(wr[s][nb], xr[s % PFX][mb], acc[nb][mb]);
          const int kw = ks + s + PFW, kx = ks + s + PFX;
          if (kw < k1) {
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) wr[s][nb] = load_frag(wp[nb] + (size_t)kw * 512, 0);
          }
          if (kx < k1) {
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) xr[s % PFX][mb] = load_frag(xp[mb] + (size_t)kx * xstep, 0);
          }
        }
      }
    }
  }
};

__device__ __forceinline__ float silu_d(float g) { return g / (1.0f + expf(-g)); }

enum { DEPI_STORE = DEC_STORE, DEPI_RESID = DEC_RESID, DEPI_SWIGLU = DEC_SWIGLU, DEPI_SAMPLE = DEC_SAMPLE,
       DEPI_PARTIAL = DEC_PARTIAL };

template <int NB, int MB, int WAVES, int PFW, int PFX, int MINW, int EPI, int NBP = NB>
__global__ __launch_bounds__(WAVES * 64, MINW) void k_gemm_dec(DecGemmArgs a) {
  // NBP = row tiles summed and finished per pass over the LDS exchange buffer (NB / NBP passes)
  static_assert(NB % NBP == 0 && (EPI != DEPI_SWIGLU || NBP % 2 == 0 || NB == 1) && (EPI != DEPI_SAMPLE || MB <= WAVES),
                "bad tiles-per-pass");
  __shared__ float red[WAVES][NBP * MB * 4][64];
  __shared__ float s_scale[128];
  __shared__ float s_part[2][WAVES * 64];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  // weight row tiles nt0 .. nt0 + NB - 1 (group grp of n_groups), token tiles mt0 .. mt0 + MB - 1: the launch may
  // split the rows over gridDim.y (split-K uses that index itself) or over pairs of workgroups along x
  int grp = blockIdx.x, n_groups = gridDim.x, mpart = (EPI == DEPI_PARTIAL) ? 0 : blockIdx.y;
  // split-K: this workgroup's K split and their number.  XCD-aligned form (8 splits, one-dimensional grid): workgroups
  // go to the 8 XCDs round-robin in launch order, so split s = launch index % 8 runs on XCD s alone and every XCD's
  // L2 fetches one eighth of the activation operand instead of all of it
  int ksp = blockIdx.y, nsp = gridDim.y;
  if (EPI == DEPI_PARTIAL && a.xcd_split) {
    ksp = blockIdx.x & 7;
    nsp = 8;
    grp = blockIdx.x >> 3;
    n_groups = gridDim.x >> 3;
  }
  if (a.row_pairs) {
    grp = (blockIdx.x >> 4) * 8 + (blockIdx.x & 7);
    mpart = (blockIdx.x >> 3) & 1;
    n_groups = (a.n_tiles + NB - 1) / NB;
    if (grp >= n_groups) return;  // the grid is rounded up to whole sets of 8 pairs
  }
  const int nt0 = grp * NB;
  const int mt0 = mpart * MB;
  const int Mpad = a.m_tiles * 16;
  // Row scales (consumers need r_new / r_old, producers r of the state they update).  Thread t sums
  // tiles part, part + P, ... of row t % Mpad; the P partial sums are then added in index order.
  // A split-K launch only needs them in the kernel that finishes the sum: its first workgroup
  // computes them on the side and leaves them in rs_out.
  constexpr bool kProducer = (EPI == DEPI_RESID || EPI == DEPI_PARTIAL);
  const bool do_rs = EPI != DEPI_PARTIAL || (grp == 0 && ksp == 0);  // workgroup-uniform (x 0: group 0, rows 0..)
  constexpr int NT = WAVES * 64;
  constexpr int BT = (WAVES >= 8) ? 8 : 24;  // loads per batch (all tiles of d = 1536 in one batch)
  const int P = NT / Mpad;  // Mpad <= 128 <= NT
  const int m = tid % Mpad, part = tid / Mpad;
  const bool two = !kProducer && a.ss_cur && a.ss_old != a.ss_cur;
  float sa = 0.f, sb = 0.f;
  float va[BT], vb[BT];  // the last batch stays pending while the operand streams are started
#pragma unroll
  for (int u = 0; u < BT; ++u) va[u] = vb[u] = 0.f;
  if (do_rs && a.ss_cur && part < P) {
    int t0 = part;
    for (; t0 + BT * P < a.ss_tiles; t0 += BT * P) {  // full batches: independent loads, then adds in index order
      float fa[BT], fb[BT];
#pragma unroll
      for (int u = 0; u < BT; ++u) {
        fa[u] = a.ss_cur[(size_t)(t0 + u * P) * Mpad + m];
        fb[u] = two ? a.ss_old[(size_t)(t0 + u * P) * Mpad + m] : 0.f;
      }
#pragma unroll
      for (int u = 0; u < BT; ++u) {
        sa += fa[u];
        sb += fb[u];
      }
    }
#pragma unroll
    for (int u = 0; u < BT; ++u) {
      const int t = t0 + u * P;
      va[u] = (t < a.ss_tiles) ? a.ss_cur[(size_t)t * Mpad + m] : 0.f;
      vb[u] = (two && t < a.ss_tiles) ? a.ss_old[(size_t)t * Mpad + m] : 0.f;
    }
  }
  // ---- operand streams: issued behind the row-scale loads, in flight while the scales are worked out
  int kbeg = 0, kend = a.k_tiles;
  if (EPI == DEPI_PARTIAL) {
    const int per_split = (a.k_tiles + nsp - 1) / nsp;
    kbeg = ksp * per_split;
    kend = min(a.k_tiles, kbeg + per_split);
  }
  const int per_wave = (max(kend - kbeg, 0) + WAVES - 1) / WAVES;
  const int k0 = kbeg + wave * per_wave, k1 = min(kend, k0 + per_wave);
  // O projection behind a context-split attention: the operand comes in chunks that are combined below
  bool chunked = false;
  if constexpr (EPI == DEPI_RESID && NB == 1 && (WAVES == 8 || WAVES == 12) && MB <= 4) chunked = a.n_xchunks > 1;  // workgroup-uniform
  DecStream<NB, MB, PFW, PFX> stream;
  stream.start(a.Wt, a.k_tiles, a.n_tiles, nt0, a.Xt, a.m_tiles, mt0, k0, chunked ? k0 : k1, lane);
  // Chunk-combining form: what one head needs (its weight tiles, the operand tiles of every chunk, the chunk
  // statistics).  chunks at most: the host keeps MB * chunks <= 8; the 12-wavefront form, which only ever runs with
  // two chunks, holds two in half the registers and requests its first head here, in the shadow of the row scales.
  constexpr bool kCombines = (EPI == DEPI_RESID && NB == 1 && (WAVES == 8 || WAVES == 12) && MB <= 4);
  constexpr int NCM = !kCombines ? 1 : WAVES == 12 ? 2 : MB >= 4 ? 2 : MB == 2 ? 4 : 8;
  v8h c_wf[4], c_xf[NCM][4][MB];
  float c_m[NCM][MB], c_l[NCM][MB];
  auto load_head = [&](int j) {
    const int HT = a.head_tiles, n_heads = a.k_tiles / HT, NC = a.n_xchunks;
    const int col = lane & 15;
    const h16_t* wp = a.Wt + (size_t)min(nt0, a.n_tiles - 1) * a.k_tiles * 512 + lane * 8;
#pragma unroll
    for (int t = 0; t < 4; ++t) c_wf[t] = load_frag(wp + (size_t)(j * HT + min(t, HT - 1)) * 512, 0);
#pragma unroll
    for (int c = 0; c < NCM; ++c)
#pragma unroll
      for (int mb = 0; mb < MB; ++mb) {
        const int row = (mt0 + mb) * 16 + col;
        const bool live = c < NC && row < a.M;
        const float* ml = a.chunk_ml + (((size_t)row * n_heads + j) * NC + c) * 2;
        c_m[c][mb] = live ? ml[0] : -INFINITY;
        c_l[c][mb] = live ? ml[1] : 0.f;
      }
#pragma unroll
    for (int c = 0; c < NCM; ++c) {
      if (c >= NC) break;  // NC is uniform: the chunks that do not exist are neither loaded nor multiplied
      const h16_t* xp = a.Xt + (size_t)c * a.x_chunk_stride + lane * 8;
#pragma unroll
      for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
          c_xf[c][t][mb] =
              load_frag(xp + ((size_t)(j * HT + min(t, HT - 1)) * a.m_tiles + min(mt0 + mb, a.m_tiles - 1)) * 512, 0);
    }
  };
  if constexpr (kCombines && WAVES == 12) load_head(min(wave, a.k_tiles / a.head_tiles - 1));
#pragma unroll
  for (int u = 0; u < BT; ++u) {
    sa += va[u];
    sb += vb[u];
  }
  if (do_rs) {
    if (part < P) {
      s_part[0][tid] = sa;
      s_part[1][tid] = sb;
    }
    // workgroup barrier on the LDS writes only (a __syncthreads() would also wait for the operand streams)
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    if (tid < Mpad) {
      float sc = 1.f;
      if (a.ss_cur && (kProducer || two)) {
        float ta = 0.f, tb = 0.f;
        for (int q = 0; q < P; ++q) {
          ta += s_part[0][q * Mpad + tid];
          tb += s_part[1][q * Mpad + tid];
        }
        sc = 1.0f / sqrtf(ta * a.inv_d + a.eps);
        if (two) sc *= sqrtf(tb * a.inv_d + a.eps);
      }
      s_scale[tid] = sc;
      if (EPI == DEPI_PARTIAL) a.rs_out[tid] = sc;
    }
  }
  v4f acc[NB][MB];
#pragma unroll
  for (int nb = 0; nb < NB; ++nb)
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) acc[nb][mb] = v4f{0.f, 0.f, 0.f, 0.f};
  stream.run(acc);
  if constexpr (EPI == DEPI_RESID && NB == 1 && (WAVES == 8 || WAVES == 12) && MB <= 4) {
    if (chunked) {
      // out[n][row] = sum_head sum_chunk share(row, head, chunk) * (W[n, head] . o_chunk[head, row]), where o_chunk is
      // the attention output over the chunk's keys normalised by the chunk's own sum l, and
      // share = l exp(m - max_c m) / sum_c l exp(m - max_c m).  Wavefront w takes heads w, w + WAVES, ...
      const int HT = a.head_tiles, n_heads = a.k_tiles / HT, NC = a.n_xchunks;
      for (int j = wave; j < n_heads; j += WAVES) {
        if (WAVES != 12 || j != wave) load_head(j);
        float mx[MB], den[MB];
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
          mx[mb] = c_m[0][mb];
#pragma unroll
          for (int c = 1; c < NCM; ++c) mx[mb] = fmaxf(mx[mb], c_m[c][mb]);
          den[mb] = 0.f;
#pragma unroll
          for (int c = 0; c < NCM; ++c) {
            c_l[c][mb] = (c_l[c][mb] > 0.f) ? c_l[c][mb] * expf(c_m[c][mb] - mx[mb]) : 0.f;  // un-normalised share
            den[mb] += c_l[c][mb];
          }
        }
#pragma unroll
        for (int c = 0; c < NCM; ++c) {
          if (c >= NC) break;
#pragma unroll
          for (int mb = 0; mb < MB; ++mb) {
            v4f part = v4f{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int t = 0; t < 4; ++t)
              if (t < HT) part = mfma16(c_wf[t], c_xf[c][t][mb], part);
            const float share = (den[mb] > 0.f) ? c_l[c][mb] / den[mb] : 0.f;
            acc[0][mb] = acc[0][mb] + part * share;
          }
        }
      }
    }
  }
  // Sum over the K slices: every wavefront publishes its accumulators; wavefront w then adds the WAVES
  // slices of token tiles w, w + WAVES, ... in index order and runs the epilogue for those tokens.
  // SAMPLE: a wavefront has at most one token tile (MB <= WAVES); its sampler state lives across the passes.
  Lse smp_lse = lse_empty();
  float smp_y = -INFINITY, smp_z = 0.f;
  int smp_i = 0x7fffffff;
#pragma unroll
  for (int ph = 0; ph < NB / NBP; ++ph) {
  const int nbase = nt0 + ph * NBP;  // first row tile of this pass
  if (ph) __syncthreads();            // the previous pass has been read
#pragma unroll
  for (int j = 0; j < NBP; ++j)
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
      for (int r = 0; r < 4; ++r) red[wave][(j * MB + mb) * 4 + r][lane] = acc[ph * NBP + j][mb][r];
  __syncthreads();
  for (int mb = wave; mb < MB && mt0 + mb < a.m_tiles; mb += WAVES) {
  v4f sum[NBP];
#pragma unroll
  for (int nb = 0; nb < NBP; ++nb) {
    sum[nb] = v4f{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int w = 0; w < WAVES; ++w)
#pragma unroll
      for (int r = 0; r < 4; ++r) sum[nb][r] += red[w][(nb * MB + mb) * 4 + r][lane];
  }
  const int col = lane & 15, rq = (lane >> 4) * 4;
  const int m = (mt0 + mb) * 16 + col;
  const float sc = (EPI == DEPI_PARTIAL) ? 1.f : s_scale[m];

  if (EPI == DEPI_PARTIAL) {
    float* P = a.out_f32 + (size_t)ksp * Mpad * a.ld_out;
#pragma unroll
    for (int nb = 0; nb < NBP; ++nb) {
      if (nbase + nb >= a.n_tiles) continue;
      *reinterpret_cast<v4f*>(P + (size_t)m * a.ld_out + (nbase + nb) * 16 + rq) = sum[nb];
    }
  } else if (EPI == DEPI_STORE) {
#pragma unroll
    for (int nb = 0; nb < NBP; ++nb) {
      if (nbase + nb >= a.n_tiles || m >= a.M) continue;
      *reinterpret_cast<v4f*>(a.out_f32 + (size_t)m * a.ld_out + (nbase + nb) * 16 + rq) = sum[nb] * sc;
    }
  } else if (EPI == DEPI_RESID) {
#pragma unroll
    for (int nb = 0; nb < NBP; ++nb) {
      if (nbase + nb >= a.n_tiles) continue;
      const int n = (nbase + nb) * 16 + rq;
      const v4f g = *reinterpret_cast<const v4f*>(a.gain + n);
      const bool live = m < a.M;
      v4f hv = v4f{0.f, 0.f, 0.f, 0.f};
      if (live) {
        float* hp = a.out_f32 + (size_t)m * a.ld_out + n;
        hv = *reinterpret_cast<const v4f*>(hp) + sum[nb];
        *reinterpret_cast<v4f*>(hp) = hv;
        uint2 pk;
        pk.x = pack_h16x2_flag(hv[0] * g[0] * sc, hv[1] * g[1] * sc, a.err_flag);
        pk.y = pack_h16x2_flag(hv[2] * g[2] * sc, hv[3] * g[3] * sc, a.err_flag);
        *reinterpret_cast<uint2*>(a.out_h16 + act_off(m, n, Mpad)) = pk;
      }
      float ss = (hv[0] * hv[0] + hv[1] * hv[1]) + (hv[2] * hv[2] + hv[3] * hv[3]);
      ss += __shfl_xor(ss, 16, 64);
      ss += __shfl_xor(ss, 32, 64);
      if (lane < 16 && live) a.ss_out[(size_t)(nbase + nb) * Mpad + m] = ss;
    }
  } else if (EPI == DEPI_SWIGLU) {
    // weight row tiles alternate gate / up: tile 2j holds gate rows 16j.., tile 2j+1 the up rows
#pragma unroll
    for (int nb = 0; nb < NBP; nb += 2) {
      if (nbase + nb >= a.n_tiles || m >= a.M) continue;
      const int f = ((nbase + nb) >> 1) * 16 + rq;
      const v4f g = sum[nb] * sc, u = sum[(nb + 1) % NBP] * sc;
      uint2 pk;
      pk.x = pack_h16x2_flag(silu_d(g[0]) * u[0], silu_d(g[1]) * u[1], a.err_flag);
      pk.y = pack_h16x2_flag(silu_d(g[2]) * u[2], silu_d(g[3]) * u[3], a.err_flag);
      *reinterpret_cast<uint2*>(a.out_h16 + act_off(m, f, Mpad)) = pk;
    }
  } else {  // DEPI_SAMPLE: log-sum-exp and Gumbel arg-max over this pass's part of the workgroup's vocabulary slice
    const SampleCtl ctl = *a.ctl;
    // the random numbers of a row follow the row and its own step, whatever slot it sits in and whenever it joined
    // (an empty slot draws row 0's: unused)
    const int smp_row = (ctl.slot_row && m < a.M) ? max(ctl.slot_row[m], 0) : m;
    const int step = *a.d_step - ((ctl.row_step0 && m < a.M) ? ctl.row_step0[m] : 0);
#pragma unroll
    for (int nb = 0; nb < NBP; ++nb) {
      if (nbase + nb >= a.n_tiles) continue;
      const int v0 = (nbase + nb) * 16 + rq;  // multiple of 4: one generator block per 4 entries
      uint4 rb = make_uint4(0, 0, 0, 0);
      if (!ctl.greedy)
        rb = philox4x32_10(make_uint4((uint32_t)(v0 >> 2), (uint32_t)step, ctl.seq_offset + smp_row, 0u), ctl.key0,
                           ctl.key1);
      const uint32_t rr[4] = {rb.x, rb.y, rb.z, rb.w};
      float zt[4];
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const float z = sum[nb][r] * sc;
        zt[r] = ctl.greedy ? z : z * ctl.inv_temp;
      }
      lse_push4(smp_lse, zt[0], zt[1], zt[2], zt[3]);
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const float y = ctl.greedy ? zt[r] : zt[r] + gumbel_from_bits(rr[r]);
        if (y > smp_y) { smp_y = y; smp_i = v0 + r; smp_z = zt[r]; }  // ascending index: the first maximum wins
      }
    }
  }
  }  // token tiles of this wavefront
  }  // passes
  if (EPI == DEPI_SAMPLE) {
    if (wave < MB && mt0 + wave < a.m_tiles) {
      const int col = lane & 15, m = (mt0 + wave) * 16 + col;
#pragma unroll
      for (int o = 16; o <= 32; o <<= 1) {
        const Lse ol = {__shfl_xor(smp_lse.m, o, 64), __shfl_xor(smp_lse.s, o, 64)};
        const float oy = __shfl_xor(smp_y, o, 64), oz = __shfl_xor(smp_z, o, 64);
        const int oi = __shfl_xor(smp_i, o, 64);
        smp_lse = lse_merge(smp_lse, ol);
        if (oy > smp_y || (oy == smp_y && oi < smp_i)) { smp_y = oy; smp_i = oi; smp_z = oz; }
      }
      if (lane < 16 && m < a.M) {
        // row-major per token row, so that the merge reads a row's partials as one contiguous run
        DecSamplePartial* p = reinterpret_cast<DecSamplePartial*>(a.out_f32) + (size_t)m * n_groups + grp;
        p->m = smp_lse.m; p->s = smp_lse.s; p->y = smp_y; p->idx = smp_i; p->zt = smp_z;
      }
    }
  }
}

template <int NB, int MB, int WAVES, int PFW, int PFX, int MINW, int NBP = NB>
static void launch_dec_t(const DecGemmArgs& a0, int epi, hipStream_t st, int msplit = 1, bool row_pairs = false) {
  DecGemmArgs a = a0;
  a.row_pairs = row_pairs ? 1 : 0;
  const int groups = (a.n_tiles + NB - 1) / NB;
  const int gx = row_pairs ? (groups + 7) / 8 * 16 : groups;
  if constexpr (NBP != NB) {  // several passes over the exchange buffer: SwiGLU and split-K shapes only
    const dim3 grid(gx, epi == DEPI_PARTIAL ? a.ksplit : 1), block(WAVES * 64);
    if (epi == DEPI_PARTIAL) k_gemm_dec<NB, MB, WAVES, PFW, PFX, MINW, DEPI_PARTIAL, NBP><<<grid, block, 0, st>>>(a);
    else if (epi == DEPI_SAMPLE) {
      if constexpr (MB <= WAVES) k_gemm_dec<NB, MB, WAVES, PFW, PFX, MINW, DEPI_SAMPLE, NBP><<<grid, block, 0, st>>>(a);
    } else k_gemm_dec<NB, MB, WAVES, PFW, PFX, MINW, DEPI_SWIGLU, NBP><<<grid, block, 0, st>>>(a);
  } else {
    const dim3 grid(gx, epi == DEPI_PARTIAL ? a.ksplit : msplit);
    const dim3 block(WAVES * 64);
    switch (epi) {
      case DEPI_PARTIAL: k_gemm_dec<NB, MB, WAVES, PFW, PFX, MINW, DEPI_PARTIAL><<<grid, block, 0, st>>>(a); break;
      case DEPI_STORE: k_gemm_dec<NB, MB, WAVES, PFW, PFX, MINW, DEPI_STORE><<<grid, block, 0, st>>>(a); break;
      case DEPI_RESID: k_gemm_dec<NB, MB, WAVES, PFW, PFX, MINW, DEPI_RESID><<<grid, block, 0, st>>>(a); break;
      case DEPI_SWIGLU: k_gemm_dec<NB, MB, WAVES, PFW, PFX, MINW, DEPI_SWIGLU><<<grid, block, 0, st>>>(a); break;
      default: k_gemm_dec<NB, MB, WAVES, PFW, PFX, MINW, DEPI_SAMPLE><<<grid, block, 0, st>>>(a); break;
    }
  }
}

// Narrow shape: one weight row tile per workgroup, K split over 8 or 16 wavefronts (QKV, O, down).
template <int MB>
static void launch_dec_narrow(const DecGemmArgs& a, int epi, hipStream_t st, int msplit = 1) {
  // 16 wavefronts split long K ranges; the chunked O projection, where a wavefront holds a whole head's operands of
  // every chunk at once, takes 12 wavefronts for two chunks (12 heads: one round of loads) and 8 for more
  if (a.k_tiles >= 48 && !(epi == DEPI_RESID && a.n_xchunks > 1)) launch_dec_t<1, MB, 16, 3, 3, 1>(a, epi, st, msplit);
  else if (epi == DEPI_RESID && MB <= 2 && a.n_xchunks == 2) launch_dec_t<1, MB, 12, 3, 3, 1>(a, DEPI_RESID, st, msplit);
  else launch_dec_t<1, MB, 8, 3, 3, 1>(a, epi, st, msplit);
}
// Wide shape: many row tiles (gate/up, LM head) or a split K (down): NB tiles per workgroup, K split over its wavefronts.
// What a CU pulls from L2 and HBM grows with the wavefronts it hosts, so the forms below put 8 to 12 on a CU where the
// registers and LDS allow (LDS: the exchange buffer is walked in NB / NBP passes).
template <int MB>
static void launch_dec_wide(const DecGemmArgs& a, int epi, hipStream_t st) {
  if constexpr (MB > 4) {
    // 65..128 rows: the activation operand is 8 KiB per k step against 1 KiB per weight row tile and every workgroup
    // reads its rows of it from L2: four row tiles x 64 rows per workgroup, the two workgroups of a tile set 8 apart in
    // launch order (one XCD: the second read of the weights hits L2), three workgroups per CU
    launch_dec_t<4, 4, 4, 2, 2, 3, 2>(a, epi, st, 1, true);
  } else {
    // every workgroup reads the whole activation operand, so a CU that hosts two workgroups takes about
    // twice as long as one that hosts one: one round of workgroups with 6 row tiles beats 1.x rounds with 4
    if (epi == DEPI_SWIGLU && a.n_tiles > 4 * 256 && a.n_tiles <= 6 * 256) launch_dec_t<6, MB, 8, 2, 2, 1, 2>(a, epi, st);
    else if (epi == DEPI_PARTIAL && a.partial_nb == 3) {
      // 8 K splits, one per XCD; three row tiles and 5 wavefronts per workgroup, rings three deep (1.5 B shape: down
      // projection 11.3 -> 10.6 us, HBM fetch of the launch 36.8 -> 29 MB; 7 wavefronts or rings two deep: 0.2 % slower)
      DecGemmArgs x = a;
      x.xcd_split = 1;
      x.row_pairs = 0;
      k_gemm_dec<3, MB, 5, 3, 3, 1, DEPI_PARTIAL, 3><<<dim3(8 * ((a.n_tiles + 2) / 3)), 5 * 64, 0, st>>>(x);
    } else if (epi == DEPI_PARTIAL && a.partial_nb == 2) launch_dec_t<2, MB, 8, 2, 2, 1>(a, epi, st);
    else if (epi == DEPI_SAMPLE) launch_dec_t<4, MB, 4, 2, 2, 3, 2>(a, epi, st);  // three workgroups per CU
    else launch_dec_t<4, MB, 4, 2, 2, 2>(a, epi, st);
  }
}

// Weight row tiles per workgroup of the wide launches (what the sampler's partial results are counted in).
int dec_wide_nb(int m_tiles) { return m_tiles > 4 ? kRows128WideTiles : 4; }
int dec_sample_groups(int n_tiles, int k_tiles, int m_tiles) {
  const int persistent = lmhead_sample_persistent_groups(n_tiles, k_tiles, m_tiles);
  if (persistent > 0) return persistent;
  return (n_tiles + dec_wide_nb(m_tiles) - 1) / dec_wide_nb(m_tiles);
}

void gemm_dec(const DecGemmArgs& a, int epi, hipStream_t st) {
  const bool wide = (epi == DEPI_SWIGLU || epi == DEPI_SAMPLE || epi == DEPI_PARTIAL);
  const int mb = a.m_tiles <= 1 ? 1 : a.m_tiles <= 2 ? 2 : a.m_tiles <= 4 ? 4 : 8;
  // 65..128 rows: the form whose wavefronts share the activation operand through LDS (rows128)
  if (mb == 8 && gemm_dec_rows128(a, epi, st)) return;
  // sampling LM head up to 64 rows: the persistent form where the model width allows it
  if (epi == DEPI_SAMPLE && mb <= 4 && lmhead_sample_persistent(a, st)) return;
  if (wide) {
    switch (mb) {
      case 1: launch_dec_wide<1>(a, epi, st); break;
      case 2: launch_dec_wide<2>(a, epi, st); break;
      case 4: launch_dec_wide<4>(a, epi, st); break;
      default: launch_dec_wide<8>(a, epi, st); break;
    }
  } else {
    switch (mb) {
      case 1: launch_dec_narrow<1>(a, epi, st); break;
      case 2: launch_dec_narrow<1>(a, epi, st, 2); break;
      // 33..64 rows: every workgroup reads the whole activation operand of its rows from L2, four times the bytes
      // of its weight tile, and with one workgroup per weight row tile only 100-odd CUs work: two workgroups per
      // row tile, 32 rows each (placed on the same XCD by the launch order, so the tile's second read hits L2)
      case 4: launch_dec_narrow<2>(a, epi, st, 2); break;
      // 65..128 rows: two weight row tiles per workgroup (the activation operand outweighs the weights) and two
      // workgroups of 64 rows per pair of tiles; behind a context-split attention the form that combines chunks
      default:
        if (epi == DEPI_RESID && a.n_xchunks > 1) launch_dec_narrow<2>(a, epi, st, (a.m_tiles + 1) / 2);
        // ... in one round on the 256 CUs: a CU that hosts two of these workgroups takes twice as long, so a launch of
        // more than 128 pairs of tiles takes three tiles per workgroup
        else if ((a.n_tiles + 1) / 2 * 2 <= 256) launch_dec_t<2, 4, 8, 2, 2, 1>(a, epi, st, 2);
        else {
          DecGemmArgs a3 = a;
          a3.row_pairs = 0;
          const dim3 grid((a.n_tiles + 2) / 3, 2), block(8 * 64);
          if (epi == DEPI_STORE) k_gemm_dec<3, 4, 8, 2, 2, 1, DEPI_STORE><<<grid, block, 0, st>>>(a3);
          else k_gemm_dec<3, 4, 8, 2, 2, 1, DEPI_RESID><<<grid, block, 0, st>>>(a3);
        }
        break;
    }
  }
}

// ---------------------------------------------------------------- split-K sum + residual epilogue
// h += sum_s P[s]; x' = fp16(h g r_old); per-tile sums of squares.  One workgroup per 16 output
// columns and 64 rows; a thread owns (row, 4 consecutive columns).  The partial sums are added in split order.
__global__ __launch_bounds__(128) void k_resid_reduce(const float* __restrict__ P, int ksplit, int Mpad, int N,
                                                      float* h, const float* __restrict__ gain,
                                                      const float* __restrict__ rs, h16_t* x, float* ss_out, int M,
                                                      int* err_flag) {
  const int nt = blockIdx.x, cg = threadIdx.x & 3;
  const int n = nt * 16 + cg * 4;
  const v4f g = *reinterpret_cast<const v4f*>(gain + n);
  {
    const int m = (threadIdx.x >> 2) + 32 * blockIdx.y;
    const bool live = m < M;
    v4f hv = v4f{0.f, 0.f, 0.f, 0.f};
    if (live) {
      v4f acc = v4f{0.f, 0.f, 0.f, 0.f};
      for (int s0 = 0; s0 < ksplit; s0 += 8) {
        v4f v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u)
          v[u] = (s0 + u < ksplit) ? *reinterpret_cast<const v4f*>(P + ((size_t)(s0 + u) * Mpad + m) * N + n)
                                   : v4f{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int u = 0; u < 8; ++u) acc = acc + v[u];
      }
      float* hp = h + (size_t)m * N + n;
      hv = *reinterpret_cast<const v4f*>(hp) + acc;
      *reinterpret_cast<v4f*>(hp) = hv;
      const float sc = rs[m];
      uint2 pk;
      pk.x = pack_h16x2_flag(hv[0] * g[0] * sc, hv[1] * g[1] * sc, err_flag);
      pk.y = pack_h16x2_flag(hv[2] * g[2] * sc, hv[3] * g[3] * sc, err_flag);
      *reinterpret_cast<uint2*>(x + act_off(m, n, Mpad)) = pk;
    }
    float ss = (hv[0] * hv[0] + hv[1] * hv[1]) + (hv[2] * hv[2] + hv[3] * hv[3]);
    ss += __shfl_xor(ss, 1, 64);
    ss += __shfl_xor(ss, 2, 64);
    if (cg == 0 && live) ss_out[(size_t)nt * Mpad + m] = ss;
  }
}
void resid_reduce(const float* P, int ksplit, int m_tiles, int N, float* h, const float* gain, const float* rs,
                  h16_t* x, float* ss_out, int M, int* err_flag, hipStream_t st) {
  k_resid_reduce<<<dim3(N / 16, (m_tiles + 1) / 2), 128, 0, st>>>(P, ksplit, m_tiles * 16, N, h, gain, rs, x, ss_out, M, err_flag);
}

// ---------------------------------------------------------------- embedding of the fed-back token
// Row m of the residual for the next step: h = E[id]; exact row norm (the workgroup holds the whole row);
// x' = fp16(h g r); per-tile sums of squares.  Runs at the end of the sampler merge, by all 256 threads of the
// row's workgroup (16 elements each: d <= 4096).
__device__ __forceinline__ void embed_row(const EmbedNextArgs& e, int m, int id, float* red) {
  float v[16];
  float ss = 0.f;
  const int d = e.d, k = threadIdx.x * 16;
  const bool live = k < d;
  if (live) {
    const v4u r0 = *reinterpret_cast<const v4u*>(e.E + (size_t)id * d + k);
    const v4u r1 = *reinterpret_cast<const v4u*>(e.E + (size_t)id * d + k + 8);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      v[2 * i] = __uint_as_float(r0[i] << 16);
      v[2 * i + 1] = __uint_as_float(r0[i] & 0xffff0000u);
      v[8 + 2 * i] = __uint_as_float(r1[i] << 16);
      v[8 + 2 * i + 1] = __uint_as_float(r1[i] & 0xffff0000u);
    }
#pragma unroll
    for (int i = 0; i < 16; ++i) ss += v[i] * v[i];
#pragma unroll
    for (int i = 0; i < 16; i += 4)
      *reinterpret_cast<v4f*>(e.h + (size_t)m * d + k + i) = v4f{v[i], v[i + 1], v[i + 2], v[i + 3]};
    e.ss_out[(size_t)(k >> 4) * e.Mpad + m] = ss;
  }
  const float tot = block_sum(ss, red);
  const float r = 1.0f / sqrtf(tot / (float)d + e.eps);
  if (live) {
#pragma unroll
    for (int half = 0; half < 2; ++half) {
      v4u pk;
#pragma unroll
      for (int i = 0; i < 4; ++i)
        pk[i] = pack_h16x2_flag(v[half * 8 + 2 * i] * e.gain[k + half * 8 + 2 * i] * r,
                                v[half * 8 + 2 * i + 1] * e.gain[k + half * 8 + 2 * i + 1] * r, e.err_flag);
      *reinterpret_cast<v4u*>(e.x + act_off(m, k + half * 8, e.Mpad)) = pk;
    }
  }
}

// ---------------------------------------------------------------- sampler merge (per row)
__global__ __launch_bounds__(256) void k_sample_merge(const DecSamplePartial* part, int n_groups, int M,
                                                      const SampleCtl* ctlp, int* d_step, int* cur_ids,
                                                      EmbedNextArgs emb) {
  __shared__ float red[16];
  __shared__ int s_tok;
  __shared__ Lse s_lse[4];
  __shared__ float s_y[4], s_z[4];
  __shared__ int s_i[4];
  const int b = blockIdx.x;
  Lse lse = lse_empty();
  float by = -INFINITY, bz = 0.f;
  int bi = 0x7fffffff;
  // batches of independent loads (a partial per iteration would serialise one memory round trip each)
  constexpr int kBatch = 5;
  for (int g0 = threadIdx.x; g0 < n_groups; g0 += kBatch * blockDim.x) {
    DecSamplePartial p[kBatch];
#pragma unroll
    for (int u = 0; u < kBatch; ++u) {
      const int g = g0 + u * blockDim.x;
      p[u] = part[(size_t)b * n_groups + min(g, n_groups - 1)];
    }
#pragma unroll
    for (int u = 0; u < kBatch; ++u) {
      if (g0 + u * (int)blockDim.x >= n_groups) break;
      lse = lse_merge(lse, Lse{p[u].m, p[u].s});
      if (p[u].y > by || (p[u].y == by && p[u].idx < bi)) { by = p[u].y; bi = p[u].idx; bz = p[u].zt; }
    }
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    const Lse ol = {__shfl_xor(lse.m, o, 64), __shfl_xor(lse.s, o, 64)};
    const float oy = __shfl_xor(by, o, 64), oz = __shfl_xor(bz, o, 64);
    const int oi = __shfl_xor(bi, o, 64);
    lse = lse_merge(lse, ol);
    if (oy > by || (oy == by && oi < bi)) { by = oy; bi = oi; bz = oz; }
  }
  const int lane = threadIdx.x & 63, wid = threadIdx.x >> 6;
  if (lane == 0) { s_lse[wid] = lse; s_y[wid] = by; s_z[wid] = bz; s_i[wid] = bi; }
  __syncthreads();
  if (threadIdx.x == 0) {
    for (int w = 1; w < 4; ++w) {
      lse = lse_merge(lse, s_lse[w]);
      if (s_y[w] > by || (s_y[w] == by && s_i[w] < bi)) { by = s_y[w]; bi = s_i[w]; bz = s_z[w]; }
    }
    const SampleCtl ctl = *ctlp;
    const int step = *d_step;
    const int row = ctl.slot_row ? ctl.slot_row[b] : b;   // b is the slot
    int tok = bi;
    float lp = bz - (lse.m + logf(lse.s));
    if (row < 0) {
      tok = 0;  // nobody in this slot: nothing is reported, the slot keeps computing on token 0
    } else {
      if ((unsigned)tok >= (unsigned)emb.vocab) {  // no logit of the row compared greater than -inf: every one is NaN
        tok = 0;
        atomicOr(emb.err_flag, kErrFp16Range);
      }
      if (ctl.row_step0) {
        // a batch that takes in new prompts as it runs (its caller passes stop flags and has filled the outputs
        // with what a finished row reports): this row is at its own step, and the batch may run on after its end
        const int own = step - ctl.row_step0[b];
        if (ctl.done[row] || own >= ctl.max_new) {
          tok = ctl.stop_id;
        } else {
          if (tok == ctl.stop_id) {
            ctl.done[row] = 1;
            ctl.out_lens[row] = own + 1;
          } else if (own == ctl.max_new - 1) {
            ctl.done[row] = 1;
          }
          ctl.out_ids[(size_t)row * ctl.max_new + own] = tok;
          ctl.out_logprobs[(size_t)row * ctl.max_new + own] = lp;
        }
        cur_ids[row] = tok;
      } else {
        if (ctl.done) {
          if (ctl.done[row]) {
            tok = ctl.stop_id;
            lp = 0.f;
          } else if (tok == ctl.stop_id) {
            ctl.done[row] = 1;
            ctl.out_lens[row] = step + 1;
          }
        }
        cur_ids[row] = tok;
        ctl.out_ids[(size_t)row * ctl.max_new + step] = tok;
        ctl.out_logprobs[(size_t)row * ctl.max_new + step] = lp;
      }
    }
    s_tok = tok;
    // the last row to get here advances the step counter: by then every row has read it (d_step[1] counts
    // arrivals and is left at zero for the next launch)
    __atomic_signal_fence(__ATOMIC_SEQ_CST);
    if (atomicAdd(d_step + 1, 1) == M - 1) {
      d_step[1] = 0;
      d_step[0] = step + 1;
    }
  }
  __syncthreads();
  embed_row(emb, b, s_tok, red);  // the row's operand of the next step's first GEMM
}
void sample_merge(const float* part, int n_groups, int M, const SampleCtl* ctl, int* d_step, int* cur_ids,
                  const EmbedNextArgs& emb, hipStream_t st) {
  k_sample_merge<<<M, 256, 0, st>>>(reinterpret_cast<const DecSamplePartial*>(part), n_groups, M, ctl, d_step,
                                    cur_ids, emb);
}


// ---------------------------------------------------------------- decode attention, fused
// One workgroup per (sequence, kv head, context chunk).  Prologue: rotate the G query heads of the
// row (fp32 qkv -> fp16, through LDS); the workgroup whose chunk holds the current position also
// rotates the new key, converts the new value and stores both into their page before attending.
// Epilogue: the wavefronts' partial (max, sum, O) are merged through LDS and the workgroup writes
// the output over ITS chunk of the context, normalised by the chunk's own sum, together with the
// chunk's (max, sum) per head.  Chunks are combined by the consumer (the O projection weights the
// per-chunk products by their softmax shares): no cross-workgroup hand-over inside this kernel.
// (A merge by the last workgroup to arrive needs device-scope fences around an atomic counter,
// which cost more than the split saved.)
template <int HD>
__device__ __forceinline__ h16_t* dec_page(const KvPool& pool, int layer, int which, int page, int g) {
  return (h16_t*)pool.base +
         ((((size_t)layer * 2 + which) * pool.n_pages + page) * pool.n_kv_heads + g) * (size_t)(kPageTokens * HD);
}

constexpr int AW = 8;        // wavefronts per workgroup
constexpr int AGMAX = 8;     // query heads per kv head at most
constexpr int ATAB = 512;    // page-table entries of one chunk kept in LDS

template <int HD>
struct KvFrags {
  v8h k[2][HD / 32];
  v4u v[HD / 16];
};
template <int HD>
__device__ __forceinline__ KvFrags<HD> load_kv(const h16_t* K0, const h16_t* K1, const h16_t* V0, const h16_t* V1,
                                               int lane) {
  KvFrags<HD> f;
#pragma unroll
  for (int kb = 0; kb < HD / 32; ++kb) {
    f.k[0][kb] = load_frag(K0 + kb * 512, lane);
    f.k[1][kb] = load_frag(K1 + kb * 512, lane);
  }
  const int voff = (lane & 15) * kPageTokens + 4 * (lane >> 4);
#pragma unroll
  for (int cb = 0; cb < HD / 16; ++cb) {
    const uint2 x = *reinterpret_cast<const uint2*>(V0 + cb * 256 + voff);
    const uint2 y = *reinterpret_cast<const uint2*>(V1 + cb * 256 + voff);
    f.v[cb] = v4u{x.x, x.y, y.x, y.y};
  }
  return f;
}

// One step (two pages, 32 tokens from tok0) of a single block of query columns on loaded fragments.
// The softmax state is kept in base-2 units: scale2 = log2(e) / sqrt(head_dim), st.m = running maximum of
// scale2 * score, weights = 2^(scale2 * score - m) (one v_exp_f32 each).  MASK = false: every token of the step
// is visible to the query (tok0 + 31 <= position), so nothing is compared; the unused columns (zero queries)
// then carry finite garbage that nobody reads.
template <int HD, bool MASK>
__device__ __forceinline__ void attn_step1(const KvFrags<HD>& f, int tok0, const v8h (&qf)[HD / 32], int qpos,
                                           float scale2, AttnState<HD / 16>& st, int lane) {
  const int lg = lane >> 4;
  v4f s0 = v4f{0.f, 0.f, 0.f, 0.f}, s1 = s0;
#pragma unroll
  for (int kb = 0; kb < HD / 32; ++kb) {
    s0 = mfma16(f.k[0][kb], qf[kb], s0);
    s1 = mfma16(f.k[1][kb], qf[kb], s1);
  }
  float sv[8];
  float tmax = -INFINITY;
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    const int t0 = tok0 + 4 * lg + r, t1 = t0 + 16;
    sv[r] = (!MASK || t0 <= qpos) ? s0[r] * scale2 : -INFINITY;
    sv[4 + r] = (!MASK || t1 <= qpos) ? s1[r] * scale2 : -INFINITY;
    tmax = fmaxf(tmax, fmaxf(sv[r], sv[4 + r]));
  }
  tmax = fmaxf(tmax, __shfl_xor(tmax, 16, 64));
  tmax = fmaxf(tmax, __shfl_xor(tmax, 32, 64));
  const float m_new = fmaxf(st.m, tmax);
  const float m_safe = (MASK && m_new == -INFINITY) ? 0.f : m_new;
  const float corr = __builtin_amdgcn_exp2f(st.m - m_safe);
  float p[8], psum = 0.f;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    p[e] = __builtin_amdgcn_exp2f(sv[e] - m_safe);
    psum += p[e];
  }
  st.l = st.l * corr + psum;
  st.m = m_new;
  v4u pk;
  pk[0] = pack_h16x2_inrange(p[0], p[1]);  // weights lie in [0, 1]
  pk[1] = pack_h16x2_inrange(p[2], p[3]);
  pk[2] = pack_h16x2_inrange(p[4], p[5]);
  pk[3] = pack_h16x2_inrange(p[6], p[7]);
  const v8h pf = __builtin_bit_cast(v8h, pk);
  if (__any(corr != 1.0f)) {  // the running maximum of some column moved: rescale what has been summed
#pragma unroll
    for (int cb = 0; cb < HD / 16; ++cb) st.o[cb] = st.o[cb] * corr;
  }
#pragma unroll
  for (int cb = 0; cb < HD / 16; ++cb) st.o[cb] = mfma16(__builtin_bit_cast(v8h, f.v[cb]), pf, st.o[cb]);
}

template <int DHD>
__global__ __launch_bounds__(AW * 64) void k_attn_dec(AttnDecArgs a) {
  constexpr int HALF = DHD / 2;
  __shared__ __attribute__((aligned(16))) h16_t q_s[16][DHD];
  __shared__ float s_o[AW][AGMAX][DHD + 1];
  __shared__ float s_m[AW][16], s_l[AW][16];
  __shared__ int s_table[ATAB];
  // Workgroups are handed to the 8 XCDs round-robin in launch order, and each XCD has its own L2.
  // The `share` sequences that sample from one prompt read the same prompt pages, so their
  // workgroups (for one kv head) are given launch indices that are congruent modulo 8: the pages
  // then come from HBM once per XCD instead of once per sequence.
  int b = blockIdx.x, g = blockIdx.y;
  {
    const int B = gridDim.x, total = B * gridDim.y, S = a.share;
    if (S > 1 && total % (8 * S) == 0) {
      const int L = b + B * g, xcd = L & 7, slot = L >> 3;
      const int item = ((slot / S) * 8 + xcd) * S + slot % S;
      g = item / B;
      b = item - g * B;
    }
  }
  const int chunk = blockIdx.z;
  const int Hq = a.Hq, Hkv = a.Hkv, G = Hq / Hkv;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int col = lane & 15, lg = lane >> 4;
  const KvPool& pool = a.pool;
  const int* table = pool.page_table + (size_t)b * pool.max_pages;
  const int pos0 = a.row_pos ? a.row_pos[b] : a.pos_base;
  const int step0 = a.row_step0 ? a.row_step0[b] : 0;
  // Pages [p_lo, p_end) of the sequence are this workgroup's.  Either equal chunks, or (two chunks, split_at_prompt)
  // the whole pages of the prompt and the rest: a boundary that depends on the sequence alone, so that a sequence
  // gets the same arithmetic whatever else is in the batch and however many tokens the call may generate (given
  // that the call splits at all: contexts of more than 8 pages).
  int p_lo = chunk * a.chunk_pages, p_end = p_lo + a.chunk_pages;
  if (a.split_at_prompt) {
    const int nb = ((pos0 + 1) / kPageTokens) & ~1;  // even: the steps below take pages in pairs
    p_lo = chunk ? nb : 0;
    p_end = chunk ? pool.max_pages : nb;
  }
  // ---- loads that do not depend on the position: step counter, this chunk's page ids, the raw
  // q/k/v row, and (speculatively) the first pair of pages of this wavefront
  const int step = *a.d_step;
  for (int i = tid; i < p_end - p_lo; i += AW * 64) s_table[i] = table[min(p_lo + i, pool.max_pages - 1)];
  const float* row = a.qkv + (size_t)b * (Hq + 2 * Hkv) * DHD;
  float qraw[2] = {0.f, 0.f};
  const int qj = tid >> 6, qi = tid & 63;  // wavefront j rotates head j (AW >= G)
  if (qj < G && qi < HALF) {
    qraw[0] = row[(size_t)(g * G + qj) * DHD + qi];
    qraw[1] = row[(size_t)(g * G + qj) * DHD + qi + HALF];
  }
  const int pg0 = p_lo + 2 * wave;
  KvFrags<DHD> cur;
  {
    const int i0 = table[min(pg0, pool.max_pages - 1)], i1 = table[min(pg0 + 1, pool.max_pages - 1)];
    cur = load_kv<DHD>(dec_page<DHD>(pool, a.layer, 0, i0, g), dec_page<DHD>(pool, a.layer, 0, i1, g),
                  dec_page<DHD>(pool, a.layer, 1, i0, g), dec_page<DHD>(pool, a.layer, 1, i1, g), lane);
  }
  // ---- position-dependent part
  const int pos = pos0 + (a.row_step0 ? min(step - step0, a.max_step) : step);
  const int n_ctx_pages = pos / kPageTokens + 1;
  // a negative position base marks a slot that holds no sequence (rows packed into fewer slots): nothing to attend
  const int p_hi = pos0 < 0 ? p_lo : min(n_ctx_pages, p_end);
  if (p_lo >= p_hi) {
    // this chunk lies beyond the context: it contributes nothing, which its consumer learns from a zero sum;
    // the operand slice is cleared so that stale bits (possibly NaN patterns) never meet a zero weight
    if (tid < G * (DHD / 8)) {
      const int c = tid / (DHD / 8), d0 = (tid % (DHD / 8)) * 8;
      *reinterpret_cast<v4u*>(a.o + chunk * a.o_chunk_stride + act_off(b, (g * G + c) * DHD + d0, a.m_tiles * 16)) =
          v4u{0u, 0u, 0u, 0u};
      if (d0 == 0) {
        float* ml = a.ml + (((size_t)b * Hq + g * G + c) * a.n_chunks + chunk) * 2;
        ml[0] = -INFINITY;
        ml[1] = 0.f;
      }
    }
    return;
  }
  const float* cs = a.cos + (size_t)pos * (DHD / 2);
  const float* sn = a.sin + (size_t)pos * (DHD / 2);
  if (qj < G && qi < HALF) {
    const float c = cs[qi], s = sn[qi];
    q_s[qj][qi] = f32_to_h16_flag(qraw[0] * c - qraw[1] * s, a.err_flag);
    q_s[qj][qi + HALF] = f32_to_h16_flag(qraw[1] * c + qraw[0] * s, a.err_flag);
  }
  // the owner of the current position appends K and V to the cache (last wavefront: it is idle above when G < AW)
  const int cur_page = pos / kPageTokens;
  const bool owner_wg = cur_page >= p_lo && cur_page < p_hi;
  if (owner_wg && wave == AW - 1 && lane < HALF) {
    const int page = table[cur_page], slot = pos % kPageTokens;
    h16_t* kp = dec_page<DHD>(pool, a.layer, 0, page, g);
    h16_t* vp = dec_page<DHD>(pool, a.layer, 1, page, g);
    const int i = lane;
    const float x0 = row[(size_t)(Hq + g) * DHD + i], x1 = row[(size_t)(Hq + g) * DHD + i + HALF];
    const float v0 = row[(size_t)(Hq + Hkv + g) * DHD + i], v1 = row[(size_t)(Hq + Hkv + g) * DHD + i + HALF];
    const float c = cs[i], s = sn[i];
    const int c0 = i, c1 = i + HALF;
    kp[(c0 >> 3) * 128 + slot * 8 + (c0 & 7)] = f32_to_h16_flag(x0 * c - x1 * s, a.err_flag);
    kp[(c1 >> 3) * 128 + slot * 8 + (c1 & 7)] = f32_to_h16_flag(x1 * c + x0 * s, a.err_flag);
    vp[c0 * kPageTokens + slot] = f32_to_h16_flag(v0, a.err_flag);
    vp[c1 * kPageTokens + slot] = f32_to_h16_flag(v1, a.err_flag);
  }
  __syncthreads();  // q_s, s_table complete; this workgroup's K/V stores are visible to its own loads

  v8h qf[DHD / 32];
#pragma unroll
  for (int kb = 0; kb < DHD / 32; ++kb) {
    v4u raw = {0u, 0u, 0u, 0u};
    if (col < G) raw = *reinterpret_cast<const v4u*>(&q_s[col][kb * 32 + 8 * lg]);
    qf[kb] = __builtin_bit_cast(v8h, raw);
  }
  const int qpos = (col < G) ? pos : -1;
  AttnState<DHD / 16> st;
  attn_init(st);
  const float scale2 = (DHD == 128 ? 0.08838834764831845f : 0.125f) * 1.4426950408889634f;  // log2(e) / sqrt(head_dim)
  auto page_id = [&](int pg) { return s_table[min(pg, n_ctx_pages - 1) - p_lo]; };
  // the speculative load may have raced with the append above: redo it if it covers the current page
  if (owner_wg && (cur_page == pg0 || cur_page == pg0 + 1) && pg0 < p_hi) {
    const int i0 = page_id(pg0), i1 = page_id(pg0 + 1);
    cur = load_kv<DHD>(dec_page<DHD>(pool, a.layer, 0, i0, g), dec_page<DHD>(pool, a.layer, 0, i1, g),
                  dec_page<DHD>(pool, a.layer, 1, i0, g), dec_page<DHD>(pool, a.layer, 1, i1, g), lane);
  }
  // Stage j of this wavefront = pages pg0 + 2 AW j, +1.  Two register sets alternate: while one is multiplied the
  // loads of the next stage fill the other.  The loop body has no conditional load (a load behind a branch makes
  // the compiler wait for every outstanding load at the join, i.e. for the prefetch it has just issued) and no
  // copies between the sets; the last one or two stages are taken outside the loop.
  const h16_t* kbase = dec_page<DHD>(pool, a.layer, 0, 0, g);
  const h16_t* vbase = dec_page<DHD>(pool, a.layer, 1, 0, g);
  const size_t pstride = (size_t)pool.n_kv_heads * (kPageTokens * DHD);
  auto load_stage = [&](int j) {
    const int pg = pg0 + 2 * AW * j;
    const size_t o0 = (size_t)page_id(pg) * pstride, o1 = (size_t)page_id(pg + 1) * pstride;
    return load_kv<DHD>(kbase + o0, kbase + o1, vbase + o0, vbase + o1, lane);
  };
  // a stage that is followed by another stage of this wavefront lies wholly before the current position
  auto attend_full = [&](const KvFrags<DHD>& f, int j) {
    attn_step1<DHD, false>(f, (pg0 + 2 * AW * j) * kPageTokens, qf, qpos, scale2, st, lane);
  };
  auto attend_last = [&](const KvFrags<DHD>& f, int j) {
    attn_step1<DHD, true>(f, (pg0 + 2 * AW * j) * kPageTokens, qf, qpos, scale2, st, lane);
  };
  const int n_st = pg0 < p_hi ? (p_hi - pg0 + 2 * AW - 1) / (2 * AW) : 0;
  KvFrags<DHD> alt;
  int j = 0;
  for (; j + 2 < n_st; j += 2) {
    alt = load_stage(j + 1);
    attend_full(cur, j);
    cur = load_stage(j + 2);
    attend_full(alt, j + 1);
  }
  if (j + 1 < n_st) {
    alt = load_stage(j + 1);
    attend_full(cur, j);
    attend_last(alt, j + 1);
  } else if (j < n_st) {
    attend_last(cur, j);
  }
  float l = st.l;
  l += __shfl_xor(l, 16, 64);
  l += __shfl_xor(l, 32, 64);
  if (col < AGMAX) {
#pragma unroll
    for (int cb = 0; cb < DHD / 16; ++cb)
#pragma unroll
      for (int r = 0; r < 4; ++r) s_o[wave][col][cb * 16 + 4 * lg + r] = st.o[cb][r];
  }
  if (lg == 0) {
    s_m[wave][col] = st.m;
    s_l[wave][col] = l;
  }
  __syncthreads();
  // ---- merge the wavefronts: thread t < 16 G owns (column c, 8 consecutive dims)
  const bool owner = tid < G * (DHD / 8);
  const int c = tid / (DHD / 8), d0 = (tid % (DHD / 8)) * 8;
  float mm = -INFINITY, ll = 0.f, acc[8] = {};
  if (owner) {
#pragma unroll
    for (int w = 0; w < AW; ++w) mm = fmaxf(mm, s_m[w][c]);
#pragma unroll
    for (int w = 0; w < AW; ++w) {
      const float f = __builtin_amdgcn_exp2f(s_m[w][c] - mm);
      ll += f * s_l[w][c];
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[e] += f * s_o[w][c][d0 + e];
    }
  }
  const int Mpad = a.m_tiles * 16;
  if (owner) {
    const float inv = 1.0f / ll;  // every page of an active chunk holds at least one visible key
    v4u pk;
#pragma unroll
    for (int e = 0; e < 4; ++e) pk[e] = pack_h16x2_flag(acc[2 * e] * inv, acc[2 * e + 1] * inv, a.err_flag);
    *reinterpret_cast<v4u*>(a.o + chunk * a.o_chunk_stride + act_off(b, (g * G + c) * DHD + d0, Mpad)) = pk;
    if (a.n_chunks > 1 && d0 == 0) {
      float* ml = a.ml + (((size_t)b * Hq + g * G + c) * a.n_chunks + chunk) * 2;
      ml[0] = mm * 0.6931471805599453f;  // the consumer works in natural units
      ml[1] = ll;
    }
  }
}

// ---------------------------------------------------------------- packing live rows into the leading slots
__global__ void k_count_live(const int* done, int B, int* live) {
  __shared__ float red[16];
  float n = 0.f;
  for (int b = threadIdx.x; b < B; b += blockDim.x) n += done[b] ? 0.f : 1.f;
  const float tot = block_sum(n, red);
  if (threadIdx.x == 0) live[0] = (int)tot;
}
void count_live(const int* done, int B, int* live, hipStream_t st) { k_count_live<<<1, 256, 0, st>>>(done, B, live); }

// One workgroup; B is small (the rows of one group).  Thread 0 walks the flags in row order (a stable packing),
// then all threads gather the page-table rows.
__global__ __launch_bounds__(256) void k_compact_rows(const int* done, int B, int slots, int* slot_row,
                                                      const int* page_table, const int* row_pos, int max_pages,
                                                      int* page_table_c, int* row_pos_c) {
  __shared__ int s_row[256];
  if (threadIdx.x == 0) {
    int n = 0;
    for (int b = 0; b < B && n < slots; ++b)
      if (!done[b]) s_row[n++] = b;
    for (; n < slots; ++n) s_row[n] = -1;
  }
  __syncthreads();
  for (int s = threadIdx.x; s < slots; s += blockDim.x) {
    slot_row[s] = s_row[s];
    row_pos_c[s] = s_row[s] >= 0 ? row_pos[s_row[s]] : -1;
  }
  for (int i = threadIdx.x; i < slots * max_pages; i += blockDim.x) {
    const int s = i / max_pages, j = i - s * max_pages;
    page_table_c[i] = s_row[s] >= 0 ? page_table[(size_t)s_row[s] * max_pages + j] : 0;
  }
}
void compact_rows(const int* done, int B, int slots, int* slot_row, const int* page_table, const int* row_pos,
                  int max_pages, int* page_table_c, int* row_pos_c, hipStream_t st) {
  k_compact_rows<<<1, 256, 0, st>>>(done, B, slots, slot_row, page_table, row_pos, max_pages, page_table_c, row_pos_c);
}

__global__ __launch_bounds__(256) void k_embed_slots(const int* slot_row, const int* cur_ids, EmbedNextArgs emb) {
  __shared__ float red[16];
  const int s = blockIdx.x, row = slot_row[s];
  int tok = row >= 0 ? cur_ids[row] : 0;
  tok = min(max(tok, 0), emb.vocab - 1);
  embed_row(emb, s, tok, red);
}
void embed_slots(const int* slot_row, const int* cur_ids, int slots, const EmbedNextArgs& emb, hipStream_t st) {
  k_embed_slots<<<slots, 256, 0, st>>>(slot_row, cur_ids, emb);
}

// ---------------------------------------------------------------- a batch that takes in new prompts as it runs
__global__ void k_admit_init(int* slot_row, int* row_step0, int B, int Mpad) {
  const int s = blockIdx.x * blockDim.x + threadIdx.x;
  if (s < Mpad) {
    slot_row[s] = s < B ? s : -1;
    row_step0[s] = 0;
  }
}
void admit_init(int* slot_row, int* row_step0, int B, int Mpad, hipStream_t st) {
  k_admit_init<<<(Mpad + 255) / 256, 256, 0, st>>>(slot_row, row_step0, B, Mpad);
}

__global__ __launch_bounds__(256) void k_admit_prompt(AdmitArgs a) {
  const int j = blockIdx.x, slot = a.slots[j];
  const int raw = *a.len, len = min(max(raw, 1), a.Lmax);
  if (threadIdx.x == 0) {
    if (raw != len && j == 0) atomicOr(a.err_flag, 4);
    a.row_pos[slot] = len - 1;
    a.slot_row[slot] = a.prompt_index * a.n_samples + j;
    a.row_step0[slot] = a.step0;
  }
  // whole prompt pages: the region's, shared by the prompt's sequences; the rest: the slot's own
  const int n_full = len / kPageTokens;
  for (int i = threadIdx.x; i < a.max_pages; i += blockDim.x) {
    const int page = (i < n_full) ? a.region * a.nf_max + i : a.shared_total + slot * a.max_pages + i;
    a.page_table[(size_t)slot * a.max_pages + i] = page;
    if (j == 0) a.prefill_row[i] = page;
  }
  if (j == 0)
    for (int i = threadIdx.x; i < a.Lmax; i += blockDim.x) a.ids_out[i] = (i < len) ? a.prompt[i] : 0;
}
void admit_prompt(const AdmitArgs& a, hipStream_t st) { k_admit_prompt<<<a.n_samples, 256, 0, st>>>(a); }

// the prompt's last, partly filled page (written into the first slot's own page by the prefill) goes to the other slots
__global__ void k_fork_tail_slots(AdmitArgs a, KvPool pool, int words_per_page) {
  const int j = blockIdx.x + 1;
  const int len = min(max(*a.len, 1), a.Lmax);
  if (len % kPageTokens == 0) return;
  const int page_idx = len / kPageTokens;
  const int lw = blockIdx.y;  // layer * 2 + which
  const int src = a.shared_total + a.slots[0] * a.max_pages + page_idx;
  const int dst = a.shared_total + a.slots[j] * a.max_pages + page_idx;
  const uint32_t* s = (const uint32_t*)pool.base + ((size_t)lw * pool.n_pages + src) * words_per_page;
  uint32_t* d = (uint32_t*)pool.base + ((size_t)lw * pool.n_pages + dst) * words_per_page;
  for (int i = threadIdx.x; i < words_per_page; i += blockDim.x) d[i] = s[i];
}
void fork_tail_slots(const AdmitArgs& a, KvPool pool, int n_layers, hipStream_t st) {
  if (a.n_samples < 2) return;
  const int words = pool.n_kv_heads * kPageTokens * pool.head_dim * 2 / 4;
  k_fork_tail_slots<<<dim3(a.n_samples - 1, n_layers * 2), 256, 0, st>>>(a, pool, words);
}

// live[s] = 1 when the sequence in slot s still runs (s < n_slots <= 256)
__global__ __launch_bounds__(256) void k_slot_live(const int* done, const int* slot_row, int n_slots, int* live) {
  const int s = threadIdx.x;
  if (s >= n_slots) return;
  const int row = slot_row[s];
  live[s] = (row >= 0 && !done[row]) ? 1 : 0;
}
void slot_live(const int* done, const int* slot_row, int n_slots, int* live, hipStream_t st) {
  k_slot_live<<<1, 256, 0, st>>>(done, slot_row, n_slots, live);
}

// The sequences that still run, in slot order, move to the leading `slots` slots of a second set of tables
// (one workgroup; B <= 256).
__global__ __launch_bounds__(256) void k_compact_slots(const int* done, int B, int slots, const int* slot_row,
                                                       const int* page_table, const int* row_pos, const int* row_step0,
                                                       int max_pages, int* slot_row_c, int* page_table_c, int* row_pos_c,
                                                       int* row_step0_c) {
  __shared__ int s_src[256];
  if (threadIdx.x == 0) {
    int n = 0;
    for (int s = 0; s < B && n < slots; ++s) {
      const int row = slot_row[s];
      if (row >= 0 && !done[row]) s_src[n++] = s;
    }
    for (; n < slots; ++n) s_src[n] = -1;
  }
  __syncthreads();
  for (int s = threadIdx.x; s < slots; s += blockDim.x) {
    const int src = s_src[s];
    slot_row_c[s] = src >= 0 ? slot_row[src] : -1;
    row_pos_c[s] = src >= 0 ? row_pos[src] : -1;
    row_step0_c[s] = src >= 0 ? row_step0[src] : 0;
  }
  for (int i = threadIdx.x; i < slots * max_pages; i += blockDim.x) {
    const int s = i / max_pages, j = i - s * max_pages;
    page_table_c[i] = s_src[s] >= 0 ? page_table[(size_t)s_src[s] * max_pages + j] : 0;
  }
}
void compact_slots(const int* done, int B, int slots, const int* slot_row, const int* page_table, const int* row_pos,
                   const int* row_step0, int max_pages, int* slot_row_c, int* page_table_c, int* row_pos_c,
                   int* row_step0_c, hipStream_t st) {
  k_compact_slots<<<1, 256, 0, st>>>(done, B, slots, slot_row, page_table, row_pos, row_step0, max_pages, slot_row_c,
                                     page_table_c, row_pos_c, row_step0_c);
}

void attention_dec(const AttnDecArgs& a, int B, hipStream_t st) {
  const dim3 grid(B, a.Hkv, a.n_chunks);
  if (a.pool.head_dim == 64) k_attn_dec<64><<<grid, AW * 64, 0, st>>>(a);
  else k_attn_dec<128><<<grid, AW * 64, 0, st>>>(a);
}

}  // namespace bf16
}  // namespace mtmc
