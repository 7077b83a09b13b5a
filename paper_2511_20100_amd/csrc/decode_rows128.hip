// Decode GEMMs for 65..128 rows: the wide launches (gate/up, down projection, sampling LM head).
//
// The general decode GEMM (decode_bf16.hip) splits K over the wavefronts of a workgroup, so every wavefront
// reads its own part of the activation operand and a workgroup reads all of it.  Up to 64 rows that operand is
// small beside the weights a workgroup streams; at 128 rows it is 8 KiB per k tile against 1 KiB per weight row
// tile, every workgroup pulls more activation bytes from L2 than weight bytes from HBM, and the launch is bound
// by L2-to-CU traffic (272 MB of gate/up weights took 96 us where 32 rows take 62).
//
// Here the wavefronts of a workgroup own different weight row tiles and ALL walk the same k range together: the
// activation tiles of a k step (8 token tiles x 1 KiB) are copied into LDS once per workgroup (LDS-direct 16-byte
// loads, a ring of stages filled some steps ahead) and every wavefront reads them from there, while its own
// weight tiles stream from HBM straight into a register ring.  A wavefront ends with complete sums for its tiles
// and all rows: the epilogues run from registers, without the cross-wavefront sum of the general form.
// Same arithmetic per output element (one accumulator over K in ascending order, per K split).
#include "bf16_kernels.h"
#include "device_utils.h"
#include "frag.h"

namespace mtmc {
namespace bf16 {

namespace {

typedef __attribute__((address_space(3))) void* lds_ptr_t;
typedef const __attribute__((address_space(1))) void* glb_ptr_t;

constexpr int kMB = 8;                              // token tiles of 16 rows
constexpr int kKT = 2;                              // k tiles per step (one LDS stage)
constexpr int kNSX = 4;                             // LDS stages
constexpr int kD = kNSX - 1;                        // steps the copies and the weight loads run ahead
static_assert(kD == 3, "the tail of the k loop names the three register sets");
constexpr int kXStageBytes = kKT * kMB * 1024;      // 16 KiB
constexpr int kXRingBytes = kNSX * kXStageBytes;    // 64 KiB: two workgroups per CU

template <int N>
__device__ __forceinline__ void wait_vm() {
  static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
  __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | (7 << 4) | (15 << 8));
}

__device__ __forceinline__ float silu_r(float g) { return g / (1.0f + expf(-g)); }

// NBW weight row tiles per wavefront, WAVES wavefronts per workgroup.
template <int NBW, int WAVES, int EPI, int MINB>
__global__ __launch_bounds__(WAVES * 64, MINB) void k_gemm_rows128(DecGemmArgs a) {
  static_assert(EPI == DEC_SWIGLU || EPI == DEC_PARTIAL || EPI == DEC_SAMPLE, "the wide launches only");
  static_assert(EPI != DEC_SWIGLU || NBW % 2 == 0, "gate and up tiles come in pairs");
  constexpr int NT = WAVES * 64;
  // 1 KiB copies per wavefront and step: every wavefront issues the same number (the waits count operations), so
  // when WAVES does not divide the stage's 16 blocks the last wavefronts copy the last block more than once
  constexpr int XC = (kKT * kMB + WAVES - 1) / WAVES;
  constexpr int OPS = XC + kKT * NBW;               // vector-memory operations a wavefront issues per step
  static_assert((kD - 1) * OPS < 64, "the wait counts the operations of kD - 1 steps");
  extern __shared__ __attribute__((aligned(1024))) uint8_t lds[];
  __shared__ float s_scale[128];
  __shared__ float s_part[2][NT];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int grp = blockIdx.x;
  const int nt0 = (grp * WAVES + wave) * NBW;       // this wavefront's first weight row tile
  const int Mpad = a.m_tiles * 16;                  // 80 .. 128

  // ---- row scales (consumers: r_new / r_old; producers: r of the state they update): thread t sums the tiles
  // part, part + P, ... of row t % Mpad, the P partial sums are then added in index order.  A split-K launch needs
  // them only in the kernel that finishes the sum: its first workgroup leaves them in rs_out.
  constexpr bool kProducer = EPI == DEC_PARTIAL;
  const bool do_rs = EPI != DEC_PARTIAL || (blockIdx.x == 0 && blockIdx.y == 0);
  const int P = NT / Mpad, m_rs = tid % Mpad, part = tid / Mpad;
  const bool two = !kProducer && a.ss_cur && a.ss_old != a.ss_cur;
  float sa = 0.f, sb = 0.f;
  if (do_rs && a.ss_cur && part < P) {
    constexpr int BT = 8;
    for (int t0 = part; t0 < a.ss_tiles; t0 += BT * P) {  // batches of independent loads, added in index order
      float fa[BT], fb[BT];
#pragma unroll
      for (int u = 0; u < BT; ++u) {
        const int t = t0 + u * P;
        fa[u] = t < a.ss_tiles ? a.ss_cur[(size_t)t * Mpad + m_rs] : 0.f;
        fb[u] = (two && t < a.ss_tiles) ? a.ss_old[(size_t)t * Mpad + m_rs] : 0.f;
      }
#pragma unroll
      for (int u = 0; u < BT; ++u) {
        sa += fa[u];
        sb += fb[u];
      }
    }
  }
  if (do_rs) {
    if (part < P) {
      s_part[0][tid] = sa;
      s_part[1][tid] = sb;
    }
    __syncthreads();
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
      if (EPI == DEC_PARTIAL) a.rs_out[tid] = sc;
    }
    __syncthreads();
  }

  // ---- k range of this workgroup (split-K: grid.y), in steps of kKT tiles
  int kbeg = 0, kend = a.k_tiles;
  if (EPI == DEC_PARTIAL) {
    const int per_split = (a.k_tiles + gridDim.y - 1) / gridDim.y;
    kbeg = blockIdx.y * per_split;
    kend = min(a.k_tiles, kbeg + per_split);
  }
  const int n_steps = (max(kend - kbeg, 0) + kKT - 1) / kKT;
  v4f acc[NBW][kMB];
#pragma unroll
  for (int nb = 0; nb < NBW; ++nb)
#pragma unroll
    for (int mb = 0; mb < kMB; ++mb) acc[nb][mb] = v4f{0.f, 0.f, 0.f, 0.f};

  if (n_steps > 0) {
    const int klast = kend - 1;
    // activation block (k tile kk, token tile mt): 1 KiB at Xt + (kk * m_tiles + mt) * 512 halves
    const h16_t* xsrc = a.Xt + lane * 8;
    const h16_t* wp[NBW];
#pragma unroll
    for (int nb = 0; nb < NBW; ++nb) wp[nb] = a.Wt + (size_t)min(nt0 + nb, a.n_tiles - 1) * a.k_tiles * 512 + lane * 8;
    v8h wr[kD][kKT][NBW];
    // one step's copies (this wavefront's XC of the stage's 16 blocks) and weight loads; tile indices past the
    // range are clamped: such blocks are fetched again but never multiplied
    auto issue_x = [&](int step) {
      uint8_t* stage = lds + (step % kNSX) * kXStageBytes;
#pragma unroll
      for (int i = 0; i < XC; ++i) {
        const int c = min(wave * XC + i, kKT * kMB - 1), t = c / kMB, mt = c % kMB;
        const int kk = min(kbeg + step * kKT + t, klast);
        __builtin_amdgcn_global_load_lds((glb_ptr_t)(xsrc + ((size_t)kk * a.m_tiles + min(mt, a.m_tiles - 1)) * 512),
                                         (lds_ptr_t)(stage + c * 1024), 16, 0, 0);
      }
    };
    auto load_w = [&](v8h (&dst)[kKT][NBW], int step) {
#pragma unroll
      for (int t = 0; t < kKT; ++t) {
        const int kk = min(kbeg + step * kKT + t, klast);
#pragma unroll
        for (int nb = 0; nb < NBW; ++nb) dst[t][nb] = load_frag(wp[nb] + (size_t)kk * 512, 0);
      }
    };
    auto multiply = [&](const v8h (&w)[kKT][NBW], int step) {
      const uint8_t* stage = lds + (step % kNSX) * kXStageBytes + lane * 16;
#pragma unroll
      for (int t = 0; t < kKT; ++t) {
        if (kbeg + step * kKT + t > klast) break;  // uniform: the last step of an odd range
        v8h xf[kMB];
#pragma unroll
        for (int mb = 0; mb < kMB; ++mb) xf[mb] = *reinterpret_cast<const v8h*>(stage + (t * kMB + mb) * 1024);
#pragma unroll
        for (int nb = 0; nb < NBW; ++nb)
#pragma unroll
          for (int mb = 0; mb < kMB; ++mb) acc[nb][mb] = mfma16(w[t][nb], xf[mb], acc[nb][mb]);
      }
    };
    // prologue: steps 0 .. kD - 1 in flight
#pragma unroll
    for (int s = 0; s < kD; ++s) {
      issue_x(s);
      load_w(wr[s], s);
    }
    int j = 0;
    // steady state: every step that is multiplied is followed by the issue of step j + kD, unconditionally (clamped
    // past the end); at the top of a step the operations of the kD - 1 younger steps may still be in flight
    for (; j + kD <= n_steps; j += kD) {
#pragma unroll
      for (int s = 0; s < kD; ++s) {
        wait_vm<(kD - 1) * OPS>();
        __builtin_amdgcn_s_barrier();   // the stage is complete for every wavefront; the stage read last is free
        multiply(wr[s], j + s);
        __builtin_amdgcn_sched_barrier(0);
        issue_x(j + s + kD);
        load_w(wr[s], j + s + kD);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    // the last n_steps % kD steps: everything they need has been issued
    for (int s = 0; s < kD; ++s) {
      if (j + s >= n_steps) break;
      wait_vm<0>();
      __builtin_amdgcn_s_barrier();
      if (s == 0) multiply(wr[0], j);
      else if (s == 1) multiply(wr[1], j + 1);
      else multiply(wr[2], j + 2);
    }
    wait_vm<0>();  // clamped copies past the end still target this workgroup's LDS
  }

  // ---- epilogues: lane holds features n = tile * 16 + rq .. + 3 of token m = mb * 16 + col
  const int col = lane & 15, rq = (lane >> 4) * 4;
  if (EPI == DEC_PARTIAL) {
    float* Pout = a.out_f32 + (size_t)blockIdx.y * Mpad * a.ld_out;
#pragma unroll
    for (int nb = 0; nb < NBW; ++nb) {
      if (nt0 + nb >= a.n_tiles) continue;
#pragma unroll
      for (int mb = 0; mb < kMB; ++mb) {
        const int m = mb * 16 + col;
        if (m < Mpad) *reinterpret_cast<v4f*>(Pout + (size_t)m * a.ld_out + (nt0 + nb) * 16 + rq) = acc[nb][mb];
      }
    }
  } else if (EPI == DEC_SWIGLU) {
    // weight row tiles alternate gate / up: tile 2 j holds gate rows 16 j .., tile 2 j + 1 the up rows
#pragma unroll
    for (int nb = 0; nb < NBW; nb += 2) {
      if (nt0 + nb >= a.n_tiles) continue;
      const int f = ((nt0 + nb) >> 1) * 16 + rq;
#pragma unroll
      for (int mb = 0; mb < kMB; ++mb) {
        const int m = mb * 16 + col;
        if (m >= a.M) continue;
        const float sc = s_scale[m];
        const v4f g = acc[nb][mb] * sc, u = acc[(nb + 1) % NBW][mb] * sc;
        uint2 pk;
        pk.x = pack_h16x2_flag(silu_r(g[0]) * u[0], silu_r(g[1]) * u[1], a.err_flag);
        pk.y = pack_h16x2_flag(silu_r(g[2]) * u[2], silu_r(g[3]) * u[3], a.err_flag);
        *reinterpret_cast<uint2*>(a.out_h16 + act_off(m, f, Mpad)) = pk;
      }
    }
  } else {  // DEC_SAMPLE: log-sum-exp and Gumbel arg-max of every row over this wavefront's columns, then over the workgroup's
    const SampleCtl ctl = *a.ctl;
    const int step = *a.d_step;
    // per-wavefront results of all 128 rows go through LDS (the operand ring is free now: every wavefront has
    // passed the last barrier of the loop and waited for its own copies)
    __syncthreads();
    DecSamplePartial* sm = reinterpret_cast<DecSamplePartial*>(lds);   // [WAVES][128]
#pragma unroll
    for (int mb = 0; mb < kMB; ++mb) {
      const int m = mb * 16 + col;
      const float sc = m < Mpad ? s_scale[m] : 1.f;
      const int row = (ctl.slot_row && m < a.M) ? max(ctl.slot_row[m], 0) : m;
      const int row_step = step - ((ctl.row_step0 && m < a.M) ? ctl.row_step0[m] : 0);  // a row that joined later
      Lse lse = lse_empty();
      float by = -INFINITY, bz = 0.f;
      int bi = 0x7fffffff;
#pragma unroll
      for (int nb = 0; nb < NBW; ++nb) {
        if (nt0 + nb >= a.n_tiles) continue;
        const int v0 = (nt0 + nb) * 16 + rq;  // multiple of 4: one generator block per 4 entries
        uint4 rb = make_uint4(0, 0, 0, 0);
        if (!ctl.greedy)
          rb = philox4x32_10(make_uint4((uint32_t)(v0 >> 2), (uint32_t)row_step, ctl.seq_offset + row, 0u), ctl.key0, ctl.key1);
        const uint32_t rr[4] = {rb.x, rb.y, rb.z, rb.w};
        float zt[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const float z = acc[nb][mb][r] * sc;
          zt[r] = ctl.greedy ? z : z * ctl.inv_temp;
        }
        lse_push4(lse, zt[0], zt[1], zt[2], zt[3]);
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const float y = ctl.greedy ? zt[r] : zt[r] + gumbel_from_bits(rr[r]);
          if (y > by) { by = y; bi = v0 + r; bz = zt[r]; }  // ascending index: the first maximum wins
        }
      }
#pragma unroll
      for (int o = 16; o <= 32; o <<= 1) {
        const Lse ol = {__shfl_xor(lse.m, o, 64), __shfl_xor(lse.s, o, 64)};
        const float oy = __shfl_xor(by, o, 64), oz = __shfl_xor(bz, o, 64);
        const int oi = __shfl_xor(bi, o, 64);
        lse = lse_merge(lse, ol);
        if (oy > by || (oy == by && oi < bi)) { by = oy; bi = oi; bz = oz; }
      }
      if (lane < 16) {
        DecSamplePartial* p = sm + wave * 128 + m;
        p->m = lse.m; p->s = lse.s; p->y = by; p->idx = bi; p->zt = bz;
      }
    }
    __syncthreads();
    // thread t < 128 merges row t over the wavefronts in ascending column order
    if (tid < a.M && tid < 128) {
      Lse lse = lse_empty();
      float by = -INFINITY, bz = 0.f;
      int bi = 0x7fffffff;
      for (int w = 0; w < WAVES; ++w) {
        const DecSamplePartial p = sm[w * 128 + tid];
        lse = lse_merge(lse, Lse{p.m, p.s});
        if (p.y > by || (p.y == by && p.idx < bi)) { by = p.y; bi = p.idx; bz = p.zt; }
      }
      DecSamplePartial* o = reinterpret_cast<DecSamplePartial*>(a.out_f32) + (size_t)tid * gridDim.x + grp;
      o->m = lse.m; o->s = lse.s; o->y = by; o->idx = bi; o->zt = bz;
    }
  }
}

template <int NBW, int WAVES, int EPI, int MINB = 2>
void launch_rows128(const DecGemmArgs& a, hipStream_t st) {
  static bool configured = false;  // per process; the attribute is a property of the function
  if (!configured) {
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&k_gemm_rows128<NBW, WAVES, EPI, MINB>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, kXRingBytes);
    configured = true;
  }
  const int per_wg = NBW * WAVES;
  const dim3 grid((a.n_tiles + per_wg - 1) / per_wg, EPI == DEC_PARTIAL ? a.ksplit : 1);
  k_gemm_rows128<NBW, WAVES, EPI, MINB><<<grid, WAVES * 64, kXRingBytes, st>>>(a);
}

}  // namespace

bool gemm_dec_rows128(const DecGemmArgs& a, int epi, hipStream_t st) {
  if (a.m_tiles <= 4 || a.m_tiles > kMB) return false;
  // The narrow matrices (QKV, O projection: a few hundred row tiles) stay with the general form: four tiles per
  // workgroup leave 56 .. 72 workgroups, far too few to pull the weights (49 and 54 us against 23 and 18 at the
  // 7 B shape), and fewer tiles per workgroup bring back the activation reads this form exists to avoid.
  if (epi == DEC_STORE || epi == DEC_RESID) return false;
  switch (epi) {
    case DEC_SWIGLU: {
      // One round on the 256 CUs with as many workgroups as that allows: a CU that hosts two workgroups pulls two
      // activation copies and takes nearly twice as long, and workgroups of more tiles leave CUs idle (7 B shape,
      // 2368 tiles: 8 tiles x 296 workgroups 89 us, 10 x 237 67 us, 12 x 198 69 us, 16 x 148 76 us).
      const auto groups = [&](int waves) { return (a.n_tiles + 2 * waves - 1) / (2 * waves); };
      if (groups(4) <= 256) launch_rows128<2, 4, DEC_SWIGLU>(a, st);
      else if (groups(5) <= 256) launch_rows128<2, 5, DEC_SWIGLU, 1>(a, st);
      else if (groups(6) <= 256) launch_rows128<2, 6, DEC_SWIGLU, 1>(a, st);
      else launch_rows128<2, 8, DEC_SWIGLU, 1>(a, st);
      return true;
    }
    // one tile per wavefront, eight wavefronts: 6.21 against 6.31 ms per step at the 7 B shape and 2.57 against
    // 2.68 ms at the 1.5 B shape (two tiles on each of four; the LM head is no faster that way)
    case DEC_PARTIAL: launch_rows128<1, kRows128WideTiles, DEC_PARTIAL, 1>(a, st); return true;
    case DEC_SAMPLE: launch_rows128<kRows128WideTiles / 4, 4, DEC_SAMPLE>(a, st); return true;
    default: return false;
  }
}

}  // namespace bf16
}  // namespace mtmc
