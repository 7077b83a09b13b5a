// Sampling LM head of a decode step for up to 64 rows and a narrow model: a PERSISTENT form.
//
// The general decode GEMM gives every workgroup a few weight row tiles and makes it fetch the whole activation
// operand and the row scales for them: at a vocabulary of 150 k entries that is thousands of workgroups, each with
// its own prologue, and as many activation bytes from L2 as weight bytes from HBM.  Here one workgroup per CU keeps
// its share of the activation operand in registers for the whole launch (wavefront w owns the k range w of four, as
// in the general form's LM-head launch) and walks over pairs of weight row tiles: the tiles of step s + 2 are
// requested while step s is multiplied, the four wavefronts' partial sums of a step meet in LDS (added in wavefront
// order, which with the same k ranges gives the logits of the general form bit for bit), and every lane folds its
// four logits per block into a running (log-sum-exp, Gumbel arg-max) of its row that leaves the kernel once, as one
// partial result per row and workgroup.
//
// Taken when the k range of a wavefront fits the registers: k_tiles = 4 KPW with KPW x (row tiles) fragments.
#include <algorithm>

#include "bf16_kernels.h"
#include "device_utils.h"
#include "frag.h"

namespace mtmc {
namespace bf16 {

namespace {

constexpr int kLW = 4;    // wavefronts per workgroup = K splits
constexpr int kLNB = 2;   // weight row tiles per step

template <int MB, int KPW>
__global__ __launch_bounds__(kLW * 64, 1) void k_lmhead_sample(DecGemmArgs a) {
  constexpr int NT = kLW * 64;
  constexpr int BLK = kLNB * MB;                     // accumulator blocks (row tile x token tile) per step
  constexpr int BPW = BLK >= kLW ? BLK / kLW : 1;    // blocks a wavefront finishes per step
  constexpr int WPM = kLNB / BPW;                    // wavefronts that finish blocks of one token tile
  static_assert(BLK % BPW == 0 && kLNB % BPW == 0, "a wavefront's blocks belong to one token tile");
  __shared__ v4f red[2][kLW][BLK][64];
  __shared__ float s_scale[64];
  __shared__ float s_part[2][NT];
  __shared__ DecSamplePartial s_fin[kLW][16];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int Mpad = a.m_tiles * 16;   // <= 64
  const int total = (a.n_tiles + kLNB - 1) / kLNB, G = gridDim.x;

  // ---- the first two steps' weight tiles and this wavefront's activation fragments are requested first
  const int k0 = wave * KPW;
  const h16_t* wbase = a.Wt + (size_t)k0 * 512 + lane * 8;
  v8h wr[2][kLNB][KPW];
  auto load_w = [&](v8h (&dst)[kLNB][KPW], int g) {
#pragma unroll
    for (int nb = 0; nb < kLNB; ++nb) {
      const h16_t* wp = wbase + (size_t)min(g * kLNB + nb, a.n_tiles - 1) * a.k_tiles * 512;
#pragma unroll
      for (int kk = 0; kk < KPW; ++kk) dst[nb][kk] = load_frag(wp + (size_t)kk * 512, 0);
    }
  };
  v8h xf[KPW][MB];
#pragma unroll
  for (int kk = 0; kk < KPW; ++kk)
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
      xf[kk][mb] = load_frag(a.Xt + ((size_t)(k0 + kk) * a.m_tiles + min(mb, a.m_tiles - 1)) * 512, lane);
  int g = blockIdx.x;
  load_w(wr[0], g);
  load_w(wr[1], g + G);

  // ---- row scales r_new / r_old of the normalisation that the producer of the operand deferred: thread t sums
  // the tiles part, part + P, ... of row t % Mpad, the P partial sums are added in index order
  {
    const int P = NT / Mpad, m = tid % Mpad, part = tid / Mpad;
    const bool two = a.ss_cur && a.ss_old != a.ss_cur;
    float sa = 0.f, sb = 0.f;
    if (a.ss_cur && part < P) {
      constexpr int BT = 8;
      for (int t0 = part; t0 < a.ss_tiles; t0 += BT * P) {
        float fa[BT], fb[BT];
#pragma unroll
        for (int u = 0; u < BT; ++u) {
          const int t = t0 + u * P;
          fa[u] = t < a.ss_tiles ? a.ss_cur[(size_t)t * Mpad + m] : 0.f;
          fb[u] = (two && t < a.ss_tiles) ? a.ss_old[(size_t)t * Mpad + m] : 0.f;
        }
#pragma unroll
        for (int u = 0; u < BT; ++u) {
          sa += fa[u];
          sb += fb[u];
        }
      }
    }
    if (part < P) {
      s_part[0][tid] = sa;
      s_part[1][tid] = sb;
    }
    __syncthreads();
    if (tid < 64) {
      float sc = 1.f;
      if (tid < Mpad && two) {
        float ta = 0.f, tb = 0.f;
        for (int q = 0; q < P; ++q) {
          ta += s_part[0][q * Mpad + tid];
          tb += s_part[1][q * Mpad + tid];
        }
        sc = 1.0f / sqrtf(ta * a.inv_d + a.eps);   // the same operations as the general form: the same bits
        sc *= sqrtf(tb * a.inv_d + a.eps);
      }
      s_scale[tid] = sc;
    }
    __syncthreads();
  }

  // ---- this wavefront's blocks of a step: q = wave BPW + j -> row tile nb = q % 2 of the pair, token tile mb = q / 2
  const int col = lane & 15, rq = (lane >> 4) * 4;
  const int q0 = wave * BPW, my_mb = q0 / kLNB;
  const bool has_blocks = q0 < BLK;
  const int m = my_mb * 16 + col;   // this lane's row, the same in every step
  const SampleCtl ctl = *a.ctl;
  const float sc = (has_blocks && m < Mpad) ? s_scale[m] : 1.f;
  // the random numbers of a row follow the row and its own step, whatever slot it sits in and whenever it joined
  // (an empty slot draws row 0's: unused)
  const int smp_row = (ctl.slot_row && m < a.M) ? max(ctl.slot_row[m], 0) : m;
  const int step_no = *a.d_step - ((ctl.row_step0 && m < a.M) ? ctl.row_step0[m] : 0);
  Lse lse = lse_empty();
  float by = -INFINITY, bz = 0.f;
  int bi = 0x7fffffff;

  auto step = [&](v8h (&w)[kLNB][KPW], int gs, int par) {
    v4f acc[kLNB][MB];
#pragma unroll
    for (int nb = 0; nb < kLNB; ++nb)
#pragma unroll
      for (int mb = 0; mb < MB; ++mb) acc[nb][mb] = v4f{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int kk = 0; kk < KPW; ++kk)
#pragma unroll
      for (int nb = 0; nb < kLNB; ++nb)
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) acc[nb][mb] = mfma16(w[nb][kk], xf[kk][mb], acc[nb][mb]);
    // the tiles of step + 2 go out before the exchange (unconditionally, clamped past the end: a refill behind a
    // branch would make the compiler wait for every outstanding load where the branch joins)
    __builtin_amdgcn_sched_barrier(0);
    load_w(w, gs + 2 * G);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int nb = 0; nb < kLNB; ++nb)
#pragma unroll
      for (int mb = 0; mb < MB; ++mb) red[par][wave][mb * kLNB + nb][lane] = acc[nb][mb];
    __syncthreads();   // one barrier per step: the exchange buffer alternates
    if (has_blocks) {
#pragma unroll
      for (int j = 0; j < BPW; ++j) {
        const int q = q0 + j, nb = q % kLNB;
        v4f sum = red[par][0][q][lane];
#pragma unroll
        for (int ww = 1; ww < kLW; ++ww) sum = sum + red[par][ww][q][lane];
        const int tile = gs * kLNB + nb;
        if (gs < total && tile < a.n_tiles) {   // uniform; no memory access inside
          const int v0 = tile * 16 + rq;        // multiple of 4: one generator block per 4 entries
          uint4 rb = make_uint4(0, 0, 0, 0);
          if (!ctl.greedy)
            rb = philox4x32_10(make_uint4((uint32_t)(v0 >> 2), (uint32_t)step_no, ctl.seq_offset + smp_row, 0u), ctl.key0,
                               ctl.key1);
          const uint32_t rr[4] = {rb.x, rb.y, rb.z, rb.w};
          float zt[4];
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            const float z = sum[r] * sc;
            zt[r] = ctl.greedy ? z : z * ctl.inv_temp;
          }
          lse_push4(lse, zt[0], zt[1], zt[2], zt[3]);
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            const float y = ctl.greedy ? zt[r] : zt[r] + gumbel_from_bits(rr[r]);
            if (y > by) { by = y; bi = v0 + r; bz = zt[r]; }  // ascending index: the first maximum wins
          }
        }
      }
    }
  };
  for (; g < total; g += 2 * G) {
    step(wr[0], g, 0);
    step(wr[1], g + G, 1);
  }

  // ---- a row's four column groups (lane / 16), then the wavefronts that share its token tile, in column order
#pragma unroll
  for (int o = 16; o <= 32; o <<= 1) {
    const Lse ol = {__shfl_xor(lse.m, o, 64), __shfl_xor(lse.s, o, 64)};
    const float oy = __shfl_xor(by, o, 64), oz = __shfl_xor(bz, o, 64);
    const int oi = __shfl_xor(bi, o, 64);
    lse = lse_merge(lse, ol);
    if (oy > by || (oy == by && oi < bi)) { by = oy; bi = oi; bz = oz; }
  }
  if (lane < 16) {
    DecSamplePartial* p = &s_fin[wave][lane];
    p->m = lse.m; p->s = lse.s; p->y = by; p->idx = bi; p->zt = bz;
  }
  __syncthreads();
  if (tid < a.M) {
    const int mb = tid >> 4, c = tid & 15;
    Lse fl = lse_empty();
    float fy = -INFINITY, fz = 0.f;
    int fi = 0x7fffffff;
    for (int j = 0; j < WPM; ++j) {
      const DecSamplePartial p = s_fin[mb * WPM + j][c];
      fl = lse_merge(fl, Lse{p.m, p.s});
      if (p.y > fy || (p.y == fy && p.idx < fi)) { fy = p.y; fi = p.idx; fz = p.zt; }
    }
    DecSamplePartial* o = reinterpret_cast<DecSamplePartial*>(a.out_f32) + (size_t)tid * G + blockIdx.x;
    o->m = fl.m; o->s = fl.s; o->y = fy; o->idx = fi; o->zt = fz;
  }
}

template <int KPW>
void launch_lmhead_sample(const DecGemmArgs& a, int grid, hipStream_t st) {
  if (a.m_tiles <= 1) k_lmhead_sample<1, KPW><<<grid, kLW * 64, 0, st>>>(a);
  else if (a.m_tiles <= 2) k_lmhead_sample<2, KPW><<<grid, kLW * 64, 0, st>>>(a);
  else k_lmhead_sample<4, KPW><<<grid, kLW * 64, 0, st>>>(a);
}

}  // namespace

int lmhead_sample_persistent_groups(int n_tiles, int k_tiles, int m_tiles) {
  if (m_tiles > 4 || k_tiles % kLW != 0) return 0;
  const int kpw = k_tiles / kLW;
  if (kpw != 3 && kpw != 4 && kpw != 12) return 0;       // widths the kernel is built for (d = 384, 512, 1536)
  return std::min((n_tiles + kLNB - 1) / kLNB, 256);
}

bool lmhead_sample_persistent(const DecGemmArgs& a, hipStream_t st) {
  const int grid = lmhead_sample_persistent_groups(a.n_tiles, a.k_tiles, a.m_tiles);
  if (grid == 0) return false;
  switch (a.k_tiles / kLW) {
    case 3: launch_lmhead_sample<3>(a, grid, st); break;
    case 4: launch_lmhead_sample<4>(a, grid, st); break;
    default: launch_lmhead_sample<12>(a, grid, st); break;
  }
  return true;
}

}  // namespace bf16
}  // namespace mtmc
