// Large-batch GEMM of the prefill / scoring pass, staged through LDS.
//
// Workgroup tile: 256 output features x 256 tokens, full K.  Four wavefronts (one per SIMD) in a
// 2 x 2 arrangement own 128 x 128 each: 4 x 4 accumulator blocks of v_mfma_f32_32x32x16_f16 per
// wavefront (a single wavefront per SIMD keeps the matrix pipe above 90 % busy with this shape, but
// only near 55 % with the 16x16x32 shape), which puts the LDS read rate at 16 KiB per k-step per
// wavefront (about half of what the LDS can deliver) and the global rate at 32 KiB per k-step per
// workgroup.
//
// Both operands already sit in memory as 1 KiB MFMA operand blocks (frag.h), so staging is a plain
// copy: every k-step (32 columns of K) needs 16 weight blocks and 16 activation blocks, which the
// wavefronts fetch with LDS-direct 16-byte loads (no registers involved) into a ring of kStages
// buffers, kStages - 1 steps ahead of the one being multiplied.  One workgroup barrier per step:
// it makes the step's blocks visible to every wavefront and at the same time guarantees that
// the buffer refilled next (read in the previous step) is no longer in use.
#include <algorithm>

#include "bf16_kernels.h"
#include "device_utils.h"
#include "frag.h"

namespace mtmc {
namespace bf16 {

namespace {

constexpr int kStages = 4;
constexpr int kPersistentGrid = 256;                 // CUs of the device; a multiple of the 8 XCDs
constexpr int kBlkTiles = 16;                       // 16-row tiles per workgroup tile side
constexpr int kStageBytes = 2 * kBlkTiles * 1024;   // weight blocks, then activation blocks
constexpr int kTrRow = 36;                          // floats per row of the epilogue's 32 x 32 transposition tile
constexpr int kTrBytes = 4 * 32 * kTrRow * 4;       // one tile per wavefront, behind the ring
constexpr int kLoadsPerStage = 2 * kBlkTiles / 4;   // LDS-direct loads each wavefront issues per step

typedef __attribute__((ext_vector_type(16))) float v16f;
typedef __attribute__((address_space(3))) void* lds_ptr_t;
typedef const __attribute__((address_space(1))) void* glb_ptr_t;

__device__ __forceinline__ void copy_block_to_lds(const uint8_t* src_lane, uint8_t* dst_block) {
  __builtin_amdgcn_global_load_lds((glb_ptr_t)src_lane, (lds_ptr_t)dst_block, 16, 0, 0);
}

// s_waitcnt on the vector-memory counter alone (the other counters left at their maxima).
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
  __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | (7 << 4) | (15 << 8));
}

// acc += A B with the accumulator pinned to the AGPR half of the register file (the 256 accumulator
// registers of a wavefront fill it exactly; left to itself the register allocator spreads them over both
// halves and spills).  Consecutive uses of one accumulator are 16 MFMAs apart, far beyond the
// dependent-issue distance of the instruction.
__device__ __forceinline__ void mfma32_acc(v16f& acc, v8h a, v8h b) {
  asm volatile("v_mfma_f32_32x32x16_f16 %0, %1, %2, %0" : "+a"(acc) : "v"(a), "v"(b) : "memory");
}

// silu with the hardware exp2 / reciprocal (about 1e-6 relative error; the result is rounded to fp16 anyway):
// the 128 evaluations per lane and output block would otherwise take a tenth of the block's time
__device__ __forceinline__ float silu_l(float g) {
  return g * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-1.4426950408889634f * g));
}

// Launch index -> output block: XCD (L % 8) owns token blocks xcd + 8 i and walks them in bands of
// kBand token blocks x all feature blocks, so workgroups resident together on an XCD share panels
// in its L2.  With fewer token blocks than XCDs (a prompt or two) the XCDs share out the feature blocks
// instead, or most of them would have nothing to do.
constexpr int kBand = 4;
struct Block { int nb, mb; bool valid; };
__device__ __forceinline__ Block block_of(int L, int nb_n, int nb_m) {
  const bool by_feature = nb_m < 8 && nb_n > nb_m;
  const int n_walk = by_feature ? nb_m : nb_n, n_own = by_feature ? nb_n : nb_m;
  const int xcd = L & 7, j = L >> 3;
  const int band = j / (kBand * n_walk), r = j - band * (kBand * n_walk);
  const int wb = r / kBand, oi = band * kBand + (r - wb * kBand);
  const int ob = xcd + 8 * oi;
  return by_feature ? Block{ob, wb, ob < n_own} : Block{wb, ob, ob < n_own};
}
// The same order without the gaps: the t-th block of those an XCD owns (t < blocks_of_xcd), band by band; the
// last band of an XCD is as high as the blocks it has left.  What a persistent workgroup walks: striding over
// launch indices instead would give the indices that name no block to always the same workgroups.
__host__ __device__ __forceinline__ int blocks_of_xcd(int xcd, int nb_n, int nb_m) {
  const bool by_feature = nb_m < 8 && nb_n > nb_m;
  const int n_walk = by_feature ? nb_m : nb_n, n_own = by_feature ? nb_n : nb_m;
  return xcd < n_own ? (n_own - xcd + 7) / 8 * n_walk : 0;
}
__device__ __forceinline__ Block block_of_xcd(int xcd, int t, int nb_n, int nb_m) {
  const bool by_feature = nb_m < 8 && nb_n > nb_m;
  const int n_walk = by_feature ? nb_m : nb_n, n_own = by_feature ? nb_n : nb_m;
  const int count = (n_own - xcd + 7) / 8;
  const int band = t / (kBand * n_walk), r = t - band * (kBand * n_walk);
  const int height = min(kBand, count - band * kBand);
  const int wb = r / height, ob = xcd + 8 * (band * kBand + (r - wb * height));
  return by_feature ? Block{ob, wb, true} : Block{wb, ob, true};
}
int grid_of(int nb_n, int nb_m) {
  const bool by_feature = nb_m < 8 && nb_n > nb_m;
  const int n_walk = by_feature ? nb_m : nb_n, n_own = by_feature ? nb_n : nb_m;
  const int per_xcd = (n_own + 7) / 8, bands = (per_xcd + kBand - 1) / kBand;
  return 8 * bands * kBand * n_walk;
}

enum { LEPI_STORE = 0, LEPI_ADD = 1, LEPI_SWIGLU = 2 };

// This wavefront's share of the copies of one 256 x 256 output block: weight blocks 4 wave .. + 3 and
// activation blocks 4 wave .. + 3 of every k-step (tile indices past the end are clamped: such blocks are
// multiplied but never stored).  Wavefront-uniform addresses of k-step 0; the lane adds its 16-byte slot.
struct TileSrc {
  const uint8_t* w[4];
  const uint8_t* x[4];
};
__device__ __forceinline__ TileSrc tile_src(const uint8_t* Wt, const uint8_t* Xt, int n_tiles, int m_tiles, int K,
                                            int nt_base, int mt_base, int uwave, int k0 = 0) {
  TileSrc t;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    t.w[j] = Wt + ((size_t)min(nt_base + 4 * uwave + j, n_tiles - 1) * K + k0) * 1024;
    t.x[j] = Xt + ((size_t)k0 * m_tiles + min(mt_base + 4 * uwave + j, m_tiles - 1)) * 1024;
  }
  return t;
}

// The matrix pipeline of a workgroup over a SEQUENCE of output blocks.  `tile_at(i, nt_base, mt_base)`
// names the i-th block (false: no more), `epilogue(acc, nt_base, mt_base)` consumes a finished one:
// acc = 4 x 4 accumulator blocks of 32 x 32 (v_mfma_f32_32x32x16_f16, 16 registers each) = the 128 x 128
// part of this wavefront (wn, wm).  The k-steps of consecutive blocks form one stream through the ring of
// kStages LDS buffers: while the last steps of a block are multiplied the first steps of the next one are
// already being fetched, and its first fragments are read, so that a new block starts without refilling
// the pipeline and its copies run under the epilogue of the previous one.  K >= kStages and even.
// SPLIT: a work item is an output block over k-steps k0 .. k0 + Ks - 1 only (tile_at also names k0, the epilogue
// gets it); the rows of W are still K k-steps long.  Ks >= kStages and even.
template <bool SPLIT = false, typename TileAt, typename Epilogue>
__device__ __forceinline__ void lds_gemm_stream(const uint8_t* Wt, const uint8_t* Xt, int n_tiles, int m_tiles, int K,
                                                uint8_t* lds, int lane, int uwave, int wn, int wm, TileAt tile_at,
                                                Epilogue epilogue, int Ks = 0) {
  int nt_base = 0, mt_base = 0, k0 = 0;
  const int KL = SPLIT ? Ks : K;  // k-steps of a work item
  bool any;
  if constexpr (SPLIT) any = tile_at(0, nt_base, mt_base, k0);
  else any = tile_at(0, nt_base, mt_base);
  if (!any) return;  // whole workgroup
  const size_t xstep = (size_t)m_tiles * 1024;
  const uint32_t lane16 = lane * 16;
  // A 32-row operand of the 32x32x16 MFMA (lane l: row l % 32, 8 consecutive k of half l / 32) is
  // gathered from two adjacent 16-row blocks: lane -> (block (l % 32) / 16, row l % 16, k group
  // 2 p + l / 32) for the p-th pair of k groups; the two pairs of a k-step are 512 bytes apart.
  const int r32 = lane & 31;
  const int lane_off = (r32 >> 4) * 1024 + (((lane >> 5) << 4) + (r32 & 15)) * 16;
  // Fragments of one k-step: per 32-row block two operands (k groups 0,1 and 2,3).
  struct Frags { v8h w[4][2], x[4][2]; };
  auto read_frag = [&](Frags& f, const uint8_t* sb, int i) {  // i = 0..15
    const int blk = (i >> 1) & 3, p = i & 1;
    if (i < 8) f.x[blk][p] = *reinterpret_cast<const v8h*>(sb + (kBlkTiles + 8 * wm + 2 * blk) * 1024 + p * 512);
    else f.w[blk][p] = *reinterpret_cast<const v8h*>(sb + (8 * wn + 2 * blk) * 1024 + p * 512);
  };
  auto issue_one = [&](const TileSrc& t, int kk, uint8_t* sb, int j) {  // j = 0..7; sb = this wavefront's part of a buffer
    if (j < 4) copy_block_to_lds(t.w[j] + (size_t)kk * 1024 + lane16, sb + j * 1024);
    else copy_block_to_lds(t.x[j - 4] + (size_t)kk * xstep + lane16, sb + (kBlkTiles + j - 4) * 1024);
  };

  TileSrc cur = tile_src(Wt, Xt, n_tiles, m_tiles, K, nt_base, mt_base, uwave, k0);
  // ---- fill the ring with the first kStages steps of the first block, read its first fragments
#pragma unroll
  for (int s = 0; s < kStages; ++s)
#pragma unroll
    for (int j = 0; j < 8; ++j) issue_one(cur, s, lds + s * kStageBytes + uwave * 4096, j);
  Frags fa, fb;
  wait_vmcnt<(kStages - 1) * kLoadsPerStage>();
  __builtin_amdgcn_s_barrier();
#pragma unroll
  for (int i = 0; i < 16; ++i) read_frag(fa, lds + lane_off, i);

  int g0 = 0;  // stream index of step 0 of the current block (step g lives in buffer g % kStages)
  for (int ti = 0;; ++ti) {
    int nt_next = 0, mt_next = 0, k0_next = 0;
    bool has_next;
    if constexpr (SPLIT) has_next = tile_at(ti + 1, nt_next, mt_next, k0_next);
    else has_next = tile_at(ti + 1, nt_next, mt_next);
    const TileSrc nxt = has_next ? tile_src(Wt, Xt, n_tiles, m_tiles, K, nt_next, mt_next, uwave, k0_next) : cur;
    v16f acc[4][4];
#pragma unroll
    for (int nb = 0; nb < 4; ++nb)
#pragma unroll
      for (int mb = 0; mb < 4; ++mb)
#pragma unroll
        for (int j = 0; j < 16; ++j) acc[nb][mb][j] = 0.f;
    asm volatile("s_nop 7" ::: "memory");  // accumulator writes settle before the first (inline-asm) MFMA reads them
    // Step kt multiplies the fragments already in registers; spread between its 32 MFMAs (which take 32
    // cycles each and leave the issue slots free) are the 16 LDS reads of the fragments of stream step
    // g + 1 and the 8 block fetches of stream step g + kStages, into the buffer step g was read from.
    auto step = [&](const Frags& fc, Frags& fn, int kt) {
      // own LDS reads done (they all feed `fc`); blocks of step g + 1 landed, g + 2 and g + 3 may fly
      __builtin_amdgcn_s_waitcnt((((kStages - 2) * kLoadsPerStage) & 15) | ((((kStages - 2) * kLoadsPerStage) >> 4) << 14) |
                                 (7 << 4) | (0 << 8));
      __builtin_amdgcn_s_barrier();
      const int g = g0 + kt;
      const uint8_t* rb = lds + ((g + 1) % kStages) * kStageBytes + lane_off;
      uint8_t* fbuf = lds + (g % kStages) * kStageBytes + uwave * 4096;
      // step g + kStages: of this block, else of the next one, else (nothing follows) a clamped copy nobody reads
      const int ka = kt + kStages;
      const bool own = ka < KL;
      const TileSrc& src = own ? cur : nxt;
      const int kk = own ? ka : (has_next ? ka - KL : KL - 1);
#pragma unroll
      for (int i = 0; i < 32; ++i) {
        const int pp = i >> 4, nb = (i >> 2) & 3, mb = i & 3;
        mfma32_acc(acc[nb][mb], fc.w[nb][pp], fc.x[mb][pp]);
        if ((i & 1) == 0) read_frag(fn, rb, i >> 1);
        if ((i & 3) == 1) issue_one(src, kk, fbuf, i >> 2);
      }
    };
    for (int kt = 0; kt < KL; kt += 2) {
      step(fa, fb, kt);
      step(fb, fa, kt + 1);
    }
    g0 += KL;
    // the last MFMAs were issued from inline assembly: give them time to retire before their accumulators
    // are read (16 passes of 4 cycles cover the longest one)
    asm volatile("s_nop 15\n\ts_nop 15\n\ts_nop 15\n\ts_nop 15\n\ts_nop 15" ::: "memory");
    if constexpr (SPLIT) epilogue(acc, nt_base, mt_base, k0);
    else epilogue(acc, nt_base, mt_base);
    if (!has_next) break;
    // the epilogue's stores (and loads) share the counter with the copies: drain it so that the waits of the
    // next block count copies only (they have been flying under the epilogue)
    wait_vmcnt<0>();
    nt_base = nt_next;
    mt_base = mt_next;
    k0 = k0_next;
    cur = nxt;
  }
  wait_vmcnt<0>();  // the clamped copies past the last step still target this workgroup's LDS
}

template <int EPI>
__global__ __launch_bounds__(256, 1) void k_gemm_lds(LargeArgs a) {
  extern __shared__ __attribute__((aligned(1024))) uint8_t lds[];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wn = wave & 1, wm = wave >> 1;
  const int nb_n = (a.n_tiles + kBlkTiles - 1) / kBlkTiles;
  int nb_m = (a.m_tiles + kBlkTiles - 1) / kBlkTiles;
  // rows packed on the device: only the row blocks that hold tokens are walked (the operand layout keeps the
  // stride of the full capacity)
  if (a.d_rows) nb_m = min(nb_m, (*a.d_rows + kBlkTiles * 16 - 1) / (kBlkTiles * 16));
  // persistent workgroup: gridDim.x is a multiple of 8, so this workgroup and the gridDim.x / 8 - 1 others of its
  // XCD share out the blocks the XCD owns, in the order block_of_xcd gives them
  const int xcd = blockIdx.x & 7, stride = gridDim.x >> 3;
  const int total = blocks_of_xcd(xcd, nb_n, nb_m);
  int t = (int)(blockIdx.x >> 3) - stride;
  auto tile_at = [&](int, int& nt_base, int& mt_base) {
    t += stride;
    if (t >= total) return false;
    const Block blk = block_of_xcd(xcd, t, nb_n, nb_m);
    nt_base = blk.nb * kBlkTiles;
    mt_base = blk.mb * kBlkTiles;
    return true;
  };
  auto epilogue = [&](v16f (&acc)[4][4], int nt_base, int mt_base) {
  // ---- epilogue: in a 32 x 32 block, lane holds token lane % 32 and features 8 q + 4 (lane / 32) + 0..3
  // (q = 0..3) in registers 4 q .. 4 q + 3
  const int col = lane & 31, rh = (lane >> 5) * 4;
  const int Mpad = a.m_tiles * 16;
  // accumulate form: the old values of a group of four blocks (one nb, the four mb) are requested while the
  // group before it is worked on; pass by pass, each block would wait a whole memory round trip for them
  v4f old[2][4][4];
  const int f = (lane & 7) * 4, trow = lane >> 3;
  auto fetch_old = [&](int nb, v4f (&dst)[4][4]) {
    const int n = (nt_base + 8 * wn + 2 * nb) * 16 + f;
#pragma unroll
    for (int mb = 0; mb < 4; ++mb)
#pragma unroll
      for (int pass = 0; pass < 4; ++pass) {
        const int mm = (mt_base + 8 * wm + 2 * mb) * 16 + pass * 8 + trow;
        dst[mb][pass] = v4f{0.f, 0.f, 0.f, 0.f};
        if (mm < a.M && n < a.N) dst[mb][pass] = *reinterpret_cast<const v4f*>(a.out_f32 + (size_t)mm * a.ld_out + n);
      }
  };
  if (EPI == LEPI_ADD) fetch_old(0, old[0]);
  bool out_of_range = false;  // SwiGLU form: a product that does not fit fp16 (reported once per block, below)
#pragma unroll
  for (int nb = 0; nb < 4; ++nb) {
    if (EPI == LEPI_ADD && nb + 1 < 4) fetch_old(nb + 1, old[(nb + 1) & 1]);
#pragma unroll
    for (int mb = 0; mb < 4; ++mb) {
      // one accumulator block at a time: it is taken from its registers here, not earlier (volatile statements
      // keep their order), which keeps the 256 accumulators out of the VGPR half until they are needed
      asm volatile("" : "+a"(acc[nb][mb])::"memory");
      const int m = (mt_base + 8 * wm + 2 * mb) * 16 + col;
      const int n0 = (nt_base + 8 * wn + 2 * nb) * 16;  // first feature row of the block
      if (EPI == LEPI_SWIGLU) {
        // rows 0..15 of the block are gate rows, rows 16..31 the matching up rows
        if (m >= a.M || n0 >= a.n_tiles * 16) continue;
#pragma unroll
        for (int q = 0; q < 2; ++q) {
          const int fo = (n0 >> 1) + 8 * q + rh;
          uint2 pk;
          pk.x = pack_h16x2_track(silu_l(acc[nb][mb][4 * q + 0]) * acc[nb][mb][4 * q + 8],
                                  silu_l(acc[nb][mb][4 * q + 1]) * acc[nb][mb][4 * q + 9], out_of_range);
          pk.y = pack_h16x2_track(silu_l(acc[nb][mb][4 * q + 2]) * acc[nb][mb][4 * q + 10],
                                  silu_l(acc[nb][mb][4 * q + 3]) * acc[nb][mb][4 * q + 11], out_of_range);
          *reinterpret_cast<uint2*>(a.out_bf16 + act_off(m, fo, Mpad)) = pk;
        }
      } else {
        // fp32 output, row-major [token][feature]: a lane's 4 consecutive features of ONE token would make every
        // store instruction touch 32 different rows; the 32 x 32 block is turned round in a wavefront-private
        // LDS tile (behind the ring) so that an instruction covers 8 rows of 128 contiguous bytes
        float* tb = reinterpret_cast<float*>(lds + kStages * kStageBytes) + wave * (32 * kTrRow);
#pragma unroll
        for (int q = 0; q < 4; ++q)
          *reinterpret_cast<v4f*>(tb + col * kTrRow + 8 * q + rh) =
              v4f{acc[nb][mb][4 * q], acc[nb][mb][4 * q + 1], acc[nb][mb][4 * q + 2], acc[nb][mb][4 * q + 3]};
        __builtin_amdgcn_wave_barrier();
        const int m0 = (mt_base + 8 * wm + 2 * mb) * 16, n = n0 + f;
#pragma unroll
        for (int pass = 0; pass < 4; ++pass) {
          const int row = pass * 8 + trow, mm = m0 + row;
          v4f v = *reinterpret_cast<const v4f*>(tb + row * kTrRow + f);
          if (EPI == LEPI_ADD) v = v + old[nb & 1][mb][pass];
          if (mm < a.M && n < a.N) *reinterpret_cast<v4f*>(a.out_f32 + (size_t)mm * a.ld_out + n) = v;
        }
        __builtin_amdgcn_wave_barrier();  // the tile is reused by the next accumulator block
      }
    }
  }
  if (EPI == LEPI_SWIGLU && out_of_range) atomicOr(a.err_flag, kErrFp16Range);
};
  lds_gemm_stream(reinterpret_cast<const uint8_t*>(a.Wt), reinterpret_cast<const uint8_t*>(a.Xt), a.n_tiles, a.m_tiles,
                  a.k_tiles, lds, lane, __builtin_amdgcn_readfirstlane(wave), wn, wm, tile_at, epilogue);
}

// Split-K form for outputs of few blocks and a long reduction (the O and down projections, and the QKV projection,
// of a prompt or a few: 12-128 blocks for 256 CUs): a work item is one output block over one of a.k_split equal
// ranges of k-steps, the items of a block are neighbours in an XCD's walk, and every item stores its sum as fp32
// into its own slice of a.part ([k_split][M][N]); k_splitk_reduce then adds the slices in order, so the result does
// not depend on which workgroup ran when.
__global__ __launch_bounds__(256, 1) void k_gemm_lds_split(LargeArgs a) {
  extern __shared__ __attribute__((aligned(1024))) uint8_t lds[];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wn = wave & 1, wm = wave >> 1;
  const int nb_n = (a.n_tiles + kBlkTiles - 1) / kBlkTiles;
  int nb_m = (a.m_tiles + kBlkTiles - 1) / kBlkTiles;
  if (a.d_rows) nb_m = min(nb_m, (*a.d_rows + kBlkTiles * 16 - 1) / (kBlkTiles * 16));
  const int S = a.k_split, Ks = a.k_tiles / S;
  const int xcd = blockIdx.x & 7, stride = gridDim.x >> 3;
  const int total = blocks_of_xcd(xcd, nb_n, nb_m) * S;
  int t = (int)(blockIdx.x >> 3) - stride;
  auto tile_at = [&](int, int& nt_base, int& mt_base, int& k0) {
    t += stride;
    if (t >= total) return false;
    const Block blk = block_of_xcd(xcd, t / S, nb_n, nb_m);
    nt_base = blk.nb * kBlkTiles;
    mt_base = blk.mb * kBlkTiles;
    k0 = (t % S) * Ks;
    return true;
  };
  auto epilogue = [&](v16f (&acc)[4][4], int nt_base, int mt_base, int k0) {
    // as the store form of k_gemm_lds: every 32 x 32 block is turned round in a wavefront-private LDS tile so that
    // a store instruction covers 8 rows of 128 contiguous bytes
    float* out = a.part + (size_t)(k0 / Ks) * a.M * a.N;
    const int col = lane & 31, rh = (lane >> 5) * 4;
    const int f = (lane & 7) * 4, trow = lane >> 3;
    float* tb = reinterpret_cast<float*>(lds + kStages * kStageBytes) + wave * (32 * kTrRow);
#pragma unroll
    for (int nb = 0; nb < 4; ++nb) {
#pragma unroll
      for (int mb = 0; mb < 4; ++mb) {
        asm volatile("" : "+a"(acc[nb][mb])::"memory");
        const int n0 = (nt_base + 8 * wn + 2 * nb) * 16;
#pragma unroll
        for (int q = 0; q < 4; ++q)
          *reinterpret_cast<v4f*>(tb + col * kTrRow + 8 * q + rh) =
              v4f{acc[nb][mb][4 * q], acc[nb][mb][4 * q + 1], acc[nb][mb][4 * q + 2], acc[nb][mb][4 * q + 3]};
        __builtin_amdgcn_wave_barrier();
        const int m0 = (mt_base + 8 * wm + 2 * mb) * 16, n = n0 + f;
#pragma unroll
        for (int pass = 0; pass < 4; ++pass) {
          const int row = pass * 8 + trow, mm = m0 + row;
          const v4f v = *reinterpret_cast<const v4f*>(tb + row * kTrRow + f);
          if (mm < a.M && n < a.N) *reinterpret_cast<v4f*>(out + (size_t)mm * a.N + n) = v;
        }
        __builtin_amdgcn_wave_barrier();  // the tile is reused by the next accumulator block
      }
    }
  };
  lds_gemm_stream<true>(reinterpret_cast<const uint8_t*>(a.Wt), reinterpret_cast<const uint8_t*>(a.Xt), a.n_tiles,
                        a.m_tiles, a.k_tiles, lds, lane, __builtin_amdgcn_readfirstlane(wave), wn, wm, tile_at, epilogue,
                        Ks);
}

// out (+)= part[0] + part[1] + ... in that order; four features per thread
__global__ __launch_bounds__(256) void k_splitk_reduce(float* out, int ld_out, const float* part, int S, int M, int N,
                                                       int accumulate, const int* d_rows) {
  const int n4 = N >> 2;
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= (size_t)M * n4) return;
  const int m = (int)(i / n4), n = (int)(i - (size_t)m * n4) * 4;
  if (d_rows && m >= *d_rows) return;
  float* o = out + (size_t)m * ld_out + n;
  v4f acc = accumulate ? *reinterpret_cast<const v4f*>(o) : v4f{0.f, 0.f, 0.f, 0.f};
  for (int s = 0; s < S; ++s) acc = acc + *reinterpret_cast<const v4f*>(part + ((size_t)s * M + m) * N + n);
  *reinterpret_cast<v4f*>(o) = acc;
}

// Scoring LM head on the same engine: a workgroup owns 256 rows and one vocabulary slice (8 blocks of
// 256 entries), computes the logits block by block and folds them into running per-row results
// (log-sum-exp, two largest logits, logit of the target token); logits are never stored.
__global__ __launch_bounds__(256, 1) void k_lmhead_lds(ScoreHeadArgs a, int slices) {
  extern __shared__ __attribute__((aligned(1024))) uint8_t lds[];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wn = wave & 1, wm = wave >> 1;
  const int nb_m = (a.m_tiles + kBlkTiles - 1) / kBlkTiles;
  const Block blk = block_of(blockIdx.x, slices, nb_m);
  if (!blk.valid) return;  // whole workgroup
  const int mt_base = blk.mb * kBlkTiles;
  if (a.d_rows && mt_base * 16 >= *a.d_rows) return;  // rows packed on the device: this block holds no token
  const int col = lane & 31, rh = (lane >> 5) * 4;
  const int uwave = __builtin_amdgcn_readfirstlane(wave);
  // The per-row running results live in LDS behind the ring (28 words per thread, word-interleaved over the
  // threads) and are loaded only inside the epilogue, so that they take no registers from the matrix loop.
  float* st_f = reinterpret_cast<float*>(lds + kStages * kStageBytes) + threadIdx.x;
  int* st_i = reinterpret_cast<int*>(st_f);
  constexpr int SM = 0, SS = 4, SV1 = 8, SI1 = 12, SV2 = 16, SZT = 20, STG = 24;  // word index + mb, x 256 threads
#pragma unroll
  for (int mb = 0; mb < 4; ++mb) {
    const int m = (mt_base + 8 * wm + 2 * mb) * 16 + col;
    st_f[(SM + mb) * 256] = -INFINITY;
    st_f[(SS + mb) * 256] = 0.f;
    st_f[(SV1 + mb) * 256] = -INFINITY;
    st_i[(SI1 + mb) * 256] = 0x7fffffff;
    st_f[(SV2 + mb) * 256] = -INFINITY;
    st_f[(SZT + mb) * 256] = -INFINITY;
    st_i[(STG + mb) * 256] = (m < a.M) ? a.targets[m] : -1;
  }
  const int nb_n = (a.n_tiles + kBlkTiles - 1) / kBlkTiles;
  const int vocab = a.n_tiles * 16;
  const int nbk0 = blk.nb * 8, nbk1 = min(blk.nb * 8 + 8, nb_n);
  auto tile_at = [&](int i, int& nt_base, int& mt_b) {
    nt_base = (nbk0 + i) * kBlkTiles;
    mt_b = mt_base;
    return nbk0 + i < nbk1;
  };
  auto epilogue = [&](v16f (&acc)[4][4], int nt_base, int) {
    const int nbk = nt_base / kBlkTiles;
    const bool full = (nbk + 1) * kBlkTiles <= a.n_tiles;  // all 256 entries of the block exist (workgroup-uniform)
    // one group of 32 rows (mb) at a time, so that only its running results and one accumulator block are live
#pragma unroll
    for (int mb = 0; mb < 4; ++mb) {
      Lse lse = Lse{st_f[(SM + mb) * 256], st_f[(SS + mb) * 256]};
      Top2 top = Top2{st_f[(SV1 + mb) * 256], st_i[(SI1 + mb) * 256], st_f[(SV2 + mb) * 256]};
      float zt = st_f[(SZT + mb) * 256];
      const int target = st_i[(STG + mb) * 256];
#pragma unroll
      for (int nb = 0; nb < 4; ++nb) {
        // the accumulator block is taken from its registers here, not earlier (volatile statements keep their order)
        asm volatile("" : "+a"(acc[nb][mb])::"memory");
        // this lane's 16 entries of the block: n0 + 8 q + r (q, r = 0..3) in register 4 q + r
        const int n0 = (nbk * kBlkTiles + 8 * wn + 2 * nb) * 16 + rh;
        v16f z = acc[nb][mb];
        if (!full) {
#pragma unroll
          for (int j = 0; j < 16; ++j)
            if (n0 + 8 * (j >> 2) + (j & 3) >= vocab) z[j] = -INFINITY;
        }
        float bm = z[0];
#pragma unroll
        for (int j = 1; j < 16; ++j) bm = fmaxf(bm, z[j]);
        if (bm > lse.m) {  // -inf never gets here: an empty block leaves the state untouched
          lse.s *= __expf(lse.m - bm);
          lse.m = bm;
        }
        if (lse.m > -INFINITY) {
          const float mm = lse.m;
          float add = 0.f;
#pragma unroll
          for (int j = 0; j < 16; ++j) add += __expf(z[j] - mm);  // exp(-inf) = 0 for missing entries
          lse.s += add;
        }
        if (a.want_top && (bm > top.v2 || bm == top.v1)) {  // only then can the two largest (or a tie) change
#pragma unroll
          for (int j = 0; j < 16; ++j) top2_push(top, z[j], n0 + 8 * (j >> 2) + (j & 3));
        }
        const int d = target - n0;
        if (d >= 0 && d < 32 && (d & 4) == 0) {
          const int idx = (d >> 3) * 4 + (d & 3);
#pragma unroll
          for (int j = 0; j < 16; ++j)
            if (j == idx) zt = z[j];
        }
      }
      st_f[(SM + mb) * 256] = lse.m;
      st_f[(SS + mb) * 256] = lse.s;
      st_f[(SV1 + mb) * 256] = top.v1;
      st_i[(SI1 + mb) * 256] = top.i1;
      st_f[(SV2 + mb) * 256] = top.v2;
      st_f[(SZT + mb) * 256] = zt;
    }
  };
  lds_gemm_stream(reinterpret_cast<const uint8_t*>(a.Wt), reinterpret_cast<const uint8_t*>(a.Xt), a.n_tiles, a.m_tiles,
                  a.k_tiles, lds, lane, uwave, wn, wm, tile_at, epilogue);
  Lse lse[4];
  Top2 top[4];
  float zt[4];
#pragma unroll
  for (int mb = 0; mb < 4; ++mb) {
    lse[mb] = Lse{st_f[(SM + mb) * 256], st_f[(SS + mb) * 256]};
    top[mb] = Top2{st_f[(SV1 + mb) * 256], st_i[(SI1 + mb) * 256], st_f[(SV2 + mb) * 256]};
    zt[mb] = st_f[(SZT + mb) * 256];
  }
#pragma unroll
  for (int mb = 0; mb < 4; ++mb) {
    const Lse ol = {__shfl_xor(lse[mb].m, 32, 64), __shfl_xor(lse[mb].s, 32, 64)};
    const Top2 ot = {__shfl_xor(top[mb].v1, 32, 64), __shfl_xor(top[mb].i1, 32, 64), __shfl_xor(top[mb].v2, 32, 64)};
    lse[mb] = lse_merge(lse[mb], ol);
    top[mb] = top2_merge(top[mb], ot);
    zt[mb] = fmaxf(zt[mb], __shfl_xor(zt[mb], 32, 64));
    const int m = (mt_base + 8 * wm + 2 * mb) * 16 + col;
    if (lane < 32 && m < a.M) {
      ScorePartial* p = reinterpret_cast<ScorePartial*>(a.part) + ((size_t)(blk.nb * 2 + wn)) * a.M + m;
      p->m = lse[mb].m; p->s = lse[mb].s; p->v1 = top[mb].v1; p->i1 = top[mb].i1; p->v2 = top[mb].v2;
      p->zt = zt[mb];
    }
  }
}

template <int EPI>
void launch_one(const LargeArgs& a, hipStream_t st) {
  static bool configured = false;  // per process; the attribute is a property of the function
  const int lds_bytes = kStages * kStageBytes + kTrBytes;
  if (!configured) {
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&k_gemm_lds<EPI>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
    configured = true;
  }
  const int nb_n = (a.n_tiles + kBlkTiles - 1) / kBlkTiles, nb_m = (a.m_tiles + kBlkTiles - 1) / kBlkTiles;
  // persistent: one workgroup per CU (the kernel fills a CU), each walks launch indices i, i + grid, ...
  const int grid = std::min(grid_of(nb_n, nb_m), kPersistentGrid);
  k_gemm_lds<EPI><<<grid, 256, lds_bytes, st>>>(a);
}

}  // namespace

void lmhead_score_lds(const ScoreHeadArgs& a, int slices, hipStream_t st) {
  static bool configured = false;
  const int lds_bytes = kStages * kStageBytes + 28 * 256 * 4;  // ring + per-thread running results
  if (!configured) {
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&k_lmhead_lds), hipFuncAttributeMaxDynamicSharedMemorySize,
                              lds_bytes);
    configured = true;
  }
  k_lmhead_lds<<<grid_of(slices, (a.m_tiles + kBlkTiles - 1) / kBlkTiles), 256, lds_bytes, st>>>(a, slices);
}

bool gemm_lds_split(const LargeArgs& a0, bool accumulate, float* part, size_t part_floats, hipStream_t st) {
  const int nb_n = (a0.n_tiles + kBlkTiles - 1) / kBlkTiles, nb_m = (a0.m_tiles + kBlkTiles - 1) / kBlkTiles;
  const int blocks = nb_n * nb_m;
  if (!part || blocks > kPersistentGrid / 2 || a0.N % 4 != 0) return false;
  // the most splits, up to 8 and to one round of workgroups, that leave every range even and at least 8 k-steps long
  int S = 0;
  for (int s = std::min(8, kPersistentGrid / blocks); s >= 2 && !S; --s)
    if (a0.k_tiles % s == 0 && (a0.k_tiles / s) % 2 == 0 && a0.k_tiles / s >= 8 &&
        (size_t)s * a0.M * a0.N <= part_floats)
      S = s;
  if (!S) return false;
  static bool configured = false;
  const int lds_bytes = kStages * kStageBytes + kTrBytes;
  if (!configured) {
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&k_gemm_lds_split), hipFuncAttributeMaxDynamicSharedMemorySize,
                              lds_bytes);
    configured = true;
  }
  LargeArgs a = a0;
  a.k_split = S;
  a.part = part;
  const int grid = std::min(kPersistentGrid, 8 * blocks_of_xcd(0, nb_n, nb_m) * S);
  k_gemm_lds_split<<<grid, 256, lds_bytes, st>>>(a);
  const size_t quads = (size_t)a.M * (a.N / 4);
  k_splitk_reduce<<<(unsigned)((quads + 255) / 256), 256, 0, st>>>(a.out_f32, a.ld_out, part, S, a.M, a.N,
                                                                  accumulate ? 1 : 0, a.d_rows);
  return true;
}

void gemm_lds(const LargeArgs& a, int epi, hipStream_t st) {
  if (epi == LEPI_STORE) launch_one<LEPI_STORE>(a, st);
  else if (epi == LEPI_ADD) launch_one<LEPI_ADD>(a, st);
  else launch_one<LEPI_SWIGLU>(a, st);
}

}  // namespace bf16
}  // namespace mtmc
