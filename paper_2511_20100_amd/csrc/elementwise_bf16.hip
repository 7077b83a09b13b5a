// Row-wise and layout kernels of the bf16 path: weight re-tiling, embedding, residual-add +
// RMSNorm (-> tiled bf16 GEMM operand), split-K sum + rotary embedding + KV page write.
#include "bf16_kernels.h"
#include "device_utils.h"
#include "frag.h"

namespace mtmc {
namespace bf16 {

// ---------------------------------------------------------------- weight re-tiling
__global__ void k_retile(h16_t* dst, const bf16_t* src0, const bf16_t* src1, int N, int K, int n_tiles,
                         int k_tiles, int interleave, int* err_flag) {
  const size_t chunk = (size_t)blockIdx.x * blockDim.x + threadIdx.x;  // one 8-element chunk
  const size_t total = (size_t)n_tiles * k_tiles * 64;
  if (chunk >= total) return;
  const int lane = (int)(chunk & 63);
  const size_t tile = chunk >> 6;
  const int kt = (int)(tile % k_tiles), nt = (int)(tile / k_tiles);
  const int k = kt * 32 + (lane >> 4) * 8;
  const bf16_t* src = src0;
  int n;
  if (interleave) {
    src = (nt & 1) ? src1 : src0;
    n = (nt >> 1) * 16 + (lane & 15);
  } else {
    n = nt * 16 + (lane & 15);
  }
  v4u v = {0u, 0u, 0u, 0u};
  if (n < N && k < K) {
    const v4u raw = *reinterpret_cast<const v4u*>(src + (size_t)n * K + k);
    bool overflow = false;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const float lo = __uint_as_float(raw[e] << 16), hi = __uint_as_float(raw[e] & 0xffff0000u);
      overflow |= !(fabsf(lo) <= 65504.f) || !(fabsf(hi) <= 65504.f);
      v[e] = pack_h16x2(lo, hi);
    }
    if (overflow) atomicOr(err_flag, 2);
  }
  *reinterpret_cast<v4u*>(dst + chunk * 8) = v;
}
void retile_weight(h16_t* dst, const bf16_t* src, int N, int K, int n_tiles, int k_tiles, int* err_flag,
                   hipStream_t st) {
  const size_t total = (size_t)n_tiles * k_tiles * 64;
  k_retile<<<(unsigned)((total + 255) / 256), 256, 0, st>>>(dst, src, nullptr, N, K, n_tiles, k_tiles, 0, err_flag);
}
void retile_gate_up(h16_t* dst, const bf16_t* gate, const bf16_t* up, int F, int K, int f_tiles,
                    int k_tiles, int* err_flag, hipStream_t st) {
  const size_t total = (size_t)2 * f_tiles * k_tiles * 64;
  k_retile<<<(unsigned)((total + 255) / 256), 256, 0, st>>>(dst, gate, up, F, K, 2 * f_tiles, k_tiles, 1, err_flag);
}

// The embedding table stays bf16 (it is gathered, not multiplied): only its finiteness is checked at load.
__global__ void k_check_finite_bf16(const bf16_t* src, size_t n, int* err_flag) {
  bool bad = false;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x)
    bad |= (src[i] & 0x7f80u) == 0x7f80u;  // exponent all ones: infinity or NaN
  if (bad) atomicOr(err_flag, 2);
}
void check_finite_bf16(const bf16_t* src, size_t n, int* err_flag, hipStream_t st) {
  if (n == 0) return;
  k_check_finite_bf16<<<1024, 256, 0, st>>>(src, n, err_flag);
}

// ---------------------------------------------------------------- control
__global__ void k_set_ctl(SampleCtl* dst, SampleCtl v) { *dst = v; }
void set_sample_ctl(SampleCtl* dst, const SampleCtl& v, hipStream_t st) { k_set_ctl<<<1, 1, 0, st>>>(dst, v); }

// ---------------------------------------------------------------- embedding
__global__ void k_embed(float* h, const int* ids, const bf16_t* E, int d, int vocab, int* err_flag,
                        const int* d_rows) {
  const int t = blockIdx.x;
  if (d_rows && t >= *d_rows) {
    // rows packed on the device: no token here.  The rows that share a 256-row block with tokens still go through
    // the matrix kernels: they are cleared, so that what is computed from them is zero (and finite)
    if (t < ((*d_rows + 255) & ~255))
      for (int c = threadIdx.x; c < d; c += blockDim.x) h[(size_t)t * d + c] = 0.f;
    return;
  }
  int id = ids[t];
  if (id < 0 || id >= vocab) {
    if (threadIdx.x == 0) atomicOr(err_flag, 1);
    id = id < 0 ? 0 : vocab - 1;
  }
  for (int c = threadIdx.x; c < d; c += blockDim.x) h[(size_t)t * d + c] = bf16_to_f32(E[(size_t)id * d + c]);
}
void embed(float* h, const int* ids, int T, const bf16_t* E, int d, int vocab, int* err_flag, hipStream_t st,
           const int* d_rows) {
  if (T == 0) return;
  k_embed<<<T, 256, 0, st>>>(h, ids, E, d, vocab, err_flag, d_rows);
}

// ---------------------------------------------------------------- residual add + RMSNorm
// One workgroup per row; a thread owns 8 consecutive features (one 16-byte chunk of the tiled
// operand).  Pass 1 folds the split-K partial sums into the fp32 residual and accumulates the
// sum of squares; pass 2 writes bf16(h * rsqrt(mean + eps) * gain).
__global__ __launch_bounds__(256) void k_add_norm(float* h, const float* P, int n_split, int ldp, int Mpad_p,
                                                  const float* gain, float eps, h16_t* x, int Mpad, int d,
                                                  int* err_flag, const int* d_rows) {
  __shared__ float red[16];
  const int m = blockIdx.x;
  if (d_rows && m >= ((*d_rows + 255) & ~255)) return;  // rows packed on the device: no token in this 256-row block
  float* hr = h + (size_t)m * d;
  float ss = 0.f;
  for (int k = threadIdx.x * 8; k < d; k += blockDim.x * 8) {
    v4f a = *reinterpret_cast<const v4f*>(hr + k), b = *reinterpret_cast<const v4f*>(hr + k + 4);
#pragma unroll 8
    for (int s = 0; s < n_split; ++s) {
      const float* pr = P + ((size_t)s * Mpad_p + m) * ldp + k;
      a = a + *reinterpret_cast<const v4f*>(pr);
      b = b + *reinterpret_cast<const v4f*>(pr + 4);
    }
    if (n_split > 0) {
      *reinterpret_cast<v4f*>(hr + k) = a;
      *reinterpret_cast<v4f*>(hr + k + 4) = b;
    }
#pragma unroll
    for (int e = 0; e < 4; ++e) ss += a[e] * a[e] + b[e] * b[e];
  }
  ss = block_sum(ss, red);
  const float r = 1.0f / sqrtf(ss / (float)d + eps);
  for (int k = threadIdx.x * 8; k < d; k += blockDim.x * 8) {
    const v4f a = *reinterpret_cast<const v4f*>(hr + k), b = *reinterpret_cast<const v4f*>(hr + k + 4);
    const v4f ga = *reinterpret_cast<const v4f*>(gain + k), gb = *reinterpret_cast<const v4f*>(gain + k + 4);
    v4u pk;
    pk[0] = pack_h16x2_flag(a[0] * r * ga[0], a[1] * r * ga[1], err_flag);
    pk[1] = pack_h16x2_flag(a[2] * r * ga[2], a[3] * r * ga[3], err_flag);
    pk[2] = pack_h16x2_flag(b[0] * r * gb[0], b[1] * r * gb[1], err_flag);
    pk[3] = pack_h16x2_flag(b[2] * r * gb[2], b[3] * r * gb[3], err_flag);
    *reinterpret_cast<v4u*>(x + act_off(m, k, Mpad)) = pk;
  }
}
// Large-batch form without partial sums: one workgroup per tile of 16 rows, 16 threads per row.  The
// normalised row tile is collected in LDS (row-major, rows 16 bytes longer than d values so that both the
// row-wise writes and the column-wise reads below are free of bank conflicts) and leaves as whole 1 KiB blocks
// of the fragment layout (the per-row kernel above writes 16 bytes of every 256: sixteen workgroups share
// each cache line).
__global__ __launch_bounds__(256) void k_norm_tile16(const float* __restrict__ h, const float* __restrict__ gain,
                                                     float eps, h16_t* x, int M, int m_tiles, int d,
                                                     int* err_flag, const int* d_rows) {
  extern __shared__ __attribute__((aligned(16))) uint8_t xs[];  // 16 rows of 2 d + 16 bytes
  const int row_bytes = 2 * d + 16;
  const int mt = blockIdx.x, r = threadIdx.x >> 4, sub = threadIdx.x & 15;
  if (d_rows && mt * 16 >= ((*d_rows + 255) & ~255)) return;  // rows packed on the device: no token in this 256-row block
  const int m = mt * 16 + r;
  const bool valid = m < M;
  const float* hr = h + (size_t)min(m, M - 1) * d;
  // the row is read once: up to kKeep chunks of 8 values per thread stay in registers between the two passes
  constexpr int kKeep = 12;  // d <= 1536; wider rows read their tail a second time (from cache)
  v4f ka[kKeep], kb[kKeep];
  float ss = 0.f;
#pragma unroll
  for (int it = 0; it < kKeep; ++it) {
    const int k = sub * 8 + it * 128;
    ka[it] = kb[it] = v4f{0.f, 0.f, 0.f, 0.f};
    if (k < d) {
      ka[it] = *reinterpret_cast<const v4f*>(hr + k);
      kb[it] = *reinterpret_cast<const v4f*>(hr + k + 4);
    }
#pragma unroll
    for (int e = 0; e < 4; ++e) ss += ka[it][e] * ka[it][e] + kb[it][e] * kb[it][e];
  }
  for (int k = sub * 8 + kKeep * 128; k < d; k += 128) {
    const v4f a = *reinterpret_cast<const v4f*>(hr + k), b = *reinterpret_cast<const v4f*>(hr + k + 4);
#pragma unroll
    for (int e = 0; e < 4; ++e) ss += a[e] * a[e] + b[e] * b[e];
  }
#pragma unroll
  for (int o = 1; o < 16; o <<= 1) ss += __shfl_xor(ss, o, 64);  // the 16 threads of a row are adjacent lanes
  const float rr = valid ? 1.0f / sqrtf(ss / (float)d + eps) : 0.f;  // padding rows become zeros
  auto emit = [&](int k, const v4f& a, const v4f& b) {
    const v4f ga = *reinterpret_cast<const v4f*>(gain + k), gb = *reinterpret_cast<const v4f*>(gain + k + 4);
    v4u pk;
    pk[0] = pack_h16x2_flag(a[0] * rr * ga[0], a[1] * rr * ga[1], err_flag);
    pk[1] = pack_h16x2_flag(a[2] * rr * ga[2], a[3] * rr * ga[3], err_flag);
    pk[2] = pack_h16x2_flag(b[0] * rr * gb[0], b[1] * rr * gb[1], err_flag);
    pk[3] = pack_h16x2_flag(b[2] * rr * gb[2], b[3] * rr * gb[3], err_flag);
    *reinterpret_cast<v4u*>(xs + r * row_bytes + k * 2) = pk;
  };
#pragma unroll
  for (int it = 0; it < kKeep; ++it) {
    const int k = sub * 8 + it * 128;
    if (k < d) emit(k, ka[it], kb[it]);
  }
  for (int k = sub * 8 + kKeep * 128; k < d; k += 128)
    emit(k, *reinterpret_cast<const v4f*>(hr + k), *reinterpret_cast<const v4f*>(hr + k + 4));
  __syncthreads();
  // block kt of the fragment layout: piece (dim group dg, row) = 8 values of one row, at offset 16 (16 dg + row)
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  uint8_t* dst = reinterpret_cast<uint8_t*>(x);
  for (int kt = wave; kt < d / 32; kt += 4)
    *reinterpret_cast<v4u*>(dst + ((size_t)kt * m_tiles + mt) * 1024 + lane * 16) =
        *reinterpret_cast<const v4u*>(xs + (lane & 15) * row_bytes + (kt * 32 + (lane >> 4) * 8) * 2);
}

void add_norm(float* h, const float* P, int n_split, int ldp, int Mpad_p, const float* gain, float eps,
              h16_t* x, int M, int m_tiles, int d, int* err_flag, hipStream_t st, const int* d_rows) {
  if (M == 0) return;
  if (n_split == 0 && M >= 1024 && d % 32 == 0 && d * 32 + 256 <= 160 * 1024) {
    static bool configured = false;
    if (!configured) {
      (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&k_norm_tile16), hipFuncAttributeMaxDynamicSharedMemorySize,
                                160 * 1024);
      configured = true;
    }
    k_norm_tile16<<<(M + 15) / 16, 256, 16 * (2 * d + 16), st>>>(h, gain, eps, x, M, m_tiles, d, err_flag, d_rows);
    return;
  }
  k_add_norm<<<M, 256, 0, st>>>(h, P, n_split, ldp, Mpad_p, gain, eps, x, m_tiles * 16, d, err_flag, d_rows);
}

// ---------------------------------------------------------------- rotary embedding + KV write
// qkv [T, (Hq + 2 Hkv) HD] fp32 (row stride ld).  q heads are rotated and stored fp16 row-major [T, Hq HD];
// k heads are rotated and written into the K pages ([dim/8][token][dim%8]); v into the V pages ([dim][token]).
// Rotation pairs are (i, i + HD / 2) of a head.
//
// One workgroup per (page, sequence): the up to 16 tokens of the sequence whose positions fall into one page.
// Thread (token, quad) rotates 4 + 4 values of a head at a time.  The K and V values of a kv head are collected
// token-major in LDS and leave as the page's 16-byte pieces (one per thread, 4 KiB contiguous at HD = 128); a
// page that the launch fills only partly is written value by value for its live slots instead.
template <int HD>
__global__ __launch_bounds__(256) void k_rope_kv_page(h16_t* q, const float* qkv, int ld, int S, int Hq, int Hkv,
                                                      const float* cos, const float* sin, int row_stride, int pos_base,
                                                      KvPool pool, int layer, int* err_flag, const int* seq_start) {
  constexpr int HALF = HD / 2, QUADS = HALF / 4;  // quads of rotation pairs per head
  constexpr int ROW = HD + 8;                     // LDS row stride in halfs: 16-byte reads down a column stay conflict-free
  __shared__ __attribute__((aligned(16))) h16_t k_s[kPageTokens][ROW];
  __shared__ __attribute__((aligned(16))) h16_t v_s[kPageTokens][ROW];
  const int seq = blockIdx.y;
  // sequences of different lengths packed back to back: this one holds the tokens tok0 .. tok0 + S - 1
  size_t tok0 = (size_t)seq * S;
  if (seq_start) {
    tok0 = (size_t)seq_start[seq];
    S = seq_start[seq + 1] - seq_start[seq];
  }
  const int pg = pos_base / kPageTokens + blockIdx.x;          // page index of the sequence
  const int p_lo = max(pg * kPageTokens, pos_base), p_hi = min((pg + 1) * kPageTokens, pos_base + S);
  if (p_lo >= p_hi) return;  // whole workgroup: the sequence has no token in this page
  const bool whole = p_hi - p_lo == kPageTokens;
  const int page = pool.page_table[(size_t)seq * row_stride * pool.max_pages + pg];
  h16_t* kv = (h16_t*)pool.base;
  const size_t page_elems = (size_t)kPageTokens * HD;
  const int tid = threadIdx.x;
  // ---- rotation of the q and k heads: unit = (slot, quad)
  for (int head = 0; head < Hq + Hkv; ++head) {
    for (int u = tid; u < kPageTokens * QUADS; u += 256) {
      const int slot = u / QUADS, i = (u % QUADS) * 4;
      const int pos = pg * kPageTokens + slot;
      if (pos < p_lo || pos >= p_hi) continue;
      const size_t t = tok0 + (pos - pos_base);
      const float* pr = qkv + t * ld + (size_t)head * HD;
      const v4f a = *reinterpret_cast<const v4f*>(pr + i), b = *reinterpret_cast<const v4f*>(pr + i + HALF);
      const v4f c = *reinterpret_cast<const v4f*>(cos + (size_t)pos * HALF + i);
      const v4f sn = *reinterpret_cast<const v4f*>(sin + (size_t)pos * HALF + i);
      const v4f ra = a * c - b * sn, rb = b * c + a * sn;
      uint2 lo, hi;
      lo.x = pack_h16x2_flag(ra[0], ra[1], err_flag); lo.y = pack_h16x2_flag(ra[2], ra[3], err_flag);
      hi.x = pack_h16x2_flag(rb[0], rb[1], err_flag); hi.y = pack_h16x2_flag(rb[2], rb[3], err_flag);
      if (head < Hq) {
        h16_t* qr = q + t * Hq * HD + (size_t)head * HD;
        *reinterpret_cast<uint2*>(qr + i) = lo;
        *reinterpret_cast<uint2*>(qr + i + HALF) = hi;
      } else {
        *reinterpret_cast<uint2*>(&k_s[slot][i]) = lo;
        *reinterpret_cast<uint2*>(&k_s[slot][i + HALF]) = hi;
      }
    }
    if (head < Hq) continue;
    // ---- a kv head: its v values next to the rotated k values, then both pages
    const int g = head - Hq;
    for (int u = tid; u < kPageTokens * (HD / 4); u += 256) {
      const int slot = u / (HD / 4), i = (u % (HD / 4)) * 4;
      const int pos = pg * kPageTokens + slot;
      if (pos < p_lo || pos >= p_hi) continue;
      const size_t t = tok0 + (pos - pos_base);
      const v4f v = *reinterpret_cast<const v4f*>(qkv + t * ld + (size_t)(Hq + Hkv + g) * HD + i);
      uint2 pk;
      pk.x = pack_h16x2_flag(v[0], v[1], err_flag); pk.y = pack_h16x2_flag(v[2], v[3], err_flag);
      *reinterpret_cast<uint2*>(&v_s[slot][i]) = pk;
    }
    __syncthreads();
    h16_t* kp = kv + ((((size_t)layer * 2 + 0) * pool.n_pages + page) * pool.n_kv_heads + g) * page_elems;
    h16_t* vp = kv + ((((size_t)layer * 2 + 1) * pool.n_pages + page) * pool.n_kv_heads + g) * page_elems;
    if (whole) {
      // K piece (dim group dg, token): 8 dims of one token.  V piece (dim c, token half th): 8 tokens of one dim.
      for (int u = tid; u < kPageTokens * HD / 8; u += 256) {
        const int dg = u / kPageTokens, tok = u % kPageTokens;
        *reinterpret_cast<v4u*>(kp + (size_t)u * 8) = *reinterpret_cast<const v4u*>(&k_s[tok][dg * 8]);
        const int c = u >> 1, th = u & 1;
        v4u col;
#pragma unroll
        for (int e = 0; e < 4; ++e)
          col[e] = (uint32_t)v_s[th * 8 + 2 * e][c] | ((uint32_t)v_s[th * 8 + 2 * e + 1][c] << 16);
        *reinterpret_cast<v4u*>(vp + (size_t)u * 8) = col;
      }
    } else {
      for (int u = tid; u < kPageTokens * HD; u += 256) {
        const int slot = u / HD, c = u % HD;
        const int pos = pg * kPageTokens + slot;
        if (pos < p_lo || pos >= p_hi) continue;
        kp[(c >> 3) * 128 + slot * 8 + (c & 7)] = k_s[slot][c];
        vp[c * kPageTokens + slot] = v_s[slot][c];
      }
    }
    __syncthreads();  // the next kv head reuses k_s / v_s
  }
}
void rope_kv_write(h16_t* q, const float* qkv, int ld, int T, int S, int Hq, int Hkv, const float* cos,
                   const float* sin, TokMap map, KvPool pool, int layer, int* err_flag, hipStream_t st,
                   const int* seq_start, int n_seqs) {
  if (seq_start ? (n_seqs == 0 || S == 0) : T == 0) return;
  // pages that the positions pos_base .. pos_base + S - 1 of a sequence touch
  const int n_pg = (map.pos_base + S - 1) / kPageTokens - map.pos_base / kPageTokens + 1;
  const dim3 grid(n_pg, seq_start ? n_seqs : T / S);
  if (pool.head_dim == 64)
    k_rope_kv_page<64><<<grid, 256, 0, st>>>(q, qkv, ld, S, Hq, Hkv, cos, sin, map.row_stride, map.pos_base, pool, layer,
                                             err_flag, seq_start);
  else
    k_rope_kv_page<128><<<grid, 256, 0, st>>>(q, qkv, ld, S, Hq, Hkv, cos, sin, map.row_stride, map.pos_base, pool,
                                              layer, err_flag, seq_start);
}

}  // namespace bf16
}  // namespace mtmc
