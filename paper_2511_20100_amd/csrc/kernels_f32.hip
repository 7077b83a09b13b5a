// fp32 path: plain HIP kernels for the small all-fp32 configuration, plus the layout/control
// kernels both paths use.  Correctness vehicle; the bf16 path has its own tuned kernels.
#include <algorithm>

#include "device_utils.h"
#include "kernels.h"

namespace mtmc {

// =====================================================================================
// layout / control
// =====================================================================================
__global__ void k_build_page_table(int* table, int rows, int max_pages, int n_samples, int n_full,
                                   int shared_total) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= rows * max_pages) return;
  const int b = i / max_pages, j = i % max_pages;
  table[i] = (j < n_full) ? (b / n_samples) * n_full + j
                          : shared_total + b * (max_pages - n_full) + (j - n_full);
}
void launch_build_page_table(int* table, int rows, int max_pages, int n_samples, int n_full,
                             int shared_total, hipStream_t st) {
  const int n = rows * max_pages;
  k_build_page_table<<<(n + 255) / 256, 256, 0, st>>>(table, rows, max_pages, n_samples, n_full,
                                                     shared_total);
}

__global__ void k_set_int(int* p, int v) { *p = v; }
__global__ void k_add_int(int* p, int v) { *p += v; }
void launch_set_int(int* p, int v, hipStream_t st) { k_set_int<<<1, 1, 0, st>>>(p, v); }
void launch_add_int(int* p, int v, hipStream_t st) { k_add_int<<<1, 1, 0, st>>>(p, v); }

__global__ void k_fill_u32(uint32_t* p, uint32_t v, size_t n) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n;
       i += (size_t)gridDim.x * blockDim.x)
    p[i] = v;
}
void launch_fill_u32(uint32_t* p, uint32_t v, size_t n, hipStream_t st) {
  if (n == 0) return;
  const int blocks = (int)((n + 255) / 256 < 2048 ? (n + 255) / 256 : 2048);
  k_fill_u32<<<blocks, 256, 0, st>>>(p, v, n);
}

// Plain 16-byte-per-lane copy: a kernel of exactly known traffic for calibrating byte counters.
__global__ void k_copy_probe(uint4* dst, const uint4* src, size_t n) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x)
    dst[i] = src[i];
}
void launch_copy_probe(void* dst, const void* src, size_t bytes, hipStream_t st) {
  const size_t n = bytes / 16;
  if (n == 0) return;
  k_copy_probe<<<4096, 256, 0, st>>>((uint4*)dst, (const uint4*)src, n);
}

__global__ void k_gather_rows(float* dst, const float* src, int d, int n_rep, int src_stride,
                              int src_offset, int rep_stride) {
  const int r = blockIdx.x;
  const size_t s = (size_t)(r / n_rep) * src_stride + src_offset + (size_t)(r % n_rep) * rep_stride;
  for (int c = threadIdx.x; c < d; c += blockDim.x) dst[(size_t)r * d + c] = src[s * d + c];
}
void launch_gather_rows(float* dst, const float* src, int rows, int d, int n_rep, int src_stride,
                        int src_offset, int rep_stride, hipStream_t st) {
  if (rows == 0) return;
  k_gather_rows<<<rows, 256, 0, st>>>(dst, src, d, n_rep, src_stride, src_offset, rep_stride);
}

__global__ void k_fork_tail_pages(KvPool pool, int n_samples, int page_idx, int words_per_page) {
  const int b = blockIdx.x;
  if (b % n_samples == 0) return;
  const int lw = blockIdx.y;  // layer * 2 + which
  const int src = pool.page_table[(size_t)(b - b % n_samples) * pool.max_pages + page_idx];
  const int dst = pool.page_table[(size_t)b * pool.max_pages + page_idx];
  const uint32_t* s = (const uint32_t*)pool.base + ((size_t)lw * pool.n_pages + src) * words_per_page;
  uint32_t* d = (uint32_t*)pool.base + ((size_t)lw * pool.n_pages + dst) * words_per_page;
  for (int i = threadIdx.x; i < words_per_page; i += blockDim.x) d[i] = s[i];
}
void launch_fork_tail_pages(KvPool pool, int n_layers, int rows, int n_samples, int page_idx,
                            int elem_bytes, hipStream_t st) {
  const int words = pool.n_kv_heads * kPageTokens * pool.head_dim * elem_bytes / 4;
  k_fork_tail_pages<<<dim3(rows, n_layers * 2), 256, 0, st>>>(pool, n_samples, page_idx, words);
}

// =====================================================================================
// rollout of prompts of different lengths
// =====================================================================================
__device__ __forceinline__ int clamp_len(int len, int Lmax) { return min(max(len, 1), Lmax); }

__global__ void k_ragged_setup(int* table, int* row_pos, int* done, int* out_lens, int* prompt_ids, int* suffix_ids,
                               const int* prompts, const int* lens, int n_samples, int Lmax, int max_pages,
                               int nf_max, int shared_total, int max_new, int reuse_len, int* err_flag) {
  const int b = blockIdx.x, p = b / n_samples;
  const int raw = lens[p], len = clamp_len(raw, Lmax);
  if (threadIdx.x == 0) {
    if (raw != len) atomicOr(err_flag, 4);
    // cached prefix: the previous call's prompt (row_pos still holds its last position) must cover it, and
    // the new prompt must reach beyond it
    if (reuse_len > 0 && (row_pos[b] + 1 < reuse_len || len <= reuse_len)) atomicOr(err_flag, 16);
    row_pos[b] = len - 1;
    done[b] = 0;
    out_lens[b] = max_new;
  }
  const int n_full = len / kPageTokens;
  for (int j = threadIdx.x; j < max_pages; j += blockDim.x)
    table[(size_t)b * max_pages + j] = (j < n_full) ? p * nf_max + j : shared_total + b * max_pages + j;
  if (b % n_samples == 0) {
    bool changed = false;
    for (int j = threadIdx.x; j < Lmax; j += blockDim.x) {
      const int id = (j < len) ? prompts[(size_t)p * Lmax + j] : 0;
      if (j < reuse_len) changed |= prompt_ids[(size_t)p * Lmax + j] != id;
      else suffix_ids[(size_t)p * (Lmax - reuse_len) + (j - reuse_len)] = id;
      prompt_ids[(size_t)p * Lmax + j] = id;
    }
    if (changed) atomicOr(err_flag, 16);
  }
}
void launch_ragged_setup(int* table, int* row_pos, int* done, int* out_lens, int* prompt_ids, int* suffix_ids,
                         const int* prompts, const int* lens, int n_prompts, int n_samples, int Lmax, int max_pages,
                         int nf_max, int shared_total, int max_new, int reuse_len, int* err_flag, hipStream_t st) {
  k_ragged_setup<<<n_prompts * n_samples, 256, 0, st>>>(table, row_pos, done, out_lens, prompt_ids, suffix_ids,
                                                        prompts, lens, n_samples, Lmax, max_pages, nf_max,
                                                        shared_total, max_new, reuse_len, err_flag);
}

__global__ void k_fork_tail_pages_ragged(KvPool pool, int n_samples, const int* lens, int Lmax, int words_per_page) {
  const int b = blockIdx.x;
  if (b % n_samples == 0) return;
  const int len = clamp_len(lens[b / n_samples], Lmax);
  if (len % kPageTokens == 0) return;
  const int page_idx = len / kPageTokens;
  const int lw = blockIdx.y;  // layer * 2 + which
  const int src = pool.page_table[(size_t)(b - b % n_samples) * pool.max_pages + page_idx];
  const int dst = pool.page_table[(size_t)b * pool.max_pages + page_idx];
  const uint32_t* s = (const uint32_t*)pool.base + ((size_t)lw * pool.n_pages + src) * words_per_page;
  uint32_t* d = (uint32_t*)pool.base + ((size_t)lw * pool.n_pages + dst) * words_per_page;
  for (int i = threadIdx.x; i < words_per_page; i += blockDim.x) d[i] = s[i];
}
void launch_fork_tail_pages_ragged(KvPool pool, int n_layers, int rows, int n_samples, const int* lens, int Lmax,
                                   int elem_bytes, hipStream_t st) {
  const int words = pool.n_kv_heads * kPageTokens * pool.head_dim * elem_bytes / 4;
  k_fork_tail_pages_ragged<<<dim3(rows, n_layers * 2), 256, 0, st>>>(pool, n_samples, lens, Lmax, words);
}

__global__ void k_gather_last_rows(float* dst, const float* src, int d, int n_samples, int Lmax, const int* lens,
                                   int pos_base) {
  const int r = blockIdx.x, p = r / n_samples;
  const size_t s = (size_t)p * (Lmax - pos_base) + max(clamp_len(lens[p], Lmax) - 1 - pos_base, 0);
  for (int c = threadIdx.x; c < d; c += blockDim.x) dst[(size_t)r * d + c] = src[s * d + c];
}
void launch_gather_last_rows(float* dst, const float* src, int d, int n_prompts, int n_samples, int Lmax,
                             const int* lens, int pos_base, hipStream_t st) {
  if (n_prompts == 0) return;
  k_gather_last_rows<<<n_prompts * n_samples, 256, 0, st>>>(dst, src, d, n_samples, Lmax, lens, pos_base);
}

// =====================================================================================
// action-level scoring: inputs of the two passes, and the sums / softmax over the candidates
// =====================================================================================
// Row b = n K + k of vseq is [last state token, action tokens ..., 0 padding]; prefix row n is the
// state without its last token.
__global__ void k_build_action_seqs(int* vseq, int* prefix, const int* states, const int* actions,
                                    const int* action_len, int n_states, int P, int K, int A, int* err_flag) {
  const int W = A + 1;
  const size_t n_v = (size_t)n_states * K * W, n_p = (size_t)n_states * (P - 1);
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n_v + n_p;
       i += (size_t)gridDim.x * blockDim.x) {
    if (i < n_v) {
      const int b = (int)(i / W), j = (int)(i % W);
      int len = action_len[b];
      if (len < 0 || len > A) {
        if (j == 0) atomicOr(err_flag, 4);
        len = len < 0 ? 0 : A;
      }
      vseq[i] = (j == 0) ? states[(size_t)(b / K) * P + P - 1] : (j <= len ? actions[(size_t)b * A + j - 1] : 0);
    } else {
      const size_t r = i - n_v;
      prefix[r] = states[(r / (P - 1)) * P + r % (P - 1)];
    }
  }
}
void launch_build_action_seqs(int* vseq, int* prefix, const int* states, const int* actions,
                              const int* action_len, int n_states, int P, int K, int A, int* err_flag,
                              hipStream_t st) {
  const size_t n = (size_t)n_states * K * (A + 1) + (size_t)n_states * (P - 1);
  const int blocks = (int)std::min<size_t>((n + 255) / 256, 2048);
  k_build_action_seqs<<<blocks, 256, 0, st>>>(vseq, prefix, states, actions, action_len, n_states, P, K, A,
                                              err_flag);
}

// One workgroup per state.  Candidate k: padding terms of token_lp are cleared, the others summed
// in position order (double), divided by the length if asked; then the log-softmax over the K
// sums, with the maximum and the sum of exponentials reduced in a fixed tree order.
__global__ __launch_bounds__(256) void k_action_reduce(float* token_lp, const int* action_len, int K, int A,
                                                       int normalize, float* out_action, float* out_policy) {
  __shared__ double red[256];
  const int n = blockIdx.x, tid = threadIdx.x;
  auto total_of = [&](int k) {
    const int b = n * K + k;
    const int len = min(max(action_len[b], 0), A);
    const float* row = token_lp + (size_t)b * A;
    double s = 0.0;
    for (int j = 0; j < len; ++j) s += (double)row[j];
    return (normalize && len > 0) ? s / (double)len : s;
  };
  auto block_reduce = [&](double v, bool take_max) {
    red[tid] = v;
    __syncthreads();
    for (int w = 128; w > 0; w >>= 1) {
      if (tid < w) red[tid] = take_max ? fmax(red[tid], red[tid + w]) : red[tid] + red[tid + w];
      __syncthreads();
    }
    const double r = red[0];
    __syncthreads();
    return r;
  };
  double mx = -INFINITY;
  for (int k = tid; k < K; k += 256) {
    const int b = n * K + k;
    const int len = min(max(action_len[b], 0), A);
    for (int j = len; j < A; ++j) token_lp[(size_t)b * A + j] = 0.f;
    const double t = total_of(k);
    out_action[b] = (float)t;
    mx = fmax(mx, t);
  }
  mx = block_reduce(mx, true);
  double se = 0.0;
  for (int k = tid; k < K; k += 256) se += exp(total_of(k) - mx);
  se = block_reduce(se, false);
  const double lse = mx + log(se);
  for (int k = tid; k < K; k += 256) out_policy[n * K + k] = (float)(total_of(k) - lse);
}
void launch_action_reduce(float* token_lp, const int* action_len, int n_states, int K, int A, int normalize,
                          float* out_action, float* out_policy, hipStream_t st) {
  k_action_reduce<<<n_states, 256, 0, st>>>(token_lp, action_len, K, A, normalize, out_action, out_policy);
}

namespace f32 {

// =====================================================================================
// embedding, RMSNorm, SwiGLU
// =====================================================================================
__global__ void k_embed(float* h, const int* ids, const float* E, int d, int vocab, int* err_flag) {
  const int t = blockIdx.x;
  int id = ids[t];
  if (id < 0 || id >= vocab) {
    if (threadIdx.x == 0) atomicOr(err_flag, 1);
    id = id < 0 ? 0 : vocab - 1;
  }
  for (int c = threadIdx.x; c < d; c += blockDim.x) h[(size_t)t * d + c] = E[(size_t)id * d + c];
}
void embed(float* h, const int* ids, int T, const float* E, int d, int vocab, int* err_flag,
           hipStream_t st) {
  k_embed<<<T, 256, 0, st>>>(h, ids, E, d, vocab, err_flag);
}

__global__ void k_rmsnorm(float* x, const float* h, const float* gain, float eps, int d) {
  __shared__ float red[16];
  const size_t row = (size_t)blockIdx.x * d;
  float ss = 0.f;
  for (int c = threadIdx.x; c < d; c += blockDim.x) {
    const float v = h[row + c];
    ss += v * v;
  }
  ss = block_sum(ss, red);
  const float r = 1.0f / sqrtf(ss / (float)d + eps);
  for (int c = threadIdx.x; c < d; c += blockDim.x) x[row + c] = h[row + c] * r * gain[c];
}
void rmsnorm(float* x, const float* h, const float* gain, float eps, int T, int d, hipStream_t st) {
  k_rmsnorm<<<T, 256, 0, st>>>(x, h, gain, eps, d);
}

__global__ void k_swiglu(float* a, const float* gu, size_t n, int F) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  const size_t t = i / F, c = i % F;
  const float g = gu[t * 2 * F + c], u = gu[t * 2 * F + F + c];
  a[i] = g / (1.0f + expf(-g)) * u;
}
void swiglu(float* a, const float* gu, int T, int F, hipStream_t st) {
  const size_t n = (size_t)T * F;
  k_swiglu<<<(unsigned)((n + 255) / 256), 256, 0, st>>>(a, gu, n, F);
}

// =====================================================================================
// GEMM: C[M, N] (+)= A[M, K] W[N, K]^T, 64x64 tile per block, 4x4 per thread, K step 16
// =====================================================================================
__global__ __launch_bounds__(256) void k_gemm(float* C, int ldc, const float* A, int lda,
                                              const float* W, int M, int N, int K, int accumulate) {
  __shared__ float As[16][64 + 4];
  __shared__ float Ws[16][64 + 4];
  const int tid = threadIdx.x;
  const int m0 = blockIdx.y * 64, n0 = blockIdx.x * 64;
  const int lr = tid >> 2, lk = (tid & 3) * 4;  // load: row lr of the tile, k offset lk..lk+3
  const int tm = (tid >> 4) * 4, tn = (tid & 15) * 4;
  float acc[4][4] = {};
  for (int k0 = 0; k0 < K; k0 += 16) {
    float4 a = make_float4(0.f, 0.f, 0.f, 0.f), w = a;
    if (m0 + lr < M) a = *(const float4*)(A + (size_t)(m0 + lr) * lda + k0 + lk);
    if (n0 + lr < N) w = *(const float4*)(W + (size_t)(n0 + lr) * K + k0 + lk);
    __syncthreads();
    As[lk + 0][lr] = a.x; As[lk + 1][lr] = a.y; As[lk + 2][lr] = a.z; As[lk + 3][lr] = a.w;
    Ws[lk + 0][lr] = w.x; Ws[lk + 1][lr] = w.y; Ws[lk + 2][lr] = w.z; Ws[lk + 3][lr] = w.w;
    __syncthreads();
#pragma unroll
    for (int k = 0; k < 16; ++k) {
      float av[4], wv[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) { av[i] = As[k][tm + i]; wv[i] = Ws[k][tn + i]; }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(av[i], wv[j], acc[i][j]);
    }
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int m = m0 + tm + i;
    if (m >= M) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int n = n0 + tn + j;
      if (n >= N) continue;
      float* c = C + (size_t)m * ldc + n;
      *c = accumulate ? (*c + acc[i][j]) : acc[i][j];
    }
  }
}
void gemm(float* C, int ldc, const float* A, int lda, const float* W, int M, int N, int K,
          bool accumulate, hipStream_t st) {
  if (M == 0 || N == 0) return;
  k_gemm<<<dim3((N + 63) / 64, (M + 63) / 64), 256, 0, st>>>(C, ldc, A, lda, W, M, N, K,
                                                            accumulate ? 1 : 0);
}

// =====================================================================================
// rotary embedding + KV page write; attention over the pages
// =====================================================================================
__device__ __forceinline__ float* page_ptr(const KvPool& pool, int layer, int which, int page, int g) {
  return (float*)pool.base +
         ((((size_t)layer * 2 + which) * pool.n_pages + page) * pool.n_kv_heads + g) *
             (size_t)(kPageTokens * pool.head_dim);
}

__global__ void k_rope_kv_write(float* qkv, int Hq, int Hkv, int hd, const float* cos,
                                const float* sin, TokMap map, KvPool pool, int layer) {
  const int t = blockIdx.x;
  const int pos = tok_pos(map, t);
  const int row = tok_seq(map, t) * map.row_stride;
  const int page = pool.page_table[(size_t)row * pool.max_pages + pos / kPageTokens];
  const int slot = pos % kPageTokens;
  const int half = hd / 2;
  float* base = qkv + (size_t)t * (Hq + 2 * Hkv) * hd;
  // q and k heads: rotate pairs (i, i + hd/2)
  for (int e = threadIdx.x; e < (Hq + Hkv) * half; e += blockDim.x) {
    const int head = e / half, i = e % half;
    const float c = cos[(size_t)pos * half + i], s = sin[(size_t)pos * half + i];
    float* w = base + (size_t)head * hd;
    const float a = w[i], b = w[i + half];
    const float ra = a * c - b * s, rb = b * c + a * s;
    if (head < Hq) {
      w[i] = ra;
      w[i + half] = rb;
    } else {
      float* kp = page_ptr(pool, layer, 0, page, head - Hq) + (size_t)slot * hd;
      kp[i] = ra;
      kp[i + half] = rb;
    }
  }
  for (int e = threadIdx.x; e < Hkv * hd; e += blockDim.x) {
    const int g = e / hd, c = e % hd;
    page_ptr(pool, layer, 1, page, g)[(size_t)slot * hd + c] = base[(size_t)(Hq + Hkv) * hd + e];
  }
}
void rope_kv_write(float* qkv, int T, int Hq, int Hkv, int hd, const float* cos, const float* sin,
                   TokMap map, KvPool pool, int layer, hipStream_t st) {
  k_rope_kv_write<<<T, 128, 0, st>>>(qkv, Hq, Hkv, hd, cos, sin, map, pool, layer);
}

// One block (128 threads) per (token, query head).  Keys are taken 128 at a time with an
// online softmax; thread i scores key i, then thread c accumulates output component c.
__global__ __launch_bounds__(128) void k_attention(float* o, const float* qkv, int Hq, int Hkv,
                                                   int hd, TokMap map, KvPool pool, int layer) {
  __shared__ float q[128];
  __shared__ float p[128];
  __shared__ float red[16];
  const int t = blockIdx.x, j = blockIdx.y;
  const int g = j / (Hq / Hkv);
  const int pos = tok_pos(map, t);
  const int* table = pool.page_table + (size_t)tok_seq(map, t) * map.row_stride * pool.max_pages;
  const int tid = threadIdx.x;
  const float scale = 1.0f / sqrtf((float)hd);
  if (tid < hd) q[tid] = qkv[(size_t)t * (Hq + 2 * Hkv) * hd + (size_t)j * hd + tid];
  __syncthreads();
  float m = -INFINITY, l = 0.f, acc = 0.f;
  const int n_ctx = pos + 1;
  for (int c0 = 0; c0 < n_ctx; c0 += 128) {
    const int key = c0 + tid;
    float s = -INFINITY;
    if (key < n_ctx) {
      const float* kp = page_ptr(pool, layer, 0, table[key / kPageTokens], g) +
                        (size_t)(key % kPageTokens) * hd;
      float d = 0.f;
      for (int c = 0; c < hd; ++c) d = fmaf(q[c], kp[c], d);
      s = d * scale;
    }
    const float m_new = fmaxf(m, block_max(s, red));
    const float pe = (key < n_ctx) ? expf(s - m_new) : 0.f;
    const float corr = expf(m - m_new);  // exp(-inf) = 0 on the first chunk
    const float sum = block_sum(pe, red);
    l = l * corr + sum;
    p[tid] = pe;
    __syncthreads();
    acc *= corr;
    if (tid < hd) {
      const int n_here = min(128, n_ctx - c0);
      for (int i = 0; i < n_here; ++i) {
        const int kk = c0 + i;
        const float* vp = page_ptr(pool, layer, 1, table[kk / kPageTokens], g) +
                          (size_t)(kk % kPageTokens) * hd;
        acc = fmaf(p[i], vp[tid], acc);
      }
    }
    m = m_new;
    __syncthreads();
  }
  if (tid < hd) o[(size_t)t * Hq * hd + (size_t)j * hd + tid] = acc / l;
}
void attention(float* o, const float* qkv, int T, int Hq, int Hkv, int hd, TokMap map, KvPool pool,
               int layer, hipStream_t st) {
  k_attention<<<dim3(T, Hq), 128, 0, st>>>(o, qkv, Hq, Hkv, hd, map, pool, layer);
}

// =====================================================================================
// sampling and scoring from materialised logits
// =====================================================================================
__global__ __launch_bounds__(256) void k_sample(const float* logits, int V, float inv_temp,
                                                int greedy, uint32_t key0, uint32_t key1,
                                                uint32_t seq_offset, const int* d_step, int max_new,
                                                int* cur_ids, int* out_ids, float* out_logprobs, int stop_id,
                                                int* done, int* out_lens) {
  __shared__ Lse s_lse[4];
  __shared__ Best s_best[4];
  const int b = blockIdx.x;
  const int step = *d_step;
  const float* z = logits + (size_t)b * V;
  Lse lse = lse_empty();
  Best best = best_empty();
  for (int v4 = threadIdx.x; v4 * 4 < V; v4 += blockDim.x) {
    uint4 r = make_uint4(0, 0, 0, 0);
    if (!greedy) r = philox4x32_10(make_uint4((uint32_t)v4, (uint32_t)step, seq_offset + b, 0u), key0, key1);
    const uint32_t rr[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const int v = v4 * 4 + k;
      if (v >= V) break;
      const float zt = greedy ? z[v] : z[v] * inv_temp;
      lse_push(lse, zt);
      const float y = greedy ? zt : zt + gumbel_from_bits(rr[k]);
      best = best_merge(best, Best{y, v});
    }
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    Lse ol = {__shfl_xor(lse.m, o, 64), __shfl_xor(lse.s, o, 64)};
    Best ob = {__shfl_xor(best.y, o, 64), __shfl_xor(best.idx, o, 64)};
    lse = lse_merge(lse, ol);
    best = best_merge(best, ob);
  }
  const int lane = threadIdx.x & 63, wid = threadIdx.x >> 6;
  if (lane == 0) { s_lse[wid] = lse; s_best[wid] = best; }
  __syncthreads();
  if (threadIdx.x == 0) {
    for (int i = 1; i < 4; ++i) { lse = lse_merge(lse, s_lse[i]); best = best_merge(best, s_best[i]); }
    const float zt = greedy ? z[best.idx] : z[best.idx] * inv_temp;
    int tok = best.idx;
    float lp = zt - (lse.m + logf(lse.s));
    if (done) {
      if (done[b]) {
        tok = stop_id;
        lp = 0.f;
      } else if (tok == stop_id) {
        done[b] = 1;
        out_lens[b] = step + 1;
      }
    }
    cur_ids[b] = tok;
    out_ids[(size_t)b * max_new + step] = tok;
    out_logprobs[(size_t)b * max_new + step] = lp;
  }
}
void sample(const float* logits, int B, int V, float inv_temp, int greedy, uint64_t seed,
            uint32_t seq_offset, const int* d_step, int max_new, int* cur_ids, int* out_ids,
            float* out_logprobs, int stop_id, int* done, int* out_lens, hipStream_t st) {
  k_sample<<<B, 256, 0, st>>>(logits, V, inv_temp, greedy, (uint32_t)(seed & 0xffffffffu),
                              (uint32_t)(seed >> 32), seq_offset, d_step, max_new, cur_ids, out_ids,
                              out_logprobs, stop_id, done, out_lens);
}

__global__ __launch_bounds__(256) void k_score_rows(const float* logits, int V, const int* seqs,
                                                    int S, int first, int n_scored, int seq0,
                                                    int row0, float* out_logprobs, int* out_top1,
                                                    float* out_margin, int* err_flag) {
  __shared__ Lse s_lse[4];
  __shared__ Top2 s_top[4];
  const int r = blockIdx.x;
  const int n = seq0 + (row0 + r) / n_scored, i = first + (row0 + r) % n_scored;
  const float* z = logits + (size_t)r * V;
  Lse lse = lse_empty();
  Top2 top = top2_empty();
  for (int v = threadIdx.x; v < V; v += blockDim.x) {
    const float x = z[v];
    lse_push(lse, x);
    top2_push(top, x, v);
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    Lse ol = {__shfl_xor(lse.m, o, 64), __shfl_xor(lse.s, o, 64)};
    Top2 ot = {__shfl_xor(top.v1, o, 64), __shfl_xor(top.i1, o, 64), __shfl_xor(top.v2, o, 64)};
    lse = lse_merge(lse, ol);
    top = top2_merge(top, ot);
  }
  const int lane = threadIdx.x & 63, wid = threadIdx.x >> 6;
  if (lane == 0) { s_lse[wid] = lse; s_top[wid] = top; }
  __syncthreads();
  if (threadIdx.x == 0) {
    for (int k = 1; k < 4; ++k) { lse = lse_merge(lse, s_lse[k]); top = top2_merge(top, s_top[k]); }
    int target = seqs[(size_t)n * S + i + 1];
    if (target < 0 || target >= V) {
      atomicOr(err_flag, 1);
      target = target < 0 ? 0 : V - 1;
    }
    const size_t slot = (size_t)n * (S - 1) + i;
    out_logprobs[slot] = z[target] - (lse.m + logf(lse.s));
    if (out_top1) out_top1[slot] = top.i1;
    if (out_margin) out_margin[slot] = top.v1 - top.v2;
  }
}
void score_rows(const float* logits, int R, int V, const int* seqs, int S, int first, int n_scored,
                int seq0, int row0, float* out_logprobs, int* out_top1, float* out_margin,
                int* err_flag, hipStream_t st) {
  if (R == 0) return;
  k_score_rows<<<R, 256, 0, st>>>(logits, V, seqs, S, first, n_scored, seq0, row0, out_logprobs,
                                  out_top1, out_margin, err_flag);
}

}  // namespace f32
}  // namespace mtmc
