// Workspace plans, auxiliary tables and the fp32 schedulers.
#include <cmath>

#include "engine.h"
#include "kernels.h"

namespace mtmc {

// Tokens per prefill / scoring chunk: bounds activation memory, keeps every launch large.  The
// bf16 scoring pass takes up to 128 Ki tokens at once (about 5 GB of activations at d = 1536,
// F = 8960), so that even the narrowest GEMM of a chunk fills the 256 CUs several times over with
// 256 x 256 output blocks, and splits longer jobs into equal chunks.
static constexpr int kChunkTokens = 8192;
static constexpr int kScoreChunkTokensBf16 = 131072;
static constexpr int kMaxBf16Batch = 128;  // rows the decode GEMMs take
static constexpr size_t kLogitBytes = (size_t)256 << 20;

int build_aux(mtmc_weights* w, hipStream_t st) {
  const mtmc_config& c = w->cfg;
  const int half = c.head_dim / 2;
  const size_t n = (size_t)c.max_positions * half;
  std::vector<float> tab(2 * n);
  for (int i = 0; i < half; ++i) {
    const double theta = std::pow((double)c.rope_base, -2.0 * i / c.head_dim);
    for (int t = 0; t < c.max_positions; ++t) {
      const double ang = (double)t * theta;
      tab[(size_t)t * half + i] = (float)std::cos(ang);
      tab[n + (size_t)t * half + i] = (float)std::sin(ang);
    }
  }
  const size_t bytes = 2 * n * sizeof(float) + 256;
  if (hipMalloc(&w->aux, bytes) != hipSuccess) {
    set_error("hipMalloc failed for the rotary tables");
    return MTMC_ENOMEM;
  }
  // err flag first (256 B), then cos, then sin
  MTMC_HIP_CHECK(hipMemsetAsync(w->aux, 0, 256, st));
  MTMC_HIP_CHECK(hipMemcpyAsync((char*)w->aux + 256, tab.data(), 2 * n * sizeof(float),
                                hipMemcpyHostToDevice, st));
  MTMC_HIP_CHECK(hipStreamSynchronize(st));  // tab goes out of scope
  w->err_flag = (int*)w->aux;
  w->rope_cos = (const float*)((char*)w->aux + 256);
  w->rope_sin = w->rope_cos + n;
  return MTMC_OK;
}

RolloutPlan plan_rollout(const mtmc_weights* w, int n_prompts, int prompt_len, int n_samples,
                         int max_new, char* base, bool ragged) {
  const mtmc_config& c = w->cfg;
  const bool bf = c.dtype == MTMC_BF16;
  RolloutPlan p{};
  p.total_prompts = n_prompts;
  if (bf) n_prompts = std::min(n_prompts, std::max(1, kMaxBf16Batch / n_samples));
  p.n_prompts = n_prompts; p.prompt_len = prompt_len; p.n_samples = n_samples; p.max_new = max_new;
  p.B = n_prompts * n_samples;
  p.bt = (p.B + 15) / 16;
  p.ragged = ragged ? 1 : 0;
  p.nf_max = prompt_len / kPageTokens;
  p.n_full = ragged ? 0 : p.nf_max;
  p.max_pages = (prompt_len + max_new + kPageTokens - 1) / kPageTokens;
  p.n_regions = n_prompts;
  if (bf && ragged && p.total_prompts > n_prompts) p.n_regions = std::min({p.total_prompts, 4 * n_prompts, 128});
  p.shared_total = p.n_regions * p.nf_max;
  p.n_pages = p.shared_total + p.B * (p.max_pages - p.n_full);
  p.chunk_prompts = std::max(1, std::min(n_prompts, kChunkTokens / prompt_len));
  p.Tmax = (std::max(p.chunk_prompts * prompt_len, p.B) + 127) / 128 * 128;
  const size_t act = bf ? 2 : 4;
  const size_t d = c.d_model, nq = (size_t)c.n_q_heads * c.head_dim;
  const size_t nqkv = nq + 2 * (size_t)c.n_kv_heads * c.head_dim;
  const size_t F = bf ? w->d_ffn_pad : c.d_ffn;
  Carver cv(base);
  p.page_table = cv.take<int>((size_t)p.B * p.max_pages);
  p.d_step = cv.take<int>(64);
  // bf16, ragged: a call of several groups may run as one batch whose places pass from prompt to prompt
  const size_t n_flag_rows = (bf && ragged) ? (size_t)p.total_prompts * n_samples : (size_t)p.B;
  p.cur_ids = cv.take<int>(n_flag_rows);
  if (ragged) {
    p.row_pos = cv.take<int>(p.B);
    p.done = cv.take<int>(n_flag_rows);
    p.prompt_ids = cv.take<int>((size_t)n_prompts * prompt_len);
    p.suffix_ids = cv.take<int>((size_t)n_prompts * prompt_len);
  }
  p.kv = cv.take<char>((size_t)c.n_layers * 2 * p.n_pages * c.n_kv_heads * kPageTokens * c.head_dim * act);
  p.h = cv.take<float>((size_t)p.Tmax * d);
  p.x = cv.take<char>((size_t)p.Tmax * d * act);
  p.qkv = cv.take<float>((size_t)p.Tmax * nqkv);
  p.o = cv.take<char>((size_t)p.Tmax * nq * act);
  p.a = cv.take<char>((size_t)p.Tmax * F * act);
  p.hB = cv.take<float>((size_t)p.B * d);
  p.xB = cv.take<char>((size_t)p.bt * 16 * d * act);
  if (!bf) {
    p.gu = cv.take<float>((size_t)p.Tmax * 2 * F);
    p.logits = cv.take<float>((size_t)p.B * c.vocab);
  } else {
    bf16_plan_rollout_extra(w, p, cv);
  }
  p.total_bytes = (cv.off + 255) / 256 * 256;
  return p;
}

ScorePlan plan_score(const mtmc_weights* w, int n_seqs, int S, char* base) {
  const mtmc_config& c = w->cfg;
  const bool bf = c.dtype == MTMC_BF16;
  ScorePlan p{};
  p.n_seqs = n_seqs; p.S = S;
  p.chunk_seqs = std::max(1, std::min(n_seqs, (bf ? kScoreChunkTokensBf16 : kChunkTokens) / S));
  if (bf) {  // equal chunks
    const int n_chunks = (n_seqs + p.chunk_seqs - 1) / p.chunk_seqs;
    p.chunk_seqs = (n_seqs + n_chunks - 1) / n_chunks;
  }
  p.pages_per_seq = (S + kPageTokens - 1) / kPageTokens;
  p.n_pages = p.chunk_seqs * p.pages_per_seq;
  p.T = (p.chunk_seqs * S + 127) / 128 * 128;
  p.rows_max = (p.chunk_seqs * (S - 1) + 127) / 128 * 128;
  const size_t act = bf ? 2 : 4;
  const size_t d = c.d_model, nq = (size_t)c.n_q_heads * c.head_dim;
  const size_t nqkv = nq + 2 * (size_t)c.n_kv_heads * c.head_dim;
  const size_t F = bf ? w->d_ffn_pad : c.d_ffn;
  Carver cv(base);
  p.page_table = cv.take<int>((size_t)p.n_pages);
  p.kv = cv.take<char>((size_t)2 * p.n_pages * c.n_kv_heads * kPageTokens * c.head_dim * act);
  p.h = cv.take<float>((size_t)p.T * d);
  p.x = cv.take<char>((size_t)p.T * d * act);
  p.qkv = cv.take<float>((size_t)p.T * nqkv);
  p.o = cv.take<char>((size_t)p.T * nq * act);
  p.a = cv.take<char>((size_t)p.T * F * act);
  p.hs = cv.take<float>((size_t)p.rows_max * d);
  p.xs = cv.take<char>((size_t)p.rows_max * d * act);
  if (!bf) {
    p.gu = cv.take<float>((size_t)p.T * 2 * F);
    p.logit_rows = (int)std::max<size_t>(1, std::min<size_t>(p.rows_max, kLogitBytes / ((size_t)c.vocab * 4)));
    p.logits = cv.take<float>((size_t)p.logit_rows * c.vocab);
  } else {
    bf16_plan_score_extra(w, p, cv);
  }
  p.total_bytes = (cv.off + 255) / 256 * 256;
  return p;
}

ActionPlan plan_actions(const mtmc_weights* w, int n_states, int P, int K, int A, char* base) {
  const mtmc_config& c = w->cfg;
  const bool bf = c.dtype == MTMC_BF16;
  ActionPlan p{};
  p.n_states = n_states; p.P = P; p.K = K; p.A = A; p.B = n_states * K;
  p.Pp = P - 1; p.W = A + 1;
  p.n_full = p.Pp / kPageTokens;
  p.max_pages = (p.Pp + p.W + kPageTokens - 1) / kPageTokens;
  p.shared_total = n_states * p.n_full;
  p.n_pages = p.shared_total + p.B * (p.max_pages - p.n_full);
  const int chunk = bf ? kScoreChunkTokensBf16 : kChunkTokens;
  p.chunk_states = std::max(1, std::min(n_states, chunk / std::max(1, p.Pp)));
  p.chunk_rows = std::max(1, std::min(p.B, chunk / p.W));
  p.Tmax = (std::max(p.chunk_states * p.Pp, p.chunk_rows * p.W) + 127) / 128 * 128;
  p.rows_max = (p.chunk_rows * A + 127) / 128 * 128;
  const size_t act = bf ? 2 : 4;
  const size_t d = c.d_model, nq = (size_t)c.n_q_heads * c.head_dim;
  const size_t nqkv = nq + 2 * (size_t)c.n_kv_heads * c.head_dim;
  const size_t F = bf ? w->d_ffn_pad : c.d_ffn;
  Carver cv(base);
  p.page_table = cv.take<int>((size_t)p.B * p.max_pages);
  p.vseq = cv.take<int>((size_t)p.B * p.W);
  p.prefix = cv.take<int>((size_t)n_states * p.Pp + 1);
  p.kv = cv.take<char>((size_t)c.n_layers * 2 * p.n_pages * c.n_kv_heads * kPageTokens * c.head_dim * act);
  p.h = cv.take<float>((size_t)p.Tmax * d);
  p.x = cv.take<char>((size_t)p.Tmax * d * act);
  p.qkv = cv.take<float>((size_t)p.Tmax * nqkv);
  p.o = cv.take<char>((size_t)p.Tmax * nq * act);
  p.a = cv.take<char>((size_t)p.Tmax * F * act);
  p.hs = cv.take<float>((size_t)p.rows_max * d);
  p.xs = cv.take<char>((size_t)p.rows_max * d * act);
  if (!bf) {
    p.gu = cv.take<float>((size_t)p.Tmax * 2 * F);
    p.logit_rows = (int)std::max<size_t>(1, std::min<size_t>(p.rows_max, kLogitBytes / ((size_t)c.vocab * 4)));
    p.logits = cv.take<float>((size_t)p.logit_rows * c.vocab);
  } else {
    bf16_plan_actions_extra(w, p, cv);
  }
  p.total_bytes = (cv.off + 255) / 256 * 256;
  return p;
}

// ======================================================================================
// fp32 path
// ======================================================================================
int f32_store_weights(mtmc_weights* w, const BlobLayout& lay, const void* blob, bool on_device,
                      hipStream_t st) {
  if (hipMalloc(&w->storage, lay.total) != hipSuccess) {
    set_error("hipMalloc failed for the weights (" + std::to_string(lay.total) + " bytes)");
    return MTMC_ENOMEM;
  }
  w->storage_bytes = lay.total;
  MTMC_HIP_CHECK(hipMemcpyAsync(w->storage, blob, lay.total,
                                on_device ? hipMemcpyDeviceToDevice : hipMemcpyHostToDevice, st));
  const char* b = (const char*)w->storage;
  w->embed = b + lay.embed;
  w->final_norm = (const float*)(b + lay.final_norm);
  w->lm_head = b + lay.lm_head;
  w->d_ffn_pad = w->cfg.d_ffn;
  w->layers.resize(w->cfg.n_layers);
  for (int l = 0; l < w->cfg.n_layers; ++l) {
    const BlobLayerOffsets& o = lay.layers[l];
    LayerWeights& L = w->layers[l];
    L.attn_norm = (const float*)(b + o.attn_norm);
    L.ffn_norm = (const float*)(b + o.ffn_norm);
    // Wq, Wk, Wv are adjacent in the blob (sizes are multiples of 256 bytes), and so are
    // Wgate, Wup: each group is used as one stacked [out, in] matrix.
    if (o.wk != o.wq + (size_t)w->cfg.n_q_heads * w->cfg.head_dim * w->cfg.d_model * 4 ||
        o.wv != o.wk + (size_t)w->cfg.n_kv_heads * w->cfg.head_dim * w->cfg.d_model * 4 ||
        o.wup != o.wgate + (size_t)w->cfg.d_ffn * w->cfg.d_model * 4) {
      set_error("fp32 path needs Wq/Wk/Wv and Wgate/Wup to be contiguous in the blob");
      return MTMC_EINVAL;
    }
    L.wqkv = b + o.wq;
    L.wo = b + o.wo;
    L.wgu = b + o.wgate;
    L.wdown = b + o.wdown;
  }
  return MTMC_OK;
}

namespace {
struct F32Acts {
  float *h, *x, *qkv, *o, *gu, *a;
};

// All residual blocks over T tokens (h in, h out).  `layer_stride` is 1 when every layer has
// its own pages (rollout) and 0 when one layer's worth of pages is reused (scoring).
void f32_layers(const mtmc_weights* w, const F32Acts& A, int T, TokMap map, KvPool pool,
                int layer_stride, hipStream_t st) {
  const mtmc_config& c = w->cfg;
  const int d = c.d_model, Hq = c.n_q_heads, Hkv = c.n_kv_heads, hd = c.head_dim, F = c.d_ffn;
  const int nq = Hq * hd, nqkv = (Hq + 2 * Hkv) * hd;
  for (int l = 0; l < c.n_layers; ++l) {
    const LayerWeights& L = w->layers[l];
    const int kvl = l * layer_stride;
    f32::rmsnorm(A.x, A.h, L.attn_norm, c.rms_eps, T, d, st);
    f32::gemm(A.qkv, nqkv, A.x, d, (const float*)L.wqkv, T, nqkv, d, false, st);
    f32::rope_kv_write(A.qkv, T, Hq, Hkv, hd, w->rope_cos, w->rope_sin, map, pool, kvl, st);
    f32::attention(A.o, A.qkv, T, Hq, Hkv, hd, map, pool, kvl, st);
    f32::gemm(A.h, d, A.o, nq, (const float*)L.wo, T, d, nq, true, st);
    f32::rmsnorm(A.x, A.h, L.ffn_norm, c.rms_eps, T, d, st);
    f32::gemm(A.gu, 2 * F, A.x, d, (const float*)L.wgu, T, 2 * F, d, false, st);
    f32::swiglu(A.a, A.gu, T, F, st);
    f32::gemm(A.h, d, A.a, F, (const float*)L.wdown, T, d, F, true, st);
  }
}
}  // namespace

int f32_rollout(const mtmc_weights* w, const RolloutPlan& p, const int* prompts, const SampleArgs& sa,
                hipStream_t st) {
  // the fp32 path runs the whole call as one group (plan_rollout keeps n_prompts == total_prompts)
  const mtmc_config& c = w->cfg;
  const int d = c.d_model, V = c.vocab;
  F32Acts A{p.h, (float*)p.x, p.qkv, (float*)p.o, p.gu, (float*)p.a};
  KvPool pool{p.kv, p.n_pages, c.n_kv_heads, c.head_dim, p.page_table, p.max_pages};
  const bool ragged = sa.prompt_lens != nullptr;
  const int R = ragged ? sa.reuse_len : 0;   // cached prefix: only positions R .. prompt_len - 1 are prefilled
  const int S = p.prompt_len - R;
  if (ragged) {
    launch_ragged_setup(p.page_table, p.row_pos, p.done, sa.out_lens, p.prompt_ids, p.suffix_ids, prompts,
                        sa.prompt_lens, p.n_prompts, p.n_samples, p.prompt_len, p.max_pages, p.nf_max,
                        p.shared_total, p.max_new, R, w->err_flag, st);
    prompts = p.suffix_ids;
  } else {
    launch_build_page_table(p.page_table, p.B, p.max_pages, p.n_samples, p.n_full, p.shared_total, st);
  }
  launch_set_int(p.d_step, 0, st);
  // ---- prefill: whole prompts, chunk by chunk; the prompt's pages are those of its first sample
  for (int p0 = 0; p0 < p.n_prompts; p0 += p.chunk_prompts) {
    const int np = std::min(p.chunk_prompts, p.n_prompts - p0);
    const int T = np * S;
    KvPool chunk_pool = pool;
    chunk_pool.page_table = p.page_table + (size_t)p0 * p.n_samples * p.max_pages;
    TokMap map{S, p.n_samples, R, nullptr};
    f32::embed(A.h, prompts + (size_t)p0 * S, T, (const float*)w->embed, d, V, w->err_flag, st);
    f32_layers(w, A, T, map, chunk_pool, 1, st);
    if (ragged)
      launch_gather_last_rows(p.hB + (size_t)p0 * p.n_samples * d, A.h, d, np, p.n_samples, p.prompt_len,
                              sa.prompt_lens + p0, R, st);
    else
      launch_gather_rows(p.hB + (size_t)p0 * p.n_samples * d, A.h, np * p.n_samples, d, p.n_samples,
                         p.prompt_len, p.prompt_len - 1, 0, st);
  }
  if (ragged)
    launch_fork_tail_pages_ragged(pool, c.n_layers, p.B, p.n_samples, sa.prompt_lens, p.prompt_len, 4, st);
  else if (p.prompt_len % kPageTokens != 0)
    launch_fork_tail_pages(pool, c.n_layers, p.B, p.n_samples, p.n_full, 4, st);
  // ---- step 0 samples from the prompt's last position; step i > 0 first feeds token i-1
  TokMap dmap{1, 1, p.prompt_len - 1, p.d_step, ragged ? p.row_pos : nullptr};
  int* done = (ragged && sa.stop_id >= 0) ? p.done : nullptr;
  for (int i = 0; i < p.max_new; ++i) {
    if (i > 0) {
      f32::embed(p.hB, p.cur_ids, p.B, (const float*)w->embed, d, V, w->err_flag, st);
      F32Acts D{p.hB, (float*)p.x, p.qkv, (float*)p.o, p.gu, (float*)p.a};
      f32_layers(w, D, p.B, dmap, pool, 1, st);
    }
    f32::rmsnorm((float*)p.xB, p.hB, w->final_norm, c.rms_eps, p.B, d, st);
    f32::gemm(p.logits, V, (const float*)p.xB, d, (const float*)w->lm_head, p.B, V, d, false, st);
    f32::sample(p.logits, p.B, V, sa.inv_temp, sa.greedy, sa.seed, sa.seq_offset, p.d_step, sa.max_new,
                p.cur_ids, sa.out_ids, sa.out_logprobs, sa.stop_id, done, sa.out_lens, st);
    launch_add_int(p.d_step, 1, st);
  }
  return MTMC_OK;
}

int f32_score(const mtmc_weights* w, const ScorePlan& p, const ScoreArgs& a, hipStream_t st) {
  const mtmc_config& c = w->cfg;
  const int d = c.d_model, V = c.vocab, S = a.S;
  const int n_scored = S - 1 - a.first;
  const size_t n_out = (size_t)a.n_seqs * (S - 1);
  launch_fill_u32((uint32_t*)a.out_logprobs, 0u, n_out, st);
  if (a.out_top1) launch_fill_u32((uint32_t*)a.out_top1, 0u, n_out, st);
  if (a.out_margin) launch_fill_u32((uint32_t*)a.out_margin, 0u, n_out, st);
  F32Acts A{p.h, (float*)p.x, p.qkv, (float*)p.o, p.gu, (float*)p.a};
  KvPool pool{p.kv, p.n_pages, c.n_kv_heads, c.head_dim, p.page_table, p.pages_per_seq};
  launch_build_page_table(p.page_table, p.chunk_seqs, p.pages_per_seq, 1, 0, 0, st);
  TokMap map{S, 1, 0, nullptr};
  for (int s0 = 0; s0 < a.n_seqs; s0 += p.chunk_seqs) {
    const int ns = std::min(p.chunk_seqs, a.n_seqs - s0);
    const int T = ns * S;
    f32::embed(A.h, a.seqs + (size_t)s0 * S, T, (const float*)w->embed, d, V, w->err_flag, st);
    f32_layers(w, A, T, map, pool, 0, st);
    const int R = ns * n_scored;
    if (R == 0) continue;
    launch_gather_rows(p.hs, A.h, R, d, n_scored, S, a.first, 1, st);
    f32::rmsnorm((float*)p.xs, p.hs, w->final_norm, c.rms_eps, R, d, st);
    for (int r0 = 0; r0 < R; r0 += p.logit_rows) {
      const int nr = std::min(p.logit_rows, R - r0);
      f32::gemm(p.logits, V, (const float*)p.xs + (size_t)r0 * d, d, (const float*)w->lm_head, nr, V, d,
                false, st);
      f32::score_rows(p.logits, nr, V, a.seqs, S, a.first, n_scored, s0, r0, a.out_logprobs, a.out_top1,
                      a.out_margin, w->err_flag, st);
    }
  }
  return MTMC_OK;
}

int f32_score_actions(const mtmc_weights* w, const ActionPlan& p, const ActionArgs& a, hipStream_t st) {
  const mtmc_config& c = w->cfg;
  const int d = c.d_model, V = c.vocab;
  F32Acts A{p.h, (float*)p.x, p.qkv, (float*)p.o, p.gu, (float*)p.a};
  KvPool pool{p.kv, p.n_pages, c.n_kv_heads, c.head_dim, p.page_table, p.max_pages};
  launch_build_page_table(p.page_table, p.B, p.max_pages, p.K, p.n_full, p.shared_total, st);
  launch_build_action_seqs(p.vseq, p.prefix, a.states, a.actions, a.action_len, p.n_states, p.P, p.K, p.A,
                           w->err_flag, st);
  launch_fill_u32((uint32_t*)a.out_token, 0u, (size_t)p.B * p.A, st);
  // ---- the states without their last token, once per state, into the pages of their first candidate
  if (p.Pp > 0) {
    for (int n0 = 0; n0 < p.n_states; n0 += p.chunk_states) {
      const int ns = std::min(p.chunk_states, p.n_states - n0);
      const int T = ns * p.Pp;
      KvPool chunk_pool = pool;
      chunk_pool.page_table = p.page_table + (size_t)n0 * p.K * p.max_pages;
      TokMap map{p.Pp, p.K, 0, nullptr};
      f32::embed(A.h, p.prefix + (size_t)n0 * p.Pp, T, (const float*)w->embed, d, V, w->err_flag, st);
      f32_layers(w, A, T, map, chunk_pool, 1, st);
    }
    if (p.Pp % kPageTokens != 0) launch_fork_tail_pages(pool, c.n_layers, p.B, p.K, p.n_full, 4, st);
  }
  // ---- the candidates: W tokens per row on top of the shared pages, every position scored
  TokMap map{p.W, 1, p.Pp, nullptr};
  for (int r0 = 0; r0 < p.B; r0 += p.chunk_rows) {
    const int nr = std::min(p.chunk_rows, p.B - r0);
    const int T = nr * p.W;
    KvPool chunk_pool = pool;
    chunk_pool.page_table = p.page_table + (size_t)r0 * p.max_pages;
    f32::embed(A.h, p.vseq + (size_t)r0 * p.W, T, (const float*)w->embed, d, V, w->err_flag, st);
    f32_layers(w, A, T, map, chunk_pool, 1, st);
    const int R = nr * p.A;
    launch_gather_rows(p.hs, A.h, R, d, p.A, p.W, 0, 1, st);
    f32::rmsnorm((float*)p.xs, p.hs, w->final_norm, c.rms_eps, R, d, st);
    for (int q0 = 0; q0 < R; q0 += p.logit_rows) {
      const int nq = std::min(p.logit_rows, R - q0);
      f32::gemm(p.logits, V, (const float*)p.xs + (size_t)q0 * d, d, (const float*)w->lm_head, nq, V, d,
                false, st);
      f32::score_rows(p.logits, nq, V, p.vseq, p.W, 0, p.A, r0, q0, a.out_token, nullptr, nullptr, w->err_flag,
                      st);
    }
  }
  launch_action_reduce(a.out_token, a.action_len, p.n_states, p.K, p.A, a.normalize, a.out_action, a.out_policy,
                       st);
  return MTMC_OK;
}

}  // namespace mtmc
