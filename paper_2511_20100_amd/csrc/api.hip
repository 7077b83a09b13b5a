// C boundary, argument checks, weight store, workspace carving and the step schedulers.
#include <cmath>
#include <cstring>
#include <new>

#include "engine.h"
#include "kernels.h"

namespace mtmc {

static thread_local std::string g_last_error;
void set_error(const std::string& msg) { g_last_error = msg; }

static inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

static int check_config(const mtmc_config* c) {
  MTMC_REQUIRE(c != nullptr, "cfg is NULL");
  MTMC_REQUIRE(c->n_layers > 0 && c->d_model > 0 && c->n_q_heads > 0 && c->n_kv_heads > 0 &&
                   c->head_dim > 0 && c->d_ffn > 0 && c->vocab > 0,
               "all model dimensions must be positive");
  MTMC_REQUIRE(c->dtype == MTMC_F32 || c->dtype == MTMC_BF16, "dtype must be MTMC_F32 or MTMC_BF16");
  MTMC_REQUIRE(c->head_dim == 64 || c->head_dim == 128, "head_dim must be 64 or 128");
  MTMC_REQUIRE(c->n_q_heads % c->n_kv_heads == 0, "n_q_heads must be a multiple of n_kv_heads");
  MTMC_REQUIRE(c->dtype != MTMC_BF16 || c->n_q_heads / c->n_kv_heads <= 8,
               "MTMC_BF16 kernels need at most 8 query heads per kv head");
  MTMC_REQUIRE(c->d_model % 16 == 0 && c->d_ffn % 16 == 0 && c->vocab % 16 == 0,
               "d_model, d_ffn and vocab must be multiples of 16");
  MTMC_REQUIRE(c->dtype != MTMC_BF16 || (c->d_model % 32 == 0 && c->d_model <= 4096),
               "MTMC_BF16 kernels need d_model % 32 == 0 and d_model <= 4096");
  MTMC_REQUIRE(c->page_tokens == kPageTokens, "page_tokens must be 16");
  MTMC_REQUIRE(c->max_positions > 0, "max_positions must be positive");
  MTMC_REQUIRE(c->rms_eps >= 0.f && c->rope_base > 0.f, "rms_eps >= 0 and rope_base > 0 required");
  MTMC_REQUIRE(c->tie_embeddings == 0 || c->tie_embeddings == 1, "tie_embeddings must be 0 or 1");
  return MTMC_OK;
}

BlobLayout blob_layout(const mtmc_config& c) {
  BlobLayout b;
  const size_t eb = c.dtype == MTMC_BF16 ? 2 : 4;
  const size_t d = c.d_model, q = (size_t)c.n_q_heads * c.head_dim, kv = (size_t)c.n_kv_heads * c.head_dim;
  const size_t F = c.d_ffn, V = c.vocab;
  size_t off = 0;
  auto take = [&](size_t bytes) {
    off = align_up(off, 256);
    const size_t at = off;
    off += bytes;
    return at;
  };
  b.embed = take(V * d * eb);
  b.layers.resize(c.n_layers);
  for (auto& l : b.layers) {
    l.attn_norm = take(d * 4);
    l.wq = take(q * d * eb);
    l.wk = take(kv * d * eb);
    l.wv = take(kv * d * eb);
    l.wo = take(d * q * eb);
    l.ffn_norm = take(d * 4);
    l.wgate = take(F * d * eb);
    l.wup = take(F * d * eb);
    l.wdown = take(d * F * eb);
  }
  b.final_norm = take(d * 4);
  b.lm_head = c.tie_embeddings ? b.embed : take(V * d * eb);  // tied: the embedding matrix is the LM head
  b.total = off;
  return b;
}

}  // namespace mtmc

using namespace mtmc;

extern "C" const char* mtmc_last_error(void) { return g_last_error.c_str(); }

extern "C" size_t mtmc_blob_bytes(const mtmc_config* cfg) {
  if (check_config(cfg) != MTMC_OK) return 0;
  return blob_layout(*cfg).total;
}

extern "C" int mtmc_weights_create(const mtmc_config* cfg, const void* blob, size_t blob_bytes,
                                   int blob_on_device, void* stream, mtmc_weights** out) {
  if (int rc = check_config(cfg)) return rc;
  MTMC_REQUIRE(blob != nullptr && out != nullptr, "blob and out must not be NULL");
  const BlobLayout lay = blob_layout(*cfg);
  MTMC_REQUIRE(blob_bytes >= lay.total, "blob is smaller than the canonical layout of this configuration");
  hipStream_t st = (hipStream_t)stream;
  mtmc_weights* w = new (std::nothrow) mtmc_weights();
  if (!w) { set_error("out of host memory"); return MTMC_ENOMEM; }
  w->cfg = *cfg;
  w->storage = nullptr;
  w->aux = nullptr;
  w->opt_hip_graph = 1;
  w->opt_lds_min_blocks = 32;
  w->opt_stop_poll = 32;
  w->opt_admit = 1;
  w->graphs = nullptr;
  w->ragged_mu = new (std::nothrow) std::mutex();
  if (!w->ragged_mu) { delete w; set_error("out of host memory"); return MTMC_ENOMEM; }
  int rc = hipGetDevice(&w->device) == hipSuccess ? MTMC_OK : MTMC_EHIP;
  if (rc == MTMC_OK) rc = build_aux(w, st);
  if (rc == MTMC_OK)
    rc = cfg->dtype == MTMC_F32 ? f32_store_weights(w, lay, blob, blob_on_device != 0, st)
                                : bf16_store_weights(w, lay, blob, blob_on_device != 0, st);
  if (rc == MTMC_OK && hipStreamSynchronize(st) != hipSuccess) {
    set_error("hipStreamSynchronize failed after the weight upload");
    rc = MTMC_EHIP;
  }
  if (rc != MTMC_OK) {
    mtmc_weights_destroy(w);
    return rc;
  }
  *out = w;
  return MTMC_OK;
}

extern "C" void mtmc_weights_destroy(mtmc_weights* w) {
  if (!w) return;
  destroy_graph_cache(w);
  if (w->storage) (void)hipFree(w->storage);
  if (w->aux) (void)hipFree(w->aux);
  delete w->ragged_mu;
  delete w;
}

extern "C" int mtmc_admission_plan(const int32_t* live, const int32_t* slot_region, int32_t n_slots, int32_t n_regions,
                                   int32_t n_samples, int32_t prompts_left, int32_t max_at_once, int32_t wait_for,
                                   int32_t* out_slots, int32_t* out_regions) {
  if (!live || !slot_region || !out_slots || !out_regions || n_slots < 1 || n_regions < 1 || n_samples < 1 ||
      prompts_left < 0 || max_at_once < 1 || wait_for < 1) {
    set_error("invalid argument: mtmc_admission_plan needs its arrays and counts of at least 1");
    return MTMC_EINVAL;
  }
  return admission_plan(live, slot_region, n_slots, n_regions, n_samples, prompts_left, max_at_once, wait_for,
                        out_slots, out_regions);
}

extern "C" int mtmc_set_option(mtmc_weights* w, int option, int value) {
  MTMC_REQUIRE(w != nullptr, "weights is NULL");
  MTMC_REQUIRE(option == MTMC_OPT_HIP_GRAPH || option == MTMC_OPT_GEMM_LDS_MIN_BLOCKS ||
                   option == MTMC_OPT_STOP_POLL_STEPS || option == MTMC_OPT_ADMIT_PROMPTS,
               "unknown option");
  if (option == MTMC_OPT_HIP_GRAPH) {
    w->opt_hip_graph = value ? 1 : 0;
  } else if (option == MTMC_OPT_STOP_POLL_STEPS) {
    MTMC_REQUIRE(value >= 0 && value <= (1 << 20), "MTMC_OPT_STOP_POLL_STEPS needs a value in [0, 2^20]");
    w->opt_stop_poll = value;
  } else if (option == MTMC_OPT_ADMIT_PROMPTS) {
    w->opt_admit = value ? 1 : 0;
  } else {
    MTMC_REQUIRE(value >= 1, "MTMC_OPT_GEMM_LDS_MIN_BLOCKS needs a value >= 1");
    w->opt_lds_min_blocks = value;
  }
  return MTMC_OK;
}

extern "C" int mtmc_kernel_timer(mtmc_weights* w, int kernel_class, int every_n_steps) {
  MTMC_REQUIRE(w != nullptr, "weights is NULL");
  MTMC_REQUIRE(w->cfg.dtype == MTMC_BF16, "the kernel timer covers the MTMC_BF16 decode kernels");
  MTMC_REQUIRE(kernel_class >= 0 && kernel_class <= MTMC_KERNEL_LM_HEAD && every_n_steps >= 0, "bad kernel class or period");
  return kernel_timer_set(w, kernel_class, every_n_steps);
}

extern "C" int mtmc_kernel_timer_read(mtmc_weights* w, void* stream, double* total_ms, int64_t* launches,
                                      double* empty_pair_ms) {
  MTMC_REQUIRE(w != nullptr && total_ms != nullptr && launches != nullptr, "NULL pointer argument");
  return kernel_timer_read(w, (hipStream_t)stream, total_ms, launches, empty_pair_ms);
}

extern "C" int mtmc_copy_probe(void* dst, const void* src, size_t bytes, void* stream) {
  MTMC_REQUIRE(dst != nullptr && src != nullptr, "NULL pointer argument");
  MTMC_REQUIRE(bytes % 16 == 0 && ((uintptr_t)dst & 15) == 0 && ((uintptr_t)src & 15) == 0,
               "bytes and both pointers must be multiples of 16");
  launch_copy_probe(dst, src, bytes, (hipStream_t)stream);
  MTMC_HIP_CHECK(hipGetLastError());
  return MTMC_OK;
}

extern "C" int mtmc_read_probe(const void* src, size_t bytes, void* sink, void* stream) {
  MTMC_REQUIRE(src != nullptr && sink != nullptr, "NULL pointer argument");
  MTMC_REQUIRE(bytes >= (size_t)16384 && bytes % 16384 == 0 && ((uintptr_t)src & 15) == 0,
               "bytes must be a positive multiple of 16384 and src 16-byte aligned");
  launch_read_probe(src, bytes, sink, (hipStream_t)stream);
  MTMC_HIP_CHECK(hipGetLastError());
  return MTMC_OK;
}

extern "C" int mtmc_mfma_probe(float* out, int32_t workgroups, int32_t iters, void* stream, double* flops) {
  MTMC_REQUIRE(out != nullptr && flops != nullptr, "NULL pointer argument");
  MTMC_REQUIRE(workgroups > 0 && workgroups <= 65536 && iters > 0 && iters <= (1 << 24), "workgroups or iters out of range");
  *flops = launch_mfma_probe(out, workgroups, iters, (hipStream_t)stream);
  MTMC_HIP_CHECK(hipGetLastError());
  return MTMC_OK;
}

extern "C" int mtmc_poll_errors(const mtmc_weights* w, void* stream) {
  MTMC_REQUIRE(w != nullptr, "weights is NULL");
  MTMC_HIP_CHECK(hipStreamSynchronize((hipStream_t)stream));
  int flag = 0;
  MTMC_HIP_CHECK(hipMemcpy(&flag, w->err_flag, sizeof(int), hipMemcpyDeviceToHost));
  if (flag) {
    MTMC_HIP_CHECK(hipMemset(w->err_flag, 0, sizeof(int)));
    set_error(mtmc_data_error_string(flag));
    return MTMC_EDATA;
  }
  return MTMC_OK;
}

extern "C" const char* mtmc_data_error_string(int bits) {
  static thread_local std::string text;
  text.clear();
  auto add = [&](int bit, const char* msg) {
    if (!(bits & bit)) return;
    if (!text.empty()) text += "; ";
    text += msg;
  };
  add(MTMC_DATA_TOKEN_ID, "a token id outside [0, vocab) was seen (and clamped) on the device");
  add(MTMC_DATA_WEIGHT, "a weight is not finite or exceeds 65504 in magnitude");
  add(MTMC_DATA_LENGTH, "an action or prompt length outside its range was seen (and clamped) on the device");
  add(MTMC_DATA_PREFIX,
      "a cached prompt prefix did not match: the ids of the first reuse_len positions differ from the previous "
      "call's, or a prompt is not longer than reuse_len, or the previous prompt was shorter (results are wrong)");
  add(MTMC_DATA_FP16_RANGE,
      "an activation, key or value left the fp16 range (magnitude above 65504, or not finite) and was clamped: "
      "the results of the calls since the last poll are unreliable");
  return text.c_str();
}

// --------------------------------------------------------------------------------------
// rollout
// --------------------------------------------------------------------------------------
static int check_rollout_shape(const mtmc_weights* w, int32_t n_prompts, int32_t prompt_len,
                               int32_t n_samples, int32_t max_new) {
  MTMC_REQUIRE(w != nullptr, "weights is NULL");
  MTMC_REQUIRE(n_prompts > 0 && prompt_len > 0 && n_samples > 0 && max_new > 0,
               "n_prompts, prompt_len, n_samples and max_new must be positive");
  MTMC_REQUIRE((int64_t)prompt_len + max_new <= w->cfg.max_positions,
               "prompt_len + max_new exceeds max_positions");
  MTMC_REQUIRE((int64_t)n_prompts * n_samples <= (1 << 20), "too many sequences");
  // the decode attention splits the context into at most 4 chunks of 512 pages (the O projection combines them)
  MTMC_REQUIRE(w->cfg.dtype != MTMC_BF16 || (int64_t)prompt_len + max_new <= MTMC_MAX_DECODE_CONTEXT,
               "prompt_len + max_new exceeds MTMC_MAX_DECODE_CONTEXT (32768) of the MTMC_BF16 path");
  return MTMC_OK;
}

extern "C" size_t mtmc_rollout_workspace_bytes(const mtmc_weights* w, int32_t n_prompts,
                                               int32_t prompt_len, int32_t n_samples,
                                               int32_t max_new) {
  if (check_rollout_shape(w, n_prompts, prompt_len, n_samples, max_new) != MTMC_OK) return 0;
  RolloutPlan p = plan_rollout(w, n_prompts, prompt_len, n_samples, max_new, nullptr);
  return p.total_bytes;
}

extern "C" int mtmc_rollout(const mtmc_weights* w, const int32_t* prompts, int32_t n_prompts,
                            int32_t prompt_len, int32_t n_samples, int32_t max_new,
                            float temperature, uint64_t seed, uint32_t seq_offset, int32_t* out_ids,
                            float* out_logprobs, void* workspace, size_t workspace_bytes,
                            void* stream) {
  if (int rc = check_rollout_shape(w, n_prompts, prompt_len, n_samples, max_new)) return rc;
  MTMC_REQUIRE(prompts && out_ids && out_logprobs && workspace, "NULL pointer argument");
  MTMC_REQUIRE(temperature >= 0.f && std::isfinite(temperature), "temperature must be finite and >= 0");
  MTMC_REQUIRE(((uintptr_t)workspace & 255) == 0, "workspace must be 256-byte aligned");
  RolloutPlan p = plan_rollout(w, n_prompts, prompt_len, n_samples, max_new, (char*)workspace);
  if (workspace_bytes < p.total_bytes) {
    set_error("workspace too small for mtmc_rollout: need " + std::to_string(p.total_bytes) + " bytes");
    return MTMC_ENOMEM;
  }
  SampleArgs sa;
  sa.greedy = temperature == 0.f ? 1 : 0;
  sa.inv_temp = sa.greedy ? 1.0f : (float)(1.0 / (double)temperature);
  sa.seed = seed;
  sa.seq_offset = seq_offset;
  sa.max_new = max_new;
  sa.out_ids = out_ids;
  sa.out_logprobs = out_logprobs;
  sa.prompt_lens = nullptr;
  sa.stop_id = -1;
  sa.out_lens = nullptr;
  sa.reuse_len = 0;
  hipStream_t st = (hipStream_t)stream;
  int rc = w->cfg.dtype == MTMC_F32 ? f32_rollout(w, p, prompts, sa, st)
                                    : bf16_rollout(w, p, prompts, sa, st);
  if (rc != MTMC_OK) return rc;
  MTMC_HIP_CHECK(hipGetLastError());
  return MTMC_OK;
}

extern "C" size_t mtmc_rollout_ragged_workspace_bytes(const mtmc_weights* w, int32_t n_prompts,
                                                      int32_t max_prompt_len, int32_t n_samples,
                                                      int32_t max_new) {
  if (check_rollout_shape(w, n_prompts, max_prompt_len, n_samples, max_new) != MTMC_OK) return 0;
  return plan_rollout(w, n_prompts, max_prompt_len, n_samples, max_new, nullptr, true).total_bytes;
}

static int rollout_ragged(const mtmc_weights* w, const int32_t* prompts, const int32_t* prompt_lens,
                          int32_t n_prompts, int32_t max_prompt_len, int32_t n_samples, int32_t max_new,
                          float temperature, uint64_t seed, uint32_t seq_offset, int32_t stop_id, int32_t reuse_len,
                          int32_t* out_ids, float* out_logprobs, int32_t* out_lens, void* workspace,
                          size_t workspace_bytes, void* stream) {
  if (int rc = check_rollout_shape(w, n_prompts, max_prompt_len, n_samples, max_new)) return rc;
  MTMC_REQUIRE(reuse_len >= 0 && reuse_len % kPageTokens == 0 && reuse_len < max_prompt_len,
               "reuse_len must be a non-negative multiple of 16 below max_prompt_len");
  MTMC_REQUIRE(prompts && prompt_lens && out_ids && out_logprobs && out_lens && workspace, "NULL pointer argument");
  MTMC_REQUIRE(temperature >= 0.f && std::isfinite(temperature), "temperature must be finite and >= 0");
  MTMC_REQUIRE(stop_id < w->cfg.vocab, "stop_id must be a token id, or negative for none");
  MTMC_REQUIRE(((uintptr_t)workspace & 255) == 0, "workspace must be 256-byte aligned");
  RolloutPlan p = plan_rollout(w, n_prompts, max_prompt_len, n_samples, max_new, (char*)workspace, true);
  if (workspace_bytes < p.total_bytes) {
    set_error("workspace too small for mtmc_rollout_ragged: need " + std::to_string(p.total_bytes) + " bytes");
    return MTMC_ENOMEM;
  }
  {
    // the cached prefix of a workspace: valid for the shape of the last call on it, gone with any other use
    mtmc_weights* mw = const_cast<mtmc_weights*>(w);
    std::lock_guard<std::mutex> lock(*mw->ragged_mu);
    auto& calls = mw->ragged_calls;
    auto it = calls.begin();
    while (it != calls.end() && it->workspace != workspace) ++it;
    if (reuse_len > 0) {
      MTMC_REQUIRE(p.n_prompts == p.total_prompts,
                   "a cached prefix needs the whole call in one group (at most 128 sequences with MTMC_BF16)");
      MTMC_REQUIRE(it != calls.end() && it->n_prompts == n_prompts && it->max_prompt_len == max_prompt_len &&
                       it->n_samples == n_samples && it->max_new == max_new,
                   "reuse_len > 0 needs a previous mtmc_rollout_ragged call on this workspace with the same "
                   "n_prompts, max_prompt_len, n_samples and max_new");
    }
    if (it != calls.end()) calls.erase(it);
    if (calls.size() >= 16) calls.erase(calls.begin());
    calls.push_back(RaggedCallRecord{workspace, n_prompts, max_prompt_len, n_samples, max_new});
  }
  SampleArgs sa;
  sa.greedy = temperature == 0.f ? 1 : 0;
  sa.inv_temp = sa.greedy ? 1.0f : (float)(1.0 / (double)temperature);
  sa.seed = seed;
  sa.seq_offset = seq_offset;
  sa.max_new = max_new;
  sa.out_ids = out_ids;
  sa.out_logprobs = out_logprobs;
  sa.prompt_lens = prompt_lens;
  sa.stop_id = stop_id < 0 ? -1 : stop_id;
  sa.out_lens = out_lens;
  sa.reuse_len = reuse_len;
  hipStream_t st = (hipStream_t)stream;
  int rc = w->cfg.dtype == MTMC_F32 ? f32_rollout(w, p, prompts, sa, st)
                                    : bf16_rollout(w, p, prompts, sa, st);
  if (rc != MTMC_OK) return rc;
  MTMC_HIP_CHECK(hipGetLastError());
  return MTMC_OK;
}

extern "C" int mtmc_rollout_ragged(const mtmc_weights* w, const int32_t* prompts, const int32_t* prompt_lens,
                                   int32_t n_prompts, int32_t max_prompt_len, int32_t n_samples,
                                   int32_t max_new, float temperature, uint64_t seed, uint32_t seq_offset,
                                   int32_t stop_id, int32_t* out_ids, float* out_logprobs, int32_t* out_lens,
                                   void* workspace, size_t workspace_bytes, void* stream) {
  return rollout_ragged(w, prompts, prompt_lens, n_prompts, max_prompt_len, n_samples, max_new, temperature, seed,
                        seq_offset, stop_id, 0, out_ids, out_logprobs, out_lens, workspace, workspace_bytes, stream);
}

extern "C" int mtmc_rollout_ragged_cached(const mtmc_weights* w, const int32_t* prompts, const int32_t* prompt_lens,
                                          int32_t n_prompts, int32_t max_prompt_len, int32_t n_samples,
                                          int32_t max_new, float temperature, uint64_t seed, uint32_t seq_offset,
                                          int32_t stop_id, int32_t reuse_len, int32_t* out_ids, float* out_logprobs,
                                          int32_t* out_lens, void* workspace, size_t workspace_bytes, void* stream) {
  return rollout_ragged(w, prompts, prompt_lens, n_prompts, max_prompt_len, n_samples, max_new, temperature, seed,
                        seq_offset, stop_id, reuse_len, out_ids, out_logprobs, out_lens, workspace, workspace_bytes,
                        stream);
}

// --------------------------------------------------------------------------------------
// scoring
// --------------------------------------------------------------------------------------
static int check_score_shape(const mtmc_weights* w, int32_t n_seqs, int32_t seq_len) {
  MTMC_REQUIRE(w != nullptr, "weights is NULL");
  MTMC_REQUIRE(n_seqs > 0 && seq_len >= 2, "n_seqs must be positive and seq_len >= 2");
  MTMC_REQUIRE(seq_len <= w->cfg.max_positions, "seq_len exceeds max_positions");
  return MTMC_OK;
}

extern "C" size_t mtmc_score_workspace_bytes(const mtmc_weights* w, int32_t n_seqs, int32_t seq_len) {
  if (check_score_shape(w, n_seqs, seq_len) != MTMC_OK) return 0;
  return plan_score(w, n_seqs, seq_len, nullptr).total_bytes;
}

extern "C" int mtmc_score(const mtmc_weights* w, const int32_t* seqs, int32_t n_seqs, int32_t seq_len,
                          int32_t prompt_len, float* out_logprobs, int32_t* out_top1,
                          float* out_margin, void* workspace, size_t workspace_bytes, void* stream) {
  if (int rc = check_score_shape(w, n_seqs, seq_len)) return rc;
  MTMC_REQUIRE(seqs && out_logprobs && workspace, "NULL pointer argument");
  MTMC_REQUIRE(prompt_len >= 1 && prompt_len <= seq_len, "prompt_len must lie in [1, seq_len]");
  MTMC_REQUIRE(((uintptr_t)workspace & 255) == 0, "workspace must be 256-byte aligned");
  ScorePlan p = plan_score(w, n_seqs, seq_len, (char*)workspace);
  if (workspace_bytes < p.total_bytes) {
    set_error("workspace too small for mtmc_score: need " + std::to_string(p.total_bytes) + " bytes");
    return MTMC_ENOMEM;
  }
  ScoreArgs a;
  a.seqs = seqs;
  a.n_seqs = n_seqs;
  a.S = seq_len;
  a.first = prompt_len - 1;
  a.out_logprobs = out_logprobs;
  a.out_top1 = out_top1;
  a.out_margin = out_margin;
  hipStream_t st = (hipStream_t)stream;
  int rc = w->cfg.dtype == MTMC_F32 ? f32_score(w, p, a, st) : bf16_score(w, p, a, st);
  if (rc != MTMC_OK) return rc;
  MTMC_HIP_CHECK(hipGetLastError());
  return MTMC_OK;
}

// --------------------------------------------------------------------------------------
// action-level scoring
// --------------------------------------------------------------------------------------
static int check_actions_shape(const mtmc_weights* w, int32_t n_states, int32_t state_len, int32_t n_actions,
                               int32_t max_action_len) {
  MTMC_REQUIRE(w != nullptr, "weights is NULL");
  MTMC_REQUIRE(n_states > 0 && state_len > 0 && n_actions > 0 && max_action_len > 0,
               "n_states, state_len, n_actions and max_action_len must be positive");
  MTMC_REQUIRE((int64_t)state_len + max_action_len <= w->cfg.max_positions,
               "state_len + max_action_len exceeds max_positions");
  MTMC_REQUIRE((int64_t)n_states * n_actions <= (1 << 20), "too many candidate actions");
  MTMC_REQUIRE((int64_t)n_states * n_actions * ((int64_t)max_action_len + 1) < (1ll << 31) &&
                   (int64_t)n_states * state_len < (1ll << 31),
               "too many tokens");
  return MTMC_OK;
}

extern "C" size_t mtmc_score_actions_workspace_bytes(const mtmc_weights* w, int32_t n_states, int32_t state_len,
                                                     int32_t n_actions, int32_t max_action_len) {
  if (check_actions_shape(w, n_states, state_len, n_actions, max_action_len) != MTMC_OK) return 0;
  return plan_actions(w, n_states, state_len, n_actions, max_action_len, nullptr).total_bytes;
}

extern "C" int mtmc_score_actions(const mtmc_weights* w, const int32_t* states, int32_t n_states,
                                  int32_t state_len, const int32_t* actions, const int32_t* action_len,
                                  int32_t n_actions, int32_t max_action_len, int32_t normalize,
                                  float* out_token_logprobs, float* out_action_logprobs,
                                  float* out_policy_logprobs, void* workspace, size_t workspace_bytes,
                                  void* stream) {
  if (int rc = check_actions_shape(w, n_states, state_len, n_actions, max_action_len)) return rc;
  MTMC_REQUIRE(states && actions && action_len && out_token_logprobs && out_action_logprobs &&
                   out_policy_logprobs && workspace,
               "NULL pointer argument");
  MTMC_REQUIRE(((uintptr_t)workspace & 255) == 0, "workspace must be 256-byte aligned");
  ActionPlan p = plan_actions(w, n_states, state_len, n_actions, max_action_len, (char*)workspace);
  if (workspace_bytes < p.total_bytes) {
    set_error("workspace too small for mtmc_score_actions: need " + std::to_string(p.total_bytes) + " bytes");
    return MTMC_ENOMEM;
  }
  ActionArgs a;
  a.states = states;
  a.actions = actions;
  a.action_len = action_len;
  a.normalize = normalize != 0;
  a.out_token = out_token_logprobs;
  a.out_action = out_action_logprobs;
  a.out_policy = out_policy_logprobs;
  hipStream_t st = (hipStream_t)stream;
  int rc = w->cfg.dtype == MTMC_F32 ? f32_score_actions(w, p, a, st) : bf16_score_actions(w, p, a, st);
  if (rc != MTMC_OK) return rc;
  MTMC_HIP_CHECK(hipGetLastError());
  return MTMC_OK;
}

// --------------------------------------------------------------------------------------
// PPO clipped surrogate
// --------------------------------------------------------------------------------------
extern "C" size_t mtmc_ppo_workspace_bytes(void) { return ppo_workspace_bytes(); }

extern "C" int mtmc_ppo_clip_loss(const float* new_logprobs, const float* old_logprobs, const float* advantages,
                                  const int32_t* mask, int64_t n, float clip_eps, double* out, void* workspace,
                                  size_t workspace_bytes, void* stream) {
  MTMC_REQUIRE(new_logprobs && old_logprobs && advantages && out && workspace, "NULL pointer argument");
  MTMC_REQUIRE(n > 0, "n must be positive");
  MTMC_REQUIRE(clip_eps >= 0.f && clip_eps < 1.f && std::isfinite(clip_eps), "clip_eps must lie in [0, 1)");
  MTMC_REQUIRE(((uintptr_t)workspace & 255) == 0, "workspace must be 256-byte aligned");
  if (workspace_bytes < ppo_workspace_bytes()) {
    set_error("workspace too small for mtmc_ppo_clip_loss: need " + std::to_string(ppo_workspace_bytes()) + " bytes");
    return MTMC_ENOMEM;
  }
  launch_ppo_clip_loss(new_logprobs, old_logprobs, advantages, mask, (long long)n, (double)clip_eps, out, workspace,
                       (hipStream_t)stream);
  MTMC_HIP_CHECK(hipGetLastError());
  return MTMC_OK;
}

extern "C" int mtmc_ppo_clip_loss_static(const float* new_logprobs, const float* old_logprobs,
                                         const float* advantages, const int32_t* mask, int64_t n, float clip_eps,
                                         double* out, void* stream) {
  MTMC_REQUIRE(new_logprobs && old_logprobs && advantages && out, "NULL pointer argument");
  MTMC_REQUIRE(n > 0, "n must be positive");
  if (n > (int64_t)MTMC_PPO_STATIC_MAX_SAMPLES) {
    set_error("invalid argument: mtmc_ppo_clip_loss_static takes at most MTMC_PPO_STATIC_MAX_SAMPLES (" +
              std::to_string((long long)MTMC_PPO_STATIC_MAX_SAMPLES) + ") samples per call, got " +
              std::to_string((long long)n) + "; use mtmc_ppo_clip_loss with a workspace, or split the samples");
    return MTMC_EINVAL;
  }
  MTMC_REQUIRE(clip_eps >= 0.f && clip_eps < 1.f && std::isfinite(clip_eps), "clip_eps must lie in [0, 1)");
  void* partials = nullptr;
  if (int rc = ppo_static_scratch(&partials)) return rc;
  launch_ppo_clip_loss(new_logprobs, old_logprobs, advantages, mask, (long long)n, (double)clip_eps, out, partials,
                       (hipStream_t)stream);
  MTMC_HIP_CHECK(hipGetLastError());
  return MTMC_OK;
}
