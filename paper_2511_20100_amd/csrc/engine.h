// Host-side engine: blob layout, workspace plans and the per-dtype schedulers.
#pragma once

#include "common.h"

namespace mtmc {

struct BlobLayerOffsets {
  size_t attn_norm, wq, wk, wv, wo, ffn_norm, wgate, wup, wdown;
};
struct BlobLayout {
  size_t embed, final_norm, lm_head, total;
  std::vector<BlobLayerOffsets> layers;
};
BlobLayout blob_layout(const mtmc_config& c);

// Bump allocator over the caller's workspace (base may be NULL to only measure).
struct Carver {
  char* base;
  size_t off = 0;
  explicit Carver(char* b) : base(b) {}
  template <class T>
  T* take(size_t n) {
    off = (off + 255) / 256 * 256;
    T* p = base ? reinterpret_cast<T*>(base + off) : nullptr;
    off += n * sizeof(T);
    return p;
  }
};

constexpr size_t kGemmPartFloats = (size_t)16 << 20;  // 64 MiB: up to 8 ranges of K for the outputs that are split

struct RolloutPlan {
  // A call is run as consecutive groups of `n_prompts` prompts (B = n_prompts * n_samples
  // sequences each); all sizes below are per group.
  int total_prompts;
  int n_prompts, prompt_len, n_samples, max_new, B;
  int ragged;        // prompts of different lengths: prompt_len is the padded length, n_full is 0 (a row
                     // has private pages for its whole length) and up to nf_max pages per prompt are shared
  int nf_max;        // ragged: shared pages reserved per prompt (prompt_len / 16)
  int n_full;        // pages per prompt that are completely filled by the prompt (shared)
  int max_pages;     // page-table row length
  int shared_total;  // pages shared by the sequences of a prompt: n_prompts * n_full; ragged: n_regions * nf_max
  int n_regions;     // ragged: regions of nf_max shared pages (n_prompts; bf16 calls of several groups: more, so that
                     // a new prompt finds one free while the last sequences of earlier prompts still run)
  int n_pages;       // pages in the pool
  int chunk_prompts, Tmax;
  // control
  int* page_table;
  int* d_step;
  int* cur_ids;      // [B]; ragged, bf16: [total_prompts * n_samples], by row of the call
  int* row_pos;      // ragged: [B] position of a row's last prompt token
  int* done;         // ragged: [B] stop flags; bf16: [total_prompts * n_samples], by row of the call
  int* prompt_ids;   // ragged: [n_prompts, prompt_len] prompts with the padding cleared
  int* slot_row;     // ragged, bf16: [bt * 16] row held by each slot once live rows are packed (-1: nobody)
  int* page_table_c; // ragged, bf16: [B, max_pages] page-table rows by slot
  int* row_pos_c;    // ragged, bf16: [bt * 16] position base by slot (-1: nobody)
  int* live;         // ragged, bf16: [16 + 256] live[0] = rows that have not stopped; from 16 on: per slot, does it hold a sequence that still runs
  int* row_step0;    // ragged, bf16: [bt * 16] step of the call at which the sequence in a slot was at its step 0
  int* prefill_table; // ragged, bf16: [bt * 16, max_pages] page-table rows through which new prompts are prefilled
  int* slot_row_c;   // ragged, bf16: [bt * 16] slot_row / row_step0 of the packed batch (page_table_c, row_pos_c)
  int* row_step0_c;
  float* hT;         // ragged, bf16: [n_samples, d] last prompt position of a prompt that joins a running batch
  void* xT;          // ragged, bf16: its normalised operand, tiled
  float* ssT;        // ragged, bf16: sums of squares that go with xT
  int* suffix_ids;   // ragged: [n_prompts, prompt_len - reuse_len] the ids that are prefilled (all, without a cached prefix)
  void* kv;
  // activations (Tmax rows unless noted)
  float* h;
  void* x;
  float* qkv;
  void* o;
  float* gu;
  void* a;
  float* hB;      // [B, d]
  void* xB;       // [B, d]
  float* logits;  // fp32 path: [B, V]
  // bf16 path scratch
  float* part;        // split-K partial sums
  void* o_chunks;     // decode-attention output per context chunk: n_chunks tiled fp16 operands [Hq*hd, bt*16]
  float* attn_ml;     // (max, sum) per (sequence, head, chunk) for the O projection to combine the chunks
  float* lm_part;     // LM-head per-tile partial reductions
  float* gemm_part;   // partial sums of the prefill GEMMs' split-K form (kGemmPartFloats)
  void* qb;           // rotated queries, bf16 row-major [Tmax, Hq*hd]
  void* ctl;          // per-call sampling parameters (device copy)
  float* ssA;         // per-tile sums of squares of the residual rows (two generations)
  float* ssB;
  float* rs_buf;      // 1/rms per row, handed from the split-K down projection to its reduction
  int chunk_pages, n_chunks;       // decode-attention context split
  int split_at_prompt;             // two chunks: the prompt's whole pages | the rest (else equal chunks)
  int ks_qkv, ks_o, ks_down;       // split-K factors of the decode GEMMs
  int down_nb;                     // weight row tiles per workgroup of the down projection (2 or 4)
  int bt;                          // 16-row tiles covering B
  size_t total_bytes;
};

struct ScorePlan {
  int n_seqs, S, chunk_seqs, pages_per_seq, n_pages, T;
  int rows_max;      // scored rows per chunk at most (chunk_seqs * (S - 1))
  int logit_rows;    // rows of the logits buffer (fp32 path)
  int* page_table;
  void* kv;
  float* h;
  void* x;
  float* qkv;
  void* o;
  float* gu;
  void* a;
  float* hs;   // [rows_max, d] gathered scored rows
  void* xs;    // [rows_max, d]
  float* logits;
  float* part;
  float* lm_part;
  float* gemm_part;   // partial sums of the split-K GEMMs (kGemmPartFloats), or NULL when the pass is too large to use them
  void* qb;
  int* targets;
  size_t total_bytes;
};

// Action-level scoring.  The states (without their last token) are prefilled once into pages that
// the K candidates of a state share; row b = n K + k then runs the A + 1 tokens
// [last state token, action tokens, padding] at positions P - 1 .. P - 1 + A on top of them.
struct ActionPlan {
  int n_states, P, K, A, B;
  int Pp;            // prefilled tokens per state (P - 1)
  int W;             // tokens per candidate row (A + 1)
  int n_full;        // pages per state completely filled by the prefilled tokens (shared)
  int max_pages;     // page-table row length
  int shared_total;  // n_states * n_full
  int n_pages;
  int chunk_states;  // states per prefill chunk
  int chunk_rows;    // candidate rows per chunk of the second pass
  int Tmax;          // token rows of the activation buffers
  int rows_max;      // scored rows per chunk at most (chunk_rows * A)
  int logit_rows;    // fp32 path: rows of the logits buffer
  int* page_table;   // [B, max_pages]
  int* vseq;         // [B, W]
  int* prefix;       // [n_states, Pp]
  void* kv;
  float* h;
  void* x;
  float* qkv;
  void* o;
  float* gu;
  void* a;
  float* hs;
  void* xs;
  float* logits;
  float* lm_part;
  float* gemm_part;   // partial sums of the split-K GEMMs (kGemmPartFloats), or NULL when the pass is too large to use them
  void* qb;
  int* targets;
  // bf16 path: the candidates of a chunk packed without padding (built on the device, see build_packed_actions)
  int* seq_start;    // [chunk_rows + 1]
  int* d_rows;       // [16] d_rows[0] = packed tokens of the chunk
  int* pids;         // [chunk_rows * A] input token of every packed token
  int* out_index;    // [chunk_rows * A] where its term goes in out_token
  size_t total_bytes;
};

struct ActionArgs {
  const int* states;
  const int* actions;
  const int* action_len;
  int normalize;
  float* out_token;
  float* out_action;
  float* out_policy;
};

struct SampleArgs {
  int greedy;
  float inv_temp;
  uint64_t seed;
  uint32_t seq_offset;
  int max_new;
  int* out_ids;
  float* out_logprobs;
  // prompts of different lengths / stop token (mtmc_rollout_ragged); prompt_lens == NULL otherwise
  const int* prompt_lens;
  int stop_id;
  int* out_lens;
  int reuse_len;     // leading positions of every prompt whose keys / values the workspace still holds (0: none)
};

struct ScoreArgs {
  const int* seqs;
  int n_seqs, S, first;
  float* out_logprobs;
  int* out_top1;
  float* out_margin;
};

RolloutPlan plan_rollout(const mtmc_weights* w, int n_prompts, int prompt_len, int n_samples,
                         int max_new, char* base, bool ragged = false);
ScorePlan plan_score(const mtmc_weights* w, int n_seqs, int S, char* base);
ActionPlan plan_actions(const mtmc_weights* w, int n_states, int P, int K, int A, char* base);

// Rotary table (angles in double) and the device error flag.
int build_aux(mtmc_weights* w, hipStream_t st);

int f32_store_weights(mtmc_weights* w, const BlobLayout& lay, const void* blob, bool on_device,
                      hipStream_t st);
int f32_rollout(const mtmc_weights* w, const RolloutPlan& p, const int* prompts, const SampleArgs& sa,
                hipStream_t st);
int f32_score(const mtmc_weights* w, const ScorePlan& p, const ScoreArgs& a, hipStream_t st);

int bf16_store_weights(mtmc_weights* w, const BlobLayout& lay, const void* blob, bool on_device,
                       hipStream_t st);
// Which prompts join a running batch at one look (host only).  live [n_slots]: the slot holds a sequence that still
// runs; slot_region [n_slots]: the region of shared prompt pages that sequence reads.  A prompt needs n_samples free
// slots and a region that no running sequence reads.  Returns k = min(free slots / n_samples, free regions,
// prompts_left, max_at_once), or 0 while k < min(prompts_left, wait_for, max_at_once) and some sequence still runs; out_slots
// [k * n_samples] = the lowest free slots, prompt by prompt, out_regions [k] = the lowest free regions.
int admission_plan(const int* live, const int* slot_region, int n_slots, int n_regions, int n_samples, int prompts_left,
                   int max_at_once, int wait_for, int* out_slots, int* out_regions);
int bf16_rollout(const mtmc_weights* w, const RolloutPlan& p, const int* prompts,
                 const SampleArgs& sa, hipStream_t st);
int bf16_score(const mtmc_weights* w, const ScorePlan& p, const ScoreArgs& a, hipStream_t st);
int f32_score_actions(const mtmc_weights* w, const ActionPlan& p, const ActionArgs& a, hipStream_t st);
int bf16_score_actions(const mtmc_weights* w, const ActionPlan& p, const ActionArgs& a, hipStream_t st);
void destroy_graph_cache(mtmc_weights* w);
int kernel_timer_set(mtmc_weights* w, int cls, int every);
int kernel_timer_read(mtmc_weights* w, hipStream_t st, double* total_ms, int64_t* launches, double* empty_pair_ms);
void bf16_plan_rollout_extra(const mtmc_weights* w, RolloutPlan& p, Carver& c);
void bf16_plan_score_extra(const mtmc_weights* w, ScorePlan& p, Carver& c);
void bf16_plan_actions_extra(const mtmc_weights* w, ActionPlan& p, Carver& c);

}  // namespace mtmc
