// Launchers of the bf16-path kernels (weights / KV cache in bf16, fp32 accumulation).
#pragma once

#include "common.h"
#include "frag.h"

namespace mtmc {
namespace bf16 {

// Per-call sampling parameters, kept in device memory so that captured launches stay valid.
struct SampleCtl {
  int greedy;
  float inv_temp;
  uint32_t key0, key1, seq_offset;
  int max_new;
  int* out_ids;
  float* out_logprobs;
  // stop token (done == NULL: none): a row whose flag is set reports stop_id with log-prob 0; a row that
  // samples stop_id sets its flag and out_lens[row] = step + 1
  int stop_id;
  int* done;
  int* out_lens;
  // Rows packed into fewer slots (a batch whose finished rows gave up their places): slot m of the decode
  // kernels holds row slot_row[m] of the call, or nobody (-1).  NULL: slot m is row m.  Outputs, stop flags, the
  // fed-back ids (cur_ids) and the random-number counters go by row.
  const int* slot_row;
  // Rows that joined the batch while it was running (a new prompt took the places of a finished one): the
  // sequence in slot m is at its own step *d_step - row_step0[m].  It reports under that step, draws that
  // step's random numbers, raises its stop flag when that step is max_new - 1 and reports nothing after that
  // or once the flag is up.  NULL: every row is at step *d_step.
  const int* row_step0;
};

struct LargeArgs {
  const h16_t* Wt;
  const h16_t* Xt;
  int n_tiles, k_tiles, m_tiles, M, N;
  float* out_f32;
  int ld_out;
  h16_t* out_bf16;
  int* err_flag;         // SwiGLU epilogue: raised when a value does not fit fp16
  const int* d_rows;     // optional (device): only the first *d_rows rows hold tokens; blocks of rows beyond are skipped
  int k_split;           // split-K form: ranges of k-steps, and the partial sums [k_split][M][N] (set by its launcher)
  float* part;
};

struct ScoreHeadArgs {
  const h16_t* Wt;
  const h16_t* Xt;
  int n_tiles, k_tiles, m_tiles, M;
  const int* targets;
  float* part;
  int n_groups, groups_per_block;
  int want_top;   // 0: the two largest logits are not tracked (the caller asked for log-probs only)
  const int* d_rows;  // optional (device): only the first *d_rows rows hold tokens
};

// ---- decode step (six launches per block; see decode_bf16.hip) ------------------------------
struct DecGemmArgs {
  const h16_t* Wt;
  const h16_t* Xt;
  int n_tiles, k_tiles, m_tiles, M;
  const float* ss_cur;   // per-tile sums of squares [ss_tiles][m_tiles*16] of the current residual (NULL: scale 1)
  const float* ss_old;   // same, of the residual whose norm scaled Xt
  int ss_tiles;
  float inv_d, eps;
  float* out_f32;        // STORE: fp32 [M, ld_out]; RESID: residual h (in/out); SAMPLE: sampler partials
  int ld_out;
  h16_t* out_h16;        // SWIGLU / RESID: tiled fp16 operand for the next GEMM
  float* ss_out;         // RESID: [n_tiles][m_tiles*16]
  const float* gain;     // RESID: gain of the next norm
  const SampleCtl* ctl;
  const int* d_step;
  int ksplit;            // PARTIAL: K splits (grid.y); out_f32 = partial sums [ksplit][m_tiles*16][ld_out]
  float* rs_out;         // PARTIAL: 1/rms of every row of the state described by ss_cur
  int partial_nb;        // PARTIAL, up to 64 rows: 2 = two weight row tiles and 8 wavefronts per workgroup, 3 = three
                         // and 5 with ksplit = 8 aligned to the XCDs, else four and 4
  int xcd_split;         // set by the launcher of the XCD-aligned form
  // RESID with n_xchunks > 1 (O projection behind a context-split attention): Xt holds n_xchunks operands
  // x_chunk_stride elements apart, each the attention output over one chunk of the context, normalised by itself;
  // chunk_ml [M][k_tiles / head_tiles][n_xchunks][2] = (running maximum, sum) of row, head, chunk.  The product is
  // taken head by head and chunk by chunk and the pieces are added with their softmax weights.
  int n_xchunks, head_tiles;
  size_t x_chunk_stride;
  const float* chunk_ml;
  // set by the launcher: the rows are split over pairs of workgroups that follow each other by 8 in launch order
  // (same XCD, dispatched together, so the second read of a weight tile hits L2); 0 = rows split over grid.y, if at all
  int row_pairs;
  int* err_flag;         // RESID / SWIGLU: raised when a value written as fp16 does not fit
};
enum { DEC_STORE = 0, DEC_RESID = 1, DEC_SWIGLU = 2, DEC_SAMPLE = 3, DEC_PARTIAL = 4 };
// One partial result of the sampling LM head: the state of a row over one workgroup's vocabulary slice.
struct DecSamplePartial {
  float m, s, y;   // log-sum-exp state (maximum, sum), largest perturbed logit
  int idx;         // its vocabulary index
  float zt;        // its unperturbed logit / T
  float pad[3];
};
// 65..128 rows (decode_rows128.hip): every wavefront of a workgroup owns its own weight row tiles and all the rows,
// the wavefronts walk K together and share the activation operand through LDS.  Returns false when the launch is
// one it does not take (the caller then uses the general form).  The down projection and the LM head give a
// workgroup kRows128WideTiles weight row tiles (the host sizes the split-K factor and the sampler's partial results
// by that); the gate/up launch picks its own shape, 8 to 16 tiles, so that the launch is one round on the CUs.
constexpr int kRows128WideTiles = 8;
bool gemm_dec_rows128(const DecGemmArgs& a, int epi, hipStream_t st);
void resid_reduce(const float* P, int ksplit, int m_tiles, int N, float* h, const float* gain, const float* rs,
                  h16_t* x, float* ss_out, int M, int* err_flag, hipStream_t st);
void gemm_dec(const DecGemmArgs& a, int epi, hipStream_t st);
int dec_wide_nb(int m_tiles);
// Sampling LM head (decode_lmhead.hip): the persistent form for up to 64 rows and the model widths it is built for.
// lmhead_sample_persistent_groups = partial results per row that launch leaves (0: the launch is not taken);
// dec_sample_groups = the same for whichever form gemm_dec(.., DEC_SAMPLE) runs (what sample_merge must be told).
int lmhead_sample_persistent_groups(int n_tiles, int k_tiles, int m_tiles);
bool lmhead_sample_persistent(const DecGemmArgs& a, hipStream_t st);
int dec_sample_groups(int n_tiles, int k_tiles, int m_tiles);
// What the sampler merge prepares for the next decode step from the token it has just chosen for a row: the
// residual h = E[token], x' = fp16(RMSNorm(h; gain)) in tiled layout (Mpad rows) and the per-tile sums of squares.
struct EmbedNextArgs {
  float* h;
  const bf16_t* E;
  int d;             // <= 4096
  const float* gain;
  float eps;
  h16_t* x;
  int Mpad;
  float* ss_out;
  int vocab;         // a chosen id outside [0, vocab) (every logit NaN) is replaced by 0 and reported
  int* err_flag;
};
// Merges the sampler partials of a step, writes the outputs of step *d_step, advances *d_step (d_step[1] is the
// kernel's arrival counter: zero before the first launch, left at zero by every launch) and embeds the chosen tokens.
void sample_merge(const float* part, int n_groups, int M, const SampleCtl* ctl, int* d_step, int* cur_ids,
                  const EmbedNextArgs& emb, hipStream_t st);
struct AttnDecArgs {
  const float* qkv;      // fp32 [B, (Hq + 2 Hkv) * 128], not yet rotated
  const float* cos;
  const float* sin;
  int Hq, Hkv, layer, pos_base;
  const int* row_pos;    // per-sequence position base (sequences of different lengths), or NULL: pos_base
  const int* d_step;
  // sequences that joined the batch while it was running: the sequence in slot b is at step
  // min(*d_step - row_step0[b], max_step) (a slot whose sequence has ended keeps rewriting its last position
  // until the host gives the slot to another sequence).  NULL: every sequence is at step *d_step.
  const int* row_step0;
  int max_step;
  KvPool pool;
  int chunk_pages, n_chunks, m_tiles;
  int split_at_prompt;   // n_chunks == 2: chunk 0 = the whole pages of the sequence's prompt (pos_base / row_pos), chunk 1 = the rest
  int share;             // consecutive sequences that share prompt pages (samples per prompt); B % share == 0
  h16_t* o;              // tiled fp16 [Hq * hd (k), m_tiles * 16], one per chunk, o_chunk_stride elements apart:
  size_t o_chunk_stride; //   the output over the chunk's keys alone, normalised by the chunk's own sum
  float* ml;             // [B, Hq, n_chunks, 2]: running maximum and sum of (sequence, head, chunk); the consumer
                         //   (O projection) combines the chunks.  Not written when n_chunks == 1.
  int* err_flag;         // raised when q, k, v or the output does not fit fp16
};
void attention_dec(const AttnDecArgs& a, int B, hipStream_t st);

// ---- packing the live rows of a batch with a stop token into the leading slots ------------------
// live[0] = number of rows whose stop flag is clear.
void count_live(const int* done, int B, int* live, hipStream_t st);
// slot_row[0 .. slots) = the rows with a clear stop flag in ascending order, then -1; the page-table rows and
// position bases of those rows gathered by slot (an empty slot gets page 0 everywhere and position base -1,
// which the attention kernel takes as "nobody here").
void compact_rows(const int* done, int B, int slots, int* slot_row, const int* page_table, const int* row_pos,
                  int max_pages, int* page_table_c, int* row_pos_c, hipStream_t st);
// The residual, its normalised fp16 operand and the sums of squares of every slot's current token
// (cur_ids by row; token 0 for an empty slot), in the layout of `slots` rows.
void embed_slots(const int* slot_row, const int* cur_ids, int slots, const EmbedNextArgs& emb, hipStream_t st);

// ---- weight re-tiling (once, at load) ------------------------------------------------------
// dst (tiled fp16, n_tiles x k_tiles blocks) <- src row-major [N, K] bf16; rows/cols past N/K are
// zero.  Sets bit 1 of *err_flag if a weight does not fit fp16 (magnitude above 65504, or not finite).
// check_finite_bf16 does the same for a matrix that is kept as bf16 (the embedding table): not finite -> bit 1.
void check_finite_bf16(const bf16_t* src, size_t n, int* err_flag, hipStream_t st);
void retile_weight(h16_t* dst, const bf16_t* src, int N, int K, int n_tiles, int k_tiles, int* err_flag,
                   hipStream_t st);
// Gate and up interleaved by 16-row tiles: tile 2j <- gate rows 16j.., tile 2j+1 <- up rows 16j..
void retile_gate_up(h16_t* dst, const bf16_t* gate, const bf16_t* up, int F, int K, int f_tiles,
                    int k_tiles, int* err_flag, hipStream_t st);

// ---- GEMMs ---------------------------------------------------------------------------------
// d_rows (device, may be NULL): the number of rows that hold tokens when it is known on the device only (rows
// packed by a kernel); M and m_tiles then give the capacity the launch is sized for.
// part (device, may be NULL) / part_floats: room for partial sums; with it, an output of few 256 x 256 blocks is
// computed over several ranges of K at once (gemm_lds_split) and summed in a fixed order.
void gemm_large_f32(float* C, int ldc, int N, bool accumulate, const h16_t* Wt, int n_tiles,
                    int k_tiles, const h16_t* Xt, int M, int m_tiles, int lds_min_blocks, const int* d_rows,
                    hipStream_t st, float* part = nullptr, size_t part_floats = 0);
void gemm_large_swiglu(h16_t* act, const h16_t* Wt, int n_tiles, int k_tiles, const h16_t* Xt,
                       int M, int m_tiles, int lds_min_blocks, int* err_flag, const int* d_rows, hipStream_t st);
// LDS-staged 256 x 256 kernel behind the two launchers above (epi: 0 store, 1 accumulate, 2 SwiGLU).
void gemm_lds(const LargeArgs& a, int epi, hipStream_t st);
// Split-K form of the store / accumulate GEMM for outputs of at most 128 blocks: false when it does not apply
// (no range count from 2 to 8 divides K into even ranges of at least 8 k-steps that fit `part`), and nothing was launched.
bool gemm_lds_split(const LargeArgs& a, bool accumulate, float* part, size_t part_floats, hipStream_t st);
int score_head_blocks(int n_tiles, int* groups_per_block);
void lmhead_score(float* part, const h16_t* Wt, int n_tiles, int k_tiles, const h16_t* Xt, int M,
                  int m_tiles, const int* targets, bool want_top, int lds_min_blocks, const int* d_rows,
                  hipStream_t st);
// One partial result of the scoring LM head: a row's state over one vocabulary slice.
struct ScorePartial {
  float m, s, v1;   // log-sum-exp state, largest logit
  int i1;           // its index
  float v2, zt;     // second largest logit, logit of the target token (-inf if not in the slice)
  float pad[2];
};
// LDS-staged version (256 rows x 256 vocabulary entries per step, `slices` vocabulary slices of 128 row tiles).
void lmhead_score_lds(const ScoreHeadArgs& a, int slices, hipStream_t st);
void score_targets(int* targets, const int* seqs, int R, int S, int first, int n_scored, int seq0,
                   int row0, int vocab, int* err_flag, hipStream_t st);
void score_reduce(const float* part, int n_parts, int R, int S, int first, int n_scored, int seq0,
                  int row0, float* out_logprobs, int* out_top1, float* out_margin, hipStream_t st);
// Rows packed by build_packed_actions: row r < *d_rows goes to out_logprobs[out_index[r]].
void score_reduce_scatter(const float* part, int n_parts, int R, const int* d_rows, const int* out_index,
                          float* out_logprobs, hipStream_t st);
// Candidate actions of different lengths packed without padding (action-level scoring).  Rows b = r0 .. r0 + nr - 1
// of the call (candidate b has len_b = action_len[b] clamped to [0, A] tokens a_1 .. a_len) become the packed
// token list of a chunk: candidate b contributes the len_b inputs [last token of its state, a_1 .. a_{len-1}]
// (none when empty), whose outputs predict a_1 .. a_len.
//   seq_start [nr + 1]  first packed token of every candidate (exclusive prefix sums); d_rows[0] = their total
//   ids, targets [cap]  input token and the token it must predict, per packed token
//   out_index [cap]     b * A + i: where the term of (candidate b, action token i) goes
// One workgroup of 1024 threads; nr * A <= cap.  An action_len outside [0, A] raises bit 4 of *err_flag.
void build_packed_actions(int* seq_start, int* d_rows, int* ids, int* targets, int* out_index, const int* states,
                          const int* actions, const int* action_len, int P, int K, int A, int r0, int nr, int vocab,
                          int* err_flag, hipStream_t st);

// ---- elementwise / row kernels -------------------------------------------------------------
void set_sample_ctl(SampleCtl* dst, const SampleCtl& v, hipStream_t st);
// A batch that takes in new prompts as it runs.  Every slot has pages of its own for a whole sequence; the whole
// pages of a prompt lie in one of the call's regions of nf_max pages, shared by the prompt's sequences.
// admit_init: slot s holds row s (nobody from B on), every row at step *d_step.
// admit_prompt: the sequences of prompt `prompt_index` of the call (rows prompt_index * n_samples + j) take the
// slots slots[j]; they are at their step *d_step - step0; their page-table rows are rebuilt over `region`; the
// prompt, its padding cleared, is left in ids_out [Lmax].  fork_tail_slots: after the prefill through slots[0].
// slot_live: which slots hold a sequence that still runs.  compact_slots: those sequences packed into the leading
// slots of a second set of tables.
struct AdmitArgs {
  int* page_table;     // [slots, max_pages]
  int* row_pos;        // [slots]
  int* slot_row;       // [slots]
  int* row_step0;      // [slots]
  int* ids_out;
  int* prefill_row;    // [max_pages] a copy of the page-table row of slots[0] (the prefill of several new prompts
                       // at once goes through a table of these rows)
  const int* prompt;   // device [Lmax]
  const int* len;      // device, the prompt's length (clamped to [1, Lmax] and reported when outside)
  int region, prompt_index, n_samples, Lmax, max_pages, nf_max, shared_total, step0;
  int* err_flag;
  int slots[128];
};
void admit_init(int* slot_row, int* row_step0, int B, int Mpad, hipStream_t st);
void admit_prompt(const AdmitArgs& a, hipStream_t st);
void fork_tail_slots(const AdmitArgs& a, KvPool pool, int n_layers, hipStream_t st);
void slot_live(const int* done, const int* slot_row, int n_slots, int* live, hipStream_t st);
void compact_slots(const int* done, int B, int slots, const int* slot_row, const int* page_table, const int* row_pos,
                   const int* row_step0, int max_pages, int* slot_row_c, int* page_table_c, int* row_pos_c,
                   int* row_step0_c, hipStream_t st);
void embed(float* h, const int* ids, int T, const bf16_t* E, int d, int vocab, int* err_flag,
           hipStream_t st, const int* d_rows = nullptr);
// h[m, :] += sum_s P[s][m][:] (n_split may be 0); x = bf16(RMSNorm(h; gain)) in tiled layout.
void add_norm(float* h, const float* P, int n_split, int ldp, int Mpad_p, const float* gain, float eps,
              h16_t* x, int M, int m_tiles, int d, int* err_flag, hipStream_t st, const int* d_rows = nullptr);
// qkv fp32 [T, (Hq + 2 Hkv) hd] (row stride ld), T = n_seqs * S tokens at positions map.pos_base + t % S: rotates q
// (-> fp16 row-major [T, Hq*hd]) and k, writes k and v into the pages.  map.d_step and map.row_pos must be NULL.
// seq_start (device, may be NULL): sequences of different lengths packed back to back: sequence s holds the
// tokens seq_start[s] .. seq_start[s + 1] - 1 at positions map.pos_base + 0, 1, ...; S is then the longest
// length a sequence can have and n_seqs the number of sequences (T is ignored).
void rope_kv_write(h16_t* q, const float* qkv, int ld, int T, int S, int Hq, int Hkv, const float* cos,
                   const float* sin, TokMap map, KvPool pool, int layer, int* err_flag, hipStream_t st,
                   const int* seq_start = nullptr, int n_seqs = 0);

// ---- attention -----------------------------------------------------------------------------
// Floats of the per-chunk partial results of the decode attention kernel.
// Prefill / scoring: causal attention of every token of T = n_seqs * S over its own sequence.
void attention_prefill(h16_t* o, const h16_t* q, int n_seqs, int S, int m_tiles, int Hq, int Hkv,
                       TokMap map, KvPool pool, int layer, int* err_flag, hipStream_t st,
                       const int* seq_start = nullptr);

}  // namespace bf16
}  // namespace mtmc
