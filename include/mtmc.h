/*
 * mtmc.h -- C boundary of the MI355X policy rollout / scoring library (libmtmc.so).
 *
 * The Macro Thinking policy of the paper is a lightweight decoder-only language model that
 * emits an action as a token sequence a_k = {w_k^1 .. w_k^N} (Method, "Training Methodology").
 * Two operations on that model are exported:
 *
 *   mtmc_score    teacher-forced per-token log-probabilities log P(w^i | s, w^1..w^{i-1}),
 *                 i.e. the logarithms of the factors of Eq. 2;
 *   mtmc_rollout  sampling such token sequences autoregressively, several continuations per
 *                 prompt (Inference Pipeline, "Macro Thinking"), returning the sampled ids and
 *                 the log-probability each was drawn with.
 *
 * and, built on the same kernels: mtmc_rollout_ragged (prompts of different lengths, stop token),
 * mtmc_score_actions (Eq. 2 summed per candidate action and the softmax over a state's candidates)
 * and mtmc_ppo_clip_loss (value of the clipped surrogate of the PPO update over scored samples).
 *
 * Model: pre-norm residual blocks (RMSNorm, rotary embedding with pairs (i, i + head_dim/2),
 * grouped-query causal attention, SwiGLU feed-forward), final RMSNorm, LM head (its own matrix,
 * or the embedding matrix when tie_embeddings is set), no biases.  Matrices are row-major [out, in], y = W x.
 *
 * General rules
 *  - All pointers marked "device" must be device memory of the current HIP device; "host"
 *    pointers are ordinary host memory.  The library never takes ownership of caller memory.
 *  - Apart from mtmc_weights_create (which allocates the library-owned, re-tiled copy of the
 *    weights) no call allocates or frees device memory: scratch comes from the caller's
 *    `workspace`, sized by the matching *_workspace_bytes query.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).  mtmc_rollout and
 *    mtmc_score only enqueue work on it and return without synchronising; outputs are valid
 *    once the caller has synchronised the stream.  Calls that share a workspace must be
 *    ordered on one stream; calls on one weights handle with distinct workspaces may overlap
 *    on different streams and give the results they give alone.
 *  - Every int-returning call gives MTMC_OK (0) or a negative code; mtmc_last_error() then
 *    holds a message for the calling thread.
 */
#ifndef MTMC_H
#define MTMC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define MTMC_OK       0
#define MTMC_EINVAL  (-1)  /* null pointer, bad shape, unsupported configuration        */
#define MTMC_ENOMEM  (-2)  /* workspace too small, or device allocation failed           */
#define MTMC_EHIP    (-3)  /* a HIP runtime call failed; message holds hipGetErrorString */
#define MTMC_EDATA   (-4)  /* the device saw bad data: see mtmc_poll_errors                */

#define MTMC_F32  0        /* matrices fp32, all arithmetic fp32                          */
/* MTMC_BF16: the caller's matrices are bf16.  The library converts them once, at load, to IEEE fp16 (exact for
 * every bf16 value of magnitude in [2^-17, 65504]; larger or non-finite weights are rejected, smaller ones lose
 * at most 3e-8) and runs the matrix cores on fp16 operands: the activations that enter a matrix product and
 * the KV cache are fp16 (11 significant bits, range +-65504), everything else -- residual stream, norms,
 * softmax statistics, log-sum-exp, all accumulators -- is fp32.  A producer that has to clamp a value into
 * the fp16 range raises MTMC_DATA_FP16_RANGE (see mtmc_poll_errors).                              */
#define MTMC_BF16 1

typedef struct {
  int32_t n_layers, d_model, n_q_heads, n_kv_heads, head_dim, d_ffn, vocab;
  float   rms_eps;        /* added to the mean square inside the square root              */
  float   rope_base;      /* theta_i = rope_base^(-2i/head_dim)                           */
  int32_t dtype;          /* MTMC_F32 or MTMC_BF16                                        */
  int32_t page_tokens;    /* tokens per KV-cache page; must be 16                         */
  int32_t max_positions;  /* rows of the rotary table: >= prompt_len + max_new, >= seq_len */
  int32_t tie_embeddings; /* 1: the LM head is the embedding matrix and the blob has no lm_head  */
} mtmc_config;

typedef struct mtmc_weights mtmc_weights; /* opaque, library-owned */

/*
 * Copies the canonical weight blob into library-owned device memory, re-tiled for the
 * kernels, and builds the rotary cos/sin table (angles in double, rounded to fp32).
 *
 * blob: tensors in this order, each starting at the next multiple of 256 bytes:
 *   embed[V,d]; per layer: attn_norm[d] Wq[Hq*hd,d] Wk[Hkv*hd,d] Wv[Hkv*hd,d] Wo[d,Hq*hd]
 *   ffn_norm[d] Wgate[F,d] Wup[F,d] Wdown[d,F]; final_norm[d]; lm_head[V,d] (absent when
 *   tie_embeddings is set: logits are then taken against embed).
 *   Norm gains are fp32; matrices are fp32 (MTMC_F32) or bf16 (MTMC_BF16).
 * blob_on_device: 0 = host pointer, 1 = device pointer.  The caller keeps and frees blob;
 * it is no longer referenced when the call returns (the call synchronises `stream`).
 * Constraints: head_dim 64 or 128, n_q_heads % n_kv_heads == 0,
 * d_model, d_ffn, n_q_heads*head_dim multiples of 16, vocab multiple of 16.
 */
int mtmc_weights_create(const mtmc_config* cfg, const void* blob, size_t blob_bytes,
                        int blob_on_device, void* stream, mtmc_weights** out);
void mtmc_weights_destroy(mtmc_weights* w);

/* Bytes of the canonical blob for a configuration (0 if cfg is invalid). */
size_t mtmc_blob_bytes(const mtmc_config* cfg);

/*
 * mtmc_rollout: for every prompt p < n_prompts and sample s < n_samples, sequence
 * b = p*n_samples + s continues prompt p by max_new tokens.  At step i, with z the logits at
 * the last position of (prompt + tokens sampled so far):
 *     y_v = z_v/T + g_v,  token = argmax_v y_v (lowest index on ties),
 *     logprob = z_token/T - logsumexp_v(z_v/T),
 * g_v = -ln(-ln u_v), u_v = ((r_v >> 9) + 0.5) * 2^-23, r_v = word (v % 4) of
 * Philox4x32-10(counter = (v/4, i, seq_offset + b, 0), key = (seed low, seed high)).
 * temperature == 0 selects greedy decoding (g = 0, T = 1).  No early stop: every sequence
 * runs max_new steps.  The returned log-probability is the factor of Eq. 2 under the
 * sampling distribution (equal to mtmc_score's term when T == 1).
 *
 * prompts      device int32 [n_prompts, prompt_len], ids in [0, vocab)
 * out_ids      device int32 [n_prompts*n_samples, max_new]
 * out_logprobs device float [n_prompts*n_samples, max_new]
 * workspace    device, >= mtmc_rollout_workspace_bytes(...) bytes, 256-byte aligned
 * Out-of-range ids are clamped on the device and reported by the next mtmc_poll_errors.
 * MTMC_BF16 decodes contexts of at most MTMC_MAX_DECODE_CONTEXT tokens: prompt_len + max_new
 * beyond that is MTMC_EINVAL.
 */
#define MTMC_MAX_DECODE_CONTEXT 32768
size_t mtmc_rollout_workspace_bytes(const mtmc_weights* w, int32_t n_prompts, int32_t prompt_len,
                                    int32_t n_samples, int32_t max_new);
int mtmc_rollout(const mtmc_weights* w, const int32_t* prompts, int32_t n_prompts,
                 int32_t prompt_len, int32_t n_samples, int32_t max_new, float temperature,
                 uint64_t seed, uint32_t seq_offset, int32_t* out_ids, float* out_logprobs,
                 void* workspace, size_t workspace_bytes, void* stream);

/*
 * mtmc_rollout_ragged: mtmc_rollout for prompts of different lengths, with an optional stop token
 * (Inference Pipeline, "Macro Thinking": the policy's output ends with a terminal action or at the
 * step limit).  Prompt p is prompts[p, :prompt_lens[p]]; the rest of its row is padding and never
 * influences a result.  Sequence b = p * n_samples + s continues prompt p exactly as mtmc_rollout
 * would continue it alone (same counters of the random generator, so the same noise whatever else is in the
 * batch; calls of the same shape give bit-identical results, and across batch sizes, which select other kernel
 * tilings and so another order of the fp32 sums, log-probabilities agree to about 1e-3 and a sampled id can
 * differ only where two candidates are that close).  With stop_id >= 0 a sequence ends with the first sampled stop_id: that token and
 * its log-probability are reported, every later slot of the row holds stop_id with log-probability
 * 0, and out_lens[b] = number of tokens generated including the stop token (max_new if none).
 * MTMC_BF16: finished sequences give up their place in the batch and the call ends when all have
 * finished (MTMC_OPT_STOP_POLL_STEPS); a call with more sequences than one batch holds (128) runs as one
 * batch that takes the call's next prompts in as sequences finish (MTMC_OPT_ADMIT_PROMPTS).  MTMC_F32: they
 * keep their place.
 *
 * prompts      device int32 [n_prompts, max_prompt_len], right-padded
 * prompt_lens  device int32 [n_prompts], values in [1, max_prompt_len]; a value outside is clamped
 *              and reported by mtmc_poll_errors
 * stop_id      a token id, or negative for none
 * out_lens     device int32 [n_prompts * n_samples]
 * other arguments, errors and workspace rules as for mtmc_rollout, with
 * mtmc_rollout_ragged_workspace_bytes(...); max_prompt_len + max_new <= max_positions.
 */
size_t mtmc_rollout_ragged_workspace_bytes(const mtmc_weights* w, int32_t n_prompts, int32_t max_prompt_len,
                                           int32_t n_samples, int32_t max_new);
int mtmc_rollout_ragged(const mtmc_weights* w, const int32_t* prompts, const int32_t* prompt_lens,
                        int32_t n_prompts, int32_t max_prompt_len, int32_t n_samples, int32_t max_new,
                        float temperature, uint64_t seed, uint32_t seq_offset, int32_t stop_id,
                        int32_t* out_ids, float* out_logprobs, int32_t* out_lens, void* workspace,
                        size_t workspace_bytes, void* stream);

/*
 * mtmc_rollout_ragged_cached: mtmc_rollout_ragged for a prompt that extends the previous call's (Inference
 * Pipeline, "Macro Thinking": the state of optimisation step t + 1 is the state of step t plus the new code and
 * history).  The workspace of a ragged call still holds the keys and values of its prompts; when the first
 * reuse_len positions of EVERY prompt are unchanged since the previous mtmc_rollout_ragged[_cached] call on the
 * same workspace, only the positions from reuse_len on are evaluated again.  Results are those of
 * mtmc_rollout_ragged on the same arguments: bit for bit when both calls run the same matrix kernels, and
 * to the rounding order of the fp32 sums (about 1e-3 in a log-probability) when the number of tokens left
 * to evaluate falls under the size from which the large-batch kernel is used (MTMC_OPT_GEMM_LDS_MIN_BLOCKS).
 *   - reuse_len: a multiple of 16 (whole cache pages), below max_prompt_len; 0 = nothing is kept.
 *   - the previous call on `workspace` must have had the same n_prompts, max_prompt_len, n_samples and max_new
 *     (the cache layout follows from them), else MTMC_EINVAL; the caller must not have written to the
 *     workspace in between, nor used it for another kind of call.
 *   - checked on the device and reported by mtmc_poll_errors as MTMC_DATA_PREFIX (the results are then wrong):
 *     every prompt's first reuse_len ids equal the previous call's, every previous prompt was at least
 *     reuse_len long, every new prompt is longer than reuse_len.
 *   - MTMC_BF16: the call must fit one group (n_prompts * n_samples <= 128).
 */
int mtmc_rollout_ragged_cached(const mtmc_weights* w, const int32_t* prompts, const int32_t* prompt_lens,
                               int32_t n_prompts, int32_t max_prompt_len, int32_t n_samples, int32_t max_new,
                               float temperature, uint64_t seed, uint32_t seq_offset, int32_t stop_id,
                               int32_t reuse_len, int32_t* out_ids, float* out_logprobs, int32_t* out_lens,
                               void* workspace, size_t workspace_bytes, void* stream);

/*
 * mtmc_score: teacher-forced pass over seqs [n_seqs, seq_len].  For i in [0, seq_len-1):
 *     out_logprobs[n, i] = z_i[seqs[n, i+1]] - logsumexp_v z_i[v]     if i + 1 >= prompt_len
 *                        = 0                                           otherwise
 * where z_i are the logits at position i: the log of the i-th factor of Eq. 2 for the
 * action that starts at position prompt_len.  The LM head is not evaluated on unscored
 * positions.  Optional outputs (may be NULL), same shape, 0 where not scored:
 *     out_top1[n, i]   = argmax_v z_i[v] (lowest index on ties)
 *     out_margin[n, i] = largest - second largest logit
 *
 * seqs         device int32 [n_seqs, seq_len]; seq_len >= 2; 1 <= prompt_len <= seq_len
 * out_*        device [n_seqs, seq_len - 1]
 * workspace    device, >= mtmc_score_workspace_bytes(...) bytes, 256-byte aligned
 */
size_t mtmc_score_workspace_bytes(const mtmc_weights* w, int32_t n_seqs, int32_t seq_len);
int mtmc_score(const mtmc_weights* w, const int32_t* seqs, int32_t n_seqs, int32_t seq_len,
               int32_t prompt_len, float* out_logprobs, int32_t* out_top1, float* out_margin,
               void* workspace, size_t workspace_bytes, void* stream);

/*
 * mtmc_score_actions: the policy over each state's candidate actions (Method, "Training
 * Methodology": the action probability of Eq. 2, then the softmax over the candidates).
 * State n has K = n_actions candidates; candidate k is the first action_len[n, k] tokens a_1..a_N
 * of actions[n, k, :] (the rest of the row is padding and never influences a result).
 *     out_token_logprobs[n, k, i] = log P(a_{i+1} | state_n, a_1..a_i)    for i < N, else 0
 *     out_action_logprobs[n, k]   = sum_i out_token_logprobs[n, k, i]     (Eq. 2 in log form);
 *                                   divided by N when normalize != 0 and N > 0 (the paper does not
 *                                   say whether lengths are normalised: off unless asked for)
 *     out_policy_logprobs[n, k]   = out_action_logprobs[n, k] - logsumexp_j out_action_logprobs[n, j]
 * An empty action (N = 0) has log-probability 0.  The state is evaluated once per state, not once
 * per candidate: the K candidates of a state read the same cached keys and values of its tokens.
 * Scoring what mtmc_rollout returned is the case states = the prompts, candidates = the samples of each
 * prompt, every action_len = max_new: out_token_logprobs is then what mtmc_score returns from position
 * prompt_len - 1 on, with each prompt evaluated once instead of once per sample.
 *
 * states       device int32 [n_states, state_len], state_len >= 1
 * actions      device int32 [n_states, n_actions, max_action_len]; padding entries are ignored
 * action_len   device int32 [n_states, n_actions], values in [0, max_action_len]; a value outside
 *              is clamped and reported by mtmc_poll_errors
 * out_token_logprobs   device fp32 [n_states, n_actions, max_action_len]
 * out_action_logprobs, out_policy_logprobs   device fp32 [n_states, n_actions]
 * workspace    device, >= mtmc_score_actions_workspace_bytes(...) bytes, 256-byte aligned
 * state_len + max_action_len must not exceed max_positions.
 */
size_t mtmc_score_actions_workspace_bytes(const mtmc_weights* w, int32_t n_states, int32_t state_len,
                                          int32_t n_actions, int32_t max_action_len);
int mtmc_score_actions(const mtmc_weights* w, const int32_t* states, int32_t n_states, int32_t state_len,
                       const int32_t* actions, const int32_t* action_len, int32_t n_actions,
                       int32_t max_action_len, int32_t normalize, float* out_token_logprobs,
                       float* out_action_logprobs, float* out_policy_logprobs, void* workspace,
                       size_t workspace_bytes, void* stream);

/*
 * mtmc_ppo_clip_loss: the clipped surrogate of the standard PPO update that the policy is trained with
 * (Method, "Training Methodology"), over the samples i < n whose mask is non-zero (all if mask is NULL):
 *     r_i  = exp(new_logprobs[i] - old_logprobs[i])
 *     loss = - mean_i min(r_i A_i, clip(r_i, 1 - clip_eps, 1 + clip_eps) A_i),   A_i = advantages[i]
 * The log-probabilities are what mtmc_score / mtmc_score_actions return (per token or per action) under
 * the current and the behaviour policy.  Value only: no gradient is formed.  clip_eps is the caller's
 * (the paper does not state it).
 *     out[0] = loss   out[1] = fraction of samples with |r_i - 1| > clip_eps
 *     out[2] = mean of old - new log-probability   out[3] = number of samples selected
 * All zero when no sample is selected.  Sums are formed in double in a fixed order (results do not
 * depend on scheduling).
 *
 * new_logprobs, old_logprobs, advantages   device fp32 [n];  mask   device int32 [n] or NULL
 * out          device double [4]
 * workspace    device, >= mtmc_ppo_workspace_bytes() bytes, 256-byte aligned
 */
size_t mtmc_ppo_workspace_bytes(void);
int mtmc_ppo_clip_loss(const float* new_logprobs, const float* old_logprobs, const float* advantages,
                       const int32_t* mask, int64_t n, float clip_eps, double* out, void* workspace,
                       size_t workspace_bytes, void* stream);

/*
 * mtmc_ppo_clip_loss_static: mtmc_ppo_clip_loss for callers that cannot allocate device memory or pass a
 * workspace -- code under HIP-graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments (without the workspace), same kernels, same results bit for bit.  The per-workgroup partial sums
 * live in a 32 KiB array that is part of the library's device code (one copy per GPU, held until the process
 * ends); the call allocates and frees nothing.  Limits and rules:
 *   - n <= MTMC_PPO_STATIC_MAX_SAMPLES, else MTMC_EINVAL (a larger job goes through mtmc_ppo_clip_loss);
 *   - every call on a GPU uses that GPU's one array: calls that may overlap on one GPU (different streams,
 *     different threads) race on it and must be ordered by the caller; calls on one stream are ordered;
 *   - the array keeps the previous call's partial sums; every call overwrites the entries it reads.
 */
#define MTMC_PPO_STATIC_MAX_SAMPLES 268435456
int mtmc_ppo_clip_loss_static(const float* new_logprobs, const float* old_logprobs, const float* advantages,
                              const int32_t* mask, int64_t n, float clip_eps, double* out, void* stream);

/*
 * Synchronises `stream`, then returns MTMC_EDATA if any kernel since the last poll raised a bit of the
 * device's sticky data flag (the flag is cleared; mtmc_last_error() names the causes), MTMC_EHIP on a
 * runtime error, else MTMC_OK.  The bits:
 *   MTMC_DATA_TOKEN_ID    a token id outside [0, vocab) (clamped into range)
 *   MTMC_DATA_WEIGHT      a weight that is not finite or, MTMC_BF16, exceeds 65504 in magnitude
 *                         (mtmc_weights_create fails with MTMC_EINVAL on it)
 *   MTMC_DATA_LENGTH      an action or prompt length outside its range (clamped)
 *   MTMC_DATA_PREFIX      mtmc_rollout_ragged_cached: the cached prefix does not match the new prompts
 *   MTMC_DATA_FP16_RANGE  MTMC_BF16: an activation, a rotated query or key, a value or an attention output
 *                         had to be clamped to +-65504 (a NaN becomes -65504) where it is stored as fp16, or
 *                         every logit of a row was NaN (token 0 is then reported).  Outputs of the calls
 *                         since the last poll are unreliable.
 * mtmc_data_error_string returns the text for a set of bits (valid until the thread's next call of it).
 */
#define MTMC_DATA_TOKEN_ID   1
#define MTMC_DATA_WEIGHT     2
#define MTMC_DATA_LENGTH     4
#define MTMC_DATA_FP16_RANGE 8
#define MTMC_DATA_PREFIX     16
/*
 * Host logic of the rollout that takes in prompts as it runs (MTMC_OPT_ADMIT_PROMPTS), exposed so that it can be
 * checked without a GPU; makes no GPU call.  Which of the call's remaining prompts join the batch at one look:
 *   live [n_slots]         1 when the slot holds a sequence that still runs, else 0
 *   slot_region [n_slots]  region of shared prompt pages that the slot's sequence reads (< n_regions)
 * A prompt needs n_samples free slots and a region that no running sequence reads.  Returns
 * k = min(free slots / n_samples, free regions, prompts_left, max_at_once), or 0 while k < min(prompts_left,
 * wait_for, max_at_once) and some sequence still runs (a prefill costs about the same for one prompt as for a few);
 * out_slots [k * n_samples] = the lowest free slots, n_samples per prompt, out_regions [k] = the lowest free
 * regions (both host arrays with room for the largest k).  MTMC_EINVAL (negative) for a NULL pointer or a
 * count below 1 (prompts_left may be 0).
 */
int mtmc_admission_plan(const int32_t* live, const int32_t* slot_region, int32_t n_slots, int32_t n_regions,
                        int32_t n_samples, int32_t prompts_left, int32_t max_at_once, int32_t wait_for,
                        int32_t* out_slots, int32_t* out_regions);

int mtmc_poll_errors(const mtmc_weights* w, void* stream);
const char* mtmc_data_error_string(int bits);

/*
 * Tuning switches.
 *   MTMC_OPT_HIP_GRAPH (default 1): mtmc_rollout captures one decode step into a HIP graph and
 *   replays it for every token.  Results do not depend on it (same kernels in the same order).
 *   Instantiated graphs are cached inside `w`, keyed by workspace address and the call's shape; replacing
 *   a cached graph (more than 8 are never kept) synchronises the device once.  When `stream` is itself being captured the steps
 *   are launched directly.
 *   MTMC_OPT_GEMM_LDS_MIN_BLOCKS (default 32, value >= 1): prefill / scoring GEMMs (MTMC_BF16)
 *   whose output has at least this many 256 x 256 blocks run in the LDS-staged kernel, smaller
 *   ones in the direct 128 x 128 kernel.  Both sum over K in the same order; results agree to
 *   the fp32 rounding inside the matrix instruction.
 *   MTMC_OPT_STOP_POLL_STEPS (default 32, 0 = off): MTMC_BF16 rollouts with a stop token look at the rows'
 *   stop flags every this many decode steps.  The look itself is queued on the stream; the host reads it one
 *   period later (so the GPU never waits for the host), ends the call once every row has stopped and packs
 *   the rows still running into fewer 16-row tiles when that frees a tile, so that a batch costs less as
 *   its rows finish.  With it the call blocks the calling thread on the stream (it returns when at most
 *   two periods of work are still queued) and calls with a stop token on one weights handle take turns;
 *   with 0, or when `stream` is being captured, the call only enqueues, as mtmc_rollout does, every row keeps
 *   its place, and the call costs what it costs without a stop token.  Packing changes the tiling, hence
 *   the order of the fp32 sums, of the steps after it: log-probabilities then agree with the unpacked call's
 *   to about 1e-3 (an id can differ where two candidates are that close), and with the definition as
 *   closely as before.
 *   MTMC_OPT_ADMIT_PROMPTS (default 1): a MTMC_BF16 mtmc_rollout_ragged call with a stop token, more than 128
 *   sequences and MTMC_OPT_STOP_POLL_STEPS > 0 runs as one batch of 128 slots; every min(8, poll steps) steps the
 *   calling thread waits for the stream, and prompts of the call that find n_samples free slots (left by
 *   sequences that have ended) are prefilled and join the batch, each sequence at its own step; when no prompt is
 *   left the sequences still running are packed as described above.  A sequence's random numbers go by its row and
 *   its own step, so results are those of the call that runs batch after batch (value 0) up to the rounding order
 *   of the fp32 sums (step 0 of a prompt that joins is sampled in a smaller batch, the packed batch runs other
 *   tilings): about 1e-3 in a log-probability, an id can differ where two candidates are that close.  Not used
 *   when `stream` is being captured, without a stop token, or with a cached prefix.
 */
#define MTMC_OPT_HIP_GRAPH 1
#define MTMC_OPT_GEMM_LDS_MIN_BLOCKS 2
#define MTMC_OPT_STOP_POLL_STEPS 3
#define MTMC_OPT_ADMIT_PROMPTS 4
int mtmc_set_option(mtmc_weights* w, int option, int value);

/*
 * Diagnostics for measurement: HIP-event timing of one class of decode kernel inside mtmc_rollout
 * (MTMC_BF16).  While a class is selected, every `every_n_steps`-th decode step is launched
 * directly instead of through the captured graph, with an event pair around each launch of
 * that class (same kernels, same results).  mtmc_kernel_timer_read synchronises `stream` and
 * returns the summed duration and the number of timed launches since the last read; if
 * `empty_pair_ms` is not NULL it receives the mean duration of event pairs recorded back to back
 * with nothing between them (one such pair per timed step: what the bracketing itself adds).
 * kernel_class 0 switches the timer off.
 */
#define MTMC_KERNEL_QKV       1  /* QKV projection                              */
#define MTMC_KERNEL_ATTENTION 2  /* rope + KV append + paged attention          */
#define MTMC_KERNEL_GATE_UP   3  /* gate/up projection with SwiGLU epilogue     */
#define MTMC_KERNEL_DOWN      4  /* down projection (split-K partial sums)      */
#define MTMC_KERNEL_LM_HEAD   5  /* LM head + log-softmax + Gumbel-max + merge  */
int mtmc_kernel_timer(mtmc_weights* w, int kernel_class, int every_n_steps);
int mtmc_kernel_timer_read(mtmc_weights* w, void* stream, double* total_ms, int64_t* launches,
                           double* empty_pair_ms);

/*
 * Diagnostics for measurement: copies `bytes` (a multiple of 16; both device pointers 16-byte
 * aligned, ranges not overlapping) from src to dst with one plain copy kernel.  A kernel that is
 * known to read and to write exactly `bytes`: hardware byte counters of a profiled run are scaled
 * by what they report for it.  Stream-ordered, does not synchronise.
 */
int mtmc_copy_probe(void* dst, const void* src, size_t bytes, void* stream);

/*
 * Diagnostics for measurement: what the device sustains, to be reported beside its published peaks.
 * mtmc_read_probe reads `bytes` (a positive multiple of 16384; src device, 16-byte aligned) once with a plain
 * streaming kernel and discards them (sink: 4 writable device bytes).  mtmc_mfma_probe runs `iters` rounds of
 * sixteen fp16 32x32x16 matrix instructions (four A fragments times four B fragments of pseudo-random values, on
 * sixteen accumulator blocks) in every wavefront of `workgroups` workgroups of four wavefronts, on registers
 * only (out: device floats [workgroups * 256], overwritten), and returns in *flops the floating-point
 * operations of the launch.  Both are stream-ordered and do not synchronise: the caller
 * brackets them with events.
 */
int mtmc_read_probe(const void* src, size_t bytes, void* sink, void* stream);
int mtmc_mfma_probe(float* out, int32_t workgroups, int32_t iters, void* stream, double* flops);

/* Message of the last failing call on this thread; valid until the next library call. */
const char* mtmc_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* MTMC_H */
