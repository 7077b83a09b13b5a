// Host-side launchers of the HIP kernels.  Every launcher only enqueues on `st`.
#pragma once

#include "common.h"

namespace mtmc {

// ---------------------------------------------------------------- shared (layout / control)
// Page table of a rollout: row b, entry j -> shared page (b / n_samples) * n_full + j for
// j < n_full, else private page shared_total + b * (max_pages - n_full) + (j - n_full).
void launch_build_page_table(int* table, int rows, int max_pages, int n_samples, int n_full,
                             int shared_total, hipStream_t st);
void launch_set_int(int* p, int v, hipStream_t st);
void launch_add_int(int* p, int v, hipStream_t st);
void launch_fill_u32(uint32_t* p, uint32_t v, size_t n, hipStream_t st);
void launch_copy_probe(void* dst, const void* src, size_t bytes, hipStream_t st);
// dst[r, :] = src[(r / n_rep) * src_stride + src_offset + (r % n_rep) * rep_stride, :]
void launch_gather_rows(float* dst, const float* src, int rows, int d, int n_rep, int src_stride,
                        int src_offset, int rep_stride, hipStream_t st);
// For every row b with b % n_samples != 0: page table[b][page_idx] := copy of page
// table[b - b % n_samples][page_idx], in every (layer, K/V).  elem_bytes is the KV element size.
void launch_fork_tail_pages(KvPool pool, int n_layers, int rows, int n_samples, int page_idx,
                            int elem_bytes, hipStream_t st);

// Rollout of prompts of different lengths (lens [n_prompts], clamped to [1, Lmax]; a value outside
// raises bit 4 of *err_flag).  Row b = p n_samples + s: table entry j is shared page p nf_max + j for
// j < lens[p] / 16, else private page shared_total + b max_pages + j; row_pos[b] = lens[p] - 1;
// done[b] = 0; out_lens[b] = max_new.  prompt_ids [n_prompts, Lmax] = prompts with the padding set to 0.
// reuse_len > 0 (a multiple of 16): the first reuse_len positions of every prompt keep the cached keys and values
// that the previous call left in the workspace.  That needs, per prompt: the same first reuse_len ids as the
// previous call's (compared with prompt_ids before it is overwritten), a previous length of at least reuse_len
// (row_pos before it is overwritten) and a new length above reuse_len; a violation raises bit 16 of *err_flag.
// suffix_ids [n_prompts, Lmax - reuse_len] = the ids from position reuse_len on (what is left to prefill).
void launch_ragged_setup(int* table, int* row_pos, int* done, int* out_lens, int* prompt_ids, int* suffix_ids,
                         const int* prompts, const int* lens, int n_prompts, int n_samples, int Lmax, int max_pages,
                         int nf_max, int shared_total, int max_new, int reuse_len, int* err_flag, hipStream_t st);
// For every row b with b % n_samples != 0 whose prompt length is not a multiple of the page size: the page
// that holds the prompt's last tokens := copy of that page of row b - b % n_samples, in every (layer, K/V).
void launch_fork_tail_pages_ragged(KvPool pool, int n_layers, int rows, int n_samples, const int* lens, int Lmax,
                                   int elem_bytes, hipStream_t st);
// dst[p n_samples + s, :] = src[p (Lmax - pos_base) + lens[p] - 1 - pos_base, :] for p < n_prompts, s < n_samples:
// the hidden row of a prompt's last token when src holds the positions pos_base .. Lmax - 1 of every prompt.
void launch_gather_last_rows(float* dst, const float* src, int d, int n_prompts, int n_samples, int Lmax,
                             const int* lens, int pos_base, hipStream_t st);

// Action-level scoring.  vseq [n_states K, A + 1]: row n K + k = last token of state n, then the
// tokens of candidate k, then zeros; prefix [n_states, P - 1]: the states without their last token.
// An action_len outside [0, A] raises bit 4 of *err_flag and is clamped.
void launch_build_action_seqs(int* vseq, int* prefix, const int* states, const int* actions,
                              const int* action_len, int n_states, int P, int K, int A, int* err_flag,
                              hipStream_t st);
// token_lp [n_states K, A] in place: padding cleared; out_action = per-candidate sums (divided by the
// length if normalize); out_policy = their log-softmax over the K candidates of a state.
void launch_action_reduce(float* token_lp, const int* action_len, int n_states, int K, int A, int normalize,
                          float* out_action, float* out_policy, hipStream_t st);

// probes.hip: a plain streaming read of `bytes` (a multiple of 16 KiB is read completely) and a register-only
// loop of matrix instructions (returns the flops the launch performs; out holds workgroups * 256 floats)
void launch_read_probe(const void* src, size_t bytes, void* sink, hipStream_t st);
double launch_mfma_probe(float* out, int workgroups, int iters, hipStream_t st);
// Clipped PPO surrogate over n samples (mask may be NULL); out = {loss, clip fraction, approx KL, count} as
// doubles; workspace of ppo_workspace_bytes() bytes holds the per-workgroup partial sums.
size_t ppo_workspace_bytes();
// Device address of the current GPU's file-scope scratch array of ppo_workspace_bytes() bytes (MTMC_OK or an error).
int ppo_static_scratch(void** out);
void launch_ppo_clip_loss(const float* new_logp, const float* old_logp, const float* adv, const int* mask,
                          long long n, double eps, double* out, void* workspace, hipStream_t st);

// ---------------------------------------------------------------- fp32 path
namespace f32 {
void embed(float* h, const int* ids, int T, const float* E, int d, int vocab, int* err_flag,
           hipStream_t st);
void rmsnorm(float* x, const float* h, const float* gain, float eps, int T, int d, hipStream_t st);
// C[M, N] (ldc) = or += A[M, K] (lda) * W[N, K]^T      (K % 16 == 0)
void gemm(float* C, int ldc, const float* A, int lda, const float* W, int M, int N, int K,
          bool accumulate, hipStream_t st);
// qkv [T, (Hq + 2 Hkv) hd]: rotates q in place, writes rotated k and v into the pages.
void rope_kv_write(float* qkv, int T, int Hq, int Hkv, int hd, const float* cos, const float* sin,
                   TokMap map, KvPool pool, int layer, hipStream_t st);
// o [T, Hq hd] = causal grouped-query attention of the (rotated) q in qkv over the pages.
void attention(float* o, const float* qkv, int T, int Hq, int Hkv, int hd, TokMap map, KvPool pool,
               int layer, hipStream_t st);
void swiglu(float* a, const float* gu, int T, int F, hipStream_t st);  // gu [T, 2F] -> a [T, F]
// Gumbel-max sampling from materialised logits [B, V] at step *d_step; writes out_ids[b, step],
// out_logprobs[b, step] and cur_ids[b].
// With done != NULL (stop token in use): a row whose done flag is set reports stop_id with log-prob 0; a row
// that samples stop_id sets its flag and out_lens[b] = step + 1.
void sample(const float* logits, int B, int V, float inv_temp, int greedy, uint64_t seed,
            uint32_t seq_offset, const int* d_step, int max_new, int* cur_ids, int* out_ids,
            float* out_logprobs, int stop_id, int* done, int* out_lens, hipStream_t st);
// Teacher-forced scoring from materialised logits [R, V].  Row r is position
// i = first + (row0 + r) % n_scored of sequence n = seq0 + (row0 + r) / n_scored; its target is
// seqs[n, i + 1] and its output slot [n, i] of the [*, S - 1] outputs.
void score_rows(const float* logits, int R, int V, const int* seqs, int S, int first, int n_scored,
                int seq0, int row0, float* out_logprobs, int* out_top1, float* out_margin,
                int* err_flag, hipStream_t st);
}  // namespace f32

}  // namespace mtmc
