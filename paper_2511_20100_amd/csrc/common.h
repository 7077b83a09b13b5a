// Internal declarations shared by the library's translation units (not part of the C boundary).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <mutex>
#include <string>
#include <vector>

#include "mtmc.h"

namespace mtmc {

constexpr int kPageTokens = 16;

void set_error(const std::string& msg);

#define MTMC_HIP_CHECK(expr)                                                              \
  do {                                                                                    \
    hipError_t e_ = (expr);                                                               \
    if (e_ != hipSuccess) {                                                               \
      ::mtmc::set_error(std::string(#expr) + ": " + hipGetErrorString(e_));              \
      return MTMC_EHIP;                                                                   \
    }                                                                                     \
  } while (0)

#define MTMC_REQUIRE(cond, msg)                                                           \
  do {                                                                                    \
    if (!(cond)) {                                                                        \
      ::mtmc::set_error(std::string("invalid argument: ") + (msg));                       \
      return MTMC_EINVAL;                                                                 \
    }                                                                                     \
  } while (0)

// How the tokens of a launch map to sequences and positions.  Token t belongs to sequence
// t / S, sits at position base + (*d_step if d_step) + t % S with base = row_pos[t / S] if row_pos
// is given (sequences of different lengths), else pos_base, and uses row (t / S) * row_stride of
// the page table.
struct TokMap {
  int S;
  int row_stride;
  int pos_base;
  const int* d_step;
  const int* row_pos;
};

// Where the KV pages live.  Page `pg` of (layer l, which in {0 = K, 1 = V}, kv head g) starts at
// element (((l * 2 + which) * n_pages + pg) * n_kv_heads + g) * 16 * head_dim.
struct KvPool {
  void* base;
  int n_pages;
  int n_kv_heads;
  int head_dim;
  const int* page_table;  // [rows, max_pages]
  int max_pages;
};

struct GraphCache;  // engine_bf16.hip

// What the library remembers (on the host) of the last mtmc_rollout_ragged* call on a workspace: a later call may
// keep that call's cached prompt prefix only if it has the same shape, hence the same page layout.
struct RaggedCallRecord {
  const void* workspace;
  int n_prompts, max_prompt_len, n_samples, max_new;
};

struct LayerWeights {
  const float* attn_norm;
  const float* ffn_norm;
  const void* wqkv;    // [(Hq + 2 Hkv) hd, d]
  const void* wo;      // [d, Hq hd]
  const void* wgu;     // fp32: [2F, d] (gate rows, then up rows); bf16: 16-row blocks gate/up interleaved
  const void* wdown;   // [d, F]
};

}  // namespace mtmc

struct mtmc_weights {
  mtmc_config cfg;
  int device;
  void* storage;        // single device allocation behind every weight pointer below
  void* aux;            // device allocation holding the rotary tables and the error flag
  size_t storage_bytes;
  const void* embed;    // [V, d] row-major in the storage type
  const float* final_norm;
  const void* lm_head;  // [V, d]
  std::vector<mtmc::LayerWeights> layers;
  const float* rope_cos;  // [max_positions, hd/2]
  const float* rope_sin;
  int* err_flag;        // device int, non-zero once a bad token id was seen
  int d_ffn_pad;        // F rounded up to the K-tile of the bf16 kernels (== F for fp32)
  int opt_hip_graph;    // replay decode steps as a captured HIP graph (default 1)
  int opt_lds_min_blocks;  // output blocks (256 x 256) from which large GEMMs use the LDS-staged kernel
  int opt_stop_poll;       // decode steps between two looks at the stop flags of a rollout with a stop token (0: never)
  int opt_admit;           // a rollout with a stop token and more sequences than one batch holds runs as one batch
                           // that takes in the next prompts as sequences finish and leave slots (0: batch after batch)
  mtmc::GraphCache* graphs;  // instantiated decode-step graphs, keyed by workspace and shape
  std::mutex* ragged_mu;     // guards ragged_calls
  std::vector<mtmc::RaggedCallRecord> ragged_calls;  // at most 16, oldest dropped first
};
