// bf16 path: weight store (re-tiled for the MFMA kernels), workspace extras and the schedulers.
// Weights and KV cache are bf16; the residual stream, norms, softmax and all accumulators fp32.
#include <algorithm>
#include <array>
#include <mutex>

#include "bf16_kernels.h"
#include "engine.h"
#include "kernels.h"

namespace mtmc {

// Instantiated decode-step graphs.  A graph bakes in the workspace pointers and the group
// shape; everything that changes between calls (seed, temperature, output pointers, step
// counter) lives in device memory that the kernels read.
struct GraphCache {
  struct Entry {
    // every pointer and split factor a captured launch holds follows from the workspace base and the shape of the
    // WHOLE call (the plan), plus the rows of the group the step belongs to
    const void* workspace;
    int total_prompts, B, prompt_len, n_samples, max_new, ragged;
    hipGraphExec_t exec;
  };
  std::mutex mu;
  std::vector<Entry> entries;
  hipStream_t capture_stream = nullptr;  // never runs work: launches on it are only recorded
  // kernel timer (diagnostics): event pairs recorded around one class of decode kernel
  int timer_class = 0, timer_every = 0;
  std::vector<hipEvent_t> events;  // pool, used pairwise
  size_t events_used = 0;
  std::vector<hipEvent_t> empty_events;  // pairs recorded back to back (what a pair costs by itself)
  size_t empty_used = 0;
  // rollouts with a stop token: where the host reads the number of live rows (pinned, two slots used in turn)
  std::mutex poll_mu;                    // one such rollout at a time per weights handle
  int* host_live = nullptr;
  hipEvent_t poll_events[2] = {nullptr, nullptr};
  int* host_slots = nullptr;            // pinned: which slots hold a sequence that still runs (a batch that takes in prompts)
};

// Brackets launches of one kernel class with HIP events while a decode step is launched directly.
struct KernelTimer {
  GraphCache* gc;
  int cls;
  hipStream_t st;
  void mark(int k) {
    if (!gc || k != cls) return;
    if (gc->events_used == gc->events.size()) {
      hipEvent_t e = nullptr;
      if (hipEventCreate(&e) != hipSuccess) return;
      gc->events.push_back(e);
    }
    (void)hipEventRecord(gc->events[gc->events_used++], st);
  }
  // Two events with nothing between them, once per timed step.
  void mark_empty_pair() {
    if (!gc || !cls) return;
    for (int i = 0; i < 2; ++i) {
      if (gc->empty_used == gc->empty_events.size()) {
        hipEvent_t e = nullptr;
        if (hipEventCreate(&e) != hipSuccess) return;
        gc->empty_events.push_back(e);
      }
      (void)hipEventRecord(gc->empty_events[gc->empty_used++], st);
    }
  }
};

void destroy_graph_cache(mtmc_weights* w) {
  if (!w->graphs) return;
  for (auto& e : w->graphs->entries) (void)hipGraphExecDestroy(e.exec);
  if (w->graphs->capture_stream) (void)hipStreamDestroy(w->graphs->capture_stream);
  for (hipEvent_t e : w->graphs->events) (void)hipEventDestroy(e);
  for (hipEvent_t e : w->graphs->empty_events) (void)hipEventDestroy(e);
  for (hipEvent_t e : w->graphs->poll_events)
    if (e) (void)hipEventDestroy(e);
  if (w->graphs->host_live) (void)hipHostFree(w->graphs->host_live);
  if (w->graphs->host_slots) (void)hipHostFree(w->graphs->host_slots);
  delete w->graphs;
  w->graphs = nullptr;
}

int kernel_timer_set(mtmc_weights* w, int cls, int every) {
  if (!w->graphs) w->graphs = new GraphCache();
  std::lock_guard<std::mutex> lock(w->graphs->mu);
  w->graphs->timer_class = cls;
  w->graphs->timer_every = every;
  w->graphs->events_used = 0;
  w->graphs->empty_used = 0;
  return MTMC_OK;
}

int kernel_timer_read(mtmc_weights* w, hipStream_t st, double* total_ms, int64_t* launches, double* empty_pair_ms) {
  *total_ms = 0.0;
  *launches = 0;
  if (empty_pair_ms) *empty_pair_ms = 0.0;
  if (!w->graphs) return MTMC_OK;
  MTMC_HIP_CHECK(hipStreamSynchronize(st));
  std::lock_guard<std::mutex> lock(w->graphs->mu);
  GraphCache& gc = *w->graphs;
  for (size_t i = 0; i + 1 < gc.events_used; i += 2) {
    float ms = 0.f;
    MTMC_HIP_CHECK(hipEventElapsedTime(&ms, gc.events[i], gc.events[i + 1]));
    *total_ms += ms;
    *launches += 1;
  }
  gc.events_used = 0;
  double empty = 0.0;
  for (size_t i = 0; i + 1 < gc.empty_used; i += 2) {
    float ms = 0.f;
    MTMC_HIP_CHECK(hipEventElapsedTime(&ms, gc.empty_events[i], gc.empty_events[i + 1]));
    empty += ms;
  }
  if (empty_pair_ms && gc.empty_used >= 2) *empty_pair_ms = empty / (double)(gc.empty_used / 2);
  gc.empty_used = 0;
  return MTMC_OK;
}

namespace {
inline int tiles16(int n) { return (n + 15) / 16; }

inline int tiles32(int n) { return (n + 31) / 32; }

// Split-K factor of a decode GEMM: as many workgroups as fit into ONE round on the 256 CUs (a CU
// that hosts two of them takes twice as long), while every wavefront (4 per workgroup) still
// walks at least two k tiles.
int choose_ksplit(int n_tiles, int k_tiles, int m_tiles) {
  const int nb = bf16::dec_wide_nb(m_tiles);
  const int groups = (n_tiles + nb - 1) / nb;
  const int want = std::max(1, 256 / groups);
  return std::max(1, std::min(want, k_tiles / 8));
}

struct Dims {
  int d, Hq, Hkv, nq, nqkv, F, V;
  int kt_d, kt_nq, kt_F;          // k tiles (32) of the three reduction widths
  int nt_qkv, nt_d, nt_gu, nt_V;  // n tiles (16) of the weight matrices
};
Dims dims_of(const mtmc_weights* w) {
  const mtmc_config& c = w->cfg;
  Dims D;
  D.d = c.d_model; D.Hq = c.n_q_heads; D.Hkv = c.n_kv_heads; D.nq = D.Hq * c.head_dim;
  D.nqkv = (D.Hq + 2 * D.Hkv) * c.head_dim; D.F = w->d_ffn_pad; D.V = c.vocab;
  D.kt_d = tiles32(D.d); D.kt_nq = tiles32(D.nq); D.kt_F = D.F / 32;
  D.nt_qkv = tiles16(D.nqkv); D.nt_d = tiles16(D.d); D.nt_gu = 2 * (D.F / 16); D.nt_V = tiles16(D.V);
  return D;
}
}  // namespace

// ======================================================================================
// weights
// ======================================================================================
int bf16_store_weights(mtmc_weights* w, const BlobLayout& lay, const void* blob, bool on_device,
                       hipStream_t st) {
  const mtmc_config& c = w->cfg;
  w->d_ffn_pad = (c.d_ffn + 31) / 32 * 32;
  const Dims D = dims_of(w);
  for (const BlobLayerOffsets& o : lay.layers) {
    if (o.wk != o.wq + (size_t)D.nq * D.d * 2 || o.wv != o.wk + (size_t)D.Hkv * c.head_dim * D.d * 2) {
      set_error("Wq/Wk/Wv must be contiguous in the blob");
      return MTMC_EINVAL;
    }
  }
  void* dev_blob = nullptr;
  const char* src = (const char*)blob;
  if (!on_device) {
    if (hipMalloc(&dev_blob, lay.total) != hipSuccess) {
      set_error("hipMalloc failed for the staging copy of the blob");
      return MTMC_ENOMEM;
    }
    if (hipMemcpyAsync(dev_blob, blob, lay.total, hipMemcpyHostToDevice, st) != hipSuccess) {
      (void)hipFree(dev_blob);
      set_error("upload of the weight blob failed");
      return MTMC_EHIP;
    }
    src = (const char*)dev_blob;
  }
  // ---- carve the library-owned storage
  Carver cv(nullptr);
  auto plan = [&](Carver& k) {
    struct Out { bf16_t* embed; h16_t* lm; float* fnorm; std::vector<std::array<void*, 6>> L; } o;
    o.embed = k.take<bf16_t>((size_t)D.V * D.d);
    o.lm = k.take<h16_t>((size_t)D.nt_V * D.kt_d * 512);
    o.fnorm = k.take<float>(D.d);
    o.L.resize(c.n_layers);
    for (auto& l : o.L) {
      l[0] = k.take<float>(D.d);
      l[1] = k.take<float>(D.d);
      l[2] = k.take<h16_t>((size_t)D.nt_qkv * D.kt_d * 512);
      l[3] = k.take<h16_t>((size_t)D.nt_d * D.kt_nq * 512);
      l[4] = k.take<h16_t>((size_t)D.nt_gu * D.kt_d * 512);
      l[5] = k.take<h16_t>((size_t)D.nt_d * D.kt_F * 512);
    }
    return o;
  };
  plan(cv);
  const size_t total = cv.off + 256;
  if (hipMalloc(&w->storage, total) != hipSuccess) {
    if (dev_blob) (void)hipFree(dev_blob);
    set_error("hipMalloc failed for the weights (" + std::to_string(total) + " bytes)");
    return MTMC_ENOMEM;
  }
  w->storage_bytes = total;
  Carver real((char*)w->storage);
  auto o = plan(real);
  int rc = MTMC_OK;
  auto copy = [&](void* dst, size_t off, size_t bytes) {
    if (rc == MTMC_OK && hipMemcpyAsync(dst, src + off, bytes, hipMemcpyDeviceToDevice, st) != hipSuccess) {
      set_error("device copy of a weight tensor failed");
      rc = MTMC_EHIP;
    }
  };
  copy(o.embed, lay.embed, (size_t)D.V * D.d * 2);
  bf16::check_finite_bf16((const bf16_t*)(src + lay.embed), (size_t)D.V * D.d, w->err_flag, st);
  copy(o.fnorm, lay.final_norm, (size_t)D.d * 4);
  bf16::retile_weight(o.lm, (const bf16_t*)(src + lay.lm_head), D.V, D.d, D.nt_V, D.kt_d, w->err_flag, st);
  w->embed = o.embed;
  w->lm_head = o.lm;
  w->final_norm = o.fnorm;
  w->layers.resize(c.n_layers);
  for (int l = 0; l < c.n_layers; ++l) {
    const BlobLayerOffsets& b = lay.layers[l];
    copy(o.L[l][0], b.attn_norm, (size_t)D.d * 4);
    copy(o.L[l][1], b.ffn_norm, (size_t)D.d * 4);
    bf16::retile_weight((h16_t*)o.L[l][2], (const bf16_t*)(src + b.wq), D.nqkv, D.d, D.nt_qkv, D.kt_d, w->err_flag, st);
    bf16::retile_weight((h16_t*)o.L[l][3], (const bf16_t*)(src + b.wo), D.d, D.nq, D.nt_d, D.kt_nq, w->err_flag, st);
    bf16::retile_gate_up((h16_t*)o.L[l][4], (const bf16_t*)(src + b.wgate), (const bf16_t*)(src + b.wup),
                         c.d_ffn, D.d, D.F / 16, D.kt_d, w->err_flag, st);
    bf16::retile_weight((h16_t*)o.L[l][5], (const bf16_t*)(src + b.wdown), D.d, c.d_ffn, D.nt_d, D.kt_F, w->err_flag, st);
    LayerWeights& L = w->layers[l];
    L.attn_norm = (const float*)o.L[l][0];
    L.ffn_norm = (const float*)o.L[l][1];
    L.wqkv = o.L[l][2];
    L.wo = o.L[l][3];
    L.wgu = o.L[l][4];
    L.wdown = o.L[l][5];
  }
  if (rc == MTMC_OK && hipGetLastError() != hipSuccess) {
    set_error("a weight re-tiling kernel failed to launch");
    rc = MTMC_EHIP;
  }
  if (hipStreamSynchronize(st) != hipSuccess && rc == MTMC_OK) {
    set_error("hipStreamSynchronize failed while re-tiling the weights");
    rc = MTMC_EHIP;
  }
  if (dev_blob) (void)hipFree(dev_blob);
  if (rc == MTMC_OK) {
    int flag = 0;
    MTMC_HIP_CHECK(hipMemcpy(&flag, w->err_flag, sizeof(int), hipMemcpyDeviceToHost));
    if (flag & 2) {
      (void)hipMemset(w->err_flag, 0, sizeof(int));
      set_error("invalid argument: a weight is not finite or exceeds 65504 in magnitude (the matrix "
                "cores run on fp16 copies of the bf16 weights)");
      return MTMC_EINVAL;
    }
  }
  return rc;
}

// ======================================================================================
// workspace extras
// ======================================================================================
namespace {
// Launch shape of the decode kernels for B rows in bt 16-row tiles.
struct DecodeTune {
  int ks_qkv, ks_o, ks_down, down_nb, n_chunks, chunk_pages, split_at_prompt;
};
DecodeTune tune_decode(const Dims& D, int B, int bt, int max_pages) {
  DecodeTune t;
  t.ks_qkv = choose_ksplit(D.nt_qkv, D.kt_d, bt);
  t.ks_o = choose_ksplit(D.nt_d, D.kt_nq, bt);
  t.ks_down = choose_ksplit(D.nt_d, D.kt_F, bt);
  // A small down projection (each workgroup's share of the weights under 256 KB) is bound by fixed costs and by
  // what few wavefronts pull per CU: two row tiles and 8 wavefronts per workgroup, half the K splits (1.3-1.7 %
  // of the step at d 1536 / F 8960; at d 3584 / F 18944 the doubled activation reads cost 1.3 % instead).
  t.down_nb = 4;
  if (bt <= 4 && 4 * (D.kt_F / t.ks_down) < 256) {
    t.down_nb = 2;
    t.ks_down = std::max(1, std::min(256 / ((D.nt_d + 1) / 2), D.kt_F / 16));
    // ... and where 8 splits of three-tile workgroups still are one round, the split is aligned to the 8 XCDs: each
    // XCD then fetches its eighth of the activation operand (64 x F fp16) instead of all of it
    if ((D.nt_d + 2) / 3 * 8 <= 256 && D.kt_F >= 8 * 10) {
      t.down_nb = 3;
      t.ks_down = 8;
    }
  }
  // context split of the decode attention: for small batches up to about 128 workgroups of 8 wavefronts, and two
  // ways at 33..64 rows when that still leaves at most 256 workgroups (the O projection combines two chunks in its 12-wavefront form at little
  // extra cost; with its 8-wavefront form the split lost what the attention gained)
  const int want = std::max(bt >= 3 && bt <= 4 && B * D.Hkv <= 128 ? 2 : 1, 128 / std::max(1, B * D.Hkv));
  // the O projection that combines the chunks holds (row tiles per workgroup) * chunks <= 8 operand sets: its
  // workgroups take one row tile up to 32 rows and two beyond
  const int max_chunks = bt <= 2 ? 8 : 4;
  t.n_chunks = std::max(1, std::min({want, (max_pages + 7) / 8, max_chunks}));
  t.chunk_pages = ((max_pages + t.n_chunks - 1) / t.n_chunks + 1) / 2 * 2;
  // page ids of a chunk are staged in LDS; kMaxDecodeContext keeps the chunk count within max_chunks
  t.chunk_pages = std::min(t.chunk_pages, 512);
  t.n_chunks = (max_pages + t.chunk_pages - 1) / t.chunk_pages;
  t.chunk_pages = ((max_pages + t.n_chunks - 1) / t.n_chunks + 1) / 2 * 2;  // equal chunks again after the clamp
  t.n_chunks = (max_pages + t.chunk_pages - 1) / t.chunk_pages;
  // the two-way split at 33..64 rows is made at the end of each sequence's prompt (its shared pages | its own):
  // independent of max_new and of the other sequences, and about even when prompts and generations are of a size
  t.split_at_prompt = (bt >= 3 && bt <= 4 && t.n_chunks == 2 && max_pages <= 512) ? 1 : 0;
  return t;
}
void apply_tune(RolloutPlan& p, const DecodeTune& t) {
  p.ks_qkv = t.ks_qkv; p.ks_o = t.ks_o; p.ks_down = t.ks_down; p.down_nb = t.down_nb;
  p.n_chunks = t.n_chunks; p.chunk_pages = t.chunk_pages; p.split_at_prompt = t.split_at_prompt;
}
}  // namespace

void bf16_plan_rollout_extra(const mtmc_weights* w, RolloutPlan& p, Carver& cv) {
  const Dims D = dims_of(w);
  apply_tune(p, tune_decode(D, p.B, p.bt, p.max_pages));
  // Buffers whose size follows from the launch shape are sized for every number of row tiles up to bt: a rollout
  // with a stop token packs its live rows into fewer tiles as rows finish, and each tile count has its own shape.
  size_t part = 0, o_chunks = 0, attn_ml = 0;
  for (int bt = 1; bt <= p.bt; ++bt) {
    const int B = bt == p.bt ? p.B : bt * 16;
    const DecodeTune t = tune_decode(D, B, bt, p.max_pages);
    const size_t Mpad = (size_t)bt * 16;
    part = std::max(part, std::max({(size_t)t.ks_qkv * D.nqkv, (size_t)t.ks_o * D.d, (size_t)t.ks_down * D.d}) * Mpad);
    o_chunks = std::max(o_chunks, (size_t)t.n_chunks * D.nq * Mpad);
    attn_ml = std::max(attn_ml, Mpad * D.Hq * t.n_chunks * 2);
  }
  const size_t Mpad = (size_t)p.bt * 16;
  p.part = cv.take<float>(part);
  p.o_chunks = cv.take<h16_t>(o_chunks);
  p.attn_ml = cv.take<float>(attn_ml);
  p.lm_part = cv.take<float>((size_t)((D.nt_V + 1) / 2) * Mpad * 8);
  p.qb = cv.take<h16_t>((size_t)p.Tmax * D.nq);
  p.gemm_part = cv.take<float>(kGemmPartFloats);
  p.ctl = cv.take<bf16::SampleCtl>(2);
  p.ssA = cv.take<float>((size_t)D.nt_d * Mpad);
  p.ssB = cv.take<float>((size_t)D.nt_d * Mpad);
  p.rs_buf = cv.take<float>(Mpad);
  if (p.ragged) {
    p.slot_row = cv.take<int>(Mpad);
    p.page_table_c = cv.take<int>(Mpad * p.max_pages);
    p.row_pos_c = cv.take<int>(Mpad);
    p.live = cv.take<int>(16 + 256);
    p.row_step0 = cv.take<int>(Mpad);
    p.prefill_table = cv.take<int>(Mpad * p.max_pages);
    p.slot_row_c = cv.take<int>(Mpad);
    p.row_step0_c = cv.take<int>(Mpad);
    const size_t MpadT = Mpad;  // the sequences of the prompts that join at one look: no more than the batch holds
    p.hT = cv.take<float>(MpadT * D.d);
    p.xT = cv.take<h16_t>(MpadT * D.d);
    p.ssT = cv.take<float>((size_t)D.nt_d * MpadT);
  }
}

// whether a pass over up to T tokens can have a d-wide output of at most 128 blocks of 256 x 256 (what gemm_lds_split takes)
static bool split_k_may_apply(int T, int d) { return (size_t)((T + 255) / 256) * ((d + 255) / 256) <= 128; }

void bf16_plan_score_extra(const mtmc_weights* w, ScorePlan& p, Carver& cv) {
  const Dims D = dims_of(w);
  int gpb = 0;
  const int blocks = bf16::score_head_blocks(D.nt_V, &gpb);
  p.lm_part = cv.take<float>((size_t)blocks * 2 * p.rows_max * 8);
  p.qb = cv.take<h16_t>((size_t)p.T * D.nq);
  p.targets = cv.take<int>(p.rows_max);
  p.gemm_part = split_k_may_apply(p.T, D.d) ? cv.take<float>(kGemmPartFloats) : nullptr;
}

void bf16_plan_actions_extra(const mtmc_weights* w, ActionPlan& p, Carver& cv) {
  const Dims D = dims_of(w);
  int gpb = 0;
  const int blocks = bf16::score_head_blocks(D.nt_V, &gpb);
  p.lm_part = cv.take<float>((size_t)blocks * 2 * p.rows_max * 8);
  p.qb = cv.take<h16_t>((size_t)p.Tmax * D.nq);
  p.targets = cv.take<int>(p.rows_max);
  p.seq_start = cv.take<int>((size_t)p.chunk_rows + 1);
  p.d_rows = cv.take<int>(16);
  p.pids = cv.take<int>(p.rows_max);
  p.out_index = cv.take<int>(p.rows_max);
  // no split-K scratch: the prefix pass keeps the sums of the scoring pass at 98 k tokens, so that scoring rollout
  // samples through this entry point gives what mtmc_score gives, bit for bit, at the sizes both are used at
  p.gemm_part = nullptr;
}

// ======================================================================================
// schedulers
// ======================================================================================
namespace {

// All residual blocks over T >= 1 tokens in the large-batch (prefill / scoring) form.
// In: h (fp32 [T, d]) and x = bf16 RMSNorm(h; attn_norm of layer 0) in tiled layout.
// Out: h after the last block (x is not refreshed after the last block).
// seq_start / d_rows (device, may be NULL): the sequences have different lengths and are packed back to back
// (sequence s = tokens seq_start[s] .. seq_start[s + 1] - 1, *d_rows tokens in all); S is then the longest
// length possible and n_seqs * S the capacity the launches are sized for.
void prefill_layers(const mtmc_weights* w, const Dims& D, float* h, h16_t* x, float* qkv, h16_t* qb,
                    h16_t* o, h16_t* a, int n_seqs, int S, TokMap map, KvPool pool, int layer_stride,
                    hipStream_t st, const int* seq_start = nullptr, const int* d_rows = nullptr, float* part = nullptr) {
  const mtmc_config& c = w->cfg;
  const int T = n_seqs * S, mt = tiles16(T), lmb = w->opt_lds_min_blocks;
  const size_t pf = part ? kGemmPartFloats : 0;  // partial sums of the split-K GEMMs (a prompt or a few)
  for (int l = 0; l < c.n_layers; ++l) {
    const LayerWeights& L = w->layers[l];
    const int kvl = l * layer_stride;
    bf16::gemm_large_f32(qkv, D.nqkv, D.nqkv, false, (const h16_t*)L.wqkv, D.nt_qkv, D.kt_d, x, T, mt, lmb, d_rows, st, part, pf);
    bf16::rope_kv_write(qb, qkv, D.nqkv, T, S, D.Hq, D.Hkv, w->rope_cos, w->rope_sin, map, pool, kvl, w->err_flag, st,
                        seq_start, n_seqs);
    bf16::attention_prefill(o, qb, n_seqs, S, mt, D.Hq, D.Hkv, map, pool, kvl, w->err_flag, st, seq_start);
    bf16::gemm_large_f32(h, D.d, D.d, true, (const h16_t*)L.wo, D.nt_d, D.kt_nq, o, T, mt, lmb, d_rows, st, part, pf);
    bf16::add_norm(h, nullptr, 0, 0, 0, L.ffn_norm, c.rms_eps, x, T, mt, D.d, w->err_flag, st, d_rows);
    bf16::gemm_large_swiglu(a, (const h16_t*)L.wgu, D.nt_gu, D.kt_d, x, T, mt, lmb, w->err_flag, d_rows, st);
    bf16::gemm_large_f32(h, D.d, D.d, true, (const h16_t*)L.wdown, D.nt_d, D.kt_F, a, T, mt, lmb, d_rows, st, part, pf);
    if (l + 1 < c.n_layers)
      bf16::add_norm(h, nullptr, 0, 0, 0, w->layers[l + 1].attn_norm, c.rms_eps, x, T, mt, D.d, w->err_flag, st, d_rows);
  }
}

// One decode step over the B sequences of a group.  In: hB / xB / ssA hold the embedded and normalised tokens of
// the step (the sampler merge of the previous step leaves them).  Runs the blocks (six launches each) against the
// paged cache at position prompt_len - 1 + *d_step and leaves in xB the operand of the LM head together with the
// row-norm bookkeeping (*ss_cur, *ss_old) its consumer needs.
void decode_layers(const mtmc_weights* w, const Dims& D, const RolloutPlan& p, KvPool pool, int pos_base,
                   const float** ss_cur_out, const float** ss_old_out, hipStream_t st, KernelTimer* tm = nullptr) {
  auto mark = [&](int k) { if (tm) tm->mark(k); };
  const mtmc_config& c = w->cfg;
  const int B = p.B, bt = p.bt;
  float* h = p.hB;
  h16_t* x = (h16_t*)p.xB;
  h16_t* o = (h16_t*)p.o;
  h16_t* a = (h16_t*)p.a;
  float* ss[2] = {p.ssA, p.ssB};
  int cur = 0, old = 0;
  bf16::DecGemmArgs g{};
  g.m_tiles = bt; g.M = B; g.ss_tiles = D.nt_d; g.inv_d = 1.0f / (float)D.d; g.eps = c.rms_eps; g.err_flag = w->err_flag;
  for (int l = 0; l < c.n_layers; ++l) {
    const LayerWeights& L = w->layers[l];
    bf16::DecGemmArgs q = g;
    q.Wt = (const h16_t*)L.wqkv; q.Xt = x; q.n_tiles = D.nt_qkv; q.k_tiles = D.kt_d;
    q.ss_cur = ss[cur]; q.ss_old = ss[old]; q.out_f32 = p.qkv; q.ld_out = D.nqkv;
    mark(MTMC_KERNEL_QKV);
    bf16::gemm_dec(q, bf16::DEC_STORE, st);
    mark(MTMC_KERNEL_QKV);
    bf16::AttnDecArgs at{};
    at.qkv = p.qkv; at.cos = w->rope_cos; at.sin = w->rope_sin; at.Hq = D.Hq; at.Hkv = D.Hkv; at.layer = l;
    at.pos_base = pos_base; at.row_pos = p.ragged ? p.row_pos : nullptr; at.d_step = p.d_step; at.pool = pool; at.chunk_pages = p.chunk_pages; at.split_at_prompt = p.split_at_prompt;
    at.n_chunks = p.n_chunks; at.m_tiles = bt; at.share = p.n_samples;
    at.row_step0 = p.ragged == 3 ? p.row_step0 : nullptr; at.max_step = p.max_new - 1;
    at.o = (h16_t*)p.o_chunks; at.o_chunk_stride = (size_t)D.nq * bt * 16; at.ml = p.attn_ml; at.err_flag = w->err_flag;
    mark(MTMC_KERNEL_ATTENTION);
    bf16::attention_dec(at, B, st);
    mark(MTMC_KERNEL_ATTENTION);
    bf16::DecGemmArgs r1 = g;
    r1.Wt = (const h16_t*)L.wo; r1.Xt = (const h16_t*)p.o_chunks; r1.n_tiles = D.nt_d; r1.k_tiles = D.kt_nq;
    r1.n_xchunks = p.n_chunks; r1.head_tiles = c.head_dim / 32; r1.x_chunk_stride = at.o_chunk_stride;
    r1.chunk_ml = p.attn_ml;
    r1.ss_cur = ss[cur]; r1.out_f32 = h; r1.ld_out = D.d; r1.out_h16 = x; r1.ss_out = ss[cur ^ 1]; r1.gain = L.ffn_norm;
    bf16::gemm_dec(r1, bf16::DEC_RESID, st);
    old = cur; cur ^= 1;
    bf16::DecGemmArgs gu = g;
    gu.Wt = (const h16_t*)L.wgu; gu.Xt = x; gu.n_tiles = D.nt_gu; gu.k_tiles = D.kt_d;
    gu.ss_cur = ss[cur]; gu.ss_old = ss[old]; gu.out_h16 = a;
    mark(MTMC_KERNEL_GATE_UP);
    bf16::gemm_dec(gu, bf16::DEC_SWIGLU, st);
    mark(MTMC_KERNEL_GATE_UP);
    // down projection: split-K partial sums (enough workgroups to pull full bandwidth), then one
    // launch that adds them in split order and does the residual / norm bookkeeping
    bf16::DecGemmArgs r2 = g;
    r2.Wt = (const h16_t*)L.wdown; r2.Xt = a; r2.n_tiles = D.nt_d; r2.k_tiles = D.kt_F;
    r2.ss_cur = ss[cur]; r2.out_f32 = p.part; r2.ld_out = D.d; r2.ksplit = p.ks_down; r2.rs_out = p.rs_buf; r2.partial_nb = p.down_nb;
    mark(MTMC_KERNEL_DOWN);
    bf16::gemm_dec(r2, bf16::DEC_PARTIAL, st);
    mark(MTMC_KERNEL_DOWN);
    bf16::resid_reduce(p.part, p.ks_down, bt, D.d, h, (l + 1 < c.n_layers) ? w->layers[l + 1].attn_norm : w->final_norm,
                       p.rs_buf, x, ss[cur ^ 1], B, w->err_flag, st);
    old = cur; cur ^= 1;
  }
  *ss_cur_out = ss[cur];
  *ss_old_out = ss[old];
}

// Returns in *out the instantiated graph of one decode step for this workspace and shape, capturing
// it on a private stream if it is not cached (or nullptr when graphs are off or `st` is already capturing).
template <class Step>
int decode_graph(const mtmc_weights* w, const RolloutPlan& gp, hipStream_t st, Step&& step,
                 hipGraphExec_t* out) {
  *out = nullptr;
  if (!w->opt_hip_graph) return MTMC_OK;
  hipStreamCaptureStatus cs = hipStreamCaptureStatusNone;
  if (hipStreamIsCapturing(st, &cs) != hipSuccess || cs != hipStreamCaptureStatusNone) {
    (void)hipGetLastError();
    return MTMC_OK;
  }
  mtmc_weights* mw = const_cast<mtmc_weights*>(w);
  if (!mw->graphs) mw->graphs = new GraphCache();
  GraphCache& gc = *mw->graphs;
  std::lock_guard<std::mutex> lock(gc.mu);
  if (!gc.capture_stream) {  // the caller's stream may be the default stream, which cannot capture
    hipError_t e = hipStreamCreateWithFlags(&gc.capture_stream, hipStreamNonBlocking);
    if (e != hipSuccess) {
      set_error(std::string("hipStreamCreateWithFlags: ") + hipGetErrorString(e));
      return MTMC_EHIP;
    }
  }
  for (auto& e : gc.entries)
    if (e.workspace == (const void*)gp.page_table && e.total_prompts == gp.total_prompts && e.B == gp.B &&
        e.prompt_len == gp.prompt_len && e.n_samples == gp.n_samples && e.max_new == gp.max_new &&
        e.ragged == gp.ragged) {
      *out = e.exec;
      return MTMC_OK;
    }
  if (gc.entries.size() >= 8) {  // evict the oldest; it may still be queued, on this stream or on another caller's
    MTMC_HIP_CHECK(hipDeviceSynchronize());
    (void)hipGraphExecDestroy(gc.entries.front().exec);
    gc.entries.erase(gc.entries.begin());
  }
  hipGraph_t graph = nullptr;
  MTMC_HIP_CHECK(hipStreamBeginCapture(gc.capture_stream, hipStreamCaptureModeThreadLocal));
  step(gc.capture_stream);
  MTMC_HIP_CHECK(hipStreamEndCapture(gc.capture_stream, &graph));
  hipGraphExec_t exec = nullptr;
  hipError_t e = hipGraphInstantiate(&exec, graph, nullptr, nullptr, 0);
  (void)hipGraphDestroy(graph);
  if (e != hipSuccess) {
    set_error(std::string("hipGraphInstantiate: ") + hipGetErrorString(e));
    return MTMC_EHIP;
  }
  gc.entries.push_back({(const void*)gp.page_table, gp.total_prompts, gp.B, gp.prompt_len, gp.n_samples, gp.max_new,
                        gp.ragged, exec});
  *out = exec;
  return MTMC_OK;
}


}  // namespace

int admission_plan(const int* live, const int* slot_region, int n_slots, int n_regions, int n_samples, int prompts_left,
                   int max_at_once, int wait_for, int* out_slots, int* out_regions) {
  std::vector<int> users(n_regions, 0);
  int n_free = 0, n_live = 0;
  for (int s = 0; s < n_slots; ++s) {
    if (live[s]) {
      ++n_live;
      if (slot_region[s] >= 0 && slot_region[s] < n_regions) ++users[slot_region[s]];
    } else {
      ++n_free;
    }
  }
  int free_regions = 0;
  for (int r = 0; r < n_regions; ++r) free_regions += users[r] == 0;
  const int k = std::min({n_free / n_samples, free_regions, prompts_left, max_at_once});
  if (k <= 0 || (k < std::min({prompts_left, wait_for, max_at_once}) && n_live > 0)) return 0;
  int ns = 0, nr = 0;
  for (int s = 0; s < n_slots && ns < k * n_samples; ++s)
    if (!live[s]) out_slots[ns++] = s;
  for (int r = 0; r < n_regions && nr < k; ++r)
    if (users[r] == 0) out_regions[nr++] = r;
  return k;
}

namespace {

// A rollout with a stop token and more sequences than one batch holds, run as ONE batch that takes in the call's
// prompts as it runs.  Every slot of the batch has pages of its own for a whole sequence; the whole pages of a prompt
// lie in one of n_regions regions shared by the prompt's sequences.  The first n_prompts prompts start together as
// in bf16_rollout.  Every few steps the host waits for the stream and reads which slots still hold a running
// sequence.  While prompts are left, the next one is taken in as soon as n_samples slots are free (any slots) and
// a region is free (one whose prompt's sequences have all ended): the slots' page-table rows are rebuilt, the
// prompt is prefilled through the first of them, its step 0 is sampled from a batch of its own (a second control
// block and step counter), and its sequences join the batch at their own step (row_step0).  A slot whose sequence
// has ended keeps computing on its own pages until it is given away.  When no prompt is left, the sequences still
// running are packed into fewer 16-row tiles as in bf16_rollout, and the call ends with the last of them.  While
// prompts are left the batch keeps its shape, so a sequence's arithmetic does not depend on when it joined.
int bf16_rollout_admit(const mtmc_weights* w, const RolloutPlan& p, const int* prompts, const SampleArgs& sa,
                       hipStream_t st) {
  const mtmc_config& c = w->cfg;
  const Dims D = dims_of(w);
  const int S = p.prompt_len, ns = p.n_samples, B = p.B;
  const size_t total_rows = (size_t)p.total_prompts * ns;
  KvPool pool{p.kv, p.n_pages, c.n_kv_heads, c.head_dim, p.page_table, p.max_pages};
  const size_t kv_words = (size_t)c.n_layers * 2 * p.n_pages * c.n_kv_heads * kPageTokens * c.head_dim / 2;
  RolloutPlan gp = p;
  gp.ragged = 3;  // the step graph of this form is its own (its launches carry row_step0)
  bf16::SampleCtl* d_ctl = (bf16::SampleCtl*)p.ctl;
  const uint32_t key0 = (uint32_t)(sa.seed & 0xffffffffu), key1 = (uint32_t)(sa.seed >> 32);
  bf16::SampleCtl ctl{sa.greedy, sa.inv_temp, key0, key1, sa.seq_offset, sa.max_new, sa.out_ids, sa.out_logprobs,
                      sa.stop_id, p.done, sa.out_lens, p.slot_row, p.row_step0};
  bf16::set_sample_ctl(d_ctl, ctl, st);
  // what a row reports after its end
  launch_fill_u32((uint32_t*)sa.out_ids, (uint32_t)sa.stop_id, total_rows * p.max_new, st);
  launch_fill_u32((uint32_t*)sa.out_logprobs, 0u, total_rows * p.max_new, st);
  launch_fill_u32((uint32_t*)p.done, 0u, total_rows, st);
  launch_fill_u32((uint32_t*)sa.out_lens, (uint32_t)p.max_new, total_rows, st);
  launch_ragged_setup(p.page_table, p.row_pos, p.done, sa.out_lens, p.prompt_ids, p.suffix_ids, prompts, sa.prompt_lens,
                      p.n_prompts, ns, S, p.max_pages, p.nf_max, p.shared_total, p.max_new, 0, w->err_flag, st);
  bf16::admit_init(p.slot_row, p.row_step0, B, p.bt * 16, st);
  launch_set_int(p.d_step, 0, st);
  launch_set_int(p.d_step + 1, 0, st);
  launch_fill_u32((uint32_t*)p.kv, 0u, kv_words, st);
  // prefill of `np` prompts (ids [np, S], padding cleared) through the page-table rows from `table` on (one row
  // per sequence, n_samples rows per prompt, the prompt's pages being those of its first row)
  auto prefill = [&](const int* ids, int np, const int* table, int rows_per_prompt) {
    const int T = np * S, mt = tiles16(T);
    KvPool ppool = pool;
    ppool.page_table = table;
    TokMap map{S, rows_per_prompt, 0, nullptr};
    bf16::embed(p.h, ids, T, (const bf16_t*)w->embed, D.d, D.V, w->err_flag, st);
    bf16::add_norm(p.h, nullptr, 0, 0, 0, w->layers[0].attn_norm, c.rms_eps, (h16_t*)p.x, T, mt, D.d, w->err_flag, st);
    prefill_layers(w, D, p.h, (h16_t*)p.x, p.qkv, (h16_t*)p.qb, (h16_t*)p.o, (h16_t*)p.a, np, S, map, ppool, 1, st, nullptr,
                   nullptr, p.gemm_part);
  };
  for (int p0 = 0; p0 < p.n_prompts; p0 += p.chunk_prompts) {
    const int np = std::min(p.chunk_prompts, p.n_prompts - p0);
    const int* table = p.page_table + (size_t)p0 * ns * p.max_pages;
    prefill(p.suffix_ids + (size_t)p0 * S, np, table, ns);
    launch_gather_last_rows(p.hB + (size_t)p0 * ns * D.d, p.h, D.d, np, ns, S, sa.prompt_lens + p0, 0, st);
    KvPool fpool = pool;
    fpool.page_table = table;
    launch_fork_tail_pages_ragged(fpool, c.n_layers, np * ns, ns, sa.prompt_lens + p0, S, 2, st);
  }
  bf16::add_norm(p.hB, nullptr, 0, 0, 0, w->final_norm, c.rms_eps, (h16_t*)p.xB, B, gp.bt, D.d, w->err_flag, st);
  auto embed_args = [&](const RolloutPlan& q) {
    return bf16::EmbedNextArgs{p.hB, (const bf16_t*)w->embed, D.d, w->layers[0].attn_norm, c.rms_eps, (h16_t*)p.xB,
                               q.bt * 16, p.ssA, D.V, w->err_flag};
  };
  // LM head + sampler over `rows` rows of the operand x; `dc` / `ds`: control block and step counter
  auto sample = [&](hipStream_t s, const h16_t* x, int rows, const float* ss_cur, const float* ss_old,
                    const bf16::SampleCtl* dc, int* ds, int* cur_ids, const bf16::EmbedNextArgs& e) {
    bf16::DecGemmArgs lm{};
    lm.Wt = (const h16_t*)w->lm_head; lm.Xt = x; lm.n_tiles = D.nt_V; lm.k_tiles = D.kt_d;
    lm.m_tiles = tiles16(rows); lm.M = rows; lm.ss_cur = ss_cur; lm.ss_old = ss_old; lm.ss_tiles = D.nt_d;
    lm.inv_d = 1.0f / (float)D.d; lm.eps = c.rms_eps; lm.out_f32 = p.lm_part;
    lm.ctl = dc; lm.d_step = ds;
    bf16::gemm_dec(lm, bf16::DEC_SAMPLE, s);
    bf16::sample_merge(p.lm_part, bf16::dec_sample_groups(D.nt_V, D.kt_d, lm.m_tiles), rows, dc, ds, cur_ids, e, s);
  };
  // cur: the shape the step runs in (the batch, or the slots its last sequences were packed into)
  RolloutPlan cur = gp;
  KvPool cur_pool = pool;
  auto decode_step = [&](hipStream_t s) {
    const float *ss_cur = nullptr, *ss_old = nullptr;
    decode_layers(w, D, cur, cur_pool, 0, &ss_cur, &ss_old, s);
    sample(s, (const h16_t*)p.xB, cur.B, ss_cur, ss_old, d_ctl, p.d_step, p.cur_ids, embed_args(cur));
  };
  sample(st, (const h16_t*)p.xB, B, nullptr, nullptr, d_ctl, p.d_step, p.cur_ids, embed_args(gp));  // step 0 of the first prompts

  mtmc_weights* mw = const_cast<mtmc_weights*>(w);
  if (!mw->graphs) mw->graphs = new GraphCache();
  GraphCache& gc = *mw->graphs;
  std::lock_guard<std::mutex> poll_lock(gc.poll_mu);
  if (!gc.host_slots) MTMC_HIP_CHECK(hipHostMalloc((void**)&gc.host_slots, 256 * sizeof(int), hipHostMallocDefault));
  const int* live = gc.host_slots;
  hipGraphExec_t exec = nullptr;
  if (int rc = decode_graph(w, cur, st, decode_step, &exec)) return rc;

  std::vector<int> slot_region(B), regions(p.n_regions);  // slot_region: the region a slot's sequence reads
  for (int s = 0; s < B; ++s) slot_region[s] = s / ns;
  int next_prompt = p.n_prompts, steps = 1;  // steps: value of *d_step once the queued work has run
  int* d_live = p.live + 16;
  const int period = std::max(1, std::min(w->opt_stop_poll, 8));
  // every sequence ends within max_new steps of its start and a prompt is taken in whenever all the sequences of
  // an earlier one have ended, at the latest
  const long long step_limit = ((long long)p.total_prompts + 2) * ((long long)p.max_new + 2LL * period);
  std::vector<int> free_slots(B);
  for (;;) {
    for (int j = 0; j < period; ++j) {
      if (exec) MTMC_HIP_CHECK(hipGraphLaunch(exec, st));
      else decode_step(st);
    }
    steps += period;
    if (steps > step_limit) {
      set_error("internal error: a rollout that takes in prompts as it runs did not end");
      return MTMC_EHIP;
    }
    // the tables by slot of the whole batch stay as they are once no prompt is left: the packed batch is always made from them
    bf16::slot_live(p.done, p.slot_row, B, d_live, st);
    MTMC_HIP_CHECK(hipMemcpyAsync(gc.host_slots, d_live, B * sizeof(int), hipMemcpyDeviceToHost, st));
    MTMC_HIP_CHECK(hipStreamSynchronize(st));
    int n_live = 0;
    for (int s = 0; s < B; ++s) n_live += live[s];
    if (next_prompt < p.total_prompts) {
      // a prefill costs about the same for one prompt as for a few: wait for a quarter of the batch, unless every
      // slot is free or fewer prompts are left
      const int left = p.total_prompts - next_prompt;
      const int k = admission_plan(live, slot_region.data(), B, p.n_regions, ns, left, p.chunk_prompts,
                                   std::max(1, p.n_prompts / 4), free_slots.data(), regions.data());
      const bool admitted = k > 0;
      if (admitted) {
        const int q0 = next_prompt;
        next_prompt += k;
        std::vector<bf16::AdmitArgs> adm(k);
        for (int i = 0; i < k; ++i) {
          const int q = q0 + i;
          adm[i] = bf16::AdmitArgs{p.page_table, p.row_pos, p.slot_row, p.row_step0, p.suffix_ids + (size_t)i * S,
                                   p.prefill_table + (size_t)i * p.max_pages, prompts + (size_t)q * S, sa.prompt_lens + q,
                                   regions[i], q, ns, S, p.max_pages, p.nf_max, p.shared_total, steps - 1, w->err_flag, {}};
          for (int j = 0; j < ns; ++j) {
            adm[i].slots[j] = free_slots[(size_t)i * ns + j];
            slot_region[adm[i].slots[j]] = regions[i];
          }
          bf16::admit_prompt(adm[i], st);
        }
        prefill(p.suffix_ids, k, p.prefill_table, 1);
        launch_gather_last_rows(p.hT, p.h, D.d, k, ns, S, sa.prompt_lens + q0, 0, st);
        for (int i = 0; i < k; ++i) bf16::fork_tail_slots(adm[i], pool, c.n_layers, st);
        const int rows = k * ns;
        bf16::add_norm(p.hT, nullptr, 0, 0, 0, w->final_norm, c.rms_eps, (h16_t*)p.xT, rows, tiles16(rows), D.d, w->err_flag, st);
        // their step 0, as a batch of its own: rows q0 * ns .. of the call, a step counter of its own
        bf16::SampleCtl ct = ctl;
        ct.seq_offset = sa.seq_offset + (uint32_t)(q0 * ns);
        ct.out_ids = sa.out_ids + (size_t)q0 * ns * p.max_new;
        ct.out_logprobs = sa.out_logprobs + (size_t)q0 * ns * p.max_new;
        ct.done = p.done + (size_t)q0 * ns;
        ct.out_lens = sa.out_lens + (size_t)q0 * ns;
        ct.slot_row = nullptr;
        ct.row_step0 = nullptr;
        bf16::set_sample_ctl(d_ctl + 1, ct, st);
        launch_set_int(p.d_step + 8, 0, st);
        launch_set_int(p.d_step + 9, 0, st);
        const bf16::EmbedNextArgs embT{p.hT, (const bf16_t*)w->embed, D.d, w->layers[0].attn_norm, c.rms_eps, (h16_t*)p.xT,
                                       tiles16(rows) * 16, p.ssT, D.V, w->err_flag};
        sample(st, (const h16_t*)p.xT, rows, nullptr, nullptr, d_ctl + 1, p.d_step + 8, p.cur_ids + (size_t)q0 * ns, embT);
      }
      // the first tokens of the new sequences become operands of the next step (the other slots get again what
      // they hold).  B, not the padded count: h has B rows
      if (admitted) bf16::embed_slots(p.slot_row, p.cur_ids, B, embed_args(gp), st);
      continue;
    }
    if (n_live == 0) break;
    const int slots = tiles16(n_live) * 16;
    if (slots < cur.bt * 16) {
      bf16::compact_slots(p.done, B, slots, p.slot_row, p.page_table, p.row_pos, p.row_step0, p.max_pages, p.slot_row_c,
                          p.page_table_c, p.row_pos_c, p.row_step0_c, st);
      cur = gp;
      cur.B = slots; cur.bt = slots / 16; cur.n_samples = 1;
      cur.row_pos = p.row_pos_c; cur.row_step0 = p.row_step0_c;
      apply_tune(cur, tune_decode(D, cur.B, cur.bt, p.max_pages));
      cur_pool.page_table = p.page_table_c;
      bf16::SampleCtl cc = ctl;
      cc.slot_row = p.slot_row_c;
      cc.row_step0 = p.row_step0_c;
      bf16::set_sample_ctl(d_ctl, cc, st);
      bf16::embed_slots(p.slot_row_c, p.cur_ids, slots, embed_args(cur), st);
      if (int rc = decode_graph(w, cur, st, decode_step, &exec)) return rc;
    }
  }
  return MTMC_OK;
}

}  // namespace

int bf16_rollout(const mtmc_weights* w, const RolloutPlan& p, const int* prompts, const SampleArgs& sa,
                 hipStream_t st) {
  const mtmc_config& c = w->cfg;
  if (p.n_samples > 128) {
    set_error("invalid argument: MTMC_BF16 rollout takes at most 128 samples per prompt");
    return MTMC_EINVAL;
  }
  if (sa.prompt_lens && sa.stop_id >= 0 && sa.reuse_len == 0 && p.total_prompts > p.n_prompts && p.max_new > 1 &&
      w->opt_admit && w->opt_stop_poll > 0) {
    // not while the caller is capturing the stream: the host must not wait then
    hipStreamCaptureStatus cs = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(st, &cs) == hipSuccess && cs == hipStreamCaptureStatusNone)
      return bf16_rollout_admit(w, p, prompts, sa, st);
    (void)hipGetLastError();
  }
  const Dims D = dims_of(w);
  KvPool pool{p.kv, p.n_pages, c.n_kv_heads, c.head_dim, p.page_table, p.max_pages};
  const size_t kv_words = (size_t)c.n_layers * 2 * p.n_pages * c.n_kv_heads * kPageTokens * c.head_dim / 2;
  for (int g0 = 0; g0 < p.total_prompts; g0 += p.n_prompts) {
    const int np_group = std::min(p.n_prompts, p.total_prompts - g0);
    RolloutPlan gp = p;  // this group's shape (the last group may be smaller)
    gp.n_prompts = np_group;
    gp.B = np_group * p.n_samples;
    gp.bt = tiles16(gp.B);
    gp.shared_total = np_group * p.nf_max;
    const bool ragged = sa.prompt_lens != nullptr;
    const int* glens = ragged ? sa.prompt_lens + g0 : nullptr;
    int* g_out_lens = ragged ? sa.out_lens + (size_t)g0 * p.n_samples : nullptr;
    const int* gprompts = prompts + (size_t)g0 * p.prompt_len;
    const size_t out_off = (size_t)g0 * p.n_samples * p.max_new;
    bf16::SampleCtl ctl{sa.greedy, sa.inv_temp, (uint32_t)(sa.seed & 0xffffffffu), (uint32_t)(sa.seed >> 32),
                        sa.seq_offset + (uint32_t)(g0 * p.n_samples), sa.max_new, sa.out_ids + out_off,
                        sa.out_logprobs + out_off, sa.stop_id, (ragged && sa.stop_id >= 0) ? p.done : nullptr,
                        g_out_lens, nullptr};
    bf16::set_sample_ctl((bf16::SampleCtl*)p.ctl, ctl, st);
    if (ragged && sa.stop_id >= 0) {
      // what a row reports after its end; rows that have given up their slot never write again
      launch_fill_u32((uint32_t*)(sa.out_ids + out_off), (uint32_t)sa.stop_id, (size_t)gp.B * p.max_new, st);
      launch_fill_u32((uint32_t*)(sa.out_logprobs + out_off), 0u, (size_t)gp.B * p.max_new, st);
    }
    const int R = ragged ? sa.reuse_len : 0;   // cached prefix: only positions R .. prompt_len - 1 are prefilled
    const int S = p.prompt_len - R;
    if (ragged) {
      launch_ragged_setup(p.page_table, p.row_pos, p.done, g_out_lens, p.prompt_ids, p.suffix_ids, gprompts, glens,
                          np_group, p.n_samples, p.prompt_len, p.max_pages, p.nf_max, gp.shared_total, p.max_new, R,
                          w->err_flag, st);
      gprompts = p.suffix_ids;
    } else {
      launch_build_page_table(p.page_table, gp.B, p.max_pages, p.n_samples, p.n_full, gp.shared_total, st);
    }
    launch_set_int(p.d_step, 0, st);
    launch_set_int(p.d_step + 1, 0, st);  // arrival counter of the sampler merge
    // stale or uninitialised cache slots must at least be finite: masked scores multiply them by 0 (with a cached
    // prefix the pool holds the previous call's values: finite, and the prefix pages must stay)
    if (R == 0) launch_fill_u32((uint32_t*)p.kv, 0u, kv_words, st);
    // ---- prefill, whole prompts per chunk; a prompt's pages are those of its first sample
    for (int p0 = 0; p0 < np_group; p0 += p.chunk_prompts) {
      const int np = std::min(p.chunk_prompts, np_group - p0);
      const int T = np * S, mt = tiles16(T);
      KvPool chunk_pool = pool;
      chunk_pool.page_table = p.page_table + (size_t)p0 * p.n_samples * p.max_pages;
      TokMap map{S, p.n_samples, R, nullptr};
      bf16::embed(p.h, gprompts + (size_t)p0 * S, T, (const bf16_t*)w->embed, D.d, D.V, w->err_flag, st);
      bf16::add_norm(p.h, nullptr, 0, 0, 0, w->layers[0].attn_norm, c.rms_eps, (h16_t*)p.x, T, mt, D.d, w->err_flag, st);
      prefill_layers(w, D, p.h, (h16_t*)p.x, p.qkv, (h16_t*)p.qb, (h16_t*)p.o, (h16_t*)p.a, np, S, map, chunk_pool, 1,
                     st, nullptr, nullptr, p.gemm_part);
      if (ragged)
        launch_gather_last_rows(p.hB + (size_t)p0 * p.n_samples * D.d, p.h, D.d, np, p.n_samples, p.prompt_len,
                                glens + p0, R, st);
      else
        launch_gather_rows(p.hB + (size_t)p0 * p.n_samples * D.d, p.h, np * p.n_samples, D.d, p.n_samples,
                           p.prompt_len, p.prompt_len - 1, 0, st);
    }
    if (ragged)
      launch_fork_tail_pages_ragged(pool, c.n_layers, gp.B, p.n_samples, glens, p.prompt_len, 2, st);
    else if (p.prompt_len % kPageTokens != 0)
      launch_fork_tail_pages(pool, c.n_layers, gp.B, p.n_samples, p.n_full, 2, st);
    // ---- step 0 samples from the prompt's last position; step i > 0 first feeds token i - 1
    bf16::add_norm(p.hB, nullptr, 0, 0, 0, w->final_norm, c.rms_eps, (h16_t*)p.xB, gp.B, gp.bt, D.d, w->err_flag, st);
    // q: the shape the step runs in (the group's rows, or the slots its live rows were packed into)
    auto embed_args = [&](const RolloutPlan& q) {
      return bf16::EmbedNextArgs{p.hB, (const bf16_t*)w->embed, D.d, w->layers[0].attn_norm, c.rms_eps, (h16_t*)p.xB,
                                 q.bt * 16, p.ssA, D.V, w->err_flag};
    };
    auto sample = [&](hipStream_t s, const float* ss_cur, const float* ss_old, const RolloutPlan& q) {
      bf16::DecGemmArgs lm{};
      lm.Wt = (const h16_t*)w->lm_head; lm.Xt = (const h16_t*)p.xB; lm.n_tiles = D.nt_V; lm.k_tiles = D.kt_d;
      lm.m_tiles = q.bt; lm.M = q.B; lm.ss_cur = ss_cur; lm.ss_old = ss_old; lm.ss_tiles = D.nt_d;
      lm.inv_d = 1.0f / (float)D.d; lm.eps = c.rms_eps; lm.out_f32 = p.lm_part;
      lm.ctl = (const bf16::SampleCtl*)p.ctl; lm.d_step = p.d_step;
      bf16::gemm_dec(lm, bf16::DEC_SAMPLE, s);
      const int groups = bf16::dec_sample_groups(D.nt_V, D.kt_d, q.bt);
      // also ++*d_step, and the embedding + first norm of the chosen tokens: the next step starts at its QKV projection
      bf16::sample_merge(p.lm_part, groups, q.B, (const bf16::SampleCtl*)p.ctl, p.d_step, p.cur_ids, embed_args(q), s);
    };
    auto decode_step_in = [&](hipStream_t s, KernelTimer* tm, const RolloutPlan& q, const KvPool& qpool) {
      const float *ss_cur = nullptr, *ss_old = nullptr;
      if (tm) tm->mark_empty_pair();
      decode_layers(w, D, q, qpool, p.prompt_len - 1, &ss_cur, &ss_old, s, tm);
      if (tm) tm->mark(MTMC_KERNEL_LM_HEAD);
      sample(s, ss_cur, ss_old, q);
      if (tm) tm->mark(MTMC_KERNEL_LM_HEAD);
    };
    auto decode_step_timed = [&](hipStream_t s, KernelTimer* tm) { decode_step_in(s, tm, gp, pool); };
    auto decode_step = [&](hipStream_t s) { decode_step_timed(s, nullptr); };
    sample(st, nullptr, nullptr, gp);  // xB holds the exactly normalised last prompt position
    // A stop token: every `poll` steps the number of rows still running goes to the host, which reads it one
    // period later, ends the group when it is zero and packs the live rows into fewer 16-row tiles when it
    // frees a tile.  Not while the caller is capturing the stream (the host must not wait then).
    int poll = (ragged && sa.stop_id >= 0) ? w->opt_stop_poll : 0;
    if (poll > 0) {
      hipStreamCaptureStatus cs = hipStreamCaptureStatusNone;
      if (hipStreamIsCapturing(st, &cs) != hipSuccess || cs != hipStreamCaptureStatusNone) {
        (void)hipGetLastError();
        poll = 0;
      }
    }
    if (p.max_new > 1 && poll > 0) {
      mtmc_weights* mw = const_cast<mtmc_weights*>(w);
      if (!mw->graphs) mw->graphs = new GraphCache();
      GraphCache& gc = *mw->graphs;
      std::lock_guard<std::mutex> poll_lock(gc.poll_mu);
      if (!gc.host_live) {
        MTMC_HIP_CHECK(hipHostMalloc((void**)&gc.host_live, 64 * sizeof(int), hipHostMallocDefault));
        for (hipEvent_t& e : gc.poll_events) MTMC_HIP_CHECK(hipEventCreateWithFlags(&e, hipEventDisableTiming));
      }
      RolloutPlan cur = gp;
      KvPool cur_pool = pool;
      auto step_cur = [&](hipStream_t s) { decode_step_in(s, nullptr, cur, cur_pool); };
      hipGraphExec_t exec = nullptr;
      if (int rc = decode_graph(w, cur, st, step_cur, &exec)) return rc;
      int i = 1, slot = 0;
      bool have_prev = false;
      while (i < p.max_new) {
        const int n = std::min(poll, p.max_new - i);
        for (int j = 0; j < n; ++j) {
          if (exec) MTMC_HIP_CHECK(hipGraphLaunch(exec, st));
          else step_cur(st);
        }
        i += n;
        if (i >= p.max_new) break;
        bf16::count_live(p.done, gp.B, p.live, st);
        MTMC_HIP_CHECK(hipMemcpyAsync(gc.host_live + 16 * slot, p.live, sizeof(int), hipMemcpyDeviceToHost, st));
        MTMC_HIP_CHECK(hipEventRecord(gc.poll_events[slot], st));
        if (have_prev) {
          MTMC_HIP_CHECK(hipEventSynchronize(gc.poll_events[slot ^ 1]));
          const int n_live = gc.host_live[16 * (slot ^ 1)];  // one period old: rows only ever finish, so an upper bound
          if (n_live <= 0) break;  // every later slot of the outputs already holds stop_id / 0
          const int slots = tiles16(n_live) * 16;
          if (slots < cur.bt * 16) {
            bf16::compact_rows(p.done, gp.B, slots, p.slot_row, p.page_table, p.row_pos, p.max_pages, p.page_table_c,
                               p.row_pos_c, st);
            cur = gp;
            cur.B = slots; cur.bt = slots / 16; cur.n_samples = 1; cur.ragged = 2;
            cur.row_pos = p.row_pos_c;
            apply_tune(cur, tune_decode(D, cur.B, cur.bt, p.max_pages));
            cur_pool.page_table = p.page_table_c;
            ctl.slot_row = p.slot_row;
            bf16::set_sample_ctl((bf16::SampleCtl*)p.ctl, ctl, st);
            bf16::embed_slots(p.slot_row, p.cur_ids, slots, embed_args(cur), st);
            if (int rc = decode_graph(w, cur, st, step_cur, &exec)) return rc;
          }
        }
        have_prev = true;
        slot ^= 1;
      }
    } else if (p.max_new > 1) {
      hipGraphExec_t exec = nullptr;
      if (int rc = decode_graph(w, gp, st, decode_step, &exec)) return rc;
      GraphCache* gc = w->graphs;
      KernelTimer tm{gc, gc ? gc->timer_class : 0, st};
      const int every = gc ? gc->timer_every : 0;
      for (int i = 1; i < p.max_new; ++i) {
        if (tm.cls && every > 0 && i % every == 1 % every) decode_step_timed(st, &tm);  // launched directly, with events
        else if (exec) MTMC_HIP_CHECK(hipGraphLaunch(exec, st));
        else decode_step(st);
      }
    }
  }
  return MTMC_OK;
}

int bf16_score(const mtmc_weights* w, const ScorePlan& p, const ScoreArgs& a, hipStream_t st) {
  const mtmc_config& c = w->cfg;
  const Dims D = dims_of(w);
  const int S = a.S, n_scored = S - 1 - a.first;
  const size_t n_out = (size_t)a.n_seqs * (S - 1);
  launch_fill_u32((uint32_t*)a.out_logprobs, 0u, n_out, st);
  if (a.out_top1) launch_fill_u32((uint32_t*)a.out_top1, 0u, n_out, st);
  if (a.out_margin) launch_fill_u32((uint32_t*)a.out_margin, 0u, n_out, st);
  KvPool pool{p.kv, p.n_pages, c.n_kv_heads, c.head_dim, p.page_table, p.pages_per_seq};
  launch_build_page_table(p.page_table, p.chunk_seqs, p.pages_per_seq, 1, 0, 0, st);
  launch_fill_u32((uint32_t*)p.kv, 0u, (size_t)2 * p.n_pages * c.n_kv_heads * kPageTokens * c.head_dim / 2, st);
  TokMap map{S, 1, 0, nullptr};
  int gpb = 0;
  const int n_parts = bf16::score_head_blocks(D.nt_V, &gpb) * 2;
  for (int s0 = 0; s0 < a.n_seqs; s0 += p.chunk_seqs) {
    const int ns = std::min(p.chunk_seqs, a.n_seqs - s0);
    const int T = ns * S, mt = tiles16(T);
    bf16::embed(p.h, a.seqs + (size_t)s0 * S, T, (const bf16_t*)w->embed, D.d, D.V, w->err_flag, st);
    bf16::add_norm(p.h, nullptr, 0, 0, 0, w->layers[0].attn_norm, c.rms_eps, (h16_t*)p.x, T, mt, D.d, w->err_flag, st);
    prefill_layers(w, D, p.h, (h16_t*)p.x, p.qkv, (h16_t*)p.qb, (h16_t*)p.o, (h16_t*)p.a, ns, S, map, pool, 0, st, nullptr,
                   nullptr, p.gemm_part);
    const int R = ns * n_scored;
    if (R == 0) continue;
    const int rt = tiles16(R);
    launch_gather_rows(p.hs, p.h, R, D.d, n_scored, S, a.first, 1, st);
    bf16::add_norm(p.hs, nullptr, 0, 0, 0, w->final_norm, c.rms_eps, (h16_t*)p.xs, R, rt, D.d, w->err_flag, st);
    bf16::score_targets(p.targets, a.seqs, R, S, a.first, n_scored, s0, 0, D.V, w->err_flag, st);
    bf16::lmhead_score(p.lm_part, (const h16_t*)w->lm_head, D.nt_V, D.kt_d, (const h16_t*)p.xs, R, rt, p.targets,
                       a.out_top1 != nullptr || a.out_margin != nullptr, w->opt_lds_min_blocks, nullptr, st);
    bf16::score_reduce(p.lm_part, n_parts, R, S, a.first, n_scored, s0, 0, a.out_logprobs, a.out_top1, a.out_margin, st);
  }
  return MTMC_OK;
}

int bf16_score_actions(const mtmc_weights* w, const ActionPlan& p, const ActionArgs& a, hipStream_t st) {
  const mtmc_config& c = w->cfg;
  const Dims D = dims_of(w);
  KvPool pool{p.kv, p.n_pages, c.n_kv_heads, c.head_dim, p.page_table, p.max_pages};
  launch_build_page_table(p.page_table, p.B, p.max_pages, p.K, p.n_full, p.shared_total, st);
  launch_build_action_seqs(p.vseq, p.prefix, a.states, a.actions, a.action_len, p.n_states, p.P, p.K, p.A,
                           w->err_flag, st);
  launch_fill_u32((uint32_t*)a.out_token, 0u, (size_t)p.B * p.A, st);
  // stale or uninitialised cache slots must at least be finite: masked scores multiply them by 0
  launch_fill_u32((uint32_t*)p.kv, 0u,
                  (size_t)c.n_layers * 2 * p.n_pages * c.n_kv_heads * kPageTokens * c.head_dim / 2, st);
  // ---- the states without their last token, once per state, into the pages of their first candidate
  if (p.Pp > 0) {
    for (int n0 = 0; n0 < p.n_states; n0 += p.chunk_states) {
      const int ns = std::min(p.chunk_states, p.n_states - n0);
      const int T = ns * p.Pp, mt = tiles16(T);
      KvPool chunk_pool = pool;
      chunk_pool.page_table = p.page_table + (size_t)n0 * p.K * p.max_pages;
      TokMap map{p.Pp, p.K, 0, nullptr};
      bf16::embed(p.h, p.prefix + (size_t)n0 * p.Pp, T, (const bf16_t*)w->embed, D.d, D.V, w->err_flag, st);
      bf16::add_norm(p.h, nullptr, 0, 0, 0, w->layers[0].attn_norm, c.rms_eps, (h16_t*)p.x, T, mt, D.d, w->err_flag, st);
      prefill_layers(w, D, p.h, (h16_t*)p.x, p.qkv, (h16_t*)p.qb, (h16_t*)p.o, (h16_t*)p.a, ns, p.Pp, map,
                     chunk_pool, 1, st, nullptr, nullptr, p.gemm_part);
    }
    if (p.Pp % kPageTokens != 0) launch_fork_tail_pages(pool, c.n_layers, p.B, p.K, p.n_full, 2, st);
  }
  // ---- the candidates, packed without padding: candidate b is the len_b tokens [last state token, a_1 ..
  // a_{len - 1}] at positions P - 1 .. on top of its state's pages, and every one of them is scored (it predicts
  // a_1 .. a_len).  The number of packed tokens is known on the device only: the launches are sized for nr * A
  // rows and the kernels skip the blocks of rows beyond *d_rows.
  TokMap map{p.A, 1, p.Pp, nullptr};
  int gpb = 0;
  const int n_parts = bf16::score_head_blocks(D.nt_V, &gpb) * 2;
  for (int r0 = 0; r0 < p.B; r0 += p.chunk_rows) {
    const int nr = std::min(p.chunk_rows, p.B - r0);
    const int T = nr * p.A, mt = tiles16(T);
    KvPool chunk_pool = pool;
    chunk_pool.page_table = p.page_table + (size_t)r0 * p.max_pages;
    bf16::build_packed_actions(p.seq_start, p.d_rows, p.pids, p.targets, p.out_index, a.states, a.actions,
                               a.action_len, p.P, p.K, p.A, r0, nr, D.V, w->err_flag, st);
    // rows without a token that share a 256-row block with tokens run through the matrix kernels: cleared inputs
    // (embedding, attention output) keep everything computed from them at zero
    launch_fill_u32((uint32_t*)p.o, 0u, (size_t)mt * 16 * D.nq / 2, st);
    bf16::embed(p.h, p.pids, T, (const bf16_t*)w->embed, D.d, D.V, w->err_flag, st, p.d_rows);
    bf16::add_norm(p.h, nullptr, 0, 0, 0, w->layers[0].attn_norm, c.rms_eps, (h16_t*)p.x, T, mt, D.d, w->err_flag, st,
                   p.d_rows);
    prefill_layers(w, D, p.h, (h16_t*)p.x, p.qkv, (h16_t*)p.qb, (h16_t*)p.o, (h16_t*)p.a, nr, p.A, map,
                   chunk_pool, 1, st, p.seq_start, p.d_rows, p.gemm_part);
    bf16::add_norm(p.h, nullptr, 0, 0, 0, w->final_norm, c.rms_eps, (h16_t*)p.xs, T, mt, D.d, w->err_flag, st, p.d_rows);
    bf16::lmhead_score(p.lm_part, (const h16_t*)w->lm_head, D.nt_V, D.kt_d, (const h16_t*)p.xs, T, mt, p.targets,
                       false, w->opt_lds_min_blocks, p.d_rows, st);
    bf16::score_reduce_scatter(p.lm_part, n_parts, T, p.d_rows, p.out_index, a.out_token, st);
  }
  launch_action_reduce(a.out_token, a.action_len, p.n_states, p.K, p.A, a.normalize, a.out_action, a.out_policy,
                       st);
  return MTMC_OK;
}

}  // namespace mtmc
