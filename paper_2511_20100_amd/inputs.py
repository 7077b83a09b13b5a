"""Seeded synthetic inputs for the policy rollout / scoring path.

This module only *describes* and *draws* inputs: model shapes, the canonical
weight blob, random weights, prompts and sequences.  It holds none of the
method's arithmetic (no norm, attention, softmax, sampling), so that both the
HIP path and the CPU oracle can be fed the very same bytes without sharing
any computation.

The policy in the paper is a lightweight (1-1.5 B parameter) decoder-only
language model (Method, "Training Methodology"); its trained weights and its
prompts (kernel code + description + history) are not available, so random
N(0, 0.02) matrices, unit norm gains and uniform random token ids of the same
shapes stand in for them.

Canonical weight blob (the layout `mtmc_weights_create` consumes)
------------------------------------------------------------------
Tensors in this order, every tensor starting at the next multiple of 256
bytes, matrices row-major ``[out, in]`` (y = W x):

    embed[V,d]
    per layer: attn_norm[d] Wq[Hq*hd,d] Wk[Hkv*hd,d] Wv[Hkv*hd,d] Wo[d,Hq*hd]
               ffn_norm[d]  Wgate[F,d]  Wup[F,d]     Wdown[d,F]
    final_norm[d]
    lm_head[V,d]

Norm gains are always fp32.  Matrices are fp32 (dtype "fp32") or bf16 bit
patterns (dtype "bf16").
"""
from __future__ import annotations

import os
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, replace
from typing import Dict, Iterable, List, Tuple

import numpy as np

BLOB_ALIGN = 256
_CHUNK = 1 << 22  # elements drawn per independent random stream


@dataclass(frozen=True)
class ModelConfig:
    n_layers: int
    d_model: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    d_ffn: int
    vocab: int
    rms_eps: float = 1e-6
    rope_base: float = 10000.0
    dtype: str = "bf16"  # "fp32" or "bf16": storage type of the matrices
    tie_embeddings: bool = False  # the LM head is the embedding matrix (no lm_head tensor)

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    def with_(self, **kw) -> "ModelConfig":
        return replace(self, **kw)


# The workload shapes (tiny fp32 parity case, 1.5 B-class headline case, 7 B-class).
TINY = ModelConfig(2, 256, 4, 2, 64, 688, 4096, dtype="fp32")
POLICY_1P5B = ModelConfig(28, 1536, 12, 2, 128, 8960, 151936, dtype="bf16")
POLICY_7B = ModelConfig(28, 3584, 28, 4, 128, 18944, 152064, dtype="bf16")
# Shapes of the classes of the paper's own policy backbones (Method, "Training Methodology"): a 1.3 B-class
# model with one kv head per query head, and a 1 B-class model with 64-dim heads and a tied LM head.
POLICY_1P3B_MHA = ModelConfig(24, 2048, 16, 16, 128, 5504, 32256, dtype="bf16")
POLICY_1B_HD64 = ModelConfig(16, 2048, 32, 8, 64, 8192, 128256, dtype="bf16", tie_embeddings=True)


def tensor_specs(cfg: ModelConfig) -> List[Tuple[str, Tuple[int, ...], bool]]:
    """(name, shape, is_matrix) of every tensor, in canonical blob order."""
    d, hd = cfg.d_model, cfg.head_dim
    q, kv, f, v = cfg.n_q_heads * hd, cfg.n_kv_heads * hd, cfg.d_ffn, cfg.vocab
    specs: List[Tuple[str, Tuple[int, ...], bool]] = [("embed", (v, d), True)]
    for l in range(cfg.n_layers):
        p = f"layers.{l}."
        specs += [
            (p + "attn_norm", (d,), False),
            (p + "wq", (q, d), True),
            (p + "wk", (kv, d), True),
            (p + "wv", (kv, d), True),
            (p + "wo", (d, q), True),
            (p + "ffn_norm", (d,), False),
            (p + "wgate", (f, d), True),
            (p + "wup", (f, d), True),
            (p + "wdown", (d, f), True),
        ]
    specs += [("final_norm", (d,), False)]
    if not cfg.tie_embeddings:
        specs += [("lm_head", (v, d), True)]
    return specs


def n_params(cfg: ModelConfig) -> int:
    return sum(int(np.prod(s)) for _, s, _ in tensor_specs(cfg))


def _elem_bytes(cfg: ModelConfig, is_matrix: bool) -> int:
    return 2 if (is_matrix and cfg.dtype == "bf16") else 4


def blob_layout(cfg: ModelConfig) -> Tuple[Dict[str, Tuple[int, Tuple[int, ...], bool]], int]:
    """name -> (byte offset, shape, is_matrix); and the total blob size."""
    off = 0
    out: Dict[str, Tuple[int, Tuple[int, ...], bool]] = {}
    for name, shape, is_matrix in tensor_specs(cfg):
        off = (off + BLOB_ALIGN - 1) // BLOB_ALIGN * BLOB_ALIGN
        out[name] = (off, shape, is_matrix)
        off += int(np.prod(shape)) * _elem_bytes(cfg, is_matrix)
    return out, off


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to the nearest bf16 (ties to even); returns the uint16 bit patterns."""
    b = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = (b + np.uint32(0x7FFF) + ((b >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Exact widening of bf16 bit patterns to fp32."""
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def _draw_normal(seed: int, tensor_idx: int, n: int, std: float, threads: int) -> np.ndarray:
    """n draws of N(0, std) as fp32.  Chunk c of tensor t always comes from the stream
    SeedSequence([seed, t, c]), so the values do not depend on the thread count."""
    out = np.empty(n, dtype=np.float32)
    chunks = [(c, lo, min(lo + _CHUNK, n)) for c, lo in enumerate(range(0, n, _CHUNK))]

    def fill(job):
        c, lo, hi = job
        rng = np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, tensor_idx, c])))
        rng.standard_normal(hi - lo, dtype=np.float32, out=out[lo:hi])
        out[lo:hi] *= np.float32(std)

    if threads > 1 and len(chunks) > 1:
        with ThreadPoolExecutor(threads) as ex:
            list(ex.map(fill, chunks))
    else:
        for job in chunks:
            fill(job)
    return out


def default_threads() -> int:
    env = os.environ.get("OMP_NUM_THREADS")
    if env and env.isdigit():
        return max(1, int(env))
    return max(1, min(16, os.cpu_count() or 1))


class Weights:
    """Named tensors of one model, as stored (fp32 arrays, or uint16 bf16 bit patterns).

    ``f32(name)`` gives the tensor's values as fp32 (an exact widening for bf16), which is
    what the CPU oracle consumes; ``blob()`` gives the canonical byte blob the library consumes.
    """

    def __init__(self, cfg: ModelConfig, tensors: Dict[str, np.ndarray]):
        self.cfg = cfg
        self.tensors = tensors
        self._cache: Dict[str, np.ndarray] = {}

    def names(self) -> Iterable[str]:
        return self.tensors.keys()

    def f32(self, name: str, cache: bool = True) -> np.ndarray:
        if name == "lm_head" and self.cfg.tie_embeddings:
            name = "embed"
        t = self.tensors[name]
        if t.dtype == np.float32:
            return t
        if name in self._cache:
            return self._cache[name]
        w = bf16_bits_to_f32(t)
        if cache:
            self._cache[name] = w
        return w

    def drop_cache(self) -> None:
        self._cache.clear()

    def blob(self) -> np.ndarray:
        layout, total = blob_layout(self.cfg)
        buf = np.zeros(total, dtype=np.uint8)
        for name, (off, _shape, _m) in layout.items():
            raw = np.ascontiguousarray(self.tensors[name]).reshape(-1).view(np.uint8)
            buf[off:off + raw.size] = raw
        return buf


def make_weights(cfg: ModelConfig, seed: int = 0, std: float = 0.02, threads: int | None = None,
                 only_layers: int | None = None, gain_std: float = 0.0) -> Weights:
    """Random weights: every matrix ~ N(0, std) (rounded to bf16 for dtype "bf16"), every
    norm gain = 1, or 1 + N(0, gain_std) per element when gain_std > 0 (a trained model's gains are
    not all one; each gain vector has its own random stream like every other tensor).
    ``only_layers`` keeps the first k layers (same values as in the full model, since each
    tensor has its own random stream) and returns a k-layer model."""
    threads = threads or default_threads()
    full_specs = tensor_specs(cfg)
    index = {name: i for i, (name, _, _) in enumerate(full_specs)}
    if only_layers is not None:
        cfg = cfg.with_(n_layers=only_layers)
    tensors: Dict[str, np.ndarray] = {}
    for name, shape, is_matrix in tensor_specs(cfg):
        if not is_matrix:
            g = np.ones(shape, dtype=np.float32)
            if gain_std > 0.0:
                g += _draw_normal(seed, index[name], int(np.prod(shape)), gain_std, 1).reshape(shape)
            tensors[name] = g
            continue
        w = _draw_normal(seed, index[name], int(np.prod(shape)), std, threads).reshape(shape)
        tensors[name] = f32_to_bf16_bits(w) if cfg.dtype == "bf16" else w
    return Weights(cfg, tensors)


def weights_from_blob(cfg: ModelConfig, blob: np.ndarray) -> Weights:
    """Views into a canonical blob (no copy)."""
    layout, total = blob_layout(cfg)
    assert blob.dtype == np.uint8 and blob.size >= total
    tensors = {}
    for name, (off, shape, is_matrix) in layout.items():
        nbytes = int(np.prod(shape)) * _elem_bytes(cfg, is_matrix)
        dt = np.uint16 if (is_matrix and cfg.dtype == "bf16") else np.float32
        tensors[name] = blob[off:off + nbytes].view(dt).reshape(shape)
    return Weights(cfg, tensors)


def make_token_ids(shape: Tuple[int, ...], vocab: int, seed: int) -> np.ndarray:
    """Uniform random token ids in [0, vocab) as int32."""
    rng = np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, 0x70726f6d])))
    return rng.integers(0, vocab, size=shape, dtype=np.int64).astype(np.int32)


def make_prompts(n_prompts: int, prompt_len: int, vocab: int, seed: int) -> np.ndarray:
    return make_token_ids((n_prompts, prompt_len), vocab, seed)


def make_sequences(n_seqs: int, seq_len: int, vocab: int, seed: int) -> np.ndarray:
    return make_token_ids((n_seqs, seq_len), vocab, seed)


def make_actions(n_states: int, n_actions: int, max_action_len: int, vocab: int, seed: int,
                 min_len: int = 1) -> Tuple[np.ndarray, np.ndarray]:
    """Candidate actions of every state: uniform random token ids [n_states, n_actions, max_action_len]
    and lengths uniform in [min_len, max_action_len] (int32 [n_states, n_actions]).  The first candidate
    of every state has the full length, so the longest row is always exercised; with min_len 0 the last
    candidate of every state is empty."""
    rng = np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, 0x61637473])))
    actions = rng.integers(0, vocab, size=(n_states, n_actions, max_action_len), dtype=np.int64).astype(np.int32)
    lens = rng.integers(min_len, max_action_len + 1, size=(n_states, n_actions), dtype=np.int64).astype(np.int32)
    if min_len == 0:
        lens[:, -1] = 0
    lens[:, 0] = max_action_len
    return actions, lens


def make_ppo_samples(n: int, seed: int) -> Tuple[np.ndarray, np.ndarray, np.ndarray, np.ndarray]:
    """Stand-ins for the scored samples of a policy update: old log-probs N(-12, 0.5) (the level of the
    synthetic policies), new = old + N(0, 0.15), advantages N(0, 1), and a mask that keeps ~80 %.
    Returns (new, old, advantages) as float32 and mask as int32."""
    rng = np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, 0x70706f])))
    old = rng.normal(-12.0, 0.5, n).astype(np.float32)
    new = (old + rng.normal(0.0, 0.15, n)).astype(np.float32)
    adv = rng.normal(0.0, 1.0, n).astype(np.float32)
    mask = (rng.random(n) < 0.8).astype(np.int32)
    return new, old, adv, mask
