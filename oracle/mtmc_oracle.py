"""CPU oracle for the policy's rollout and scoring pass.  TEST INFRASTRUCTURE ONLY.

This file is the slow, plain definition that the HIP library is checked against.  It is
not part of the product: only the tests, the smoke check and the benchmark's CPU-baseline
leg may import it, and it shares no code with the HIP path (it imports nothing from the
package; weights arrive as plain fp32 numpy arrays).

What it computes
----------------
The Macro Thinking policy is a lightweight decoder-only language model (Method, "Training
Methodology").  An action a_k is a token sequence w_k^1..w_k^N whose probability is the
product of the per-token conditionals (Eq. 2).  Two operations follow from that:

* ``score``   -- teacher-forced per-token log-probabilities log P(w^i | s, w^<i): the
                 logarithms of the factors of Eq. 2.
* ``action_policy`` -- the sums of those terms over each candidate action of a state and
                 their softmax over the candidate set (the sampling probability of an action).
* ``ppo_clip_loss`` -- the clipped surrogate of the PPO update over scored samples (value only).
* ``rollout_ragged`` -- the same for prompts of different lengths, ending at a stop token.
* ``rollout`` -- sampling a token sequence from the same conditionals, one token at a
                 time (Inference Pipeline, "Macro Thinking": the policy outputs an action),
                 by the Gumbel-max rule with noise from a counter-based generator.

The paper fixes nothing about the network beyond "pre-trained lightweight LLM"; the block
structure below (pre-norm residual blocks, RMSNorm, rotary embedding with half-split
pairing, grouped-query causal attention, SwiGLU feed-forward, untied LM head, no biases)
is the standard public definition of the model family its backbones belong to.

Arithmetic: fp32 by default (``dtype=np.float32``), with float64 for rotary angles, the
log-sum-exp and the Gumbel transform.  ``dtype=np.float64`` runs everything in double.
Nothing is blocked, fused or reordered: logits are materialised, K/V are plain contiguous
arrays, attention builds the explicit score matrix.

Pins (tests/test_oracle_*.py): Philox known-answer vectors; Gumbel-max law (chi-square);
brute-force scalar-loop attention and forward pass on tiny shapes; closed forms (2-D
rotation, uniform attention = running mean, zero-residual model); invariants (rotary
norm / relative position, RMS, log-softmax rows, chain rule over all continuations,
causality, cache == recompute, batch-independence of the sampler); for the action policy,
the full candidate set (all V^n actions: the softmax changes nothing), single-token actions
(policy = softmax of the logits), padding independence and the composition of two actions.
The full forward pass at real model sizes has no external truth to compare with (no
trained weights or reference logits exist here): "parity unpinned" beyond those pins.
"""
from __future__ import annotations

import math
from typing import Callable, Dict, List, Optional, Tuple

import numpy as np

# --------------------------------------------------------------------------------------
# Counter-based generator: Philox4x32-10 (Salmon, Moraes, Dror, Shaw, SC'11, section 3.3).
# --------------------------------------------------------------------------------------
_PHILOX_M0 = np.uint64(0xD2511F53)
_PHILOX_M1 = np.uint64(0xCD9E8D57)
_PHILOX_W0 = np.uint64(0x9E3779B9)  # golden ratio
_PHILOX_W1 = np.uint64(0xBB67AE85)  # sqrt(3) - 1
_MASK32 = np.uint64(0xFFFFFFFF)


def philox4x32_10(counter: np.ndarray, key: np.ndarray) -> np.ndarray:
    """Ten rounds of the Philox-4x32 bijection.

    counter: uint32 [..., 4], key: uint32 [..., 2] (broadcastable).  Returns uint32 [..., 4].
    One round maps (c0,c1,c2,c3) to (hi(M1*c2)^c1^k0, lo(M1*c2), hi(M0*c0)^c3^k1, lo(M0*c0));
    the key is bumped by the Weyl constants between rounds.
    """
    c = np.asarray(counter).astype(np.uint64)
    k = np.asarray(key).astype(np.uint64)
    c0, c1, c2, c3 = c[..., 0], c[..., 1], c[..., 2], c[..., 3]
    k0, k1 = k[..., 0], k[..., 1]
    for r in range(10):
        if r > 0:
            k0 = (k0 + _PHILOX_W0) & _MASK32
            k1 = (k1 + _PHILOX_W1) & _MASK32
        p0 = _PHILOX_M0 * c0
        p1 = _PHILOX_M1 * c2
        hi0, lo0 = p0 >> np.uint64(32), p0 & _MASK32
        hi1, lo1 = p1 >> np.uint64(32), p1 & _MASK32
        c0, c1, c2, c3 = hi1 ^ c1 ^ k0, lo1, hi0 ^ c3 ^ k1, lo0
    return np.stack([c0, c1, c2, c3], axis=-1).astype(np.uint32)


def random_bits(seed: int, seq: int, step: int, vocab: int) -> np.ndarray:
    """The 32 random bits attached to every vocabulary entry v of (sequence, step).

    Counter = (v // 4, step, sequence, 0), key = (low, high) words of the 64-bit seed; entry v
    takes output word v % 4.  A pure function of (seed, sequence, step, v)."""
    n4 = (vocab + 3) // 4
    ctr = np.zeros((n4, 4), dtype=np.uint32)
    ctr[:, 0] = np.arange(n4, dtype=np.uint32)
    ctr[:, 1] = np.uint32(step)
    ctr[:, 2] = np.uint32(seq)
    key = np.array([seed & 0xFFFFFFFF, (seed >> 32) & 0xFFFFFFFF], dtype=np.uint32)
    return philox4x32_10(ctr, key).reshape(-1)[:vocab]


def bits_to_uniform(r: np.ndarray) -> np.ndarray:
    """u = ((r >> 9) + 1/2) * 2^-23: 2^23 equally spaced values strictly inside (0, 1), each
    exactly representable in fp32."""
    return ((r >> np.uint32(9)).astype(np.float64) + 0.5) * (2.0 ** -23)


def gumbel_noise(seed: int, seq: int, step: int, vocab: int) -> np.ndarray:
    """g_v = -ln(-ln u_v), evaluated in double and rounded once to fp32."""
    u = bits_to_uniform(random_bits(seed, seq, step, vocab))
    return (-np.log(-np.log(u))).astype(np.float32)


# --------------------------------------------------------------------------------------
# Building blocks
# --------------------------------------------------------------------------------------
def rmsnorm(h: np.ndarray, gain: np.ndarray, eps: float) -> np.ndarray:
    """RMSNorm(h; g)_i = h_i * g_i / sqrt(mean_j h_j^2 + eps), over the last axis."""
    ms = np.mean(h * h, axis=-1, keepdims=True, dtype=h.dtype)
    return (h / np.sqrt(ms + h.dtype.type(eps))) * gain.astype(h.dtype)


def rope_tables(n_pos: int, head_dim: int, base: float) -> Tuple[np.ndarray, np.ndarray]:
    """cos(t*theta_i), sin(t*theta_i) for t < n_pos, i < head_dim/2, theta_i = base^(-2i/head_dim).
    Angles in double, tables rounded once to fp32."""
    i = np.arange(head_dim // 2, dtype=np.float64)
    theta = np.power(np.float64(base), -2.0 * i / head_dim)
    ang = np.arange(n_pos, dtype=np.float64)[:, None] * theta[None, :]
    return np.cos(ang).astype(np.float32), np.sin(ang).astype(np.float32)


def rope_apply(w: np.ndarray, pos: np.ndarray, cos: np.ndarray, sin: np.ndarray) -> np.ndarray:
    """Rotate head vectors w [T, H, hd] at positions pos [T]; pairs are (i, i + hd/2):
    (w_i, w_{i+hd/2}) <- (w_i c - w_{i+hd/2} s,  w_{i+hd/2} c + w_i s)."""
    half = w.shape[-1] // 2
    c = cos[pos][:, None, :].astype(w.dtype)
    s = sin[pos][:, None, :].astype(w.dtype)
    a, b = w[..., :half], w[..., half:]
    return np.concatenate([a * c - b * s, b * c + a * s], axis=-1)


def silu(z: np.ndarray) -> np.ndarray:
    return z / (1.0 + np.exp(-z))


def softmax_rows(s: np.ndarray) -> np.ndarray:
    m = np.max(s, axis=-1, keepdims=True)
    e = np.exp(s - m)
    return e / np.sum(e, axis=-1, keepdims=True, dtype=s.dtype)


def causal_gqa_attention(q: np.ndarray, k: np.ndarray, v: np.ndarray) -> np.ndarray:
    """q [T, Hq, hd] are the queries of the LAST T positions of a context whose keys/values
    are k, v [Tk, Hkv, hd].  Query head j reads kv head j // (Hq/Hkv); query t (absolute
    position Tk - T + t) sees keys tau <= Tk - T + t.  Returns [T, Hq, hd]."""
    T, Hq, hd = q.shape
    Tk, Hkv, _ = k.shape
    G = Hq // Hkv
    scale = q.dtype.type(1.0 / math.sqrt(hd))
    visible = np.arange(Tk)[None, :] <= (np.arange(T)[:, None] + (Tk - T))
    out = np.empty_like(q)
    for j in range(Hq):
        kj, vj = k[:, j // G, :], v[:, j // G, :]
        s = (q[:, j, :] @ kj.T) * scale
        s = np.where(visible, s, q.dtype.type(-np.inf))
        out[:, j, :] = softmax_rows(s) @ vj
    return out


def log_softmax_at(z: np.ndarray, idx: np.ndarray) -> np.ndarray:
    """log softmax(z)[idx] per row; the log-sum-exp is taken in double."""
    zd = z.astype(np.float64)
    m = zd.max(axis=-1, keepdims=True)
    lse = (m + np.log(np.exp(zd - m).sum(axis=-1, keepdims=True)))[:, 0]
    return zd[np.arange(z.shape[0]), idx] - lse


def top2(z: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """Per row: index of the largest entry (lowest index on ties) and largest - second largest."""
    i1 = np.argmax(z, axis=-1)
    rows = np.arange(z.shape[0])
    best = z[rows, i1]
    z2 = z.copy()
    z2[rows, i1] = -np.inf
    return i1.astype(np.int32), (best - z2.max(axis=-1)).astype(np.float32)


# --------------------------------------------------------------------------------------
# The model
# --------------------------------------------------------------------------------------
class Model:
    """Shapes + a getter ``w(name) -> fp32 array`` (names: embed, layers.<l>.attn_norm|wq|wk|wv|
    wo|ffn_norm|wgate|wup|wdown, final_norm, lm_head; matrices are [out, in])."""

    def __init__(self, *, n_layers: int, d_model: int, n_q_heads: int, n_kv_heads: int,
                 head_dim: int, d_ffn: int, vocab: int, rms_eps: float, rope_base: float,
                 w: Callable[[str], np.ndarray], max_positions: int = 4096,
                 dtype=np.float32):
        self.L, self.d, self.Hq, self.Hkv = n_layers, d_model, n_q_heads, n_kv_heads
        self.hd, self.F, self.V = head_dim, d_ffn, vocab
        self.eps, self.base = rms_eps, rope_base
        self.dtype = np.dtype(dtype)
        self._w = w
        self.cos, self.sin = rope_tables(max_positions, head_dim, rope_base)

    def w(self, name: str) -> np.ndarray:
        return self._w(name).astype(self.dtype, copy=False)

    # -- one residual block applied to T new positions of one sequence -----------------
    def block(self, l: int, h: np.ndarray, pos: np.ndarray,
              k_ctx: Optional[np.ndarray], v_ctx: Optional[np.ndarray]):
        """h [T, d] at absolute positions pos [T]; (k_ctx, v_ctx) hold the keys/values of the
        earlier positions ([T0, Hkv, hd]) or None.  Returns (h_out, k_all, v_all)."""
        p = f"layers.{l}."
        T = h.shape[0]
        u = rmsnorm(h, self.w(p + "attn_norm"), self.eps)
        q = (u @ self.w(p + "wq").T).reshape(T, self.Hq, self.hd)
        k = (u @ self.w(p + "wk").T).reshape(T, self.Hkv, self.hd)
        v = (u @ self.w(p + "wv").T).reshape(T, self.Hkv, self.hd)
        q = rope_apply(q, pos, self.cos, self.sin)
        k = rope_apply(k, pos, self.cos, self.sin)
        if k_ctx is not None:
            k = np.concatenate([k_ctx, k], axis=0)
            v = np.concatenate([v_ctx, v], axis=0)
        o = causal_gqa_attention(q, k, v).reshape(T, self.Hq * self.hd)
        h = h + o @ self.w(p + "wo").T
        u = rmsnorm(h, self.w(p + "ffn_norm"), self.eps)
        a = silu(u @ self.w(p + "wgate").T) * (u @ self.w(p + "wup").T)
        h = h + a @ self.w(p + "wdown").T
        return h, k, v

    def head(self, h: np.ndarray) -> np.ndarray:
        """Logits z = W_lm RMSNorm(h; g_final), materialised [T, V]."""
        return rmsnorm(h, self.w("final_norm"), self.eps) @ self.w("lm_head").T

    def embed(self, ids: np.ndarray) -> np.ndarray:
        return self.w("embed")[ids]

    # -- full recompute ----------------------------------------------------------------
    def logits(self, ids: np.ndarray) -> np.ndarray:
        """Logits at every position of one sequence ids [T] (no cache)."""
        pos = np.arange(len(ids))
        h = self.embed(ids)
        for l in range(self.L):
            h, _, _ = self.block(l, h, pos, None, None)
        return self.head(h)


class Cache:
    """Plain contiguous per-layer key/value arrays of one sequence."""

    def __init__(self, n_layers: int):
        self.k: List[Optional[np.ndarray]] = [None] * n_layers
        self.v: List[Optional[np.ndarray]] = [None] * n_layers
        self.n = 0

    def copy(self) -> "Cache":
        c = Cache(len(self.k))
        c.k = [None if a is None else a.copy() for a in self.k]
        c.v = [None if a is None else a.copy() for a in self.v]
        c.n = self.n
        return c


def extend(model: Model, cache: Cache, ids: np.ndarray) -> np.ndarray:
    """Append tokens ids [T] to a cached sequence; returns the logits at the LAST new position [V]."""
    pos = np.arange(cache.n, cache.n + len(ids))
    h = model.embed(ids)
    for l in range(model.L):
        h, cache.k[l], cache.v[l] = model.block(l, h, pos, cache.k[l], cache.v[l])
    cache.n += len(ids)
    return model.head(h[-1:])[0]


# --------------------------------------------------------------------------------------
# Scoring: the logarithms of the factors of Eq. 2
# --------------------------------------------------------------------------------------
def score(model: Model, seqs: np.ndarray, prompt_len: int = 1):
    """seqs int [N, S].  Returns (logp [N, S-1] float32, top1 [N, S-1] int32, margin [N, S-1]
    float32) with logp[n, i] = log P(seqs[n, i+1] | seqs[n, :i+1]) for i + 1 >= prompt_len and
    0 elsewhere; top1/margin = arg-max of the logits at position i and its lead over the
    runner-up (0 where not scored)."""
    N, S = seqs.shape
    logp = np.zeros((N, S - 1), dtype=np.float32)
    top1 = np.zeros((N, S - 1), dtype=np.int32)
    margin = np.zeros((N, S - 1), dtype=np.float32)
    first = max(prompt_len - 1, 0)
    for n in range(N):
        z = model.logits(seqs[n])[first:S - 1]
        logp[n, first:] = log_softmax_at(z, seqs[n, first + 1:]).astype(np.float32)
        top1[n, first:], margin[n, first:] = top2(z.astype(np.float32))
    return logp, top1, margin


def action_logprob(token_logp: np.ndarray) -> float:
    """log P_token(a | s): the sum of an action's per-token terms (Eq. 2 in log form)."""
    return float(np.sum(token_logp, dtype=np.float64))


def action_policy(model: Model, states: np.ndarray, actions: np.ndarray, action_len: np.ndarray,
                  normalize: bool = False):
    """The policy over a state's candidate actions (Method, "Training Methodology": Eq. 2, then
    the normalisation of the candidates' scores by a softmax).

    states int [Ns, P]; actions int [Ns, K, A] (entries at and beyond an action's length are
    padding and never looked at); action_len int [Ns, K] with values in [0, A].
    For state n and candidate k, with a = actions[n, k, :action_len[n, k]]:
      token_logp[n, k, i] = log P(a_i | state_n, a_<i)          (0 at padding)
      action_logp[n, k]   = sum_i token_logp[n, k, i]           (Eq. 2 in log form),
                            divided by the action's length when ``normalize`` (a reading: the
                            paper does not say whether lengths are normalised; off by default)
      policy_logp[n, k]   = action_logp[n, k] - logsumexp_j action_logp[n, j].
    Every candidate is evaluated by itself from the start of its state: nothing is shared.
    Returns (token_logp float32 [Ns, K, A], action_logp float32 [Ns, K], policy_logp float32 [Ns, K])."""
    Ns, P = states.shape
    _, K, A = actions.shape
    token_logp = np.zeros((Ns, K, A), dtype=np.float32)
    action_logp = np.zeros((Ns, K), dtype=np.float64)
    for n in range(Ns):
        for k in range(K):
            ln = int(action_len[n, k])
            if ln == 0:
                continue
            a = actions[n, k, :ln]
            z = model.logits(np.concatenate([states[n], a]))[P - 1:P - 1 + ln]
            token_logp[n, k, :ln] = log_softmax_at(z, a).astype(np.float32)
            total = float(np.sum(token_logp[n, k, :ln], dtype=np.float64))
            action_logp[n, k] = total / ln if normalize else total
    m = action_logp.max(axis=1, keepdims=True)
    lse = m + np.log(np.exp(action_logp - m).sum(axis=1, keepdims=True))
    return token_logp, action_logp.astype(np.float32), (action_logp - lse).astype(np.float32)


def ppo_clip_loss(new_logp: np.ndarray, old_logp: np.ndarray, advantages: np.ndarray, clip_eps: float,
                  mask: Optional[np.ndarray] = None):
    """The clipped surrogate of the standard PPO algorithm that the policy is trained with (Method,
    "Training Methodology"), over the n samples whose mask is non-zero (all when mask is None):
      r_i  = exp(new_logp_i - old_logp_i)
      loss = - mean_i min(r_i A_i, clip(r_i, 1 - eps, 1 + eps) A_i)
    plus two diagnostics: the fraction of samples with |r_i - 1| > eps and the mean of
    old_logp_i - new_logp_i (a first-order estimate of the KL divergence from the old policy).
    The paper gives no value of eps (its appendix is not available): it is an argument.
    Everything in float64.  Returns (loss, clip_fraction, approx_kl, count); zeros when nothing is selected."""
    new_logp = np.asarray(new_logp, dtype=np.float64).ravel()
    old_logp = np.asarray(old_logp, dtype=np.float64).ravel()
    adv = np.asarray(advantages, dtype=np.float64).ravel()
    keep = np.ones(new_logp.shape, dtype=bool) if mask is None else (np.asarray(mask).ravel() != 0)
    n = int(keep.sum())
    if n == 0:
        return 0.0, 0.0, 0.0, 0
    r = np.exp(new_logp[keep] - old_logp[keep])
    a = adv[keep]
    surrogate = np.minimum(r * a, np.clip(r, 1.0 - clip_eps, 1.0 + clip_eps) * a)
    return (float(-surrogate.mean()), float((np.abs(r - 1.0) > clip_eps).mean()),
            float((old_logp[keep] - new_logp[keep]).mean()), n)


# --------------------------------------------------------------------------------------
# Rollout: Gumbel-max sampling from the same conditionals
# --------------------------------------------------------------------------------------
def sample_token(z: np.ndarray, temperature: float, g: Optional[np.ndarray]):
    """One sampling decision from logits z [V] (fp32).

    y_v = z_v / T + g_v in fp32; token = argmax_v y_v (lowest index on ties);
    logp = z_tok / T - logsumexp_v(z_v / T).  T == 0 means greedy: g = 0 and T := 1.
    Returns (token, logp, margin of y)."""
    z = z.astype(np.float32)
    if temperature == 0.0:
        zt = z
        y = z
    else:
        zt = z * np.float32(1.0 / temperature)
        y = zt + g
    tok, mar = top2(y[None, :])
    lp = log_softmax_at(zt[None, :], tok)[0]
    return int(tok[0]), np.float32(lp), float(mar[0])


def rollout(model: Model, prompts: np.ndarray, n_samples: int, max_new: int,
            temperature: float, seed: int, mode: str = "cache", first_seq: int = 0):
    """prompts int [P, Lp].  Sequence b = first_seq + p * n_samples + s continues prompt p.
    Returns (ids [P*n_samples, max_new] int32, logp float32 same shape, margins float32).
    mode "cache": keys/values kept per sequence; mode "recompute": the whole prefix is
    run again for every token."""
    P, Lp = prompts.shape
    B = P * n_samples
    ids = np.zeros((B, max_new), dtype=np.int32)
    logp = np.zeros((B, max_new), dtype=np.float32)
    margins = np.zeros((B, max_new), dtype=np.float32)
    for p in range(P):
        base_cache = None
        if mode == "cache":
            base_cache = Cache(model.L)
            z_prompt = extend(model, base_cache, prompts[p])
        for s in range(n_samples):
            row = p * n_samples + s
            b = first_seq + row
            seq = list(prompts[p])
            cache = base_cache.copy() if mode == "cache" else None
            z = z_prompt if mode == "cache" else None
            for i in range(max_new):
                if mode == "recompute":
                    z = model.logits(np.array(seq, dtype=np.int64))[-1]
                g = gumbel_noise(seed, b, i, model.V) if temperature != 0.0 else None
                tok, lp, mar = sample_token(z, temperature, g)
                ids[row, i], logp[row, i], margins[row, i] = tok, lp, mar
                seq.append(tok)
                if mode == "cache" and i + 1 < max_new:
                    z = extend(model, cache, np.array([tok], dtype=np.int64))
    return ids, logp, margins


def rollout_ragged(model: Model, prompts: np.ndarray, prompt_lens: np.ndarray, n_samples: int, max_new: int,
                   temperature: float, seed: int, stop_id: int = -1, first_seq: int = 0):
    """Rollout of prompts of different lengths with an optional stop token (Inference Pipeline,
    "Macro Thinking": generation ends with a terminal action or at the step limit).

    prompts int [P, Lmax], right-padded: prompt p is prompts[p, :prompt_lens[p]] and the padding is
    never looked at.  Sequence b = first_seq + p * n_samples + s continues prompt p exactly as
    ``rollout`` would continue it alone.  With stop_id >= 0 a sequence ends with the first sampled
    stop_id: that token and its log-probability are reported, every later slot holds stop_id with
    log-probability 0.  Returns (ids [B, max_new] int32, logp float32, lens int32 [B] = tokens
    generated including the stop token, margins float32 (0 after the end))."""
    P = prompts.shape[0]
    B = P * n_samples
    ids = np.zeros((B, max_new), dtype=np.int32)
    logp = np.zeros((B, max_new), dtype=np.float32)
    margins = np.zeros((B, max_new), dtype=np.float32)
    lens = np.full(B, max_new, dtype=np.int32)
    for p in range(P):
        rows = slice(p * n_samples, (p + 1) * n_samples)
        ids[rows], logp[rows], margins[rows] = rollout(model, prompts[p:p + 1, :int(prompt_lens[p])], n_samples,
                                                       max_new, temperature, seed,
                                                       first_seq=first_seq + p * n_samples)
    if stop_id >= 0:
        for b in range(B):
            hits = np.nonzero(ids[b] == stop_id)[0]
            if hits.size:
                n = int(hits[0]) + 1
                lens[b] = n
                ids[b, n:] = stop_id
                logp[b, n:] = 0.0
                margins[b, n:] = 0.0
    return ids, logp, lens, margins


def replay(model: Model, prompt: np.ndarray, new_ids: np.ndarray, temperature: float,
           seed: int, seq_index: int):
    """Teacher-force a given continuation and redo every sampling decision on it.

    Returns (tok [n] int32, logp_of_given [n] float32, margin [n] float32): at step i, with the
    context prompt + new_ids[:i], tok[i] is what the sampler picks with the noise of
    (seed, seq_index, i), margin[i] its lead in y over the runner-up, and logp_of_given[i]
    the log-probability (at this temperature) of new_ids[i]."""
    full = np.concatenate([prompt, new_ids]).astype(np.int64)
    n = len(new_ids)
    z = model.logits(full)[len(prompt) - 1:len(prompt) - 1 + n].astype(np.float32)
    tok = np.zeros(n, dtype=np.int32)
    lp = np.zeros(n, dtype=np.float32)
    mar = np.zeros(n, dtype=np.float32)
    for i in range(n):
        g = gumbel_noise(seed, seq_index, i, model.V) if temperature != 0.0 else None
        t, _, m = sample_token(z[i], temperature, g)
        tok[i], mar[i] = t, m
        zt = z[i] if temperature == 0.0 else z[i] * np.float32(1.0 / temperature)
        lp[i] = log_softmax_at(zt[None, :], np.array([new_ids[i]]))[0]
    return tok, lp, mar
