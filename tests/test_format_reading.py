"""Which 16-bit format the operands of the matrix products can have (CPU only).

The workload says "bf16": that fixes the weights (both sides consume the same bf16-rounded values).  The
log-probability tolerance (1e-2 against the fp32 definition) then decides the format of what the GPU path
rounds on the way: the nine operand points of a block -- the normalised input of the QKV projection (x1),
the rotated queries and keys (q, k), the values (v), the un-normalised softmax weights (p), the attention
output (o), the normalised input of the feed-forward (x2), the SwiGLU product (a) -- and the normalised
input of the LM head (xf).  This test rounds exactly those points inside the oracle's own forward pass
(a subclass that lives here, not in the oracle) to bf16 (8 significant bits) and to IEEE fp16 (11 bits)
and compares the per-token log-probabilities with the unrounded pass, at a reduced width (the error is a
matter of depth: 28 blocks as in the 1.5 B-class policy) and with weights scaled so that the logits have
the spread of that workload.  bf16 operands break the tolerance, fp16 operands keep well inside it: the
reason the library converts the bf16 weights to fp16 (exactly, for every bf16 value of magnitude in
[2^-17, 65504]) and runs the matrix cores on fp16 operands with an fp16 KV cache.
"""
import math

import numpy as np

import mtmc_oracle as oracle
from helpers import oracle_model
from parity import LOGP_TOL_BF16
from paper_2511_20100_amd import inputs

POINTS = ("x1", "q", "k", "v", "p", "o", "x2", "a", "xf")


def round_bf16(x):
    return inputs.bf16_bits_to_f32(inputs.f32_to_bf16_bits(np.asarray(x, dtype=np.float32))).reshape(np.shape(x))


def round_fp16(x):
    return np.asarray(x, dtype=np.float32).astype(np.float16).astype(np.float32)


class RoundedOperands(oracle.Model):
    """The oracle's block and head with a rounding function applied at the chosen operand points."""

    def __init__(self, base: oracle.Model, rnd, points):
        self.__dict__.update(base.__dict__)
        self.rnd, self.points = rnd, frozenset(points)

    def r(self, name, x):
        return self.rnd(x) if name in self.points else x

    def block(self, l, h, pos, k_ctx, v_ctx):
        assert k_ctx is None and v_ctx is None
        p = f"layers.{l}."
        T = h.shape[0]
        u = self.r("x1", oracle.rmsnorm(h, self.w(p + "attn_norm"), self.eps))
        q = (u @ self.w(p + "wq").T).reshape(T, self.Hq, self.hd)
        k = (u @ self.w(p + "wk").T).reshape(T, self.Hkv, self.hd)
        v = self.r("v", (u @ self.w(p + "wv").T).reshape(T, self.Hkv, self.hd))
        q = self.r("q", oracle.rope_apply(q, pos, self.cos, self.sin))
        k = self.r("k", oracle.rope_apply(k, pos, self.cos, self.sin))
        G = self.Hq // self.Hkv
        visible = np.arange(T)[None, :] <= np.arange(T)[:, None]
        o = np.empty_like(q)
        for j in range(self.Hq):
            s = np.where(visible, (q[:, j] @ k[:, j // G].T) / math.sqrt(self.hd), -np.inf)
            e = np.exp(s - s.max(-1, keepdims=True))
            den = e.sum(-1, keepdims=True)          # the running sum stays fp32; the weights are rounded
            o[:, j] = (self.r("p", e) @ v[:, j // G]) / den
        h = h + self.r("o", o.reshape(T, -1)) @ self.w(p + "wo").T
        u = self.r("x2", oracle.rmsnorm(h, self.w(p + "ffn_norm"), self.eps))
        a = self.r("a", oracle.silu(u @ self.w(p + "wgate").T) * (u @ self.w(p + "wup").T))
        return h + a @ self.w(p + "wdown").T, k, v

    def head(self, h):
        return self.r("xf", oracle.rmsnorm(h, self.w("final_norm"), self.eps)) @ self.w("lm_head").T


def setup():
    # 28 blocks like the 1.5 B-class policy, a third of its width; std scaled by sqrt(1536 / 512) so that
    # the logits keep the workload's spread (sigma about 0.8)
    cfg = inputs.ModelConfig(28, 512, 4, 2, 128, 1376, 4096, dtype="bf16")
    w = inputs.make_weights(cfg, seed=0, std=0.035)
    ids = inputs.make_sequences(1, 96, cfg.vocab, seed=3)[0]
    return oracle_model(w, 128), ids


def logprobs(model, ids):
    return oracle.log_softmax_at(model.logits(ids)[:-1], ids[1:])


def test_unrounded_subclass_is_the_oracle():
    """With no point selected the subclass must reproduce the oracle's forward pass (it restates the block)."""
    base, ids = setup()
    same = RoundedOperands(base, round_bf16, ())
    assert np.abs(logprobs(same, ids[:24]) - logprobs(base, ids[:24])).max() < 2e-5


def test_bf16_operands_break_the_tolerance_and_fp16_operands_keep_it():
    base, ids = setup()
    ref = logprobs(base, ids)
    assert abs(np.std(base.logits(ids[:8])[-1]) - 0.8) < 0.3       # the spread the workload's logits have
    e_bf16 = np.abs(logprobs(RoundedOperands(base, round_bf16, POINTS), ids) - ref)
    e_fp16 = np.abs(logprobs(RoundedOperands(base, round_fp16, POINTS), ids) - ref)
    e_kv = np.abs(logprobs(RoundedOperands(base, round_bf16, ("k", "v")), ids) - ref)
    print(f"all nine points: bf16 max {e_bf16.max():.2e} rms {np.sqrt((e_bf16 ** 2).mean()):.2e}; "
          f"fp16 max {e_fp16.max():.2e} rms {np.sqrt((e_fp16 ** 2).mean()):.2e}; bf16 KV cache alone max {e_kv.max():.2e}")
    assert e_bf16.max() > LOGP_TOL_BF16                # bf16 activations + KV cache: outside the tolerance
    assert e_fp16.max() < 0.5 * LOGP_TOL_BF16          # fp16 at the same points: well inside
    assert e_kv.max() > 0.5 * LOGP_TOL_BF16            # a bf16 KV cache alone already spends most of the budget
    # three more significant bits: about 8 times smaller errors
    ratio = np.sqrt((e_bf16 ** 2).mean()) / np.sqrt((e_fp16 ** 2).mean())
    assert 4.0 < ratio < 16.0


def test_at_the_statistics_of_the_7b_class_fp16_operands_alone_exceed_1e_2():
    """The 7 B-class policy is 2.3 times wider: with the same N(0, 0.02) weights its attention scores, feed-forward
    pre-activations and logits have 1.5 times the spread (logit sigma about 1.2), and the same relative rounding of
    the operands moves the log-probs further.  At a seventh of its width with the standard deviation scaled to keep
    those spreads, and its full depth, fp16 rounding of the nine operand points alone exceeds 1e-2 (about 1.6e-2):
    the tolerance of the full-depth GPU test of that class is derived from this, and bf16 operands are off by an
    order of magnitude more."""
    cfg = inputs.ModelConfig(28, 512, 4, 2, 128, 2720, 4096, dtype="bf16")
    w = inputs.make_weights(cfg, seed=0, std=0.02 * math.sqrt(3584 / 512))
    ids = inputs.make_sequences(1, 160, cfg.vocab, seed=3)[0]
    base = oracle_model(w, 256)
    ref = logprobs(base, ids)
    assert abs(np.std(base.logits(ids[:8])[-1]) - 1.2) < 0.3
    e_fp16 = np.abs(logprobs(RoundedOperands(base, round_fp16, POINTS), ids) - ref)
    print(f"7 B-class statistics, all nine points fp16: max {e_fp16.max():.2e} rms {np.sqrt((e_fp16 ** 2).mean()):.2e}")
    from parity import LOGP_TOL_BF16_7B_FULL_DEPTH
    assert LOGP_TOL_BF16 < e_fp16.max() < LOGP_TOL_BF16_7B_FULL_DEPTH
    assert np.sqrt((e_fp16 ** 2).mean()) < 0.75 * LOGP_TOL_BF16
