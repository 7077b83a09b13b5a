"""Pins for the oracle's building blocks: closed forms, invariants, brute force."""
import math

import numpy as np
import pytest

import mtmc_oracle as oracle


# ---------------------------------------------------------------- RMSNorm
def test_rmsnorm_closed_form_and_invariants():
    h = np.array([[3.0, 4.0]])
    out = oracle.rmsnorm(h, np.array([1.0, 2.0]), 0.0)
    assert np.allclose(out, [[3 / math.sqrt(12.5), 2 * 4 / math.sqrt(12.5)]], atol=1e-12)
    rng = np.random.default_rng(0)
    x = rng.normal(0, 3, (5, 64))
    y = oracle.rmsnorm(x, np.ones(64), 0.0)
    assert np.allclose(np.sqrt(np.mean(y * y, axis=-1)), 1.0, atol=1e-12)
    assert np.allclose(oracle.rmsnorm(7.5 * x, np.ones(64), 0.0), y, atol=1e-12)
    # eps sits inside the square root, added to the mean square
    assert np.allclose(oracle.rmsnorm(np.array([[0.0, 0.0]]), np.ones(2), 1e-6), 0.0)
    assert np.allclose(oracle.rmsnorm(np.array([[1.0, 1.0]]), np.ones(2), 3.0), 0.5)


# ---------------------------------------------------------------- rotary embedding
def test_rope_is_a_plane_rotation():
    # head_dim 2: theta_0 = 1, so position t rotates (1, 0) to (cos t, sin t)
    cos, sin = oracle.rope_tables(16, 2, 10000.0)
    w = np.array([[[1.0, 0.0]]])
    for t in (0, 1, 5, 15):
        r = oracle.rope_apply(w, np.array([t]), cos, sin)[0, 0]
        assert np.allclose(r, [math.cos(t), math.sin(t)], atol=1e-6)


def test_rope_frequencies_and_pairing():
    hd, base = 8, 10000.0
    cos, sin = oracle.rope_tables(32, hd, base)
    t = 3
    for i in range(hd // 2):
        theta = base ** (-2.0 * i / hd)
        assert abs(cos[t, i] - math.cos(t * theta)) < 1e-6
        assert abs(sin[t, i] - math.sin(t * theta)) < 1e-6
    # the partner of component i is i + hd/2
    w = np.zeros((1, 1, hd)); w[0, 0, 1] = 1.0
    r = oracle.rope_apply(w, np.array([t]), cos, sin)[0, 0]
    expect = np.zeros(hd); expect[1] = cos[t, 1]; expect[1 + hd // 2] = sin[t, 1]
    assert np.allclose(r, expect, atol=1e-7)


def test_rope_invariants():
    hd = 16
    cos, sin = oracle.rope_tables(64, hd, 10000.0)
    rng = np.random.default_rng(1)
    q = rng.normal(size=(1, 1, hd)); k = rng.normal(size=(1, 1, hd))
    assert np.allclose(oracle.rope_apply(q, np.array([0]), cos, sin), q)
    for t in (1, 17, 63):
        assert abs(np.linalg.norm(oracle.rope_apply(q, np.array([t]), cos, sin)) - np.linalg.norm(q)) < 1e-6

    def dot(m, n):
        return float(np.sum(oracle.rope_apply(q, np.array([m]), cos, sin) *
                            oracle.rope_apply(k, np.array([n]), cos, sin)))
    assert abs(dot(5, 2) - dot(25, 22)) < 1e-5
    assert abs(dot(40, 40) - dot(0, 0)) < 1e-5
    assert abs(dot(5, 2) - dot(2, 5)) > 1e-3  # depends on the sign of m - n


# ---------------------------------------------------------------- SwiGLU pieces
def test_silu_values():
    z = np.array([0.0, 1.0, -1.0, 30.0, -30.0])
    s = oracle.silu(z)
    assert s[0] == 0.0
    assert abs(s[1] - 0.7310585786300049) < 1e-12
    assert abs(s[2] + 0.2689414213699951) < 1e-12
    assert abs(s[3] - 30.0) < 1e-10 and abs(s[4]) < 1e-10


# ---------------------------------------------------------------- softmax / log-softmax
def test_log_softmax_rows_and_shift_invariance():
    rng = np.random.default_rng(2)
    z = rng.normal(0, 2, (4, 50)).astype(np.float32)
    V = z.shape[1]
    lp = np.stack([oracle.log_softmax_at(z, np.full(4, v)) for v in range(V)], axis=1)
    assert np.allclose(np.exp(lp).sum(axis=1), 1.0, atol=1e-6)
    lp2 = np.stack([oracle.log_softmax_at(z + np.float32(8.0), np.full(4, v)) for v in range(V)], axis=1)
    assert np.allclose(lp, lp2, atol=1e-5)
    # closed form: two equal logits
    assert abs(oracle.log_softmax_at(np.array([[1.0, 1.0]]), np.array([1]))[0] + math.log(2)) < 1e-12
    assert np.allclose(oracle.softmax_rows(z.astype(np.float64)).sum(axis=-1), 1.0, atol=1e-12)


def test_top2():
    z = np.array([[1.0, 5.0, 5.0, 2.0], [0.0, -1.0, -3.0, -0.25]], dtype=np.float32)
    i, m = oracle.top2(z)
    assert list(i) == [1, 0] and np.allclose(m, [0.0, 0.25])


# ---------------------------------------------------------------- attention
def brute_attention(q, k, v):
    """Scalar loops straight from the definition."""
    T, Hq, hd = q.shape
    Tk, Hkv, _ = k.shape
    G = Hq // Hkv
    out = np.zeros((T, Hq, hd))
    for t in range(T):
        last = Tk - T + t
        for j in range(Hq):
            g = j // G
            s = [sum(q[t, j, c] * k[tau, g, c] for c in range(hd)) / math.sqrt(hd) for tau in range(last + 1)]
            m = max(s)
            e = [math.exp(x - m) for x in s]
            tot = sum(e)
            for c in range(hd):
                out[t, j, c] = sum(e[tau] / tot * v[tau, g, c] for tau in range(last + 1))
    return out


@pytest.mark.parametrize("T,Tk,Hq,Hkv,hd", [(6, 6, 4, 2, 8), (1, 9, 6, 1, 4), (3, 10, 2, 2, 16)])
def test_attention_matches_brute_force(T, Tk, Hq, Hkv, hd):
    rng = np.random.default_rng(T * 100 + Tk)
    q = rng.normal(size=(T, Hq, hd)); k = rng.normal(size=(Tk, Hkv, hd)); v = rng.normal(size=(Tk, Hkv, hd))
    assert np.allclose(oracle.causal_gqa_attention(q, k, v), brute_attention(q, k, v), atol=1e-12)


def test_gqa_equals_mha_with_replicated_kv_heads():
    rng = np.random.default_rng(3)
    T, Hq, Hkv, hd = 7, 6, 2, 8
    q = rng.normal(size=(T, Hq, hd)); k = rng.normal(size=(T, Hkv, hd)); v = rng.normal(size=(T, Hkv, hd))
    a = oracle.causal_gqa_attention(q, k, v)
    b = oracle.causal_gqa_attention(q, np.repeat(k, Hq // Hkv, axis=1), np.repeat(v, Hq // Hkv, axis=1))
    assert np.allclose(a, b, atol=1e-14)


def test_attention_zero_queries_give_running_mean():
    rng = np.random.default_rng(4)
    T, hd = 9, 4
    v = rng.normal(size=(T, 1, hd))
    out = oracle.causal_gqa_attention(np.zeros((T, 2, hd)), rng.normal(size=(T, 1, hd)), v)
    mean = np.cumsum(v[:, 0], axis=0) / np.arange(1, T + 1)[:, None]
    assert np.allclose(out[:, 0], mean, atol=1e-12) and np.allclose(out[:, 1], mean, atol=1e-12)


def test_attention_one_hot_limit_picks_the_matching_key():
    # a very sharp score on one visible key returns that key's value
    hd = 4
    k = np.eye(4)[:, None, :] * 100.0          # key tau = 100 e_tau
    v = np.arange(16, dtype=np.float64).reshape(4, 1, 4)
    q = np.zeros((1, 1, hd)); q[0, 0, 2] = 1.0  # selects key 2
    out = oracle.causal_gqa_attention(q, k, v)
    assert np.allclose(out[0, 0], v[2, 0], atol=1e-9)


# ---------------------------------------------------------------- PPO clipped surrogate
def test_ppo_surrogate_closed_forms():
    eps = 0.2
    one = lambda r, a: oracle.ppo_clip_loss([math.log(r)], [0.0], [a], eps)[0]
    assert abs(one(1.5, 2.0) + (1 + eps) * 2.0) < 1e-12     # gain capped at 1 + eps
    assert abs(one(0.5, 2.0) + 0.5 * 2.0) < 1e-12           # a lower ratio is not clipped when A > 0
    assert abs(one(0.5, -2.0) - (1 - eps) * 2.0) < 1e-12    # penalty capped at 1 - eps
    assert abs(one(1.5, -2.0) - 1.5 * 2.0) < 1e-12          # a higher ratio is not clipped when A < 0
    assert abs(one(1.1, 3.0) + 1.1 * 3.0) < 1e-12           # inside the band: plain importance weighting
    # unchanged policy: minus the mean advantage, no clipping, zero divergence
    lp = np.linspace(-5, -1, 7)
    adv = np.array([1.0, -2.0, 0.5, 3.0, -1.0, 0.0, 2.5])
    loss, frac, kl, n = oracle.ppo_clip_loss(lp, lp, adv, eps)
    assert abs(loss + adv.mean()) < 1e-12 and frac == 0.0 and kl == 0.0 and n == 7


def test_ppo_surrogate_against_a_scalar_loop_and_its_bound():
    rng = np.random.default_rng(5)
    n, eps = 200, 0.1
    new, old, adv = rng.normal(-3, 1, n), rng.normal(-3, 1, n), rng.normal(0, 1, n)
    mask = rng.integers(0, 2, n)
    tot = cnt = clipped = 0
    kl = 0.0
    for i in range(n):
        if not mask[i]:
            continue
        r = math.exp(new[i] - old[i])
        rc = min(max(r, 1 - eps), 1 + eps)
        tot += min(r * adv[i], rc * adv[i]); cnt += 1; clipped += abs(r - 1) > eps; kl += old[i] - new[i]
    loss, frac, akl, m = oracle.ppo_clip_loss(new, old, adv, eps, mask)
    assert m == cnt and abs(loss + tot / cnt) < 1e-12 and abs(frac - clipped / cnt) < 1e-12 and abs(akl - kl / cnt) < 1e-12
    # the clipped objective never exceeds the unclipped one
    keep = mask != 0
    assert -loss <= (np.exp(new - old) * adv)[keep].mean() + 1e-12
    # masked-out samples do not matter; an empty selection gives zeros
    adv2 = adv.copy(); adv2[~keep] = 1e9
    assert oracle.ppo_clip_loss(new, old, adv2, eps, mask) == (loss, frac, akl, m)
    assert oracle.ppo_clip_loss(new, old, adv, eps, np.zeros(n)) == (0.0, 0.0, 0.0, 0)
