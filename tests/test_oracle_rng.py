"""Pins for the oracle's counter-based generator, uniform mapping and Gumbel-max sampler."""
import os

import numpy as np
import pytest

import mtmc_oracle as oracle


def test_philox_known_answers(golden_dir):
    rows = [l.split() for l in open(os.path.join(golden_dir, "philox4x32_10_kat.txt"))
            if l.strip() and not l.startswith("#")]
    assert len(rows) == 3
    for r in rows:
        w = [int(x, 16) for x in r]
        got = oracle.philox4x32_10(np.array(w[0:4], dtype=np.uint32), np.array(w[4:6], dtype=np.uint32))
        assert [int(x) for x in got] == w[6:10]


def test_philox_is_a_bijection_on_a_small_slice():
    # distinct counters -> distinct outputs (a permutation of the 128-bit block)
    ctr = np.zeros((4096, 4), dtype=np.uint32)
    ctr[:, 0] = np.arange(4096)
    out = oracle.philox4x32_10(ctr, np.array([7, 9], dtype=np.uint32))
    assert len({tuple(r) for r in out.tolist()}) == 4096


def test_random_bits_counter_layout():
    # entry v takes word v % 4 of the block whose counter is (v // 4, step, seq, 0)
    seed, seq, step = (5 << 32) | 11, 3, 17
    bits = oracle.random_bits(seed, seq, step, 10)
    for v in range(10):
        blk = oracle.philox4x32_10(np.array([v // 4, step, seq, 0], dtype=np.uint32),
                                   np.array([11, 5], dtype=np.uint32))
        assert bits[v] == blk[v % 4]


def test_uniform_mapping_open_interval_and_moments():
    assert oracle.bits_to_uniform(np.array([0], dtype=np.uint32))[0] == 2.0 ** -24
    assert oracle.bits_to_uniform(np.array([0xFFFFFFFF], dtype=np.uint32))[0] == 1.0 - 2.0 ** -24
    u = oracle.bits_to_uniform(oracle.random_bits(123, 0, 0, 1 << 20))
    assert u.min() > 0.0 and u.max() < 1.0
    # every value survives a round trip through fp32 exactly
    assert np.array_equal(u.astype(np.float32).astype(np.float64), u)
    n = u.size
    assert abs(u.mean() - 0.5) < 4 * np.sqrt(1 / 12 / n)
    assert abs(u.var() - 1 / 12) < 4 * np.sqrt(1 / 180 / n)


def test_gumbel_noise_is_finite_and_has_gumbel_moments():
    g = oracle.gumbel_noise(99, 1, 2, 1 << 20).astype(np.float64)
    assert np.all(np.isfinite(g))
    n = g.size
    assert abs(g.mean() - 0.5772156649) < 4 * np.sqrt((np.pi ** 2 / 6) / n)
    assert abs(g.var() - np.pi ** 2 / 6) < 0.02


def test_gumbel_max_samples_from_softmax():
    """P(argmax_v(z_v/T + g_v) = v) = softmax(z/T)_v: chi-square on 10^6 draws, V = 16."""
    V, T = 16, 0.7
    rng = np.random.default_rng(0)
    z = rng.normal(0, 1.5, V).astype(np.float32)
    p = np.exp(z / T - np.max(z / T)); p /= p.sum()
    n_seq, n_step = 1000, 1000
    ctr = np.zeros((n_seq, n_step, V // 4, 4), dtype=np.uint32)
    ctr[..., 0] = np.arange(V // 4)[None, None, :]
    ctr[..., 1] = np.arange(n_step)[None, :, None]
    ctr[..., 2] = np.arange(n_seq)[:, None, None]
    bits = oracle.philox4x32_10(ctr, np.array([42, 0], dtype=np.uint32)).reshape(n_seq, n_step, V)
    # same bits as the per-(seq, step) generator
    assert np.array_equal(bits[3, 5], oracle.random_bits(42, 3, 5, V))
    g = (-np.log(-np.log(oracle.bits_to_uniform(bits)))).astype(np.float32)
    y = (z * np.float32(1.0 / T))[None, None, :] + g
    counts = np.bincount(np.argmax(y, axis=-1).reshape(-1), minlength=V)
    n = n_seq * n_step
    chi2 = float(np.sum((counts - n * p) ** 2 / (n * p)))
    assert chi2 < 44.3  # chi-square(15 dof) 0.9999 quantile


def test_sample_token_matches_its_parts_and_tie_break():
    V = 32
    z = np.linspace(-1, 1, V).astype(np.float32)
    g = oracle.gumbel_noise(1, 0, 0, V)
    tok, lp, mar = oracle.sample_token(z, 2.0, g)
    y = z * np.float32(0.5) + g
    assert tok == int(np.argmax(y))
    ref = z[tok] / 2.0 - np.log(np.sum(np.exp(z.astype(np.float64) / 2.0)))
    assert abs(lp - ref) < 1e-6
    s = np.sort(y)
    assert abs(mar - (s[-1] - s[-2])) < 1e-7
    # greedy (T == 0): no noise, plain log-softmax, lowest index wins ties
    zt = np.zeros(V, dtype=np.float32); zt[[5, 9]] = 3.0
    tok, lp, mar = oracle.sample_token(zt, 0.0, None)
    assert tok == 5 and mar == 0.0
    assert abs(lp - (3.0 - np.log(2 * np.exp(3.0) + (V - 2)))) < 1e-6


def test_low_temperature_recovers_argmax():
    V = 64
    z = np.random.default_rng(1).normal(0, 1, V).astype(np.float32)
    for step in range(20):
        tok, _, _ = oracle.sample_token(z, 1e-3, oracle.gumbel_noise(7, 0, step, V))
        assert tok == int(np.argmax(z))
