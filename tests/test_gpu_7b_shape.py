"""GPU parity at the layer shapes of the 7 B-class policy (d 3584, 28/4 heads of 128, F 18944,
V 152064, bf16), with 2 of its 28 blocks so that the oracle can follow: batch 128 (16 prompts x 8
samples, the widest decode batch one launch takes), rollout verified by replay of two rows on the
oracle, scoring of the same rows, decode == score."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

from parity import LOGP_TOL_BF16, check_rollout_by_replay, check_score
from paper_2511_20100_amd import inputs

CFG = inputs.ModelConfig(2, 3584, 28, 4, 128, 18944, 152064, dtype="bf16")


def test_two_blocks_of_the_7b_shape():
    from paper_2511_20100_amd import mtmc
    w = inputs.make_weights(CFG, seed=0)
    handle = mtmc.mtmc_weights_create(mtmc.make_config(CFG, 128), w.blob())
    try:
        prompts = inputs.make_prompts(16, 40, CFG.vocab, seed=2)
        rep = check_rollout_by_replay(handle, w, prompts, 8, 12, 1.0, 1, max_positions=128, rows=[0, 127],
                                      label="7b-shape")
        print("7b shape rollout: compared", rep["compared"], "of", rep["steps"], "max log-prob err", rep["max_logp_err"])
        assert rep["compared"] > 0.5 * rep["steps"]
        seqs = np.concatenate([np.repeat(prompts, 8, axis=0), rep["ids"]], axis=1)
        sc = check_score(handle, w, seqs, 40, max_positions=128, rows=[0, 127], label="7b-shape")
        print("7b shape score: max log-prob err", sc["max_logp_err"])
        assert np.abs(sc["logprobs"][:, 39:] - rep["logprobs"]).max() <= 2 * LOGP_TOL_BF16
    finally:
        mtmc.mtmc_weights_destroy(handle)


def test_long_context_and_long_scoring_at_the_7b_shape():
    """One block of the 7 B shape at the context lengths of its long workloads: decode over 2048-token prompts
    (batch 32, the decode attention walks 129 pages per sequence in several chunks) and scoring of a
    3072-token sequence (the prefill attention's longest column blocks)."""
    import torch
    from paper_2511_20100_amd import mtmc
    cfg = CFG.with_(n_layers=1)
    w = inputs.make_weights(cfg, seed=0, gain_std=0.1)
    handle = mtmc.mtmc_weights_create(mtmc.make_config(cfg, 3072), w.blob())
    try:
        prompts = inputs.make_prompts(4, 2048, cfg.vocab, seed=2)
        rep = check_rollout_by_replay(handle, w, prompts, 8, 6, 1.0, 1, max_positions=3072, rows=[31], label="7b-long")
        print("7b long context: compared", rep["compared"], "of", rep["steps"], "max log-prob err", rep["max_logp_err"])
        seqs = inputs.make_sequences(2, 3072, cfg.vocab, seed=3)
        sc = check_score(handle, w, seqs, 3040, max_positions=3072, rows=[1], label="7b-3072")
        print("7b 3072-token scoring: max log-prob err", sc["max_logp_err"], "top-1 compared", sc["compared"])
    finally:
        mtmc.mtmc_weights_destroy(handle)
