"""GPU parity at the layer shapes of the two classes of backbone the paper names for its policy (Method,
"Training Methodology"): a 1.3 B-class model with one kv head per query head (d 2048, 16 heads of 128,
F 5504, V 32256) and a 1 B-class model with grouped 64-dim heads and a tied LM head (d 2048, 32/8 heads of
64, F 8192, V 128256).  Two blocks of each so that the oracle can follow, at the benchmark's batch of 64."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

from parity import LOGP_TOL_BF16, check_actions, check_rollout_by_replay, check_score
from paper_2511_20100_amd import inputs

SHAPES = [("1p3b-mha", inputs.POLICY_1P3B_MHA.with_(n_layers=2)), ("1b-hd64", inputs.POLICY_1B_HD64.with_(n_layers=2))]


@pytest.mark.parametrize("name,cfg", SHAPES, ids=[s[0] for s in SHAPES])
def test_two_blocks_of_the_policy_shape(name, cfg):
    from paper_2511_20100_amd import mtmc
    w = inputs.make_weights(cfg, seed=0, gain_std=0.1)
    handle = mtmc.mtmc_weights_create(mtmc.make_config(cfg, 128), w.blob())
    try:
        prompts = inputs.make_prompts(8, 40, cfg.vocab, seed=2)
        rep = check_rollout_by_replay(handle, w, prompts, 8, 12, 1.0, 1, max_positions=128, rows=[0, 63], label=name)
        print(name, "rollout: compared", rep["compared"], "of", rep["steps"], "max log-prob err", rep["max_logp_err"])
        assert rep["compared"] > 0.5 * rep["steps"]
        seqs = np.concatenate([np.repeat(prompts, 8, axis=0), rep["ids"]], axis=1)
        sc = check_score(handle, w, seqs, 40, max_positions=128, rows=[0, 63], label=name)
        print(name, "score: max log-prob err", sc["max_logp_err"])
        assert np.abs(sc["logprobs"][:, 39:] - rep["logprobs"]).max() <= 2 * LOGP_TOL_BF16
        actions, lens = inputs.make_actions(2, 3, 6, cfg.vocab, seed=3)
        arep = check_actions(handle, w, prompts[:2], actions, lens, max_positions=128, tol=LOGP_TOL_BF16, label=name)
        print(name, "actions: token err", arep["max_token_err"])
    finally:
        mtmc.mtmc_weights_destroy(handle)
