"""GPU parity of the rollout over prompts of different lengths with a stop token."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

import mtmc_oracle as oracle
from helpers import oracle_model
from parity import LOGP_TOL_BF16, check_ragged_by_replay
from paper_2511_20100_amd import inputs

SMALL = inputs.ModelConfig(2, 256, 4, 2, 128, 688, 4096, dtype="bf16")
GQA6 = inputs.ModelConfig(2, 384, 6, 1, 128, 1024, 2048, dtype="bf16")


@pytest.fixture(scope="module")
def lib():
    from paper_2511_20100_amd import mtmc
    return mtmc


def junk_padding(prompts, lens, vocab):
    out = prompts.copy()
    for p in range(prompts.shape[0]):
        out[p, lens[p]:] = (out[p, lens[p]:] + 3) % vocab
    return out


def test_fp32_ids_exact_with_and_without_stop(lib):
    import torch
    cfg = inputs.TINY
    w = inputs.make_weights(cfg, seed=0, gain_std=0.1)
    handle = lib.mtmc_weights_create(lib.make_config(cfg, 128), w.blob())
    try:
        prompts = inputs.make_prompts(4, 40, cfg.vocab, seed=2)
        lens = np.array([40, 17, 32, 5], dtype=np.int32)
        model = oracle_model(w, 128)
        dev = lambda x: torch.from_numpy(x).cuda()
        ref_ids, ref_lp, ref_n, margins = oracle.rollout_ragged(model, prompts, lens, 2, 24, 1.0, seed=1)
        print("min sampling margin of the oracle:", margins.min())
        ids, lp, n = lib.mtmc_rollout_ragged(handle, dev(prompts), dev(lens), 2, 24, 1.0, 1)
        lib.mtmc_poll_errors(handle)
        assert np.array_equal(ids.cpu().numpy(), ref_ids) and np.all(n.cpu().numpy() == 24)
        assert np.abs(lp.cpu().numpy() - ref_lp).max() <= 1e-4
        # padding never matters
        ids2, lp2, _ = lib.mtmc_rollout_ragged(handle, dev(junk_padding(prompts, lens, cfg.vocab)), dev(lens), 2, 24, 1.0, 1)
        assert torch.equal(ids, ids2) and torch.equal(lp, lp2)
        # a stop token that some rows sample: a token of the free run
        stop = int(ref_ids[3, 6])
        s_ids, s_lp, s_n, _ = oracle.rollout_ragged(model, prompts, lens, 2, 24, 1.0, seed=1, stop_id=stop)
        assert s_n.min() < 24
        ids, lp, n = lib.mtmc_rollout_ragged(handle, dev(prompts), dev(lens), 2, 24, 1.0, 1, stop_id=stop)
        lib.mtmc_poll_errors(handle)
        assert np.array_equal(ids.cpu().numpy(), s_ids) and np.array_equal(n.cpu().numpy(), s_n)
        assert np.abs(lp.cpu().numpy() - s_lp).max() <= 1e-4
    finally:
        lib.mtmc_weights_destroy(handle)


CASES = [
    ("small-mixed", SMALL, 0.05, [37, 16, 1, 33], 3, 21, 0.8),
    ("gqa6-two-groups", GQA6, 0.04, [9, 3, 20, 16, 7, 32, 1, 12, 25, 31, 17, 2, 8, 30, 11, 5, 19, 14], 8, 6, 1.0),
    ("gqa6-long", GQA6, 0.05, [150, 64, 90], 4, 30, 1.0),
    # 40 rows: the context of every sequence is split at the end of its own prompt (0, 0, 2, 4 and 6 whole page pairs)
    ("small-b40-split", SMALL, 0.05, [5, 16, 33, 70, 120], 8, 14, 1.0),
    ("hd64-mixed", inputs.ModelConfig(2, 256, 4, 2, 64, 688, 4096, dtype="bf16"), 0.05, [37, 16, 1, 33, 70], 3, 21, 1.0),
]


@pytest.mark.parametrize("name,cfg,std,lens,n_samples,max_new,temp", CASES, ids=[c[0] for c in CASES])
def test_bf16_ragged_by_replay(lib, name, cfg, std, lens, n_samples, max_new, temp):
    import torch
    w = inputs.make_weights(cfg, seed=0, std=std, gain_std=0.1)
    handle = lib.mtmc_weights_create(lib.make_config(cfg, 256), w.blob())
    try:
        lens = np.array(lens, dtype=np.int32)
        prompts = inputs.make_prompts(len(lens), int(lens.max()), cfg.vocab, seed=2)
        free = check_ragged_by_replay(handle, w, prompts, lens, n_samples, max_new, temp, 1, max_positions=256, label=name)
        print(name, "free run: compared", free["compared"], "of", free["steps"], "max log-prob err", free["max_logp_err"])
        assert free["compared"] > 0.5 * free["steps"] and np.all(free["lens"] == max_new)
        # stop at a token that row 1 sampled at step 2: rows end where the free run has it, nothing changes before
        stop = int(free["ids"][1, 2])
        rep = check_ragged_by_replay(handle, w, prompts, lens, n_samples, max_new, temp, 1, stop_id=stop,
                                     max_positions=256, label=name + "-stop")
        assert rep["lens"][1] == 3 and rep["lens"].max() == max_new
        for b in range(len(lens) * n_samples):
            e = rep["lens"][b]
            assert np.array_equal(rep["ids"][b, :e], free["ids"][b, :e])
            assert np.array_equal(rep["logprobs"][b, :e], free["logprobs"][b, :e])
    finally:
        lib.mtmc_weights_destroy(handle)


def test_equal_lengths_give_the_uniform_rollout_and_padding_never_matters(lib):
    import torch
    cfg = GQA6
    w = inputs.make_weights(cfg, seed=0, std=0.05, gain_std=0.1)
    handle = lib.mtmc_weights_create(lib.make_config(cfg, 256), w.blob())
    try:
        dev = lambda x: torch.from_numpy(x).cuda()
        prompts = inputs.make_prompts(3, 21, cfg.vocab, seed=5)
        same = np.full(3, 21, dtype=np.int32)
        a_ids, a_lp = lib.mtmc_rollout(handle, dev(prompts), 4, 12, 1.0, 7)
        b_ids, b_lp, b_n = lib.mtmc_rollout_ragged(handle, dev(prompts), dev(same), 4, 12, 1.0, 7)
        assert torch.equal(a_ids, b_ids) and torch.equal(a_lp, b_lp) and bool((b_n == 12).all())
        lens = np.array([21, 4, 16], dtype=np.int32)
        c = lib.mtmc_rollout_ragged(handle, dev(prompts), dev(lens), 4, 12, 1.0, 7)
        d = lib.mtmc_rollout_ragged(handle, dev(junk_padding(prompts, lens, cfg.vocab)), dev(lens), 4, 12, 1.0, 7)
        assert all(torch.equal(x, y) for x, y in zip(c, d))
        assert torch.equal(c[0][:4], a_ids[:4])  # the full-length prompt is unaffected by its neighbours
        # each prompt alone, at its place in the batch (seq_offset), gives the same rows
        for p in range(3):
            alone = lib.mtmc_rollout_ragged(handle, dev(prompts[p:p + 1]), dev(lens[p:p + 1]), 4, 12, 1.0, 7,
                                            seq_offset=4 * p)
            assert torch.equal(alone[0], c[0][4 * p:4 * p + 4]) and torch.equal(alone[1], c[1][4 * p:4 * p + 4])
        lib.mtmc_poll_errors(handle)
    finally:
        lib.mtmc_weights_destroy(handle)


def test_bad_lengths_and_stop_ids_are_reported(lib):
    import torch
    cfg = inputs.TINY
    w = inputs.make_weights(cfg, seed=0, gain_std=0.1)
    handle = lib.mtmc_weights_create(lib.make_config(cfg, 64), w.blob())
    try:
        prompts = torch.from_numpy(inputs.make_prompts(2, 8, cfg.vocab, seed=1)).cuda()
        lib.mtmc_rollout_ragged(handle, prompts, torch.tensor([8, 9], dtype=torch.int32).cuda(), 2, 4, 1.0, 1)
        with pytest.raises(lib.MtmcError, match="length"):
            lib.mtmc_poll_errors(handle)
        lib.mtmc_rollout_ragged(handle, prompts, torch.tensor([0, 3], dtype=torch.int32).cuda(), 2, 4, 1.0, 1)
        with pytest.raises(lib.MtmcError, match="length"):
            lib.mtmc_poll_errors(handle)
        with pytest.raises(lib.MtmcError, match="stop_id"):
            lib.mtmc_rollout_ragged(handle, prompts, torch.tensor([8, 3], dtype=torch.int32).cuda(), 2, 4, 1.0, 1,
                                    stop_id=cfg.vocab)
        with pytest.raises(lib.MtmcError, match="max_positions"):
            lib.mtmc_rollout_ragged_workspace_bytes(handle, 2, 8, 2, 60)
    finally:
        lib.mtmc_weights_destroy(handle)
