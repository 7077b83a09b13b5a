"""GPU parity of action-level scoring (Eq. 2 summed per candidate action, softmax over a state's
candidates) against the oracle, which evaluates every candidate by itself from the start of its
state; the library evaluates a state once and lets its candidates share the cached keys/values."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

from parity import LOGP_TOL_BF16, check_actions
from paper_2511_20100_amd import inputs

LOGP_TOL_F32 = 1e-4
SMALL = inputs.ModelConfig(2, 256, 4, 2, 128, 688, 4096, dtype="bf16")
GQA6 = inputs.ModelConfig(2, 384, 6, 1, 128, 1024, 2048, dtype="bf16")

# (name, config, std, tol, n_states, state_len, K, A, min_len, normalize)
CASES = [
    ("f32-ragged", inputs.TINY, 0.02, LOGP_TOL_F32, 3, 37, 5, 7, 0, False),       # shared pages + a forked tail page
    ("f32-page-aligned", inputs.TINY, 0.02, LOGP_TOL_F32, 2, 33, 4, 20, 1, False),  # state fills whole pages
    ("f32-one-token-state", inputs.TINY, 0.02, LOGP_TOL_F32, 2, 1, 3, 5, 1, True),  # nothing to prefill
    ("f32-short-state", inputs.TINY, 0.02, LOGP_TOL_F32, 2, 9, 6, 3, 1, True),      # state shorter than a page
    ("f32-chunked", inputs.TINY, 0.02, LOGP_TOL_F32, 5, 2000, 10, 170, 1, False),   # states and candidate rows in 2 chunks each
    ("bf16-ragged", SMALL, 0.05, LOGP_TOL_BF16, 3, 37, 5, 7, 0, False),
    ("bf16-long-actions", SMALL, 0.05, LOGP_TOL_BF16, 2, 70, 3, 40, 1, True),      # candidates span several pages
    ("bf16-gqa6-many", GQA6, 0.05, LOGP_TOL_BF16, 4, 48, 16, 6, 1, False),
    ("bf16-one-token-state", GQA6, 0.05, LOGP_TOL_BF16, 1, 1, 2, 4, 1, False),
    ("bf16-hd64-tied", inputs.ModelConfig(2, 512, 8, 2, 64, 1024, 2048, dtype="bf16", tie_embeddings=True), 0.05,
     LOGP_TOL_BF16, 2, 45, 6, 9, 1, False),
    ("bf16-long-state", GQA6, 0.04, LOGP_TOL_BF16, 1, 300, 3, 5, 1, False),         # several 256-key blocks of context
    ("bf16-chunked", SMALL, 0.05, LOGP_TOL_BF16, 5, 20, 200, 170, 0, False),        # 1000 candidates: packed in 2 chunks
    ("bf16-one-token-actions", GQA6, 0.05, LOGP_TOL_BF16, 3, 30, 40, 1, 0, False),  # A = 1: a candidate is one token or empty
]


@pytest.fixture(scope="module")
def lib():
    from paper_2511_20100_amd import mtmc
    return mtmc


@pytest.mark.parametrize("name,cfg,std,tol,n_states,P,K,A,min_len,normalize", CASES, ids=[c[0] for c in CASES])
def test_actions_match_oracle(lib, name, cfg, std, tol, n_states, P, K, A, min_len, normalize):
    w = inputs.make_weights(cfg, seed=0, std=std, gain_std=0.1)
    handle = lib.mtmc_weights_create(lib.make_config(cfg, max(512, P + A)), w.blob())
    try:
        states = inputs.make_prompts(n_states, P, cfg.vocab, seed=21)
        actions, lens = inputs.make_actions(n_states, K, A, cfg.vocab, seed=22, min_len=min_len)
        rep = check_actions(handle, w, states, actions, lens, normalize=normalize, max_positions=max(512, P + A), tol=tol,
                            label=name)
        print(name, "token err", rep["max_token_err"], "action err", rep["max_action_err"], "policy err",
              rep["max_policy_err"])
    finally:
        lib.mtmc_weights_destroy(handle)


def test_actions_agree_with_the_scoring_pass_and_ignore_padding(lib):
    """The per-token terms equal what mtmc_score gives for state + action as one sequence (within the
    bf16 tolerance: the two passes block their sums differently), padding never matters, and two calls
    give identical bits."""
    import torch
    cfg = GQA6
    w = inputs.make_weights(cfg, seed=0, std=0.05, gain_std=0.1)
    handle = lib.mtmc_weights_create(lib.make_config(cfg, 256), w.blob())
    try:
        P, K, A = 41, 4, 9
        states = inputs.make_prompts(2, P, cfg.vocab, seed=31)
        actions, lens = inputs.make_actions(2, K, A, cfg.vocab, seed=32)
        dev = lambda x: torch.from_numpy(x).cuda()
        tok, act, pol = lib.mtmc_score_actions(handle, dev(states), dev(actions), dev(lens))
        tok2, act2, pol2 = lib.mtmc_score_actions(handle, dev(states), dev(actions), dev(lens))
        assert torch.equal(tok, tok2) and torch.equal(act, act2) and torch.equal(pol, pol2)
        other = actions.copy()
        for n in range(2):
            for k in range(K):
                other[n, k, lens[n, k]:] = (other[n, k, lens[n, k]:] + 7) % cfg.vocab
        tok3, act3, pol3 = lib.mtmc_score_actions(handle, dev(states), dev(other), dev(lens))
        assert torch.equal(tok, tok3) and torch.equal(act, act3) and torch.equal(pol, pol3)
        seqs = np.concatenate([np.repeat(states, K, axis=0), actions.reshape(2 * K, A)], axis=1)
        s = lib.mtmc_score(handle, dev(seqs), P).cpu().numpy()[:, P - 1:].reshape(2, K, A)
        live = np.arange(A)[None, None, :] < lens[:, :, None]
        assert np.abs(np.where(live, s - tok.cpu().numpy(), 0.0)).max() <= 2 * LOGP_TOL_BF16
        lib.mtmc_poll_errors(handle)
    finally:
        lib.mtmc_weights_destroy(handle)


def test_all_candidates_empty(lib):
    """No candidate has a token: nothing is evaluated in the second pass; every score is 0 and the policy uniform."""
    import torch
    cfg = SMALL
    w = inputs.make_weights(cfg, seed=0, std=0.05, gain_std=0.1)
    handle = lib.mtmc_weights_create(lib.make_config(cfg, 128), w.blob())
    try:
        states = torch.from_numpy(inputs.make_prompts(2, 19, cfg.vocab, seed=1)).cuda()
        actions, lens = inputs.make_actions(2, 4, 6, cfg.vocab, seed=2)
        tok, act, pol = lib.mtmc_score_actions(handle, states, torch.from_numpy(actions).cuda(),
                                               torch.zeros((2, 4), dtype=torch.int32, device="cuda"))
        lib.mtmc_poll_errors(handle)
        assert torch.all(tok == 0) and torch.all(act == 0)
        assert torch.allclose(pol, torch.full_like(pol, float(-np.log(4.0))), atol=1e-6)
    finally:
        lib.mtmc_weights_destroy(handle)


def test_bad_action_lengths_and_shapes_are_reported(lib):
    import torch
    cfg = inputs.TINY
    w = inputs.make_weights(cfg, seed=0, gain_std=0.1)
    handle = lib.mtmc_weights_create(lib.make_config(cfg, 64), w.blob())
    try:
        states = torch.from_numpy(inputs.make_prompts(2, 8, cfg.vocab, seed=1)).cuda()
        actions, lens = inputs.make_actions(2, 3, 4, cfg.vocab, seed=2)
        bad = lens.copy(); bad[1, 2] = 5
        lib.mtmc_score_actions(handle, states, torch.from_numpy(actions).cuda(), torch.from_numpy(bad).cuda())
        with pytest.raises(lib.MtmcError, match="length outside its range"):
            lib.mtmc_poll_errors(handle)
        lib.mtmc_poll_errors(handle)  # the flag was cleared
        with pytest.raises(lib.MtmcError, match="max_positions"):
            lib.mtmc_score_actions_workspace_bytes(handle, 1, 61, 2, 4)
        with pytest.raises(lib.MtmcError, match="positive"):
            lib.mtmc_score_actions_workspace_bytes(handle, 1, 8, 0, 4)
        with pytest.raises(lib.MtmcError, match="workspace too small"):
            lib.mtmc_score_actions(handle, states, torch.from_numpy(actions).cuda(), torch.from_numpy(lens).cuda(),
                                   workspace=torch.empty(256, dtype=torch.uint8, device="cuda"))
    finally:
        lib.mtmc_weights_destroy(handle)
