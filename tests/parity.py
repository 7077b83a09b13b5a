"""Shared parity checks (GPU library vs CPU oracle) used by the gpu-marked tests."""
import numpy as np

import mtmc_oracle as oracle
from helpers import oracle_model
from paper_2511_20100_amd import inputs

LOGP_TOL_BF16 = 1e-2   # per-token log-prob, bf16 GPU path vs fp32 oracle
# The same at the FULL depth of the 7 B-class policy (28 blocks, d 3584, logit spread 1.2 instead of 0.8): rounding
# the nine operand points of a block to fp16, and nothing else, already moves a log-prob by up to 1.6e-2 there
# (rms 5e-3; tests/test_format_reading.py reproduces that on the CPU), so 16-bit operands cannot meet 1e-2 at that
# size.  The bound below is that figure with a margin for the maximum over many more tokens than the emulation has.
LOGP_TOL_BF16_7B_FULL_DEPTH = 2.5e-2
MARGIN_GATE = 0.05     # ids are compared where the oracle's decision margin exceeds this


def check_rollout_by_replay(handle, w, prompts, n_samples, max_new, temperature, seed, *, max_positions,
                            seq_offset=0, rows=None, tol=LOGP_TOL_BF16, label=""):
    """Runs mtmc_rollout, then has the oracle teacher-force the GPU's own sequences and redo every
    sampling decision with the same noise.  Ids must agree wherever the oracle's perturbed margin
    exceeds MARGIN_GATE, log-probs everywhere within tol.  Returns a small report dict."""
    import torch
    from paper_2511_20100_amd import mtmc
    ids, lp = mtmc.mtmc_rollout(handle, torch.from_numpy(prompts).cuda(), n_samples, max_new, temperature, seed,
                                seq_offset=seq_offset)
    mtmc.mtmc_poll_errors(handle)
    ids, lp = ids.cpu().numpy(), lp.cpu().numpy()
    assert ids.min() >= 0 and ids.max() < w.cfg.vocab
    model = oracle_model(w, max_positions)
    B = prompts.shape[0] * n_samples
    rows = range(B) if rows is None else rows
    gated = total = 0
    worst = 0.0
    for b in rows:
        tok, ref_lp, margin = oracle.replay(model, prompts[b // n_samples], ids[b], temperature, seed, seq_offset + b)
        gate = margin > MARGIN_GATE
        bad = np.nonzero(gate & (tok != ids[b]))[0]
        assert bad.size == 0, f"{label} row {b}: sampled id differs from the oracle at steps {bad[:8]} " \
                              f"(margins {margin[bad[:8]]})"
        err = np.abs(ref_lp - lp[b]).max()
        worst = max(worst, float(err))
        assert err <= tol, f"{label} row {b}: log-prob error {err}"
        gated += int(gate.sum()); total += gate.size
    return {"ids": ids, "logprobs": lp, "compared": gated, "steps": total, "max_logp_err": worst}


def oracle_replay_window(model, prompt, new_ids, lo, hi, temperature, seed, seq_index):
    """oracle.replay restricted to the steps lo .. hi - 1 of a long continuation: the oracle's blocks run over
    prompt + new_ids[:hi - 1] (everything those steps can see), its LM head over the window's rows only, and
    every sampling decision of the window is redone with the noise of (seed, seq_index, step).
    Returns (tok, logp_of_given, margin), each [hi - lo]."""
    P = len(prompt)
    full = np.concatenate([prompt, new_ids[:hi - 1]]).astype(np.int64)
    pos = np.arange(len(full))
    h = model.embed(full)
    for l in range(model.L):
        h, _, _ = model.block(l, h, pos, None, None)
    z = model.head(h[P - 1 + lo:P - 1 + hi]).astype(np.float32)
    n = hi - lo
    tok, lp, mar = np.zeros(n, np.int32), np.zeros(n, np.float32), np.zeros(n, np.float32)
    for i in range(lo, hi):
        g = oracle.gumbel_noise(seed, seq_index, i, model.V) if temperature != 0.0 else None
        t, _, m = oracle.sample_token(z[i - lo], temperature, g)
        tok[i - lo], mar[i - lo] = t, m
        zt = z[i - lo] if temperature == 0.0 else z[i - lo] * np.float32(1.0 / temperature)
        lp[i - lo] = oracle.log_softmax_at(zt[None, :], np.array([new_ids[i]]))[0]
    return tok, lp, mar


def check_score(handle, w, seqs, prompt_len, *, max_positions, rows=None, tol=LOGP_TOL_BF16, label=""):
    import torch
    from paper_2511_20100_amd import mtmc
    s, top1, margin = mtmc.mtmc_score(handle, torch.from_numpy(seqs).cuda(), prompt_len, want_top1=True)
    mtmc.mtmc_poll_errors(handle)
    s, top1, margin = s.cpu().numpy(), top1.cpu().numpy(), margin.cpu().numpy()
    model = oracle_model(w, max_positions)
    rows = list(range(seqs.shape[0])) if rows is None else list(rows)
    ref_s, ref_top1, ref_margin = oracle.score(model, seqs[rows], prompt_len)
    err = np.abs(s[rows] - ref_s).max()
    assert err <= tol, f"{label}: score log-prob error {err}"
    assert np.all(s[:, :prompt_len - 1] == 0.0) and np.all(top1[:, :prompt_len - 1] == 0)
    gate = ref_margin > MARGIN_GATE
    assert np.array_equal(top1[rows][gate], ref_top1[gate]), f"{label}: top-1 ids differ above the margin gate"
    assert np.abs(margin[rows] - ref_margin).max() <= 2 * tol
    return {"logprobs": s, "max_logp_err": float(err), "compared": int(gate.sum()), "positions": int(gate.size)}


def check_actions(handle, w, states, actions, lens, *, normalize=False, max_positions, tol, label=""):
    """Runs mtmc_score_actions and compares all three outputs with the oracle's action_policy.
    Per-token terms within tol; an action's score is a sum of N terms, so N * tol bounds it (tol when
    normalised); a policy term is a score minus a weighted mean of scores: twice that bound."""
    import torch
    from paper_2511_20100_amd import mtmc
    tok, act, pol = mtmc.mtmc_score_actions(handle, torch.from_numpy(states).cuda(), torch.from_numpy(actions).cuda(),
                                            torch.from_numpy(lens).cuda(), normalize=normalize)
    mtmc.mtmc_poll_errors(handle)
    tok, act, pol = tok.cpu().numpy(), act.cpu().numpy(), pol.cpu().numpy()
    ref_tok, ref_act, ref_pol = oracle.action_policy(oracle_model(w, max_positions), states, actions, lens,
                                                     normalize=normalize)
    A = actions.shape[2]
    pad = np.arange(A)[None, None, :] >= lens[:, :, None]
    assert np.all(tok[pad] == 0.0), f"{label}: padding terms must be zero"
    e_tok = float(np.abs(tok - ref_tok).max())
    assert e_tok <= tol, f"{label}: token log-prob error {e_tok}"
    act_tol = tol * (1 if normalize else np.maximum(lens, 1))
    e_act = np.abs(act - ref_act)
    assert np.all(e_act <= act_tol), f"{label}: action log-prob error {e_act.max()}"
    e_pol = np.abs(pol - ref_pol)
    assert np.all(e_pol <= 2 * np.max(act_tol)), f"{label}: policy log-prob error {e_pol.max()}"
    assert np.allclose(np.exp(pol.astype(np.float64)).sum(axis=1), 1.0, atol=1e-5)
    return {"token": tok, "action": act, "policy": pol, "max_token_err": e_tok, "max_action_err": float(e_act.max()),
            "max_policy_err": float(e_pol.max())}


def check_ragged_by_replay(handle, w, prompts, lens, n_samples, max_new, temperature, seed, *, stop_id=-1,
                           max_positions, tol=LOGP_TOL_BF16, label=""):
    """mtmc_rollout_ragged, verified row by row: the oracle teacher-forces prompt[:len] + the tokens the GPU
    generated up to the row's end and redoes every sampling decision (ids above the margin gate, log-probs
    within tol); the row ends at the first stop token, and every slot after it holds stop_id / 0."""
    import torch
    from paper_2511_20100_amd import mtmc
    ids, lp, n = mtmc.mtmc_rollout_ragged(handle, torch.from_numpy(prompts).cuda(), torch.from_numpy(lens).cuda(),
                                          n_samples, max_new, temperature, seed, stop_id=stop_id)
    mtmc.mtmc_poll_errors(handle)
    ids, lp, n = ids.cpu().numpy(), lp.cpu().numpy(), n.cpu().numpy()
    model = oracle_model(w, max_positions)
    gated = total = 0
    worst = 0.0
    for b in range(ids.shape[0]):
        p = b // n_samples
        hits = np.nonzero(ids[b] == stop_id)[0] if stop_id >= 0 else np.array([], dtype=int)
        end = int(hits[0]) + 1 if hits.size else max_new
        assert n[b] == end, f"{label} row {b}: reported length {n[b]}, first stop token ends it at {end}"
        assert np.all(ids[b, end:] == stop_id) and np.all(lp[b, end:] == 0.0), f"{label} row {b}: slots after the end"
        tok, ref_lp, margin = oracle.replay(model, prompts[p, :lens[p]], ids[b, :end], temperature, seed, b)
        gate = margin > MARGIN_GATE
        bad = np.nonzero(gate & (tok != ids[b, :end]))[0]
        assert bad.size == 0, f"{label} row {b}: sampled id differs from the oracle at steps {bad[:8]}"
        err = float(np.abs(ref_lp - lp[b, :end]).max())
        worst = max(worst, err)
        assert err <= tol, f"{label} row {b}: log-prob error {err}"
        gated += int(gate.sum()); total += gate.size
    return {"ids": ids, "logprobs": lp, "lens": n, "compared": gated, "steps": total, "max_logp_err": worst}
