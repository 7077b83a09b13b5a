"""GPU parity at the 7 B-class policy at FULL depth, in the decode launch configuration of the second benchmark
workload: 28 layers, d 3584, 28/4 heads of 128, F 18944, V 152064, bf16 weights; 16 prompts x 8 samples = batch 128,
prompt 1024, T = 1.  The rollout is cut to 96 new tokens (the decode kernels and their launch shapes do not depend
on how long the call runs; the oracle's cost does) and the oracle teacher-forces windows of two rows: the two that
hold the largest |decode - score| of the run, i.e. where one of the two GPU paths is furthest from the exact value.
The reduced-depth cases of this shape (2 blocks, also at a context of 8224 tokens) are in test_gpu_7b_shape.py.

Tolerance: at this depth and width the fp16 rounding of the operands alone accounts for errors of 1.6e-2 (see
parity.LOGP_TOL_BF16_7B_FULL_DEPTH and tests/test_format_reading.py), so the 1e-2 of the smaller workloads cannot
hold here; the measured worst errors are printed and must stay inside what that rounding explains."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

from helpers import oracle_model
from parity import LOGP_TOL_BF16, LOGP_TOL_BF16_7B_FULL_DEPTH as TOL, MARGIN_GATE, oracle_replay_window
from paper_2511_20100_amd import inputs

CFG = inputs.POLICY_7B
N_PROMPTS, PROMPT_LEN, N_SAMPLES, MAX_NEW = 16, 1024, 8, 96
WINDOW = 32


@pytest.fixture(scope="module")
def run():
    import torch
    from paper_2511_20100_amd import mtmc
    print("7 B weights ...", flush=True)
    w = inputs.make_weights(CFG, seed=0)
    handle = mtmc.mtmc_weights_create(mtmc.make_config(CFG, PROMPT_LEN + MAX_NEW), w.blob())
    prompts = inputs.make_prompts(N_PROMPTS, PROMPT_LEN, CFG.vocab, seed=2)
    dprompts = torch.from_numpy(prompts).cuda()
    print("rollout + scoring ...", flush=True)
    ids, lp = mtmc.mtmc_rollout(handle, dprompts, N_SAMPLES, MAX_NEW, 1.0, 1)
    seqs = torch.cat([dprompts.repeat_interleave(N_SAMPLES, 0), ids], 1).contiguous()
    score = mtmc.mtmc_score(handle, seqs, PROMPT_LEN)
    mtmc.mtmc_poll_errors(handle)
    out = dict(w=w, prompts=prompts, ids=ids.cpu().numpy(), lp=lp.cpu().numpy(), score=score.cpu().numpy())
    mtmc.mtmc_weights_destroy(handle)
    return out


def test_decode_equals_score_everywhere(run):
    """At T = 1 the log-prob returned with a sampled token is the Eq. 2 factor that the scoring pass returns for it
    (two kernel paths, each within the tolerance of the exact factor)."""
    d = np.abs(run["score"][:, PROMPT_LEN - 1:] - run["lp"])
    print("7 B decode vs score: max", d.max(), "mean", d.mean())
    assert d.max() <= 2 * TOL and d.mean() <= 0.25 * TOL
    assert np.all(run["score"][:, :PROMPT_LEN - 1] == 0.0)
    assert run["ids"].min() >= 0 and run["ids"].max() < CFG.vocab
    assert abs(run["lp"].mean() + np.log(CFG.vocab)) < 1.0   # logit spread about 1.2: the mean log-prob is ln V + 0.7


def test_worst_rows_against_the_oracle(run):
    model = oracle_model(run["w"], PROMPT_LEN + MAX_NEW)
    d = np.abs(run["score"][:, PROMPT_LEN - 1:] - run["lp"])
    rows = np.argsort(d.max(axis=1))[::-1][:2]
    worst_r = worst_s = 0.0
    for row in rows:
        s_star = int(d[row].argmax())
        lo = max(0, min(s_star - WINDOW // 2, MAX_NEW - WINDOW))
        hi = lo + WINDOW
        print(f"oracle: row {row}, steps {lo}..{hi - 1} ...", flush=True)
        tok, ref_lp, mar = oracle_replay_window(model, run["prompts"][row // N_SAMPLES], run["ids"][row], lo, hi, 1.0, 1,
                                                int(row))
        gate = mar > MARGIN_GATE
        given = run["ids"][row, lo:hi]
        err_r = np.abs(ref_lp - run["lp"][row, lo:hi])
        err_s = np.abs(ref_lp - run["score"][row, PROMPT_LEN - 1 + lo:PROMPT_LEN - 1 + hi])
        print(f"row {row} steps {lo}..{hi - 1} (|decode - score| {d[row, s_star]:.2e} at step {s_star}): "
              f"rollout err max {err_r.max():.2e}, score err max {err_s.max():.2e}, "
              f"{int(gate.sum())}/{WINDOW} decisions compared", flush=True)
        assert np.array_equal(tok[gate], given[gate]), (row, np.nonzero(gate & (tok != given))[0][:8])
        assert gate.mean() > 0.7
        worst_r, worst_s = max(worst_r, float(err_r.max())), max(worst_s, float(err_s.max()))
    print(f"7 B, full depth, worst over the two windows: rollout {worst_r:.2e}, score {worst_s:.2e}")
    assert worst_r <= TOL and worst_s <= TOL
    if max(worst_r, worst_s) > LOGP_TOL_BF16:
        print(f"note: beyond the {LOGP_TOL_BF16:g} of the smaller workloads, inside the {TOL:g} that fp16 operands allow here")
