"""GPU parity of the rollout over prompts of different lengths with a stop token."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

import mtmc_oracle as oracle
from helpers import oracle_model
from parity import LOGP_TOL_BF16, MARGIN_GATE, check_ragged_by_replay
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
        # (sequences beyond the first batch of 128: with a stop token they join the running batch, without one they
        # run as a smaller batch of their own, in kernels of another tiling)
        for b in range(len(lens) * n_samples):
            e = rep["lens"][b]
            assert np.array_equal(rep["ids"][b, :e], free["ids"][b, :e])
            if b < 128:
                assert np.array_equal(rep["logprobs"][b, :e], free["logprobs"][b, :e])
            else:
                assert np.abs(rep["logprobs"][b, :e] - free["logprobs"][b, :e]).max() <= 5e-3
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


# ---------------------------------------------------------------- cached prompt prefix across calls
def grown_prompts(prompts, lens, extra, Lmax, vocab, seed):
    """State of the next optimisation step: every prompt keeps its tokens and gains extra[p] new ones."""
    new = np.zeros((prompts.shape[0], Lmax), dtype=np.int32)
    more = inputs.make_token_ids((prompts.shape[0], Lmax), vocab, seed)
    new_lens = (lens + extra).astype(np.int32)
    for p in range(prompts.shape[0]):
        new[p, :lens[p]] = prompts[p, :lens[p]]
        new[p, lens[p]:new_lens[p]] = more[p, lens[p]:new_lens[p]]
    return new, new_lens


def test_fp32_cached_prefix_equals_the_oracle_on_the_whole_prompt(lib):
    """Two optimisation steps: the second call's prompts extend the first call's; it keeps the cached keys and
    values of the first 32 positions and must give exactly what the oracle gives on the whole new prompts."""
    import torch
    cfg = inputs.TINY
    w = inputs.make_weights(cfg, seed=0, gain_std=0.1)
    handle = lib.mtmc_weights_create(lib.make_config(cfg, 128), w.blob())
    try:
        Lmax, n_new = 64, 10
        lens = np.array([40, 33, 47, 36], dtype=np.int32)
        prompts = np.zeros((4, Lmax), dtype=np.int32)
        prompts[:, :48] = inputs.make_prompts(4, 48, cfg.vocab, seed=2)
        dev = lambda x: torch.from_numpy(x).cuda()
        ws = torch.empty(lib.mtmc_rollout_ragged_workspace_bytes(handle, 4, Lmax, 2, n_new), dtype=torch.uint8, device="cuda")
        model = oracle_model(w, 128)
        ids, lp, n = lib.mtmc_rollout_ragged(handle, dev(prompts), dev(lens), 2, n_new, 1.0, 1, workspace=ws)
        ref = oracle.rollout_ragged(model, prompts, lens, 2, n_new, 1.0, seed=1)
        assert np.array_equal(ids.cpu().numpy(), ref[0])
        new, new_lens = grown_prompts(prompts, lens, np.array([9, 20, 1, 28]), Lmax, cfg.vocab, seed=7)
        ids2, lp2, n2 = lib.mtmc_rollout_ragged_cached(handle, dev(new), dev(new_lens), 2, n_new, 1.0, 5, 32, ws)
        lib.mtmc_poll_errors(handle)
        ref2 = oracle.rollout_ragged(model, new, new_lens, 2, n_new, 1.0, seed=5)
        print("min sampling margin of the oracle:", ref2[3].min())
        assert np.array_equal(ids2.cpu().numpy(), ref2[0]) and np.abs(lp2.cpu().numpy() - ref2[1]).max() <= 1e-4
        # a third step on top of the second, keeping 48 positions now
        new3, lens3 = grown_prompts(new, new_lens, np.array([5, 3, 10, 0]), Lmax, cfg.vocab, seed=8)
        ids3, lp3, _ = lib.mtmc_rollout_ragged_cached(handle, dev(new3), dev(lens3), 2, n_new, 1.0, 6, 48, ws)
        lib.mtmc_poll_errors(handle)
        ref3 = oracle.rollout_ragged(model, new3, lens3, 2, n_new, 1.0, seed=6)
        assert np.array_equal(ids3.cpu().numpy(), ref3[0]) and np.abs(lp3.cpu().numpy() - ref3[1]).max() <= 1e-4
    finally:
        lib.mtmc_weights_destroy(handle)


def test_bf16_cached_prefix_equals_a_fresh_call(lib):
    """MFMA path, 5 prompts x 8 samples: the call that keeps 3 cached pages gives what a fresh call on the same
    prompts gives (bit for bit: every token's arithmetic is the same, only the cached positions are skipped),
    with a stop token, and one row is replayed on the oracle."""
    import torch
    cfg = GQA6
    w = inputs.make_weights(cfg, seed=0, std=0.05, gain_std=0.1)
    handle = lib.mtmc_weights_create(lib.make_config(cfg, 256), w.blob())
    try:
        Lmax, n_new, ns = 120, 12, 8
        lens = np.array([50, 64, 97, 49, 80], dtype=np.int32)
        prompts = np.zeros((5, Lmax), dtype=np.int32)
        prompts[:, :100] = inputs.make_prompts(5, 100, cfg.vocab, seed=2)
        dev = lambda x: torch.from_numpy(x).cuda()
        nbytes = lib.mtmc_rollout_ragged_workspace_bytes(handle, 5, Lmax, ns, n_new)
        ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
        first = lib.mtmc_rollout_ragged(handle, dev(prompts), dev(lens), ns, n_new, 1.0, 1, workspace=ws)
        new, new_lens = grown_prompts(prompts, lens, np.array([30, 11, 23, 1, 40]), Lmax, cfg.vocab, seed=7)
        stop = 5
        cached = lib.mtmc_rollout_ragged_cached(handle, dev(new), dev(new_lens), ns, n_new, 1.0, 9, 48, ws, stop_id=stop)
        lib.mtmc_poll_errors(handle)
        fresh = lib.mtmc_rollout_ragged(handle, dev(new), dev(new_lens), ns, n_new, 1.0, 9, stop_id=stop,
                                        workspace=torch.empty(nbytes, dtype=torch.uint8, device="cuda"))
        lib.mtmc_poll_errors(handle)
        for a, b in zip(cached, fresh):
            assert torch.equal(a, b)
        rep = check_ragged_by_replay(handle, w, new, new_lens, ns, n_new, 1.0, 9, stop_id=stop, max_positions=256,
                                     label="cached-prefix")
        assert np.array_equal(rep["ids"], cached[0].cpu().numpy())
    finally:
        lib.mtmc_weights_destroy(handle)


def test_cached_prefix_misuse_is_reported(lib):
    import torch
    cfg = inputs.TINY
    w = inputs.make_weights(cfg, seed=0)
    handle = lib.mtmc_weights_create(lib.make_config(cfg, 128), w.blob())
    try:
        dev = lambda x: torch.from_numpy(x).cuda()
        prompts = inputs.make_prompts(2, 48, cfg.vocab, seed=2)
        lens = np.array([40, 48], dtype=np.int32)
        ws = torch.empty(lib.mtmc_rollout_ragged_workspace_bytes(handle, 2, 48, 2, 4), dtype=torch.uint8, device="cuda")
        with pytest.raises(lib.MtmcError, match="previous mtmc_rollout_ragged"):      # nothing cached yet
            lib.mtmc_rollout_ragged_cached(handle, dev(prompts), dev(lens), 2, 4, 1.0, 1, 16, ws)
        lib.mtmc_rollout_ragged(handle, dev(prompts), dev(lens), 2, 4, 1.0, 1, workspace=ws)
        with pytest.raises(lib.MtmcError, match="multiple of 16"):
            lib.mtmc_rollout_ragged_cached(handle, dev(prompts), dev(lens), 2, 4, 1.0, 1, 20, ws)
        with pytest.raises(lib.MtmcError, match="previous mtmc_rollout_ragged"):      # another shape
            lib.mtmc_rollout_ragged_cached(handle, dev(prompts), dev(lens), 2, 5, 1.0, 1, 16, ws)
        lib.mtmc_rollout_ragged(handle, dev(prompts), dev(lens), 2, 4, 1.0, 1, workspace=ws)
        changed = prompts.copy(); changed[1, 7] = (changed[1, 7] + 1) % cfg.vocab      # inside the kept prefix
        lib.mtmc_rollout_ragged_cached(handle, dev(changed), dev(lens), 2, 4, 1.0, 1, 16, ws)
        with pytest.raises(lib.MtmcError, match="cached prompt prefix") as e:
            lib.mtmc_poll_errors(handle)
        assert e.value.code == lib.MTMC_EDATA
        lib.mtmc_rollout_ragged(handle, dev(prompts), dev(np.array([20, 48], dtype=np.int32)), 2, 4, 1.0, 1, workspace=ws)
        lib.mtmc_rollout_ragged_cached(handle, dev(prompts), dev(lens), 2, 4, 1.0, 1, 32, ws)   # prompt 0 was 20 long
        with pytest.raises(lib.MtmcError, match="cached prompt prefix"):
            lib.mtmc_poll_errors(handle)
    finally:
        lib.mtmc_weights_destroy(handle)


# ---------------------------------------------------------------- finished rows give up their place
STOPPY = inputs.ModelConfig(2, 384, 6, 1, 128, 1024, 64, dtype="bf16")    # 64 tokens: a stop token comes up every ~64 steps
STOPPY16 = inputs.ModelConfig(2, 256, 4, 2, 128, 688, 16, dtype="bf16")   # 16 tokens: every ~16 steps


@pytest.mark.parametrize("name,cfg,lens,n_samples,max_new,poll", [
    ("b40-poll4", STOPPY, [37, 16, 1, 33, 70], 8, 96, 4),      # 48 slots -> 32 -> 16 as rows finish
    ("b64-poll8", STOPPY, [21, 40, 9, 64, 33, 17, 50, 5], 8, 80, 8),
    ("b128-poll4", STOPPY, list(range(3, 35, 2)), 8, 128, 4),   # the 128-row kernels first, then the 64-row ones
    ("b16-all-stop", STOPPY16, [30, 7], 8, 200, 4),            # every row stops long before the budget: the call ends early
], ids=lambda v: v if isinstance(v, str) else None)
def test_rows_that_stop_give_up_their_place(lib, name, cfg, lens, n_samples, max_new, poll):
    """With a stop token the library looks at the stop flags every few steps, packs the rows still running into
    fewer 16-row tiles and ends when none is left.  Every row is replayed on the oracle (decisions above the
    margin gate, log-probs, lengths, stop_id / 0 after the end); up to the first look the packed call equals the
    call that never looks."""
    import torch
    w = inputs.make_weights(cfg, seed=0, std=0.05, gain_std=0.1)
    handle = lib.mtmc_weights_create(lib.make_config(cfg, 512), w.blob())
    try:
        lens = np.array(lens, dtype=np.int32)
        prompts = inputs.make_prompts(len(lens), int(lens.max()), cfg.vocab, seed=2)
        stop = 3
        lib.mtmc_set_option(handle, lib.MTMC_OPT_STOP_POLL_STEPS, poll)
        rep = check_ragged_by_replay(handle, w, prompts, lens, n_samples, max_new, 1.0, 1, stop_id=stop,
                                     max_positions=512, label=name)
        n = rep["lens"]
        print(name, "lengths: min", n.min(), "median", int(np.median(n)), "max", n.max(), "stopped", int((n < max_new).sum()),
              "of", n.size, "; compared", rep["compared"], "of", rep["steps"], "max log-prob err", rep["max_logp_err"])
        assert (n < max_new).sum() >= n.size // 3
        again = lib.mtmc_rollout_ragged(handle, torch.from_numpy(prompts).cuda(), torch.from_numpy(lens).cuda(), n_samples,
                                        max_new, 1.0, 1, stop_id=stop)
        assert np.array_equal(again[0].cpu().numpy(), rep["ids"]) and np.array_equal(again[1].cpu().numpy(), rep["logprobs"])
        lib.mtmc_set_option(handle, lib.MTMC_OPT_STOP_POLL_STEPS, 0)
        static = lib.mtmc_rollout_ragged(handle, torch.from_numpy(prompts).cuda(), torch.from_numpy(lens).cuda(), n_samples,
                                         max_new, 1.0, 1, stop_id=stop)
        lib.mtmc_poll_errors(handle)
        s_ids, s_lp = static[0].cpu().numpy(), static[1].cpu().numpy()
        first = 2 * poll   # the first look is read one period late: no row moves before step 2 * poll
        assert np.array_equal(s_ids[:, :first], rep["ids"][:, :first]) and np.array_equal(s_lp[:, :first], rep["logprobs"][:, :first])
        same = (s_ids == rep["ids"]).all(axis=1)
        print(name, "rows identical to the unpacked call:", int(same.sum()), "of", same.size)
        assert np.abs(s_lp[same] - rep["logprobs"][same]).max() <= 5e-3
    finally:
        lib.mtmc_weights_destroy(handle)


# ---------------------------------------------------------------- new prompts take the places of finished ones
@pytest.mark.parametrize("name,cfg,n_prompts,n_samples,max_new,poll,max_len", [
    ("40x8-through-16-places", STOPPY, 40, 8, 64, 4, 40),       # 320 sequences through 128 slots
    ("11x24-through-5-places", STOPPY, 11, 24, 48, 8, 33),      # 5 places of 24 slots: 120 of the batch's 128 rows in use
    ("36x8-short-rows", STOPPY16, 36, 8, 120, 2, 70),           # nearly every row stops within 30 steps: many turnovers
], ids=lambda v: v if isinstance(v, str) else None)
def test_new_prompts_take_the_places_of_finished_ones(lib, name, cfg, n_prompts, n_samples, max_new, poll, max_len):
    """A call with a stop token and more sequences than one batch of 128 holds runs as one batch: as soon as enough
    sequences have ended, the next prompt of the call is prefilled and its sequences take the free slots, at their own
    step; when no prompt is left the sequences still running are packed into fewer tiles.  Every row is replayed on
    the oracle (a row's result does not depend on when it ran or next to whom).  Against the call that runs batch
    after batch with every row keeping its place: the sequences of the first batch are the same bit for bit while
    the batch keeps its shape (they start together in both), everything else to rounding (step 0 of a later prompt is
    sampled in a batch of another size, and the packed batch runs kernels of another tiling)."""
    import torch
    w = inputs.make_weights(cfg, seed=0, std=0.05, gain_std=0.1)
    handle = lib.mtmc_weights_create(lib.make_config(cfg, 512), w.blob())
    try:
        lens = (1 + (np.arange(n_prompts) * 7) % max_len).astype(np.int32)
        lens[3] = max_len
        prompts = inputs.make_prompts(n_prompts, max_len, cfg.vocab, seed=2)
        stop = 3
        lib.mtmc_set_option(handle, lib.MTMC_OPT_STOP_POLL_STEPS, poll)
        rep = check_ragged_by_replay(handle, w, prompts, lens, n_samples, max_new, 1.0, 1, stop_id=stop,
                                     max_positions=512, label=name)
        n = rep["lens"]
        print(name, "lengths: min", n.min(), "median", int(np.median(n)), "max", n.max(), "stopped", int((n < max_new).sum()),
              "of", n.size, "; compared", rep["compared"], "of", rep["steps"], "max log-prob err", rep["max_logp_err"])
        assert (n < max_new).sum() >= n.size // 4
        dev = lambda x: torch.from_numpy(x).cuda()
        again = lib.mtmc_rollout_ragged(handle, dev(prompts), dev(lens), n_samples, max_new, 1.0, 1, stop_id=stop)
        assert np.array_equal(again[0].cpu().numpy(), rep["ids"]) and np.array_equal(again[1].cpu().numpy(), rep["logprobs"])
        assert np.array_equal(again[2].cpu().numpy(), n)
        # batch after batch, nobody moves
        lib.mtmc_set_option(handle, lib.MTMC_OPT_ADMIT_PROMPTS, 0)
        lib.mtmc_set_option(handle, lib.MTMC_OPT_STOP_POLL_STEPS, 0)
        static = lib.mtmc_rollout_ragged(handle, dev(prompts), dev(lens), n_samples, max_new, 1.0, 1, stop_id=stop)
        lib.mtmc_poll_errors(handle)
        s_ids, s_lp, s_n = (x.cpu().numpy() for x in static)
        # while prompts are left the batch keeps its shape: the looks are `period` steps apart, one look takes in at
        # most `places` prompts, and the sequences left are packed one look after the last prompt at the earliest
        places, period = 128 // n_samples, min(poll, 8)
        first, t_safe = places * n_samples, period * (-(-(n_prompts - places) // places) + 1)
        assert np.array_equal(s_ids[:first, :t_safe], rep["ids"][:first, :t_safe])
        assert np.array_equal(s_lp[:first, :t_safe], rep["logprobs"][:first, :t_safe])
        same = (s_ids == rep["ids"]).all(axis=1)
        print(name, "rows identical to the batch-after-batch call:", int(same.sum()), "of", same.size)
        assert same.sum() >= 0.6 * same.size
        assert np.abs(s_lp[same] - rep["logprobs"][same]).max() <= 5e-3 and np.array_equal(s_n[same], n[same])
        # a prompt that joins later with a length outside [1, max_len] is reported like one of the first batch
        lib.mtmc_set_option(handle, lib.MTMC_OPT_ADMIT_PROMPTS, 1)
        lib.mtmc_set_option(handle, lib.MTMC_OPT_STOP_POLL_STEPS, poll)
        bad = lens.copy()
        bad[n_prompts - 1] = max_len + 1
        lib.mtmc_rollout_ragged(handle, dev(prompts), dev(bad), n_samples, max_new, 1.0, 1, stop_id=stop)
        with pytest.raises(lib.MtmcError, match="length"):
            lib.mtmc_poll_errors(handle)
    finally:
        lib.mtmc_weights_destroy(handle)


EDGE = [
    # name, cfg, prompt lengths (cycled over n_prompts), n_prompts, n_samples, max_new, temperature, graph
    ("one-sample-per-prompt", STOPPY, [5, 16, 33], 150, 1, 40, 1.0, 1),          # 128 places of one slot
    ("128-samples-one-place", STOPPY16, [20, 7, 48], 3, 128, 60, 1.0, 1),        # a prompt fills the batch: joins only when all have ended
    ("two-steps", STOPPY16, [9, 32], 40, 8, 2, 1.0, 1),                           # every row ends at its step 0 or 1
    ("greedy", STOPPY16, [12, 30, 16], 40, 8, 50, 0.0, 1),                        # the 8 samples of a prompt are the same sequence
    ("whole-pages-no-graph", STOPPY, [16, 32, 48], 36, 8, 48, 1.0, 0),            # no partly filled page to fork; steps launched directly
    ("long-prompts-two-per-prefill", STOPPY16, [4000, 3990], 22, 8, 24, 1.0, 1),  # a prefill takes two of these prompts at most
]


@pytest.mark.parametrize("name,cfg,lens,n_prompts,n_samples,max_new,temp,graph", EDGE, ids=[e[0] for e in EDGE])
def test_joining_prompts_edge_cases(lib, name, cfg, lens, n_prompts, n_samples, max_new, temp, graph):
    import torch
    w = inputs.make_weights(cfg, seed=0, std=0.05, gain_std=0.1)
    max_len = max(lens)
    positions = (max_len + max_new + 63) // 64 * 64
    handle = lib.mtmc_weights_create(lib.make_config(cfg, positions), w.blob())
    try:
        lens = np.array([lens[i % len(lens)] for i in range(n_prompts)], dtype=np.int32)
        prompts = inputs.make_prompts(n_prompts, max_len, cfg.vocab, seed=2)
        lib.mtmc_set_option(handle, lib.MTMC_OPT_HIP_GRAPH, graph)
        lib.mtmc_set_option(handle, lib.MTMC_OPT_STOP_POLL_STEPS, 4)
        dev = lambda x: torch.from_numpy(x).cuda()
        ids, lp, n = lib.mtmc_rollout_ragged(handle, dev(prompts), dev(lens), n_samples, max_new, temp, 3, stop_id=3)
        lib.mtmc_poll_errors(handle)
        ids, lp, n = ids.cpu().numpy(), lp.cpu().numpy(), n.cpu().numpy()
        print(name, "lengths: min", n.min(), "median", int(np.median(n)), "max", n.max(), "of", n.size, "rows")
        # every row: ends at its first stop token, stop_id / 0 behind it
        for b in range(ids.shape[0]):
            hits = np.nonzero(ids[b] == 3)[0]
            end = int(hits[0]) + 1 if hits.size else max_new
            assert n[b] == end and np.all(ids[b, end:] == 3) and np.all(lp[b, end:] == 0.0), (name, b)
            assert np.all(lp[b, :end] < 0.0) and np.all(np.isfinite(lp[b, :end]))
        if temp == 0.0:
            g = ids.reshape(n_prompts, n_samples, max_new)
            assert np.all(g == g[:, :1])
        # rows spread over the call (first batch, joined early, joined last) against the oracle
        model = oracle_model(w, positions)
        rows = sorted({0, n_samples - 1, ids.shape[0] // 2, ids.shape[0] - n_samples, ids.shape[0] - 1})
        worst = 0.0
        for b in rows:
            p, e = b // n_samples, int(n[b])
            tok, ref_lp, margin = oracle.replay(model, prompts[p, :lens[p]], ids[b, :e], temp, 3, b)
            gate = margin > MARGIN_GATE
            assert np.array_equal(tok[gate], ids[b, :e][gate]), (name, b)
            worst = max(worst, float(np.abs(ref_lp - lp[b, :e]).max()))
        print(name, "rows", rows, "max log-prob err", worst)
        assert worst <= LOGP_TOL_BF16
        # the same call again, and batch after batch
        again = lib.mtmc_rollout_ragged(handle, dev(prompts), dev(lens), n_samples, max_new, temp, 3, stop_id=3)
        assert np.array_equal(again[0].cpu().numpy(), ids) and np.array_equal(again[1].cpu().numpy(), lp)
        lib.mtmc_set_option(handle, lib.MTMC_OPT_ADMIT_PROMPTS, 0)
        other = lib.mtmc_rollout_ragged(handle, dev(prompts), dev(lens), n_samples, max_new, temp, 3, stop_id=3)
        lib.mtmc_poll_errors(handle)
        same = (other[0].cpu().numpy() == ids).all(axis=1)
        print(name, "rows identical to the batch-after-batch call:", int(same.sum()), "of", same.size)
        assert same.mean() >= 0.6
        assert np.abs(other[1].cpu().numpy()[same] - lp[same]).max() <= 5e-3
    finally:
        lib.mtmc_weights_destroy(handle)


def test_joining_calls_of_different_sizes_share_a_workspace(lib):
    """The step graphs a call replays hold pointers into its workspace that follow from the whole call's shape.  Three
    calls on ONE workspace buffer - 40 prompts (prompts join the running batch), 24 prompts (the same, another page
    layout), 16 prompts (one batch, rows give up their places) - must each give what a fresh handle gives on a buffer
    of its own, bit for bit."""
    import torch
    cfg = STOPPY
    w = inputs.make_weights(cfg, seed=0, std=0.05, gain_std=0.1)
    dev = lambda x: torch.from_numpy(x).cuda()
    ns, max_new, max_len, stop = 8, 40, 33, 3
    shapes = (40, 24, 16)
    prompts = {n: inputs.make_prompts(n, max_len, cfg.vocab, seed=10 + n) for n in shapes}
    lens = {n: (1 + (np.arange(n) * 5) % max_len).astype(np.int32) for n in shapes}

    def run(handle, n, ws):
        out = lib.mtmc_rollout_ragged(handle, dev(prompts[n]), dev(lens[n]), ns, max_new, 1.0, 2, stop_id=stop, workspace=ws)
        lib.mtmc_poll_errors(handle)
        return [x.cpu().numpy() for x in out]

    fresh = {}
    for n in shapes:
        handle = lib.mtmc_weights_create(lib.make_config(cfg, 128), w.blob())
        try:
            lib.mtmc_set_option(handle, lib.MTMC_OPT_STOP_POLL_STEPS, 4)
            fresh[n] = run(handle, n, None)
        finally:
            lib.mtmc_weights_destroy(handle)
    handle = lib.mtmc_weights_create(lib.make_config(cfg, 128), w.blob())
    try:
        lib.mtmc_set_option(handle, lib.MTMC_OPT_STOP_POLL_STEPS, 4)
        nbytes = max(lib.mtmc_rollout_ragged_workspace_bytes(handle, n, max_len, ns, max_new) for n in shapes)
        ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
        for n in shapes + shapes[::-1]:
            got = run(handle, n, ws)
            for a, b in zip(got, fresh[n]):
                assert np.array_equal(a, b), n
    finally:
        lib.mtmc_weights_destroy(handle)
