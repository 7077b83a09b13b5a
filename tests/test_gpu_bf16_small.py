"""GPU parity of the bf16 path on small models (head_dim 128): rollout verified by replay on the
oracle, scoring against the oracle, decode == score consistency, determinism."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

from parity import LOGP_TOL_BF16, check_rollout_by_replay, check_score
from paper_2511_20100_amd import inputs

# (config, std, n_prompts, prompt_len, n_samples, max_new, temperature)
SMALL = inputs.ModelConfig(2, 256, 4, 2, 128, 688, 4096, dtype="bf16")      # G = 2, ragged FFN width
GQA6 = inputs.ModelConfig(2, 384, 6, 1, 128, 1024, 2048, dtype="bf16")      # G = 6 like the 1.5 B policy
GQA7 = inputs.ModelConfig(1, 512, 7, 1, 128, 1536, 2064, dtype="bf16")      # G = 7 like the 7 B policy
MHA = inputs.ModelConfig(2, 256, 2, 2, 128, 512, 2048, dtype="bf16")        # G = 1: every query head has its own kv head
GQA4 = inputs.ModelConfig(1, 512, 4, 1, 128, 1024, 2048, dtype="bf16")
GQA8 = inputs.ModelConfig(1, 1024, 8, 1, 128, 1024, 2048, dtype="bf16")     # the widest group the kernels take
FFN_W6 = inputs.ModelConfig(1, 256, 2, 1, 128, 22016, 2048, dtype="bf16")   # 2752 gate/up row tiles: 12 per workgroup at 65..128 rows
FFN_W8 = inputs.ModelConfig(1, 256, 2, 1, 128, 25600, 2048, dtype="bf16")   # 3200 gate/up row tiles: 16 per workgroup
HD64 = inputs.ModelConfig(2, 256, 4, 2, 64, 688, 4096, dtype="bf16")        # head_dim 64
HD64_TIED = inputs.ModelConfig(2, 512, 8, 2, 64, 1024, 2048, dtype="bf16", tie_embeddings=True)  # G = 4, tied LM head
CASES = [
    ("hd64-b9", HD64, 0.05, 3, 37, 3, 21, 1.0),
    ("hd64-tied-b64", HD64_TIED, 0.05, 8, 50, 8, 24, 1.0),
    ("hd64-long", HD64, 0.05, 1, 200, 2, 40, 1.0),
    ("mha-b12", MHA, 0.05, 4, 37, 3, 24, 1.0),
    ("gqa4-b16", GQA4, 0.05, 2, 40, 8, 16, 1.0),
    ("gqa8-b10", GQA8, 0.04, 5, 33, 2, 18, 1.0),
    ("small-b8", SMALL, 0.02, 4, 32, 2, 32, 1.0),
    ("small-ragged", SMALL, 0.05, 3, 37, 3, 21, 0.8),
    ("gqa6-b24", GQA6, 0.05, 3, 50, 8, 40, 1.0),
    ("gqa7-b64", GQA7, 0.05, 8, 20, 8, 20, 1.0),
    ("gqa6-b40", GQA6, 0.05, 5, 21, 8, 12, 1.0),          # three row tiles: the second workgroup of a row split holds one
    ("gqa4-b100", GQA4, 0.05, 25, 18, 4, 10, 1.0),        # seven row tiles of the 128-row form
    ("gqa6-b128", GQA6, 0.04, 16, 16, 8, 12, 1.0),
    ("ffn-w6-b100", FFN_W6, 0.02, 25, 12, 4, 6, 1.0),     # gate/up workgroups of 6 wavefronts (5 at the 7 B width: test_gpu_7b_shape)
    ("ffn-w8-b128", FFN_W8, 0.02, 16, 12, 8, 6, 1.0),     # ... of 8 wavefronts
    ("gqa6-two-groups", GQA6, 0.04, 18, 9, 8, 6, 1.0),
    ("small-greedy", SMALL, 0.05, 2, 16, 1, 10, 0.0),
    ("small-one-token", SMALL, 0.05, 1, 1, 2, 4, 1.0),
]


@pytest.fixture(scope="module")
def lib():
    from paper_2511_20100_amd import mtmc
    return mtmc


@pytest.mark.parametrize("name,cfg,std,n_prompts,plen,n_samples,max_new,temp", CASES, ids=[c[0] for c in CASES])
def test_rollout_and_score(lib, name, cfg, std, n_prompts, plen, n_samples, max_new, temp):
    w = inputs.make_weights(cfg, seed=0, std=std, gain_std=0.1)
    handle = lib.mtmc_weights_create(lib.make_config(cfg, 256), w.blob())
    try:
        prompts = inputs.make_prompts(n_prompts, plen, cfg.vocab, seed=2)
        rep = check_rollout_by_replay(handle, w, prompts, n_samples, max_new, temp, 1, max_positions=256, label=name)
        print(name, "rollout: compared", rep["compared"], "of", rep["steps"], "max log-prob err", rep["max_logp_err"])
        assert rep["compared"] > 0.5 * rep["steps"]
        seqs = np.concatenate([np.repeat(prompts, n_samples, axis=0), rep["ids"]], axis=1)
        sc = check_score(handle, w, seqs, plen, max_positions=256, label=name)
        print(name, "score: max log-prob err", sc["max_logp_err"], "top-1 compared", sc["compared"], "of", sc["positions"])
        if temp == 1.0:  # the sampled token's log-prob is its Eq. 2 factor
            assert np.abs(sc["logprobs"][:, plen - 1:] - rep["logprobs"]).max() <= LOGP_TOL_BF16
    finally:
        lib.mtmc_weights_destroy(handle)


def test_determinism_and_offsets(lib):
    import torch
    cfg = GQA6
    w = inputs.make_weights(cfg, seed=0, std=0.05, gain_std=0.1)
    handle = lib.mtmc_weights_create(lib.make_config(cfg, 256), w.blob())
    try:
        prompts = torch.from_numpy(inputs.make_prompts(3, 20, cfg.vocab, seed=5)).cuda()
        a = lib.mtmc_rollout(handle, prompts, 4, 12, 1.0, 7)
        b = lib.mtmc_rollout(handle, prompts, 4, 12, 1.0, 7)
        c = lib.mtmc_rollout(handle, prompts, 4, 12, 1.0, 8)
        torch.cuda.synchronize()
        assert torch.equal(a[0], b[0]) and torch.equal(a[1], b[1])
        assert not torch.equal(a[0], c[0])
        s1 = lib.mtmc_score(handle, torch.cat([prompts.repeat_interleave(4, 0), a[0]], 1).contiguous(), 20)
        s2 = lib.mtmc_score(handle, torch.cat([prompts.repeat_interleave(4, 0), a[0]], 1).contiguous(), 20)
        torch.cuda.synchronize()
        assert torch.equal(s1, s2)
    finally:
        lib.mtmc_weights_destroy(handle)


def test_score_long_sequences_and_chunks(lib):
    """Sequences longer than one attention block, several sequences per chunk and several chunks."""
    cfg = GQA6
    w = inputs.make_weights(cfg, seed=3, std=0.05, gain_std=0.1)
    handle = lib.mtmc_weights_create(lib.make_config(cfg, 4096), w.blob())
    try:
        seqs = inputs.make_sequences(40, 333, cfg.vocab, seed=9)     # 40 x 333 tokens: 2 chunks of 24 + 16
        sc = check_score(handle, w, seqs, 100, max_positions=4096, rows=[0, 23, 24, 39], label="long")
        print("long score: max log-prob err", sc["max_logp_err"])
        seqs = inputs.make_sequences(2, 1500, cfg.vocab, seed=10)
        sc = check_score(handle, w, seqs, 1400, max_positions=4096, rows=[1], label="very-long")
        print("very long score: max log-prob err", sc["max_logp_err"])
    finally:
        lib.mtmc_weights_destroy(handle)


def test_graph_replay_matches_direct_launches(lib):
    """Decode steps replayed from a captured HIP graph give bit-identical results to direct
    launches, on every replay, with other work and synchronisations in between."""
    import torch
    cfg = GQA6
    w = inputs.make_weights(cfg, seed=0, std=0.05, gain_std=0.1)
    handle = lib.mtmc_weights_create(lib.make_config(cfg, 256), w.blob())
    try:
        prompts = torch.from_numpy(inputs.make_prompts(4, 19, cfg.vocab, seed=5)).cuda()
        ws = torch.empty(lib.mtmc_rollout_workspace_bytes(handle, 4, 19, 4, 24), dtype=torch.uint8, device="cuda")
        lib.mtmc_set_option(handle, lib.MTMC_OPT_HIP_GRAPH, 0)
        ref = [t.clone() for t in lib.mtmc_rollout(handle, prompts, 4, 24, 1.0, 11, workspace=ws)]
        torch.cuda.synchronize()
        lib.mtmc_set_option(handle, lib.MTMC_OPT_HIP_GRAPH, 1)
        for rep in range(3):
            got = lib.mtmc_rollout(handle, prompts, 4, 24, 1.0, 11, workspace=ws)
            torch.cuda.synchronize()
            assert torch.equal(got[0], ref[0]) and torch.equal(got[1], ref[1]), rep
            other = lib.mtmc_rollout(handle, prompts, 4, 24, 0.7, 12 + rep, workspace=ws)  # same graph, new parameters
            torch.cuda.synchronize()
            assert not torch.equal(other[0], ref[0])
    finally:
        lib.mtmc_weights_destroy(handle)


def test_calls_overlapping_on_two_streams_match_calls_in_turn(lib):
    """Two rollouts and a scoring pass on one weights handle, each with its own workspace and
    stream, give bit for bit what the same calls give one after the other."""
    import torch
    cfg = GQA6
    w = inputs.make_weights(cfg, seed=0, std=0.05, gain_std=0.1)
    handle = lib.mtmc_weights_create(lib.make_config(cfg, 256), w.blob())
    try:
        halves = [torch.from_numpy(inputs.make_prompts(3, 21, cfg.vocab, seed=5 + i)).cuda() for i in range(2)]
        seqs = torch.from_numpy(inputs.make_sequences(6, 60, cfg.vocab, seed=9)).cuda()
        wss = [torch.empty(lib.mtmc_rollout_workspace_bytes(handle, 3, 21, 4, 40), dtype=torch.uint8, device="cuda")
               for _ in range(2)]
        ws_sc = torch.empty(lib.mtmc_score_workspace_bytes(handle, 6, 60), dtype=torch.uint8, device="cuda")

        def run(streams):
            out = [lib.mtmc_rollout(handle, halves[i], 4, 40, 1.0, 3, seq_offset=12 * i, workspace=wss[i],
                                    stream=streams[i]) for i in range(2)]
            sc = lib.mtmc_score(handle, seqs, 20, workspace=ws_sc, stream=streams[2])
            torch.cuda.synchronize()
            return [t.clone() for pair in out for t in pair] + [sc.clone()]

        ref = run([None, None, None])
        streams = [torch.cuda.Stream() for _ in range(3)]
        torch.cuda.synchronize()
        for rep in range(3):
            got = run(streams)
            for a, b in zip(got, ref):
                assert torch.equal(a, b), rep
    finally:
        lib.mtmc_weights_destroy(handle)


def test_at_64_rows_the_first_tokens_do_not_depend_on_max_new(lib):
    """At 33..64 rows the decode attention splits a sequence's context at the end of its prompt, a boundary that
    depends on the sequence alone: once contexts are long enough to be split at all (more than 8 pages), a longer
    generation budget (more pages per sequence) leaves the arithmetic of the first steps unchanged, bit for bit."""
    import torch
    cfg = GQA6
    w = inputs.make_weights(cfg, seed=0, std=0.05, gain_std=0.1)
    handle = lib.mtmc_weights_create(lib.make_config(cfg, 256), w.blob())
    try:
        prompts = torch.from_numpy(inputs.make_prompts(8, 150, cfg.vocab, seed=5)).cuda()  # > 8 pages: split in both calls
        short = lib.mtmc_rollout(handle, prompts, 8, 8, 1.0, 3)
        long_ = lib.mtmc_rollout(handle, prompts, 8, 90, 1.0, 3)
        torch.cuda.synchronize()
        assert torch.equal(short[0], long_[0][:, :8]) and torch.equal(short[1], long_[1][:, :8])
    finally:
        lib.mtmc_weights_destroy(handle)


def test_kernel_timer_does_not_change_results(lib):
    import torch
    cfg = GQA6
    w = inputs.make_weights(cfg, seed=0, std=0.05, gain_std=0.1)
    handle = lib.mtmc_weights_create(lib.make_config(cfg, 256), w.blob())
    try:
        prompts = torch.from_numpy(inputs.make_prompts(2, 17, cfg.vocab, seed=5)).cuda()
        ref = [t.clone() for t in lib.mtmc_rollout(handle, prompts, 4, 20, 1.0, 3)]
        lib.mtmc_kernel_timer(handle, lib.MTMC_KERNEL_GATE_UP, 4)
        got = lib.mtmc_rollout(handle, prompts, 4, 20, 1.0, 3)
        ms, n, empty_ms = lib.mtmc_kernel_timer_read(handle)
        lib.mtmc_kernel_timer(handle, 0, 0)
        assert torch.equal(got[0], ref[0]) and torch.equal(got[1], ref[1])
        assert n == 5 * cfg.n_layers and ms > 0 and 0 <= empty_ms < ms / n      # steps 1, 5, 9, 13, 17 of 19 decode steps
    finally:
        lib.mtmc_weights_destroy(handle)


@pytest.mark.parametrize("cfg,n_seqs,seq_len", [(SMALL, 7, 211), (GQA6, 9, 300)], ids=["small-ragged", "gqa6"])
def test_lds_staged_gemm_on_ragged_shapes(lib, cfg, n_seqs, seq_len):
    """The 256 x 256 LDS-staged GEMM forced onto small problems: token counts (1477, 2700) and
    feature counts (256 ... 2 x 688) that are not multiples of its block, against the oracle and
    against the direct kernel; then the same for the prompt pass of a rollout."""
    import torch
    w = inputs.make_weights(cfg, seed=4, std=0.05, gain_std=0.1)
    handle = lib.mtmc_weights_create(lib.make_config(cfg, 512), w.blob())
    try:
        seqs = inputs.make_sequences(n_seqs, seq_len, cfg.vocab, seed=11)
        direct = lib.mtmc_score(handle, torch.from_numpy(seqs).cuda(), 50).cpu().numpy()
        lib.mtmc_set_option(handle, lib.MTMC_OPT_GEMM_LDS_MIN_BLOCKS, 1)
        sc = check_score(handle, w, seqs, 50, max_positions=512, rows=[0, n_seqs - 1], label="lds")
        print("lds-staged score: max log-prob err", sc["max_logp_err"],
              "max difference from the direct kernel", np.abs(sc["logprobs"] - direct).max())
        assert np.abs(sc["logprobs"] - direct).max() <= 3e-3   # two kernels, each rounding activations to fp16 its own way
        prompts = inputs.make_prompts(3, 130, cfg.vocab, seed=2)
        rep = check_rollout_by_replay(handle, w, prompts, 2, 6, 1.0, 1, max_positions=512, label="lds-prefill")
        assert rep["compared"] > 0.5 * rep["steps"]
    finally:
        lib.mtmc_weights_destroy(handle)


def test_long_context_over_several_attention_chunks(lib):
    """Context beyond 8192 tokens (more than the 512 pages one decode-attention workgroup stages):
    the context is then split over workgroups whose partial results the O projection combines.
    Prompt 8200 + 24 new tokens, small model, both samples replayed on the oracle."""
    cfg = GQA6
    w = inputs.make_weights(cfg, seed=6, std=0.05, gain_std=0.1)
    handle = lib.mtmc_weights_create(lib.make_config(cfg, 8256), w.blob())
    try:
        prompts = inputs.make_prompts(1, 8200, cfg.vocab, seed=8)
        rep = check_rollout_by_replay(handle, w, prompts, 2, 24, 1.0, 5, max_positions=8256, label="long-context")
        print("long context: compared", rep["compared"], "of", rep["steps"], "max log-prob err", rep["max_logp_err"])
        assert rep["compared"] > 0.5 * rep["steps"]
    finally:
        lib.mtmc_weights_destroy(handle)


def test_long_context_at_more_than_64_rows(lib):
    """72 sequences (five row tiles: the 128-row form of the decode GEMMs) with a context beyond 8192
    tokens, so that the O projection of that form has to combine two context chunks.  One prompt
    of 8200 tokens with 72 samples; three of them are replayed on the oracle."""
    cfg = GQA4
    w = inputs.make_weights(cfg, seed=6, std=0.05, gain_std=0.1)
    handle = lib.mtmc_weights_create(lib.make_config(cfg, 8256), w.blob())
    try:
        prompts = inputs.make_prompts(1, 8200, cfg.vocab, seed=8)
        rep = check_rollout_by_replay(handle, w, prompts, 72, 20, 1.0, 5, max_positions=8256, rows=[0, 37, 71],
                                      label="long-context-72")
        print("long context, 72 rows: compared", rep["compared"], "of", rep["steps"], "max log-prob err", rep["max_logp_err"])
        assert rep["compared"] > 0.5 * rep["steps"]
    finally:
        lib.mtmc_weights_destroy(handle)


def test_context_limit_is_enforced(lib):
    import torch
    cfg = GQA4
    w = inputs.make_weights(cfg, seed=6, std=0.05, gain_std=0.1)
    handle = lib.mtmc_weights_create(lib.make_config(cfg, 40000), w.blob())
    try:
        with pytest.raises(lib.MtmcError) as e:
            lib.mtmc_rollout_workspace_bytes(handle, 1, lib.MTMC_MAX_DECODE_CONTEXT - 7, 2, 8)
        assert e.value.code == lib.MTMC_EINVAL and "MTMC_MAX_DECODE_CONTEXT" in str(e.value)
        assert lib.mtmc_rollout_workspace_bytes(handle, 1, lib.MTMC_MAX_DECODE_CONTEXT - 8, 2, 8) > 0
    finally:
        lib.mtmc_weights_destroy(handle)


def test_degenerate_sizes(lib):
    """Nothing to score (prompt_len == seq_len), the shortest scorable sequence, a single new token, and
    a call split over two processes' worth of prompts (seq_offset) that must reproduce the whole call."""
    import torch
    cfg = SMALL
    w = inputs.make_weights(cfg, seed=1, std=0.05, gain_std=0.1)
    handle = lib.mtmc_weights_create(lib.make_config(cfg, 128), w.blob())
    try:
        seqs = torch.from_numpy(inputs.make_sequences(3, 20, cfg.vocab, seed=4)).cuda()
        s = lib.mtmc_score(handle, seqs, 20)
        assert s.shape == (3, 19) and torch.all(s == 0)
        two = inputs.make_sequences(5, 2, cfg.vocab, seed=6)
        sc = check_score(handle, w, two, 1, max_positions=128, label="two-token")
        assert sc["logprobs"].shape == (5, 1)
        prompts = inputs.make_prompts(4, 9, cfg.vocab, seed=3)
        rep = check_rollout_by_replay(handle, w, prompts, 3, 1, 1.0, 2, max_positions=128, label="one-new-token")
        assert rep["ids"].shape == (12, 1)
        dp = torch.from_numpy(prompts).cuda()
        whole = lib.mtmc_rollout(handle, dp, 3, 7, 1.0, 11)
        first = lib.mtmc_rollout(handle, dp[:1].contiguous(), 3, 7, 1.0, 11)
        rest = lib.mtmc_rollout(handle, dp[1:].contiguous(), 3, 7, 1.0, 11, seq_offset=3)
        assert torch.equal(whole[0], torch.cat([first[0], rest[0]]))
        assert (whole[1] - torch.cat([first[1], rest[1]])).abs().max() <= 1e-3   # batch size changes the tiling
    finally:
        lib.mtmc_weights_destroy(handle)


def test_bad_inputs_are_reported(lib):
    """A token id outside the vocabulary raises the sticky data flag; a weight beyond the fp16 range is refused."""
    import torch
    cfg = SMALL
    w = inputs.make_weights(cfg, seed=1, std=0.05, gain_std=0.1)
    handle = lib.mtmc_weights_create(lib.make_config(cfg, 128), w.blob())
    try:
        prompts = torch.from_numpy(inputs.make_prompts(2, 8, cfg.vocab, seed=5)).cuda()
        bad = prompts.clone(); bad[1, 3] = cfg.vocab
        lib.mtmc_rollout(handle, bad, 2, 3, 1.0, 1)
        with pytest.raises(lib.MtmcError) as e:
            lib.mtmc_poll_errors(handle)
        assert e.value.code == lib.MTMC_EDATA
        lib.mtmc_poll_errors(handle)
        seqs = torch.cat([prompts, prompts], 1).contiguous(); seqs[0, 10] = -1
        lib.mtmc_score(handle, seqs, 4)
        with pytest.raises(lib.MtmcError):
            lib.mtmc_poll_errors(handle)
    finally:
        lib.mtmc_weights_destroy(handle)
    blob = w.blob().copy()
    lay, _ = inputs.blob_layout(cfg)
    off = lay["layers.1.wq"][0]
    blob.view(np.uint16)[off // 2 + 5] = 0x7F00   # bf16 1.7e38: not an fp16 value
    with pytest.raises(lib.MtmcError) as e:
        lib.mtmc_weights_create(lib.make_config(cfg, 128), blob)
    assert e.value.code == lib.MTMC_EINVAL


def test_graph_of_a_tail_group_is_not_reused_by_a_call_of_its_shape(lib):
    """A call of 20 prompts x 8 samples runs as groups of 128 + 32 rows; the 32-row group's captured step holds
    pointers laid out by the 160-row plan.  A later call of 4 x 8 on the SAME workspace has its own plan: it must
    not replay that graph.  Its results equal a fresh handle's (no cached graphs) bit for bit."""
    import torch
    cfg = GQA6
    w = inputs.make_weights(cfg, seed=0, std=0.05, gain_std=0.1)
    plen, n_new = 18, 9
    prompts = torch.from_numpy(inputs.make_prompts(20, plen, cfg.vocab, seed=5)).cuda()
    tail = prompts[16:].contiguous()
    handle = lib.mtmc_weights_create(lib.make_config(cfg, 64), w.blob())
    try:
        ws = torch.empty(lib.mtmc_rollout_workspace_bytes(handle, 20, plen, 8, n_new), dtype=torch.uint8, device="cuda")
        assert ws.numel() >= lib.mtmc_rollout_workspace_bytes(handle, 4, plen, 8, n_new)
        big = lib.mtmc_rollout(handle, prompts, 8, n_new, 1.0, 3, workspace=ws)
        small = lib.mtmc_rollout(handle, tail, 8, n_new, 1.0, 3, seq_offset=128, workspace=ws)
        again = lib.mtmc_rollout(handle, prompts, 8, n_new, 1.0, 3, workspace=ws)
        lib.mtmc_poll_errors(handle)
        big, small, again = [[t.cpu() for t in r] for r in (big, small, again)]
    finally:
        lib.mtmc_weights_destroy(handle)
    fresh = lib.mtmc_weights_create(lib.make_config(cfg, 64), w.blob())
    try:
        ref = lib.mtmc_rollout(fresh, tail, 8, n_new, 1.0, 3, seq_offset=128)
        lib.mtmc_poll_errors(fresh)
        ref = [t.cpu() for t in ref]
    finally:
        lib.mtmc_weights_destroy(fresh)
    assert torch.equal(small[0], ref[0]) and torch.equal(small[1], ref[1])
    assert torch.equal(big[0], again[0]) and torch.equal(big[1], again[1])
    # the same sequences inside the 160-row call: same noise, same ids (the 32-row group runs the same tiling)
    assert torch.equal(big[0][128:], small[0])


def test_values_beyond_the_fp16_range_are_reported(lib):
    """The matrix products take fp16 operands.  A model whose value projection produces magnitudes beyond 65504
    has them clamped in the KV cache: both the scoring pass and the rollout must raise the sticky data flag, and
    the message must name the cause; the unscaled model raises nothing."""
    import torch
    cfg = SMALL
    w = inputs.make_weights(cfg, seed=1, std=0.05, gain_std=0.1)
    seqs = torch.from_numpy(inputs.make_sequences(2, 24, cfg.vocab, seed=4)).cuda()
    handle = lib.mtmc_weights_create(lib.make_config(cfg, 128), w.blob())
    try:
        lib.mtmc_score(handle, seqs, 8)
        lib.mtmc_rollout(handle, seqs[:, :8].contiguous(), 2, 4, 1.0, 1)
        lib.mtmc_poll_errors(handle)   # clean
    finally:
        lib.mtmc_weights_destroy(handle)
    # one row of Wv of the second block scaled to 2e4 per entry (a legal fp16 weight): |v| ~ 2e4 * |x|_1 >> 65504
    big = inputs.bf16_bits_to_f32(w.tensors["layers.1.wv"]).copy()
    big[5, :] = 2.0e4
    w.tensors["layers.1.wv"] = inputs.f32_to_bf16_bits(big)
    w.drop_cache()
    handle = lib.mtmc_weights_create(lib.make_config(cfg, 128), w.blob())
    try:
        lib.mtmc_score(handle, seqs, 8)
        with pytest.raises(lib.MtmcError) as e:
            lib.mtmc_poll_errors(handle)
        assert e.value.code == lib.MTMC_EDATA and "fp16 range" in str(e.value) and "token id" not in str(e.value)
        lib.mtmc_poll_errors(handle)   # the flag was cleared by the poll
        lib.mtmc_rollout(handle, seqs[:, :8].contiguous(), 2, 4, 1.0, 1)
        with pytest.raises(lib.MtmcError) as e:
            lib.mtmc_poll_errors(handle)
        assert e.value.code == lib.MTMC_EDATA and "fp16 range" in str(e.value)
    finally:
        lib.mtmc_weights_destroy(handle)
    # the same for a SwiGLU product: one row of W_up and of W_gate at 2e4 per entry, so that silu(g) u of that feature
    # leaves the range for every token whose x has a positive sum (and some do); the scoring pass is run on each of
    # its two GEMM kernels (the LDS-staged one collects the test per output block and raises the flag once)
    w = inputs.make_weights(cfg, seed=1, std=0.05, gain_std=0.1)
    for name in ("layers.0.wup", "layers.0.wgate"):
        big = inputs.bf16_bits_to_f32(w.tensors[name]).copy()
        big[7, :] = 2.0e4
        w.tensors[name] = inputs.f32_to_bf16_bits(big)
    w.drop_cache()
    handle = lib.mtmc_weights_create(lib.make_config(cfg, 128), w.blob())
    try:
        for min_blocks in (1, 1 << 20):
            lib.mtmc_set_option(handle, lib.MTMC_OPT_GEMM_LDS_MIN_BLOCKS, min_blocks)
            lib.mtmc_score(handle, seqs, 8)
            with pytest.raises(lib.MtmcError) as e:
                lib.mtmc_poll_errors(handle)
            assert e.value.code == lib.MTMC_EDATA and "fp16 range" in str(e.value), min_blocks
    finally:
        lib.mtmc_weights_destroy(handle)


def test_lds_gemm_at_its_shortest_reduction(lib):
    """The LDS-staged GEMM streams k-steps through a ring of four buffers and needs at least four of them:
    d_model = d_ffn = n_q_heads * head_dim = 128 gives every matrix product of the scoring pass (QKV, O,
    gate/up, down, LM head) exactly four k-steps, the shortest pipeline there is, with several output blocks
    per workgroup so that the stream crosses block boundaries with the ring never more than one block deep."""
    cfg = inputs.ModelConfig(2, 128, 1, 1, 128, 128, 4096, dtype="bf16")
    w = inputs.make_weights(cfg, seed=2, std=0.08, gain_std=0.1)
    handle = lib.mtmc_weights_create(lib.make_config(cfg, 512), w.blob())
    try:
        lib.mtmc_set_option(handle, lib.MTMC_OPT_GEMM_LDS_MIN_BLOCKS, 1)
        seqs = inputs.make_sequences(5, 300, cfg.vocab, seed=8)      # 1500 tokens: 6 row blocks, ragged tail
        sc = check_score(handle, w, seqs, 200, max_positions=512, rows=[0, 4], label="k4-lds")
        print("LDS GEMM with four k-steps: max log-prob err", sc["max_logp_err"], "top-1 compared", sc["compared"])
        lib.mtmc_set_option(handle, lib.MTMC_OPT_GEMM_LDS_MIN_BLOCKS, 1 << 20)   # the direct kernel on the same data
        import torch
        a = lib.mtmc_score(handle, torch.from_numpy(seqs).cuda(), 200)
        assert (a.cpu().numpy() - sc["logprobs"]).__abs__().max() <= 1e-3
    finally:
        lib.mtmc_weights_destroy(handle)


@pytest.mark.parametrize("n_seqs,S", [(2, 448), (3, 300), (7, 256), (8, 256), (9, 250), (17, 256), (33, 264)],
                         ids=lambda v: str(v))
def test_prefill_gemms_cover_every_block_at_any_number_of_token_blocks(lib, n_seqs, S):
    """The prefill / scoring GEMMs hand their output blocks to the 8 XCDs by token block, or by feature block when
    there are fewer than 8 token blocks, and the LDS-staged kernel's workgroups walk the blocks of their XCD band by
    band (the last band is lower).  Token-block counts on both sides of 8, with full and partial bands, in both
    kernels: one sequence against the oracle, and the two kernels against each other on every position (a block that
    nobody computes leaves stale values)."""
    import torch
    cfg = inputs.ModelConfig(2, 256, 2, 1, 128, 1024, 4096, dtype="bf16")   # 8 gate/up blocks of 256, 2 QKV, 1 O / down
    w = inputs.make_weights(cfg, seed=3, std=0.06, gain_std=0.1)
    handle = lib.mtmc_weights_create(lib.make_config(cfg, 512), w.blob())
    try:
        seqs = inputs.make_sequences(n_seqs, S, cfg.vocab, seed=9)
        first = S - 40
        lib.mtmc_set_option(handle, lib.MTMC_OPT_GEMM_LDS_MIN_BLOCKS, 1)
        sc = check_score(handle, w, seqs, first, max_positions=512, rows=[n_seqs - 1], label=f"lds-{n_seqs}x{S}")
        lib.mtmc_set_option(handle, lib.MTMC_OPT_GEMM_LDS_MIN_BLOCKS, 1 << 20)
        direct = check_score(handle, w, seqs, first, max_positions=512, rows=[0], label=f"direct-{n_seqs}x{S}")
        d = np.abs(direct["logprobs"] - sc["logprobs"]).max()
        print(f"{n_seqs} x {S}: LDS err {sc['max_logp_err']:.2e}, direct err {direct['max_logp_err']:.2e}, LDS vs direct {d:.2e}")
        assert d <= 3e-3   # two matrix instructions, two rounding orders; a missing block would be off by units
    finally:
        lib.mtmc_weights_destroy(handle)


@pytest.mark.parametrize("n_prompts", [1, 4])
def test_prefill_of_a_few_prompts_at_the_1p5b_widths(lib, n_prompts):
    """One and four prompts of 512 tokens at the layer widths of the 1.5 B-class policy (2 of its 28 blocks): the
    sizes at which the QKV, O and down projections of the prefill are 12-64 output blocks and run over several ranges
    of K at once, the partial sums added in a fixed order.  Rollout by replay on the oracle, the same call twice (the
    order of the sums does not depend on the schedule), and the scoring pass on the same sequences."""
    import torch
    from parity import check_rollout_by_replay
    cfg = inputs.POLICY_1P5B.with_(n_layers=2)
    w = inputs.make_weights(cfg, seed=0)
    handle = lib.mtmc_weights_create(lib.make_config(cfg, 640), w.blob())
    try:
        prompts = inputs.make_prompts(n_prompts, 512, cfg.vocab, seed=4)
        rows = sorted({0, n_prompts * 8 - 1})
        rep = check_rollout_by_replay(handle, w, prompts, 8, 6, 1.0, 1, max_positions=640, rows=rows, label=f"1p5b-{n_prompts}x512")
        print(f"{n_prompts} x 512: compared", rep["compared"], "of", rep["steps"], "max log-prob err", rep["max_logp_err"])
        again = lib.mtmc_rollout(handle, torch.from_numpy(prompts).cuda(), 8, 6, 1.0, 1)
        assert np.array_equal(again[0].cpu().numpy(), rep["ids"]) and np.array_equal(again[1].cpu().numpy(), rep["logprobs"])
        seqs = np.concatenate([np.repeat(prompts, 8, axis=0), rep["ids"]], axis=1)
        sc = check_score(handle, w, seqs, 512, max_positions=640, rows=rows[:1], label=f"1p5b-{n_prompts}x512-score")
        assert np.abs(sc["logprobs"][:, 511:] - rep["logprobs"]).max() <= 2 * LOGP_TOL_BF16
    finally:
        lib.mtmc_weights_destroy(handle)
