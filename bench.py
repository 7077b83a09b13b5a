#!/usr/bin/env python3
"""Throughput of the policy rollout + scoring path on one MI355X.

One step = one pass of the whole path over one batch: mtmc_rollout (prefill of the prompts, then
max_new Gumbel-max decode steps for every sequence) followed by mtmc_score of the sequences it
produced.  The headline value is generated tokens per second over the whole step (scored tokens
per second when the step is the scoring pass alone); inputs (weights, prompts) are resident in HBM
before the timed region.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload 1p5b|tiny|7b|...] [--no-cpu-baseline]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

from paper_2511_20100_amd import inputs  # noqa: E402

HBM_PEAK_GBS = 8000.0       # MI355X published HBM3E bandwidth
MFMA_PEAK_TFLOPS = 2500.0   # MI355X published dense 16-bit MFMA rate
# Counter summary of a workload: holds the HBM bytes one launch of its gate/up decode kernel moves
# (FETCH_SIZE / WRITE_SIZE runs scaled by the library's copy kernel), with the hash of the kernel sources the
# counters were taken on: `traffic` is reported only while those sources are unchanged.
TRAFFIC_PROFILE = os.path.join(ROOT, "profiles", "decode_kernels_{workload}_hbm_counters.txt")
DECODE_KERNEL_SOURCES = ("decode_bf16.hip", "decode_rows128.hip", "decode_lmhead.hip", "frag.h", "bf16_kernels.h", "attention_core.h",
                         "device_utils.h")


def decode_sources_hash() -> str:
    import hashlib
    h = hashlib.sha256()
    for name in DECODE_KERNEL_SOURCES:
        with open(os.path.join(ROOT, "paper_2511_20100_amd", "csrc", name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]


def gate_up_traffic_from_profile(workload):
    """Bytes per launch from the workload's committed counter summary, or None when the summary is missing, has
    no machine-readable line, or was taken on other kernel sources than the ones in the tree."""
    import re
    try:
        text = open(TRAFFIC_PROFILE.format(workload=workload)).read()
    except OSError:
        return None
    m = re.search(r"^gate_up_traffic_bytes_per_launch:\s*([0-9.]+)\s+decode_sources_sha256_16:\s*([0-9a-f]{16})", text, re.M)
    if not m or m.group(2) != decode_sources_hash():
        return None
    return float(m.group(1))

WORKLOADS = {
    # name: (config, n_prompts, prompt_len, n_samples, max_new)
    "tiny": (inputs.TINY, 4, 32, 2, 32),
    "1p5b": (inputs.POLICY_1P5B, 8, 512, 8, 1024),
    "7b": (inputs.POLICY_7B, 16, 1024, 8, 2048),
    "7b-long": (inputs.POLICY_7B, 4, 2048, 8, 8192),       # long generations: context up to 10240 tokens
    "7b-score": (inputs.POLICY_7B, 32, 1024, 8, 2048),     # scoring alone: 256 sequences of 3072 tokens
    "1p3b-mha": (inputs.POLICY_1P3B_MHA, 8, 512, 8, 1024),
    "1b-hd64": (inputs.POLICY_1B_HD64, 8, 512, 8, 1024),
}


def decode_bytes_per_step(cfg, n_prompts, prompt_len, n_samples, max_new):
    """Algorithmic HBM bytes of one average decode step: every weight matrix once (2 bytes per
    parameter, embedding table excluded) plus the KV cache of the context, with the pages of a
    prompt read once for all its samples."""
    hd = cfg.head_dim
    q, kv = cfg.n_q_heads * hd, cfg.n_kv_heads * hd
    layer = cfg.d_model * (q + 2 * kv) + q * cfg.d_model + 3 * cfg.d_model * cfg.d_ffn
    weights = 2 * (cfg.n_layers * layer + cfg.vocab * cfg.d_model)
    kv_per_token = cfg.n_layers * 2 * kv * 2
    B = n_prompts * n_samples
    avg_new = (max_new - 1) / 2.0
    kv_bytes = (n_prompts * prompt_len + B * avg_new) * kv_per_token
    return weights + kv_bytes, weights, kv_bytes


def forward_flops(cfg, n_seqs, seq_len, scored_per_seq):
    hd = cfg.head_dim
    q, kv = cfg.n_q_heads * hd, cfg.n_kv_heads * hd
    layer = cfg.d_model * (q + 2 * kv) + q * cfg.d_model + 3 * cfg.d_model * cfg.d_ffn
    gemm = 2.0 * cfg.n_layers * layer * n_seqs * seq_len
    attn = 2.0 * seq_len * seq_len * q * cfg.n_layers * n_seqs      # causal: half of 4 S^2 q
    head = 2.0 * cfg.d_model * cfg.vocab * n_seqs * scored_per_seq
    return gemm + attn + head


def cpu_baseline(weights, cfg, prompts, max_positions, score_only=False):
    """The oracle as it stands, timed on the host cores on a bounded sample of the workload: at the 1.5 B class
    one whole prompt, at the 7 B class (14 GFLOP per token) one prompt truncated to 192 tokens.  The first use of
    a bf16 tensor widens it to fp32 (an exact conversion, kept for the later tokens): that is part of the time."""
    sys.path.insert(0, os.path.join(ROOT, "oracle"))
    import mtmc_oracle as oracle
    model = oracle.Model(n_layers=cfg.n_layers, d_model=cfg.d_model, n_q_heads=cfg.n_q_heads,
                         n_kv_heads=cfg.n_kv_heads, head_dim=cfg.head_dim, d_ffn=cfg.d_ffn, vocab=cfg.vocab,
                         rms_eps=cfg.rms_eps, rope_base=cfg.rope_base, w=weights.f32, max_positions=max_positions)
    big = cfg.n_layers * cfg.d_model > 60000          # 7 B class
    if big:
        n_p, n_s, n_new, plen = 1, 1, 8, 192
    elif cfg.n_layers * cfg.d_model > 10000:
        n_p, n_s, n_new, plen = 1, 2, 128, prompts.shape[1]
    else:
        n_p, n_s, n_new, plen = prompts.shape[0], 2, 32, prompts.shape[1]
    sample_prompts = prompts[:n_p, :plen]
    t0 = time.perf_counter()
    if score_only:
        seqs = np.concatenate([sample_prompts, prompts[:n_p, plen:plen + 64]], axis=1)
        oracle.score(model, seqs, prompt_len=plen)
        dt = time.perf_counter() - t0
        n_tok, what = seqs.size, (f"scoring of {n_p} sequence of {seqs.shape[1]} tokens (the first {plen} as prompt: "
                                  f"{seqs.shape[1] - plen} scored)")
    else:
        ids, _, _ = oracle.rollout(model, sample_prompts, n_s, n_new, 1.0, seed=1)
        seqs = np.concatenate([np.repeat(sample_prompts, n_s, axis=0), ids], axis=1)[:1]
        oracle.score(model, seqs, prompt_len=plen)
        dt = time.perf_counter() - t0
        n_tok, what = n_p * n_s * n_new, (f"{n_p} prompt(s) of {plen} tokens x {n_s} samples x {n_new} new tokens "
                                          f"(cached decode), then scoring of 1 resulting sequence")
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    return {"value": n_tok / dt, "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
            "sample": f"{what}; {dt:.1f} s; subset, not extrapolated"}


def attainable_rates(torch, mtmc, dev):
    """What this GPU sustains, measured here: a plain streaming read of 2 GiB (GB/s) and a register-only loop of
    fp16 32x32x16 matrix instructions on every SIMD, with the register tile of the scoring GEMM and pseudo-random
    operands (TFLOP/s)."""
    stream = torch.cuda.current_stream()
    buf = torch.ones(2 << 30, dtype=torch.uint8, device=dev)
    sink = torch.zeros(1, dtype=torch.int32, device=dev)
    e = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    mtmc.mtmc_read_probe(buf, sink)
    e[0].record(stream)
    for _ in range(4):
        mtmc.mtmc_read_probe(buf, sink)
    e[1].record(stream)
    e[1].synchronize()
    read_gbs = 4 * buf.numel() / (e[0].elapsed_time(e[1]) * 1e-3) / 1e9
    del buf
    out = torch.empty(1024 * 256, dtype=torch.float32, device=dev)
    mtmc.mtmc_mfma_probe(out, 1024, 500)
    e[0].record(stream)
    flops = mtmc.mtmc_mfma_probe(out, 1024, 5000)
    e[1].record(stream)
    e[1].synchronize()
    return read_gbs, flops / (e[0].elapsed_time(e[1]) * 1e-3) / 1e12


def inference_legs(torch, mtmc, dev, handle, weights, cfg, prompts, n_samples, max_new, progress):
    """Beside the step, not part of `value`: what the policy's use at inference time costs (prompts that end at a
    terminal token, and a state that extends the previous step's).
    stop token: the same batch with one token made likely (its LM-head row scaled by 8: with the synthetic,
    nearly uniform policy no token would ever come up), so that rows end after tens of steps; the call that looks
    at the stop flags (rows give up their places, the call ends with the last row) against the one that does not.
    prompts join a running batch: 1024 sequences with the same stop token in one call, which takes its prompts in as
    sequences finish, against the same call run batch after batch.
    cached prefix: 32 new tokens on the same prompts, evaluating them whole against keeping all but their last
    64 positions from the previous call."""
    stream = torch.cuda.current_stream()
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    n_prompts, prompt_len = prompts.shape
    lens = torch.full((n_prompts,), prompt_len, dtype=torch.int32, device=dev)

    def timed(fn):
        fn()
        torch.cuda.synchronize()
        ev[0].record(stream)
        out = fn()
        ev[1].record(stream)
        ev[1].synchronize()
        return out, ev[0].elapsed_time(ev[1])

    out = {}
    # a long state (as much as the handle's positions allow) and a short action
    short_new = 32
    long_len = (prompt_len + max_new - short_new) // 32 * 32
    keep = long_len - 64
    if keep > 0:
        long_prompts = torch.from_numpy(inputs.make_prompts(n_prompts, long_len, cfg.vocab, seed=6)).to(dev)
        long_lens = torch.full((n_prompts,), long_len, dtype=torch.int32, device=dev)
        ws = torch.empty(mtmc.mtmc_rollout_ragged_workspace_bytes(handle, n_prompts, long_len, n_samples, short_new),
                         dtype=torch.uint8, device=dev)
        whole, ms_whole = timed(lambda: mtmc.mtmc_rollout_ragged(handle, long_prompts, long_lens, n_samples, short_new,
                                                                 1.0, 1, workspace=ws))
        kept, ms_kept = timed(lambda: mtmc.mtmc_rollout_ragged_cached(handle, long_prompts, long_lens, n_samples,
                                                                      short_new, 1.0, 1, keep, ws))
        mtmc.mtmc_poll_errors(handle)
        same_ids = (whole[0] == kept[0]).all(dim=1)
        out["cached_prefix"] = {"workload": f"{n_prompts} prompts of {long_len} tokens x {n_samples} samples, {short_new} "
                                            f"new tokens; {keep} positions of every prompt kept from the previous call",
                                "ms_whole_prompts": ms_whole, "ms_cached_prefix": ms_kept,
                                "rows_with_the_same_ids": int(same_ids.sum().item()), "rows": int(same_ids.numel()),
                                "max_logprob_difference_on_those_rows":
                                    float((whole[1][same_ids] - kept[1][same_ids]).abs().max().item()) if same_ids.any() else None,
                                "note": "512 tokens and 12 032 tokens run different matrix kernels for the O and down "
                                        "projections (same sums, another rounding order): the two calls agree to that "
                                        "rounding, not bit for bit"}
        progress(f"cached prefix: {ms_kept:.1f} ms against {ms_whole:.1f} ms")
        del ws, long_prompts
    stop = 7
    saved = weights.tensors["lm_head"]
    scaled = saved.copy()
    scaled[stop] = inputs.f32_to_bf16_bits(8.0 * inputs.bf16_bits_to_f32(saved[stop]))
    weights.tensors["lm_head"] = scaled
    try:
        blob = torch.from_numpy(weights.blob())
    finally:
        weights.tensors["lm_head"] = saved
    h2 = mtmc.mtmc_weights_create(mtmc.make_config(cfg, prompt_len + max_new), blob)
    del blob, scaled
    try:
        ws = torch.empty(mtmc.mtmc_rollout_ragged_workspace_bytes(h2, n_prompts, prompt_len, n_samples, max_new),
                         dtype=torch.uint8, device=dev)
        run = lambda: mtmc.mtmc_rollout_ragged(h2, prompts, lens, n_samples, max_new, 1.0, 1, stop_id=stop, workspace=ws)
        (ids, lp, n), ms_poll = timed(run)
        mtmc.mtmc_set_option(h2, mtmc.MTMC_OPT_STOP_POLL_STEPS, 0)
        (ids0, lp0, n0), ms_static = timed(run)
        mtmc.mtmc_poll_errors(h2)
        toks = int(n.sum().item())
        out["stop_token"] = {"workload": f"{n_prompts} x {n_samples} rows, prompt {prompt_len}, up to {max_new} new tokens, "
                                         f"stop token with its LM-head row scaled by 8",
                             "tokens_generated": toks, "longest_row": int(n.max().item()),
                             "median_row": float(n.float().median().item()),
                             "ms_rows_give_up_places": ms_poll, "ms_rows_keep_places": ms_static,
                             "tokens_per_s_rows_give_up_places": toks / (ms_poll * 1e-3),
                             "tokens_per_s_rows_keep_places": int(n0.sum().item()) / (ms_static * 1e-3)}
        progress(f"stop token: {toks} tokens, {ms_poll:.1f} ms against {ms_static:.1f} ms")
        del ws
        # eight batches of 128 sequences in one call: the slots of finished sequences go to the next prompt of the
        # call, against batch after batch (each ending with its last row, rows giving up their places as above)
        mtmc.mtmc_set_option(h2, mtmc.MTMC_OPT_STOP_POLL_STEPS, 32)
        many = 8 * (128 // n_samples)
        m_prompts = torch.from_numpy(inputs.make_prompts(many, prompt_len, cfg.vocab, seed=8)).to(dev)
        m_lens = torch.full((many,), prompt_len, dtype=torch.int32, device=dev)
        ws = torch.empty(mtmc.mtmc_rollout_ragged_workspace_bytes(h2, many, prompt_len, n_samples, max_new),
                         dtype=torch.uint8, device=dev)
        run = lambda: mtmc.mtmc_rollout_ragged(h2, m_prompts, m_lens, n_samples, max_new, 1.0, 1, stop_id=stop, workspace=ws)
        (ids, lp, n), ms_admit = timed(run)
        mtmc.mtmc_set_option(h2, mtmc.MTMC_OPT_ADMIT_PROMPTS, 0)
        (ids0, lp0, n0), ms_batches = timed(run)
        mtmc.mtmc_poll_errors(h2)
        toks, toks0 = int(n.sum().item()), int(n0.sum().item())
        same = (ids == ids0).all(dim=1)
        out["prompts_join_a_running_batch"] = {
            "workload": f"{many} x {n_samples} rows through the 128 slots of one batch, prompt {prompt_len}, up to "
                        f"{max_new} new tokens, the same stop token",
            "tokens_generated": toks, "longest_row": int(n.max().item()), "median_row": float(n.float().median().item()),
            "ms_prompts_join": ms_admit, "ms_batch_after_batch": ms_batches,
            "tokens_per_s_prompts_join": toks / (ms_admit * 1e-3),
            "tokens_per_s_batch_after_batch": toks0 / (ms_batches * 1e-3),
            "rows_with_the_same_ids": int(same.sum().item()), "rows": int(same.numel()),
            "max_logprob_difference_on_those_rows": float((lp[same] - lp0[same]).abs().max().item()) if same.any() else None}
        progress(f"prompts join a running batch: {toks} tokens, {ms_admit:.1f} ms against {ms_batches:.1f} ms")
        del ws
    finally:
        mtmc.mtmc_weights_destroy(h2)
    return out


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", default="1p5b", choices=sorted(WORKLOADS))
    ap.add_argument("--max-new", type=int, default=None, help="override the number of new tokens")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-score", action="store_true", help="time the rollout alone")
    ap.add_argument("--no-rollout", action="store_true",
                    help="time the scoring pass alone, on sequences whose new tokens are random ids (for counter runs)")
    ap.add_argument("--no-actions", action="store_true", help="skip the action-scoring leg (reported beside the step)")
    ap.add_argument("--no-inference-legs", action="store_true",
                    help="skip the stop-token and cached-prefix legs (reported beside the step, 1p5b workload only)")
    ap.add_argument("--no-graph", action="store_true", help="launch decode steps directly (for counter runs)")
    ap.add_argument("--progress", action="store_true", help="print a line to stderr as each stage ends")
    ap.add_argument("--no-kernel-timer", action="store_true", help="do not bracket the gate/up launches with events")
    ap.add_argument("--copy-probe-mib", type=int, default=0,
                    help="before the workload, copy this many MiB device to device once: a kernel of known "
                         "traffic against which hardware byte counters of the same run are scaled")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only (the path shards by prompt with no collectives; "
              "run one process per GPU on disjoint prompts). Use --gpus 1.", file=sys.stderr)
        return 2

    import torch
    from paper_2511_20100_amd import mtmc

    def progress(msg):
        if args.progress:
            print(f"[bench {time.strftime('%H:%M:%S')}] {msg}", file=sys.stderr, flush=True)

    cfg, n_prompts, prompt_len, n_samples, max_new = WORKLOADS[args.workload]
    if args.workload == "7b-score":
        args.no_rollout = args.no_actions = True
    if args.max_new:
        max_new = args.max_new
    B = n_prompts * n_samples
    seq_len = prompt_len + max_new
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    t0 = time.perf_counter()
    weights = inputs.make_weights(cfg, seed=0)
    blob = torch.from_numpy(weights.blob())
    handle = mtmc.mtmc_weights_create(mtmc.make_config(cfg, seq_len), blob)
    del blob
    if args.no_graph:
        mtmc.mtmc_set_option(handle, mtmc.MTMC_OPT_HIP_GRAPH, 0)
    if args.copy_probe_mib > 0:
        src = torch.ones(args.copy_probe_mib << 20, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        mtmc.mtmc_copy_probe(dst, src)
        torch.cuda.synchronize()
        del src, dst
    prompts_np = inputs.make_prompts(n_prompts, prompt_len, cfg.vocab, seed=2)
    prompts = torch.from_numpy(prompts_np).to(dev)
    ws_r = None if args.no_rollout else torch.empty(
        mtmc.mtmc_rollout_workspace_bytes(handle, n_prompts, prompt_len, n_samples, max_new), dtype=torch.uint8, device=dev)
    ws_s = torch.empty(mtmc.mtmc_score_workspace_bytes(handle, B, seq_len), dtype=torch.uint8, device=dev)
    out_ids = torch.empty((B, max_new), dtype=torch.int32, device=dev)
    out_lp = torch.empty((B, max_new), dtype=torch.float32, device=dev)
    seqs = torch.empty((B, seq_len), dtype=torch.int32, device=dev)
    seqs[:, :prompt_len] = prompts.repeat_interleave(n_samples, dim=0)
    score_lp = torch.empty((B, seq_len - 1), dtype=torch.float32, device=dev)
    setup_s = time.perf_counter() - t0
    progress(f"weights re-tiled and inputs resident after {setup_s:.1f} s")
    stream = torch.cuda.current_stream()

    ev = [torch.cuda.Event(enable_timing=True) for _ in range(3)]

    if args.no_rollout:
        out_ids.copy_(torch.from_numpy(inputs.make_token_ids((B, max_new), cfg.vocab, seed=5)).to(dev))

    def step(seed):
        ev[0].record(stream)
        if not args.no_rollout:
            mtmc.mtmc_rollout(handle, prompts, n_samples, max_new, 1.0, seed, workspace=ws_r, out_ids=out_ids,
                              out_logprobs=out_lp)
        ev[1].record(stream)
        if not args.no_score:
            seqs[:, prompt_len:] = out_ids
            mtmc.mtmc_score(handle, seqs, prompt_len, workspace=ws_s, out_logprobs=score_lp)
        ev[2].record(stream)

    for i in range(args.warmup):
        step(100 + i)
        torch.cuda.synchronize()
        progress(f"warm-up step {i + 1} of {args.warmup} done")
    # dominant decode kernel (gate/up projection: half of the layer weight bytes): every 32nd decode
    # step of the timed region is launched directly with a HIP-event pair around each of its launches
    timed_kernel = cfg.dtype == "bf16" and not args.no_kernel_timer and not args.no_rollout
    if timed_kernel:
        mtmc.mtmc_kernel_timer(handle, mtmc.MTMC_KERNEL_GATE_UP, 32)
    rollout_ms, score_ms = [], []
    t_begin = time.perf_counter()
    for i in range(args.steps):
        step(1 + i)
        ev[2].synchronize()  # the events are reused by the next step
        rollout_ms.append(ev[0].elapsed_time(ev[1]))
        score_ms.append(ev[1].elapsed_time(ev[2]))
        progress(f"timed step {i + 1} of {args.steps}: rollout {rollout_ms[-1]:.1f} ms, scoring {score_ms[-1]:.1f} ms")
    torch.cuda.synchronize()
    total_s = time.perf_counter() - t_begin
    mtmc.mtmc_poll_errors(handle)
    k_ms, k_launches, k_empty_ms = (0.0, 0, 0.0)
    if timed_kernel:
        k_ms, k_launches, k_empty_ms = mtmc.mtmc_kernel_timer_read(handle)
        mtmc.mtmc_kernel_timer(handle, 0, 0)

    ms_per_step = 1e3 * total_s / args.steps
    new_tokens = B * max_new
    r_ms = float(np.mean(rollout_ms))
    s_ms = float(np.mean(score_ms))
    # decode roofline: algorithmic bytes of an average decode step over the measured step time.  The
    # rollout time is prefill + (max_new - 1) decode steps; prefill is charged to the decode steps.
    step_bytes, w_bytes, kv_bytes = decode_bytes_per_step(cfg, n_prompts, prompt_len, n_samples, max_new)
    decode_ms = r_ms / max(1, max_new - 1)
    step_gbs = step_bytes / (decode_ms * 1e-3) / 1e9
    gate_up_bytes = 2 * cfg.d_ffn * cfg.d_model * 2   # gate and up matrices, 2 bytes per weight, read once
    read_gbs, mfma_tflops = attainable_rates(torch, mtmc, dev)
    hbm_attainable = {"value": read_gbs, "unit": "GB/s", "how": "plain streaming read of 2 GiB, measured in this run"}
    mfma_attainable = {"value": mfma_tflops, "unit": "TFLOP/s",
                       "how": "register-only loop of fp16 32x32x16 matrix instructions on all SIMDs (4 x 4 accumulator blocks per "
                              "wavefront, pseudo-random operands), measured in this run"}
    if k_launches > 0:
        k_us = 1e3 * k_ms / k_launches
        roofline = {"bound": "hbm", "achieved": gate_up_bytes / (k_us * 1e-6) / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": gate_up_bytes / (k_us * 1e-6) / 1e9 / HBM_PEAK_GBS,
                    "attainable": hbm_attainable,
                    "traffic": gate_up_traffic_from_profile(args.workload),
                    "kernel": "gate/up projection of a decode step, one launch per layer (k_gemm_dec<..., SWIGLU> up to "
                              "64 rows, k_gemm_rows128<..., SWIGLU> at 65..128)",
                    "bytes_per_launch": gate_up_bytes, "us_per_launch": k_us, "timed_launches": k_launches,
                    "empty_event_pair_us": 1e3 * k_empty_ms}
    else:
        roofline = {"bound": "hbm", "achieved": step_gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": step_gbs / HBM_PEAK_GBS, "attainable": hbm_attainable, "traffic": None,
                    "kernel": "whole decode step"}
    result = {
        "metric": "rollout tokens/sec @1.5B-class bs64 bf16; decode HBM GB/s + scoring MFMA % peak",
        "value": (B * seq_len if args.no_rollout else new_tokens) / (ms_per_step * 1e-3), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16 weights, f16 MFMA operands and KV cache, f32 accumulate" if cfg.dtype == "bf16" else "f32",
        "data": "synthetic",
        "config": {"workload": f"{args.workload}: {cfg.n_layers} layers d{cfg.d_model} Hq{cfg.n_q_heads}/Hkv{cfg.n_kv_heads} "
                               f"F{cfg.d_ffn} V{cfg.vocab}; {n_prompts} prompts x {n_samples} samples = batch {B}, "
                               f"prompt {prompt_len}, {max_new} new tokens at T=1; then scoring of the {B} x {seq_len} sequences",
                   "step": "mtmc_score" if args.no_rollout else "mtmc_rollout + mtmc_score" if not args.no_score
                           else "mtmc_rollout"},
        "rollout_tokens_per_s": new_tokens / (r_ms * 1e-3), "rollout_ms": r_ms,
        "roofline": roofline,
        "decode_step": {"bound": "hbm", "achieved": step_gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                        "frac": step_gbs / HBM_PEAK_GBS, "attainable": hbm_attainable,
                        "bytes_per_step": step_bytes, "ms_per_step": decode_ms,
                        "note": "algorithmic bytes of an average decode step (weights once + KV with shared prompt pages) "
                                "over rollout time / decode steps (prefill time included)"},
        "setup_s": setup_s,
    }
    if not args.no_score:
        flops = forward_flops(cfg, B, seq_len, max_new)
        result["score_tokens_per_s"] = B * seq_len / (s_ms * 1e-3)
        result["score_ms"] = s_ms
        result["score_mfma"] = {"bound": "mfma", "achieved": flops / (s_ms * 1e-3) / 1e12, "peak": MFMA_PEAK_TFLOPS,
                                "unit": "TFLOP/s", "frac": flops / (s_ms * 1e-3) / 1e12 / MFMA_PEAK_TFLOPS,
                                "attainable": mfma_attainable}
    if args.no_rollout:  # nothing was decoded: the step is the scoring pass, bound by the matrix cores
        for key in ("rollout_tokens_per_s", "rollout_ms", "decode_step"):
            del result[key]
        result["roofline"] = dict(result["score_mfma"], traffic=None,
                                  kernel="whole scoring pass (algorithmic flops of the forward pass over its time)")
    if not args.no_actions:
        # beside the step, not part of `value`: the prompts as states, 32 candidate actions of up to 32 tokens each
        K, A = 32, min(32, max_new)
        actions_np, lens_np = inputs.make_actions(n_prompts, K, A, cfg.vocab, seed=4)
        d_actions, d_lens = torch.from_numpy(actions_np).to(dev), torch.from_numpy(lens_np).to(dev)
        ws_a = torch.empty(mtmc.mtmc_score_actions_workspace_bytes(handle, n_prompts, prompt_len, K, A),
                           dtype=torch.uint8, device=dev)
        mtmc.mtmc_score_actions(handle, prompts, d_actions, d_lens, workspace=ws_a)
        ev[0].record(stream)
        for _ in range(3):
            mtmc.mtmc_score_actions(handle, prompts, d_actions, d_lens, workspace=ws_a)
        ev[1].record(stream)
        ev[1].synchronize()
        mtmc.mtmc_poll_errors(handle)
        a_ms = ev[0].elapsed_time(ev[1]) / 3
        result["action_scoring"] = {"workload": f"{n_prompts} states x {prompt_len} tokens, {K} candidate actions each, "
                                                f"1..{A} tokens per action", "ms": a_ms,
                                    "actions_per_s": n_prompts * K / (a_ms * 1e-3)}
        del ws_a
        if not args.no_rollout and not args.no_score:
            # beside the step as well: the scoring of the step's own sequences through mtmc_score_actions, with the
            # prompts as states and each prompt's samples as its candidates, so that a prompt is evaluated once instead
            # of once per sample (the same log-probs, bit for bit, wherever both routes run the same matrix kernels)
            cont = out_ids.reshape(n_prompts, n_samples, max_new)
            full = torch.full((n_prompts, n_samples), max_new, dtype=torch.int32, device=dev)
            ws_a = torch.empty(mtmc.mtmc_score_actions_workspace_bytes(handle, n_prompts, prompt_len, n_samples, max_new),
                               dtype=torch.uint8, device=dev)
            tok = mtmc.mtmc_score_actions(handle, prompts, cont, full, workspace=ws_a)[0]
            ev[0].record(stream)
            for _ in range(2):
                tok = mtmc.mtmc_score_actions(handle, prompts, cont, full, workspace=ws_a)[0]
            ev[1].record(stream)
            ev[1].synchronize()
            mtmc.mtmc_poll_errors(handle)
            ref = score_lp[:, prompt_len - 1:]
            result["scoring_with_shared_prompts"] = {
                "call": "mtmc_score_actions(states = the prompts, candidates = each prompt's samples)",
                "ms": ev[0].elapsed_time(ev[1]) / 2, "ms_mtmc_score": s_ms,
                "same_bits_as_mtmc_score": bool(torch.equal(tok.reshape(B, max_new), ref)),
                "max_difference": float((tok.reshape(B, max_new) - ref).abs().max())}
            del ws_a
    if args.workload == "1p5b" and not args.no_inference_legs and not args.no_rollout:
        result["inference"] = inference_legs(torch, mtmc, dev, handle, weights, cfg, prompts, n_samples, max_new, progress)
    if not args.no_cpu_baseline:
        progress("timing the oracle on the host cores")
        result["cpu_baseline"] = cpu_baseline(weights, cfg, prompts_np, seq_len, score_only=args.no_rollout)
    mtmc.mtmc_weights_destroy(handle)
    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
