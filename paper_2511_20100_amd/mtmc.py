"""ctypes binding of libmtmc.so: argument marshalling only.

Every function has the name and the meaning of the C entry point it wraps (include/mtmc.h).
PyTorch is used for device memory (tensors own the buffers that are passed as raw pointers)
and for the current HIP stream; no step of the computation runs in Python or in PyTorch.
There is no fallback: if the library is missing or fails to load, importing this module raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Tuple

import torch

from .inputs import ModelConfig

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libmtmc.so")

MTMC_OK, MTMC_EINVAL, MTMC_ENOMEM, MTMC_EHIP, MTMC_EDATA = 0, -1, -2, -3, -4
MTMC_F32, MTMC_BF16 = 0, 1
MTMC_DATA_TOKEN_ID, MTMC_DATA_WEIGHT, MTMC_DATA_LENGTH, MTMC_DATA_FP16_RANGE, MTMC_DATA_PREFIX = 1, 2, 4, 8, 16


class MtmcError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"libmtmc error {code}: {msg}")
        self.code = code


class mtmc_config(ctypes.Structure):
    _fields_ = [("n_layers", ctypes.c_int32), ("d_model", ctypes.c_int32), ("n_q_heads", ctypes.c_int32),
                ("n_kv_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32), ("d_ffn", ctypes.c_int32),
                ("vocab", ctypes.c_int32), ("rms_eps", ctypes.c_float), ("rope_base", ctypes.c_float),
                ("dtype", ctypes.c_int32), ("page_tokens", ctypes.c_int32), ("max_positions", ctypes.c_int32),
                ("tie_embeddings", ctypes.c_int32)]


def _load() -> ctypes.CDLL:
    if not os.path.exists(_LIB_PATH):
        raise ImportError(f"{_LIB_PATH} is missing: build it with `python -m paper_2511_20100_amd.build`")
    lib = ctypes.CDLL(_LIB_PATH)
    vp, i32, u32, u64, f32, sz = (ctypes.c_void_p, ctypes.c_int32, ctypes.c_uint32, ctypes.c_uint64,
                                  ctypes.c_float, ctypes.c_size_t)
    cfgp = ctypes.POINTER(mtmc_config)
    lib.mtmc_weights_create.argtypes = [cfgp, vp, sz, ctypes.c_int, vp, ctypes.POINTER(vp)]
    lib.mtmc_weights_create.restype = ctypes.c_int
    lib.mtmc_weights_destroy.argtypes = [vp]
    lib.mtmc_weights_destroy.restype = None
    lib.mtmc_blob_bytes.argtypes = [cfgp]
    lib.mtmc_blob_bytes.restype = sz
    lib.mtmc_rollout_workspace_bytes.argtypes = [vp, i32, i32, i32, i32]
    lib.mtmc_rollout_workspace_bytes.restype = sz
    lib.mtmc_rollout.argtypes = [vp, vp, i32, i32, i32, i32, f32, u64, u32, vp, vp, vp, sz, vp]
    lib.mtmc_rollout.restype = ctypes.c_int
    lib.mtmc_rollout_ragged_workspace_bytes.argtypes = [vp, i32, i32, i32, i32]
    lib.mtmc_rollout_ragged_workspace_bytes.restype = sz
    lib.mtmc_rollout_ragged.argtypes = [vp, vp, vp, i32, i32, i32, i32, f32, u64, u32, i32, vp, vp, vp, vp, sz, vp]
    lib.mtmc_rollout_ragged.restype = ctypes.c_int
    lib.mtmc_rollout_ragged_cached.argtypes = [vp, vp, vp, i32, i32, i32, i32, f32, u64, u32, i32, i32, vp, vp, vp, vp,
                                               sz, vp]
    lib.mtmc_rollout_ragged_cached.restype = ctypes.c_int
    lib.mtmc_score_workspace_bytes.argtypes = [vp, i32, i32]
    lib.mtmc_score_workspace_bytes.restype = sz
    lib.mtmc_score.argtypes = [vp, vp, i32, i32, i32, vp, vp, vp, vp, sz, vp]
    lib.mtmc_score.restype = ctypes.c_int
    lib.mtmc_score_actions_workspace_bytes.argtypes = [vp, i32, i32, i32, i32]
    lib.mtmc_score_actions_workspace_bytes.restype = sz
    lib.mtmc_score_actions.argtypes = [vp, vp, i32, i32, vp, vp, i32, i32, i32, vp, vp, vp, vp, sz, vp]
    lib.mtmc_score_actions.restype = ctypes.c_int
    lib.mtmc_ppo_workspace_bytes.argtypes = []
    lib.mtmc_ppo_workspace_bytes.restype = sz
    lib.mtmc_ppo_clip_loss.argtypes = [vp, vp, vp, vp, ctypes.c_int64, f32, vp, vp, sz, vp]
    lib.mtmc_ppo_clip_loss.restype = ctypes.c_int
    lib.mtmc_ppo_clip_loss_static.argtypes = [vp, vp, vp, vp, ctypes.c_int64, f32, vp, vp]
    lib.mtmc_ppo_clip_loss_static.restype = ctypes.c_int
    lib.mtmc_set_option.argtypes = [vp, ctypes.c_int, ctypes.c_int]
    lib.mtmc_set_option.restype = ctypes.c_int
    lib.mtmc_kernel_timer.argtypes = [vp, ctypes.c_int, ctypes.c_int]
    lib.mtmc_kernel_timer.restype = ctypes.c_int
    lib.mtmc_kernel_timer_read.argtypes = [vp, vp, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_int64),
                                           ctypes.POINTER(ctypes.c_double)]
    lib.mtmc_kernel_timer_read.restype = ctypes.c_int
    lib.mtmc_copy_probe.argtypes = [vp, vp, ctypes.c_size_t, vp]
    lib.mtmc_copy_probe.restype = ctypes.c_int
    lib.mtmc_read_probe.argtypes = [vp, ctypes.c_size_t, vp, vp]
    lib.mtmc_read_probe.restype = ctypes.c_int
    lib.mtmc_mfma_probe.argtypes = [vp, i32, i32, vp, ctypes.POINTER(ctypes.c_double)]
    lib.mtmc_mfma_probe.restype = ctypes.c_int
    lib.mtmc_poll_errors.argtypes = [vp, vp]
    lib.mtmc_poll_errors.restype = ctypes.c_int
    lib.mtmc_last_error.argtypes = []
    lib.mtmc_last_error.restype = ctypes.c_char_p
    lib.mtmc_data_error_string.argtypes = [ctypes.c_int]
    lib.mtmc_data_error_string.restype = ctypes.c_char_p
    lib.mtmc_admission_plan.argtypes = [vp, vp, i32, i32, i32, i32, i32, i32, vp, vp]
    lib.mtmc_admission_plan.restype = ctypes.c_int
    return lib


_lib = _load()
EXPORTS = ("mtmc_weights_create", "mtmc_weights_destroy", "mtmc_blob_bytes", "mtmc_rollout_workspace_bytes",
           "mtmc_rollout", "mtmc_score_workspace_bytes", "mtmc_score", "mtmc_poll_errors", "mtmc_last_error",
           "mtmc_set_option", "mtmc_kernel_timer", "mtmc_kernel_timer_read", "mtmc_copy_probe",
           "mtmc_score_actions_workspace_bytes", "mtmc_score_actions", "mtmc_rollout_ragged_workspace_bytes",
           "mtmc_rollout_ragged", "mtmc_ppo_workspace_bytes", "mtmc_ppo_clip_loss", "mtmc_data_error_string",
           "mtmc_ppo_clip_loss_static", "mtmc_read_probe", "mtmc_mfma_probe", "mtmc_rollout_ragged_cached",
           "mtmc_admission_plan")


def mtmc_last_error() -> str:
    return (_lib.mtmc_last_error() or b"").decode()


def _check(rc: int) -> None:
    if rc != MTMC_OK:
        raise MtmcError(rc, mtmc_last_error())


def _stream_ptr(stream: Optional[torch.cuda.Stream]) -> int:
    s = stream if stream is not None else torch.cuda.current_stream()
    return s.cuda_stream


def make_config(cfg: ModelConfig, max_positions: int) -> mtmc_config:
    return mtmc_config(cfg.n_layers, cfg.d_model, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.d_ffn,
                       cfg.vocab, cfg.rms_eps, cfg.rope_base, MTMC_BF16 if cfg.dtype == "bf16" else MTMC_F32,
                       16, max_positions, 1 if cfg.tie_embeddings else 0)


def mtmc_blob_bytes(cfg: mtmc_config) -> int:
    return int(_lib.mtmc_blob_bytes(ctypes.byref(cfg)))


def mtmc_weights_create(cfg: mtmc_config, blob, stream: Optional[torch.cuda.Stream] = None) -> int:
    """blob: a uint8 torch tensor (CPU or CUDA) or a numpy uint8 array holding the canonical blob.
    Returns the opaque handle (an integer address)."""
    if not isinstance(blob, torch.Tensor):
        blob = torch.from_numpy(blob)
    assert blob.dtype == torch.uint8 and blob.is_contiguous()
    handle = ctypes.c_void_p()
    _check(_lib.mtmc_weights_create(ctypes.byref(cfg), blob.data_ptr(), blob.numel(),
                                    1 if blob.is_cuda else 0, _stream_ptr(stream), ctypes.byref(handle)))
    return handle.value


def mtmc_weights_destroy(handle: int) -> None:
    _lib.mtmc_weights_destroy(handle)


def mtmc_rollout_workspace_bytes(handle: int, n_prompts: int, prompt_len: int, n_samples: int, max_new: int) -> int:
    n = int(_lib.mtmc_rollout_workspace_bytes(handle, n_prompts, prompt_len, n_samples, max_new))
    if n == 0:
        raise MtmcError(MTMC_EINVAL, mtmc_last_error())
    return n


def mtmc_rollout(handle: int, prompts: torch.Tensor, n_samples: int, max_new: int, temperature: float, seed: int,
                 *, seq_offset: int = 0, workspace: Optional[torch.Tensor] = None,
                 out_ids: Optional[torch.Tensor] = None, out_logprobs: Optional[torch.Tensor] = None,
                 stream: Optional[torch.cuda.Stream] = None) -> Tuple[torch.Tensor, torch.Tensor]:
    """prompts: int32 CUDA tensor [n_prompts, prompt_len].  Returns (ids, logprobs), both
    [n_prompts*n_samples, max_new] CUDA tensors, valid after the stream is synchronised."""
    assert prompts.is_cuda and prompts.dtype == torch.int32 and prompts.is_contiguous() and prompts.dim() == 2
    n_prompts, prompt_len = prompts.shape
    if workspace is None:
        workspace = torch.empty(mtmc_rollout_workspace_bytes(handle, n_prompts, prompt_len, n_samples, max_new),
                                dtype=torch.uint8, device=prompts.device)
    B = n_prompts * n_samples
    if out_ids is None:
        out_ids = torch.empty((B, max_new), dtype=torch.int32, device=prompts.device)
    if out_logprobs is None:
        out_logprobs = torch.empty((B, max_new), dtype=torch.float32, device=prompts.device)
    _check(_lib.mtmc_rollout(handle, prompts.data_ptr(), n_prompts, prompt_len, n_samples, max_new,
                             float(temperature), int(seed), int(seq_offset), out_ids.data_ptr(),
                             out_logprobs.data_ptr(), workspace.data_ptr(), workspace.numel(), _stream_ptr(stream)))
    return out_ids, out_logprobs


def mtmc_rollout_ragged_workspace_bytes(handle: int, n_prompts: int, max_prompt_len: int, n_samples: int,
                                        max_new: int) -> int:
    n = int(_lib.mtmc_rollout_ragged_workspace_bytes(handle, n_prompts, max_prompt_len, n_samples, max_new))
    if n == 0:
        raise MtmcError(MTMC_EINVAL, mtmc_last_error())
    return n


def mtmc_rollout_ragged(handle: int, prompts: torch.Tensor, prompt_lens: torch.Tensor, n_samples: int, max_new: int,
                        temperature: float, seed: int, *, stop_id: int = -1, seq_offset: int = 0,
                        workspace: Optional[torch.Tensor] = None, stream: Optional[torch.cuda.Stream] = None,
                        reuse_len: Optional[int] = None):
    """prompts int32 CUDA [n_prompts, max_prompt_len] (right-padded), prompt_lens int32 CUDA [n_prompts].
    Returns (ids [B, max_new] int32, logprobs [B, max_new] float32, lens [B] int32), B = n_prompts * n_samples.
    With reuse_len (not None) the call is mtmc_rollout_ragged_cached on the given workspace."""
    for t in (prompts, prompt_lens):
        assert t.is_cuda and t.dtype == torch.int32 and t.is_contiguous()
    n_prompts, Lmax = prompts.shape
    assert tuple(prompt_lens.shape) == (n_prompts,)
    B = n_prompts * n_samples
    if workspace is None:
        workspace = torch.empty(mtmc_rollout_ragged_workspace_bytes(handle, n_prompts, Lmax, n_samples, max_new),
                                dtype=torch.uint8, device=prompts.device)
    ids = torch.empty((B, max_new), dtype=torch.int32, device=prompts.device)
    lp = torch.empty((B, max_new), dtype=torch.float32, device=prompts.device)
    lens = torch.empty((B,), dtype=torch.int32, device=prompts.device)
    if reuse_len is None:
        _check(_lib.mtmc_rollout_ragged(handle, prompts.data_ptr(), prompt_lens.data_ptr(), n_prompts, Lmax, n_samples,
                                        max_new, temperature, seed, seq_offset, stop_id, ids.data_ptr(), lp.data_ptr(),
                                        lens.data_ptr(), workspace.data_ptr(), workspace.numel(), _stream_ptr(stream)))
    else:
        _check(_lib.mtmc_rollout_ragged_cached(handle, prompts.data_ptr(), prompt_lens.data_ptr(), n_prompts, Lmax,
                                               n_samples, max_new, temperature, seed, seq_offset, stop_id,
                                               int(reuse_len), ids.data_ptr(), lp.data_ptr(), lens.data_ptr(),
                                               workspace.data_ptr(), workspace.numel(), _stream_ptr(stream)))
    return ids, lp, lens


def mtmc_rollout_ragged_cached(handle: int, prompts: torch.Tensor, prompt_lens: torch.Tensor, n_samples: int,
                               max_new: int, temperature: float, seed: int, reuse_len: int, workspace: torch.Tensor,
                               *, stop_id: int = -1, seq_offset: int = 0,
                               stream: Optional[torch.cuda.Stream] = None):
    """mtmc_rollout_ragged that keeps the first reuse_len cached positions of every prompt in `workspace`."""
    return mtmc_rollout_ragged(handle, prompts, prompt_lens, n_samples, max_new, temperature, seed, stop_id=stop_id,
                               seq_offset=seq_offset, workspace=workspace, stream=stream, reuse_len=reuse_len)


def mtmc_score_workspace_bytes(handle: int, n_seqs: int, seq_len: int) -> int:
    n = int(_lib.mtmc_score_workspace_bytes(handle, n_seqs, seq_len))
    if n == 0:
        raise MtmcError(MTMC_EINVAL, mtmc_last_error())
    return n


def mtmc_score(handle: int, seqs: torch.Tensor, prompt_len: int = 1, *, want_top1: bool = False,
               workspace: Optional[torch.Tensor] = None, out_logprobs: Optional[torch.Tensor] = None,
               stream: Optional[torch.cuda.Stream] = None):
    """seqs: int32 CUDA tensor [n_seqs, seq_len].  Returns logprobs [n_seqs, seq_len-1], or
    (logprobs, top1, margin) when want_top1."""
    assert seqs.is_cuda and seqs.dtype == torch.int32 and seqs.is_contiguous() and seqs.dim() == 2
    n_seqs, S = seqs.shape
    if workspace is None:
        workspace = torch.empty(mtmc_score_workspace_bytes(handle, n_seqs, S), dtype=torch.uint8, device=seqs.device)
    if out_logprobs is None:
        out_logprobs = torch.empty((n_seqs, S - 1), dtype=torch.float32, device=seqs.device)
    top1 = torch.empty((n_seqs, S - 1), dtype=torch.int32, device=seqs.device) if want_top1 else None
    margin = torch.empty((n_seqs, S - 1), dtype=torch.float32, device=seqs.device) if want_top1 else None
    _check(_lib.mtmc_score(handle, seqs.data_ptr(), n_seqs, S, prompt_len, out_logprobs.data_ptr(),
                           top1.data_ptr() if want_top1 else None, margin.data_ptr() if want_top1 else None,
                           workspace.data_ptr(), workspace.numel(), _stream_ptr(stream)))
    return (out_logprobs, top1, margin) if want_top1 else out_logprobs


def mtmc_score_actions_workspace_bytes(handle: int, n_states: int, state_len: int, n_actions: int,
                                       max_action_len: int) -> int:
    n = int(_lib.mtmc_score_actions_workspace_bytes(handle, n_states, state_len, n_actions, max_action_len))
    if n == 0:
        raise MtmcError(MTMC_EINVAL, mtmc_last_error())
    return n


def mtmc_score_actions(handle: int, states: torch.Tensor, actions: torch.Tensor, action_len: torch.Tensor, *,
                       normalize: bool = False, workspace: Optional[torch.Tensor] = None,
                       stream: Optional[torch.cuda.Stream] = None):
    """states int32 [n_states, state_len], actions int32 [n_states, K, A], action_len int32 [n_states, K]
    (CUDA tensors).  Returns (token_logprobs [n_states, K, A], action_logprobs [n_states, K],
    policy_logprobs [n_states, K])."""
    for t in (states, actions, action_len):
        assert t.is_cuda and t.dtype == torch.int32 and t.is_contiguous()
    n_states, P = states.shape
    ns2, K, A = actions.shape
    assert ns2 == n_states and tuple(action_len.shape) == (n_states, K)
    if workspace is None:
        workspace = torch.empty(mtmc_score_actions_workspace_bytes(handle, n_states, P, K, A), dtype=torch.uint8,
                                device=states.device)
    tok = torch.empty((n_states, K, A), dtype=torch.float32, device=states.device)
    act = torch.empty((n_states, K), dtype=torch.float32, device=states.device)
    pol = torch.empty((n_states, K), dtype=torch.float32, device=states.device)
    _check(_lib.mtmc_score_actions(handle, states.data_ptr(), n_states, P, actions.data_ptr(), action_len.data_ptr(),
                                   K, A, 1 if normalize else 0, tok.data_ptr(), act.data_ptr(), pol.data_ptr(),
                                   workspace.data_ptr(), workspace.numel(), _stream_ptr(stream)))
    return tok, act, pol


def mtmc_ppo_workspace_bytes() -> int:
    return int(_lib.mtmc_ppo_workspace_bytes())


def mtmc_ppo_clip_loss(new_logprobs: torch.Tensor, old_logprobs: torch.Tensor, advantages: torch.Tensor,
                       clip_eps: float, mask: Optional[torch.Tensor] = None,
                       stream: Optional[torch.cuda.Stream] = None) -> torch.Tensor:
    """fp32 CUDA tensors of one size (mask: int32 or None).  Returns a CUDA double tensor
    [loss, clip fraction, approx KL, count]."""
    for t in (new_logprobs, old_logprobs, advantages):
        assert t.is_cuda and t.dtype == torch.float32 and t.is_contiguous() and t.numel() == new_logprobs.numel()
    if mask is not None:
        assert mask.is_cuda and mask.dtype == torch.int32 and mask.is_contiguous() and mask.numel() == new_logprobs.numel()
    ws = torch.empty(mtmc_ppo_workspace_bytes(), dtype=torch.uint8, device=new_logprobs.device)
    out = torch.empty(4, dtype=torch.float64, device=new_logprobs.device)
    _check(_lib.mtmc_ppo_clip_loss(new_logprobs.data_ptr(), old_logprobs.data_ptr(), advantages.data_ptr(),
                                   mask.data_ptr() if mask is not None else None, new_logprobs.numel(), clip_eps,
                                   out.data_ptr(), ws.data_ptr(), ws.numel(), _stream_ptr(stream)))
    return out


MTMC_PPO_STATIC_MAX_SAMPLES = 268435456


def mtmc_ppo_clip_loss_static(new_logprobs: torch.Tensor, old_logprobs: torch.Tensor, advantages: torch.Tensor,
                              clip_eps: float, mask: Optional[torch.Tensor] = None, *,
                              out: Optional[torch.Tensor] = None, n: Optional[int] = None,
                              stream: Optional[torch.cuda.Stream] = None) -> torch.Tensor:
    """mtmc_ppo_clip_loss without a workspace (the library's own static device array holds the partial sums).
    With ``out`` given (CUDA double [4]) nothing is allocated on the way; ``n`` (default: all) takes the first n
    samples of the tensors."""
    for t in (new_logprobs, old_logprobs, advantages):
        assert t.is_cuda and t.dtype == torch.float32 and t.is_contiguous() and t.numel() == new_logprobs.numel()
    if mask is not None:
        assert mask.is_cuda and mask.dtype == torch.int32 and mask.is_contiguous() and mask.numel() == new_logprobs.numel()
    n = new_logprobs.numel() if n is None else int(n)
    assert n <= new_logprobs.numel()
    if out is None:
        out = torch.empty(4, dtype=torch.float64, device=new_logprobs.device)
    assert out.is_cuda and out.dtype == torch.float64 and out.numel() >= 4
    _check(_lib.mtmc_ppo_clip_loss_static(new_logprobs.data_ptr(), old_logprobs.data_ptr(), advantages.data_ptr(),
                                          mask.data_ptr() if mask is not None else None, n, clip_eps,
                                          out.data_ptr(), _stream_ptr(stream)))
    return out


MTMC_MAX_DECODE_CONTEXT = 32768   # prompt_len + max_new of a MTMC_BF16 rollout
MTMC_OPT_HIP_GRAPH = 1
MTMC_OPT_GEMM_LDS_MIN_BLOCKS = 2
MTMC_OPT_STOP_POLL_STEPS = 3
MTMC_OPT_ADMIT_PROMPTS = 4


def mtmc_set_option(handle: int, option: int, value: int) -> None:
    _check(_lib.mtmc_set_option(handle, option, value))


MTMC_KERNEL_QKV, MTMC_KERNEL_ATTENTION, MTMC_KERNEL_GATE_UP, MTMC_KERNEL_DOWN, MTMC_KERNEL_LM_HEAD = 1, 2, 3, 4, 5


def mtmc_kernel_timer(handle: int, kernel_class: int, every_n_steps: int) -> None:
    _check(_lib.mtmc_kernel_timer(handle, kernel_class, every_n_steps))


def mtmc_kernel_timer_read(handle: int, stream: Optional[torch.cuda.Stream] = None) -> Tuple[float, int, float]:
    """Returns (total milliseconds, number of timed launches, mean milliseconds of an empty event
    pair) since the last read."""
    ms, n, empty = ctypes.c_double(), ctypes.c_int64(), ctypes.c_double()
    _check(_lib.mtmc_kernel_timer_read(handle, _stream_ptr(stream), ctypes.byref(ms), ctypes.byref(n),
                                       ctypes.byref(empty)))
    return ms.value, n.value, empty.value


def mtmc_copy_probe(dst: torch.Tensor, src: torch.Tensor, stream: Optional[torch.cuda.Stream] = None) -> None:
    """dst <- src with the library's plain copy kernel (same byte size, contiguous device tensors)."""
    nbytes = src.numel() * src.element_size()
    if dst.numel() * dst.element_size() != nbytes or not (src.is_cuda and dst.is_cuda):
        raise ValueError("mtmc_copy_probe needs two device tensors of the same byte size")
    _check(_lib.mtmc_copy_probe(dst.data_ptr(), src.data_ptr(), nbytes, _stream_ptr(stream)))


def mtmc_read_probe(src: torch.Tensor, sink: torch.Tensor, stream: Optional[torch.cuda.Stream] = None) -> None:
    """Streams the bytes of `src` (device tensor, a multiple of 16 KiB) through a plain read kernel once."""
    assert src.is_cuda and sink.is_cuda and src.is_contiguous() and sink.numel() * sink.element_size() >= 4
    _check(_lib.mtmc_read_probe(src.data_ptr(), src.numel() * src.element_size(), sink.data_ptr(), _stream_ptr(stream)))


def mtmc_mfma_probe(out: torch.Tensor, workgroups: int, iters: int, stream: Optional[torch.cuda.Stream] = None) -> float:
    """Launches the register-only matrix-instruction loop; returns the flops of the launch."""
    assert out.is_cuda and out.dtype == torch.float32 and out.numel() >= workgroups * 256
    flops = ctypes.c_double()
    _check(_lib.mtmc_mfma_probe(out.data_ptr(), workgroups, iters, _stream_ptr(stream), ctypes.byref(flops)))
    return flops.value


def mtmc_poll_errors(handle: int, stream: Optional[torch.cuda.Stream] = None) -> None:
    _check(_lib.mtmc_poll_errors(handle, _stream_ptr(stream)))


def mtmc_admission_plan(live, slot_region, n_regions: int, n_samples: int, prompts_left: int, max_at_once: int,
                        wait_for: int):
    """Host arrays in (numpy int32 [n_slots]); returns (slots [k, n_samples], regions [k]) as numpy arrays."""
    import numpy as np
    live = np.ascontiguousarray(live, dtype=np.int32)
    slot_region = np.ascontiguousarray(slot_region, dtype=np.int32)
    assert live.ndim == 1 and live.shape == slot_region.shape
    slots = np.zeros(max(live.size, 1), dtype=np.int32)
    regions = np.zeros(max(n_regions, 1), dtype=np.int32)
    k = _lib.mtmc_admission_plan(live.ctypes.data, slot_region.ctypes.data, live.size, n_regions, n_samples, prompts_left,
                                 max_at_once, wait_for, slots.ctypes.data, regions.ctypes.data)
    if k < 0:
        raise MtmcError(k, mtmc_last_error())
    return slots[:k * n_samples].reshape(k, n_samples).copy(), regions[:k].copy()


def mtmc_data_error_string(bits: int) -> str:
    return (_lib.mtmc_data_error_string(int(bits)) or b"").decode()
