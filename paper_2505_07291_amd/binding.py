"""Thin Python binding of libgrpo's C ABI (see include/grpo.h).

Argument marshalling only: tensors become raw device pointers, sizes and the
current HIP stream; every step of the computation runs in the library's kernels.
There is no fallback: if the shared library cannot be loaded the call raises.
"""
from __future__ import annotations

import ctypes
import os

import torch  # imported first so that the HIP runtime torch ships is the one in the process

from . import build as _build

GRPO_OK = 0
GRPO_F32, GRPO_BF16 = 0, 1
COUNT_NAMES = ("tokens", "clip_high", "clip_low", "delta", "out_of_band")

_lib = None


class GrpoError(RuntimeError):
    def __init__(self, status, where):
        self.status = int(status)
        super().__init__("%s failed: %s (status %d)" % (where, status_string(status), status))


def lib():
    """The loaded C library with argument types declared.  Builds it only if absent."""
    global _lib
    if _lib is None:
        path = _build.LIB_PATH
        if not os.path.exists(path):
            path = _build.build_library()
        L = ctypes.CDLL(path)
        vp, i64, i32, f32, f64, sz = (ctypes.c_void_p, ctypes.c_int64, ctypes.c_int,
                                      ctypes.c_float, ctypes.c_double, ctypes.c_size_t)
        L.grpo_status_string.restype = ctypes.c_char_p
        L.grpo_status_string.argtypes = [i32]
        L.grpo_workspace_bytes.restype = sz
        L.grpo_workspace_bytes.argtypes = [i64]
        L.grpo_row_kernel_plan.restype = i32
        L.grpo_row_kernel_plan.argtypes = [i32, i64, ctypes.POINTER(RowPlan)]
        L.grpo_group_advantages.restype = i32
        L.grpo_group_advantages.argtypes = [vp, i64, vp, i64, i64, f32, i32, vp, vp, i64, vp, vp]
        L.grpo_logprobs_fwd.restype = i32
        L.grpo_logprobs_fwd.argtypes = [vp, i32, i64, i64, i64, vp, vp, f32, vp, vp, sz, vp]
        L.grpo_loss_fwd_bwd.restype = i32
        L.grpo_loss_fwd_bwd.argtypes = [vp, i32, i64, i64, i64, vp, vp, vp, vp, f32, f32, f32, f32,
                                        f64, f32, vp, vp, vp, vp, vp, sz, vp]
        L.grpo_loss_fwd_bwd_noalloc.restype = i32
        L.grpo_loss_fwd_bwd_noalloc.argtypes = [vp, i32, i64, i64, i64, vp, vp, vp, vp, f32, f32, f32, f32,
                                                f64, f32, vp, vp, vp, vp, vp, vp]
        L.grpo_loss_aux_fwd_bwd.restype = i32
        L.grpo_loss_aux_fwd_bwd.argtypes = [vp, i32, i64, i64, i64, vp, vp, vp, vp, vp, vp, f32, f32, f32,
                                            f32, f32, f32, f64, f32, vp, vp, vp, vp, vp, vp, sz, vp]
        L.grpo_total_rewards.restype = i32
        L.grpo_total_rewards.argtypes = [vp, vp, vp, i64, f32, vp, vp]
        L.grpo_filter_groups.restype = i32
        L.grpo_filter_groups.argtypes = [vp, i64, vp, i64, i64, vp, vp, vp, vp, vp]
        L.grpo_packed_layout.restype = i32
        L.grpo_packed_layout.argtypes = [vp, i64, i64, i32, vp, vp, vp]
        L.grpo_workspace_error.restype = i32
        L.grpo_workspace_error.argtypes = [vp, vp, vp]
        L.grpo_lmhead_workspace_bytes.restype = sz
        L.grpo_lmhead_workspace_bytes.argtypes = [i64, i64, i64, i32]
        L.grpo_lmhead_workspace_bytes_for_chunk.restype = sz
        L.grpo_lmhead_workspace_bytes_for_chunk.argtypes = [i64, i64, i64, i64]
        L.grpo_lmhead_logprobs_fwd.restype = i32
        L.grpo_lmhead_logprobs_fwd.argtypes = [vp, i64, vp, i64, i64, i64, i64, vp, vp, f32, vp, vp, sz, vp]
        L.grpo_lmhead_loss_fwd_bwd.restype = i32
        L.grpo_lmhead_loss_fwd_bwd.argtypes = [vp, i64, vp, i64, i64, i64, i64, vp, vp, vp, vp, f32, f32,
                                               f32, f32, f64, f32, vp, vp, vp, vp, i64, vp, i64, i32,
                                               vp, sz, vp]
        L.grpo_lmhead_loss_aux_fwd_bwd.restype = i32
        L.grpo_lmhead_loss_aux_fwd_bwd.argtypes = [vp, i64, vp, i64, i64, i64, i64, vp, vp, vp, vp, vp, vp,
                                                   f32, f32, f32, f32, f32, f32, f64, f32, vp, vp, vp, vp,
                                                   vp, i64, vp, i64, i32, vp, sz, vp]
        _lib = L
    return _lib


def status_string(status) -> str:
    return lib().grpo_status_string(int(status)).decode()


def grpo_workspace_bytes(n_tokens: int) -> int:
    return int(lib().grpo_workspace_bytes(int(n_tokens)))


class RowPlan(ctypes.Structure):
    """grpo_row_plan of grpo.h."""
    _fields_ = [("vectors", ctypes.c_int64), ("resident_vectors", ctypes.c_int64), ("streaming", ctypes.c_int32),
                ("lanes", ctypes.c_int32), ("register_slots", ctypes.c_int32), ("lds_slots", ctypes.c_int32),
                ("workgroups_per_cu", ctypes.c_int32), ("ragged_tail_slot", ctypes.c_int32),
                ("streamed_remainder", ctypes.c_int32), ("reserved", ctypes.c_int32)]


def grpo_row_kernel_plan(dtype: int, vocab: int) -> dict:
    """Which row kernel serves rows of this width; see grpo_row_kernel_plan in grpo.h."""
    plan = RowPlan()
    rc = lib().grpo_row_kernel_plan(int(dtype), int(vocab), ctypes.byref(plan))
    if rc != 0:
        raise GrpoError(rc, "grpo_row_kernel_plan")
    return {name: int(getattr(plan, name)) for name, _ in RowPlan._fields_ if name != "reserved"}


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def _check(t, dtype, n, name, device):
    if t.dtype != dtype or t.dim() != 1 or t.shape[0] != n or not t.is_contiguous():
        raise ValueError("%s must be a contiguous %s tensor of length %d" % (name, dtype, n))
    if t.device != device:
        raise ValueError("%s must live on %s" % (name, device))


def _logits_args(logits, vocab):
    if logits.dim() != 2 or logits.stride(1) != 1:
        raise ValueError("logits must be [n_tokens, vocab] with unit stride along the vocabulary")
    if not logits.is_cuda:
        raise ValueError("logits must be a device tensor: libgrpo has no CPU path")
    if logits.dtype == torch.bfloat16:
        dt = GRPO_BF16
    elif logits.dtype == torch.float32:
        dt = GRPO_F32
    else:
        raise ValueError("logits must be bfloat16 or float32")
    n = logits.shape[0]
    v = logits.shape[1] if vocab is None else int(vocab)
    stride = logits.stride(0) if n > 1 else max(logits.stride(0), v)
    return dt, n, v, stride


def grpo_group_advantages(rewards, group_size=None, group_offsets=None, eps_std=1e-6, ddof=0,
                          rollout_of_token=None, adv_out=None, adv_tok_out=None, stream=None):
    """Returns (adv [n_rollouts], adv_tok [n_tokens] or None); see grpo_group_advantages in grpo.h."""
    dev = rewards.device
    R = rewards.shape[0]
    _check(rewards, torch.float32, R, "rewards", dev)
    if group_offsets is not None:
        _check(group_offsets, torch.int32, group_offsets.shape[0], "group_offsets", dev)
        n_groups, gs = group_offsets.shape[0] - 1, 0
    else:
        gs = int(group_size)
        n_groups = R // gs if gs > 0 else 0
    if adv_out is None:
        adv_out = torch.empty(R, dtype=torch.float32, device=dev)
    n_tok = 0
    if rollout_of_token is not None:
        n_tok = rollout_of_token.shape[0]
        _check(rollout_of_token, torch.int32, n_tok, "rollout_of_token", dev)
        if adv_tok_out is None:
            adv_tok_out = torch.empty(n_tok, dtype=torch.float32, device=dev)
    rc = lib().grpo_group_advantages(_ptr(rewards), R, _ptr(group_offsets), n_groups, gs,
                                     float(eps_std), int(ddof), _ptr(adv_out),
                                     _ptr(rollout_of_token), n_tok, _ptr(adv_tok_out),
                                     _stream(stream))
    if rc != GRPO_OK:
        raise GrpoError(rc, "grpo_group_advantages")
    return adv_out, adv_tok_out


_queue_workspaces = {}


def _queue_workspace(device, stream):
    """The small workspace grpo_logprobs_fwd's row queue lives in, one per device and stream, made
    on first use and kept: calls on one stream run one after the other, so they can share it, and
    the call does not allocate again (calls on different streams may overlap and must not)."""
    if stream is None:
        stream = torch.cuda.current_stream(device)
    key = (device.index if device.index is not None else torch.cuda.current_device(), stream.cuda_stream)
    ws = _queue_workspaces.get(key)
    if ws is None:
        ws = torch.empty(grpo_workspace_bytes(0), dtype=torch.uint8, device=device)
        if not torch.cuda.is_current_stream_capturing():   # memory made under capture belongs to that graph
            _queue_workspaces[key] = ws
    return ws


def grpo_logprobs_fwd(logits, tokens, mask=None, temperature=1.0, vocab=None, logprobs_out=None,
                      workspace=None, use_queue=True, stream=None):
    """log softmax(logits / T)[tokens] per row; see grpo_logprobs_fwd in grpo.h.
    Unless a workspace is passed or ``use_queue`` is False, the row queue uses a small
    workspace this module keeps per device and stream."""
    dt, n, v, stride = _logits_args(logits, vocab)
    dev = logits.device
    _check(tokens, torch.int64, n, "tokens", dev)
    if mask is not None:
        _check(mask, torch.uint8, n, "mask", dev)
    if logprobs_out is None:
        logprobs_out = torch.empty(n, dtype=torch.float32, device=dev)
    if workspace is None and use_queue and n > 0:
        workspace = _queue_workspace(dev, stream)
    rc = lib().grpo_logprobs_fwd(_ptr(logits), dt, n, v, stride, _ptr(tokens), _ptr(mask),
                                 float(temperature), _ptr(logprobs_out), _ptr(workspace),
                                 0 if workspace is None else workspace.numel(), _stream(stream))
    if rc != GRPO_OK:
        raise GrpoError(rc, "grpo_logprobs_fwd")
    return logprobs_out


def grpo_loss_fwd_bwd(logits, tokens, old_logprobs, advantages, mask=None, eps_low=0.2,
                      eps_high=0.2, delta=4.0, temperature=1.0, denom=0.0, grad_scale=1.0, *,
                      vocab=None, grad_logits=None, inplace=False, loss_out=None,
                      logprobs_out=None, counts_out=None, workspace=None, stream=None):
    """Objective forward + fused backward; see grpo_loss_fwd_bwd in grpo.h.

    Returns (loss [1] f32, logprobs [n] f32, counts [5] i64, grad_logits), all on the device and
    valid once the stream has run.  ``inplace=True`` writes the gradient over the logits.
    """
    dt, n, v, stride = _logits_args(logits, vocab)
    dev = logits.device
    _check(tokens, torch.int64, n, "tokens", dev)
    _check(old_logprobs, torch.float32, n, "old_logprobs", dev)
    _check(advantages, torch.float32, n, "advantages", dev)
    if mask is not None:
        _check(mask, torch.uint8, n, "mask", dev)
    if inplace:
        grad_logits = logits
    elif grad_logits is None:
        grad_logits = torch.empty_strided(logits.shape, logits.stride(), dtype=logits.dtype, device=dev)
    elif grad_logits.dtype != logits.dtype or grad_logits.shape != logits.shape or \
            grad_logits.stride() != logits.stride():
        raise ValueError("grad_logits must match logits in dtype, shape and strides")
    if loss_out is None:
        loss_out = torch.empty(1, dtype=torch.float32, device=dev)
    if logprobs_out is None:
        logprobs_out = torch.empty(n, dtype=torch.float32, device=dev)
    if counts_out is None:
        counts_out = torch.empty(5, dtype=torch.int64, device=dev)
    need = grpo_workspace_bytes(n)
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=dev)
    rc = lib().grpo_loss_fwd_bwd(_ptr(logits), dt, n, v, stride, _ptr(tokens), _ptr(old_logprobs),
                                 _ptr(advantages), _ptr(mask), float(eps_low), float(eps_high),
                                 float(delta), float(temperature), float(denom), float(grad_scale),
                                 _ptr(loss_out), _ptr(logprobs_out), _ptr(counts_out),
                                 _ptr(grad_logits), _ptr(workspace), workspace.numel(),
                                 _stream(stream))
    if rc != GRPO_OK:
        raise GrpoError(rc, "grpo_loss_fwd_bwd")
    return loss_out, logprobs_out, counts_out, grad_logits


NOALLOC_MAX_TOKENS = 524288  # GRPO_NOALLOC_MAX_TOKENS of grpo.h


def grpo_loss_fwd_bwd_noalloc(logits, tokens, old_logprobs, advantages, mask, eps_low, eps_high, delta,
                              temperature, denom, grad_scale, *, grad_logits, loss_out, logprobs_out=None,
                              counts_out=None, error_out=None, vocab=None, stream=None):
    """grpo_loss_fwd_bwd without a workspace; see grpo_loss_fwd_bwd_noalloc in grpo.h.  This wrapper
    allocates nothing either: every output tensor is the caller's (grad_logits may be the logits
    tensor itself).  Returns None; results are in the tensors passed."""
    dt, n, v, stride = _logits_args(logits, vocab)
    dev = logits.device
    _check(tokens, torch.int64, n, "tokens", dev)
    _check(old_logprobs, torch.float32, n, "old_logprobs", dev)
    _check(advantages, torch.float32, n, "advantages", dev)
    if mask is not None:
        _check(mask, torch.uint8, n, "mask", dev)
    if grad_logits.dtype != logits.dtype or grad_logits.shape != logits.shape or \
            grad_logits.stride() != logits.stride():
        raise ValueError("grad_logits must match logits in dtype, shape and strides")
    _check(loss_out, torch.float32, 1, "loss_out", dev)
    if logprobs_out is not None:
        _check(logprobs_out, torch.float32, n, "logprobs_out", dev)
    if counts_out is not None:
        _check(counts_out, torch.int64, 5, "counts_out", dev)
    if error_out is not None:
        _check(error_out, torch.int32, 1, "error_out", dev)
    rc = lib().grpo_loss_fwd_bwd_noalloc(_ptr(logits), dt, n, v, stride, _ptr(tokens), _ptr(old_logprobs),
                                         _ptr(advantages), _ptr(mask), float(eps_low), float(eps_high),
                                         float(delta), float(temperature), float(denom), float(grad_scale),
                                         _ptr(loss_out), _ptr(logprobs_out), _ptr(counts_out),
                                         _ptr(grad_logits), _ptr(error_out), _stream(stream))
    if rc != GRPO_OK:
        raise GrpoError(rc, "grpo_loss_fwd_bwd_noalloc")


def grpo_loss_aux_fwd_bwd(logits, tokens, old_logprobs, ref_logprobs, advantages, mask=None,
                          eps_low=0.2, eps_high=0.2, delta=4.0, temperature=1.0, kl_coef=0.0,
                          entropy_coef=0.0, denom=0.0, grad_scale=1.0, *, token_weights=None,
                          vocab=None, grad_logits=None, inplace=False, loss_out=None, logprobs_out=None,
                          entropy_out=None, want_entropy=True, counts_out=None, workspace=None,
                          stream=None):
    """Objective with the KL and entropy terms fused in; see grpo_loss_aux_fwd_bwd in grpo.h.

    Returns (loss [4] f32: total, policy, mean kl, mean entropy; logprobs [n]; entropy [n] or
    None; counts [5] i64; grad_logits)."""
    dt, n, v, stride = _logits_args(logits, vocab)
    dev = logits.device
    _check(tokens, torch.int64, n, "tokens", dev)
    _check(old_logprobs, torch.float32, n, "old_logprobs", dev)
    _check(advantages, torch.float32, n, "advantages", dev)
    if ref_logprobs is not None:
        _check(ref_logprobs, torch.float32, n, "ref_logprobs", dev)
    if token_weights is not None:
        _check(token_weights, torch.float32, n, "token_weights", dev)
    if mask is not None:
        _check(mask, torch.uint8, n, "mask", dev)
    if inplace:
        grad_logits = logits
    elif grad_logits is None:
        grad_logits = torch.empty_strided(logits.shape, logits.stride(), dtype=logits.dtype, device=dev)
    elif grad_logits.dtype != logits.dtype or grad_logits.shape != logits.shape or \
            grad_logits.stride() != logits.stride():
        raise ValueError("grad_logits must match logits in dtype, shape and strides")
    if loss_out is None:
        loss_out = torch.empty(4, dtype=torch.float32, device=dev)
    if logprobs_out is None:
        logprobs_out = torch.empty(n, dtype=torch.float32, device=dev)
    if entropy_out is None and want_entropy:
        entropy_out = torch.empty(n, dtype=torch.float32, device=dev)
    if counts_out is None:
        counts_out = torch.empty(5, dtype=torch.int64, device=dev)
    if workspace is None:
        workspace = torch.empty(grpo_workspace_bytes(n), dtype=torch.uint8, device=dev)
    rc = lib().grpo_loss_aux_fwd_bwd(
        _ptr(logits), dt, n, v, stride, _ptr(tokens), _ptr(old_logprobs), _ptr(ref_logprobs),
        _ptr(advantages), _ptr(mask), _ptr(token_weights), float(eps_low), float(eps_high),
        float(delta), float(temperature), float(kl_coef), float(entropy_coef), float(denom),
        float(grad_scale),
        _ptr(loss_out), _ptr(logprobs_out), _ptr(entropy_out), _ptr(counts_out), _ptr(grad_logits),
        _ptr(workspace), workspace.numel(), _stream(stream))
    if rc != GRPO_OK:
        raise GrpoError(rc, "grpo_loss_aux_fwd_bwd")
    return loss_out, logprobs_out, entropy_out, counts_out, grad_logits


def grpo_total_rewards(task_rewards, lengths, target_lengths, alpha, rewards_out=None, stream=None):
    """r_task - alpha |l_target - l_y| per rollout; see grpo_total_rewards in grpo.h."""
    dev = task_rewards.device
    R = task_rewards.shape[0]
    _check(task_rewards, torch.float32, R, "task_rewards", dev)
    _check(lengths, torch.int32, R, "lengths", dev)
    _check(target_lengths, torch.int32, R, "target_lengths", dev)
    if rewards_out is None:
        rewards_out = torch.empty(R, dtype=torch.float32, device=dev)
    rc = lib().grpo_total_rewards(_ptr(task_rewards), _ptr(lengths), _ptr(target_lengths), R,
                                  float(alpha), _ptr(rewards_out), _stream(stream))
    if rc != GRPO_OK:
        raise GrpoError(rc, "grpo_total_rewards")
    return rewards_out


def grpo_filter_groups(rewards, group_size=None, group_offsets=None, stream=None):
    """Returns (keep u8 [n_groups], kept_groups i32 [n_groups], n_kept i32 [1], rollout_keep u8 [R]);
    see grpo_filter_groups in grpo.h."""
    dev = rewards.device
    R = rewards.shape[0]
    _check(rewards, torch.float32, R, "rewards", dev)
    if group_offsets is not None:
        _check(group_offsets, torch.int32, group_offsets.shape[0], "group_offsets", dev)
        n_groups, gs = group_offsets.shape[0] - 1, 0
    else:
        gs = int(group_size)
        n_groups = R // gs if gs > 0 else 0
    keep = torch.empty(n_groups, dtype=torch.uint8, device=dev)
    kept = torch.empty(n_groups, dtype=torch.int32, device=dev)
    n_kept = torch.empty(1, dtype=torch.int32, device=dev)
    rk = torch.zeros(R, dtype=torch.uint8, device=dev)
    rc = lib().grpo_filter_groups(_ptr(rewards), R, _ptr(group_offsets), n_groups, gs, _ptr(keep),
                                  _ptr(kept), _ptr(n_kept), _ptr(rk), _stream(stream))
    if rc != GRPO_OK:
        raise GrpoError(rc, "grpo_filter_groups")
    return keep, kept, n_kept, rk


def grpo_packed_layout(cu_seqlens, n_tokens, sample_level, weights_out=None, rollout_of_token_out=None,
                       stream=None):
    """(weights f32 [n_tokens], rollout_of_token i32 [n_tokens]) of a packed batch whose rollout i
    owns rows [cu_seqlens[i], cu_seqlens[i+1]); see grpo_packed_layout in grpo.h."""
    dev = cu_seqlens.device
    _check(cu_seqlens, torch.int64, cu_seqlens.shape[0], "cu_seqlens", dev)
    if weights_out is None:
        weights_out = torch.empty(n_tokens, dtype=torch.float32, device=dev)
    if rollout_of_token_out is None:
        rollout_of_token_out = torch.empty(n_tokens, dtype=torch.int32, device=dev)
    rc = lib().grpo_packed_layout(_ptr(cu_seqlens), cu_seqlens.shape[0] - 1, int(n_tokens),
                                  1 if sample_level else 0, _ptr(weights_out),
                                  _ptr(rollout_of_token_out), _stream(stream))
    if rc != GRPO_OK:
        raise GrpoError(rc, "grpo_packed_layout")
    return weights_out, rollout_of_token_out


def grpo_workspace_error(workspace, stream=None) -> int:
    flag = ctypes.c_int32(0)
    rc = lib().grpo_workspace_error(_ptr(workspace), ctypes.byref(flag), _stream(stream))
    if rc != GRPO_OK:
        raise GrpoError(rc, "grpo_workspace_error")
    return int(flag.value)


def grpo_lmhead_workspace_bytes(n_tokens: int, vocab: int, d_model: int, with_backward: bool) -> int:
    return int(lib().grpo_lmhead_workspace_bytes(int(n_tokens), int(vocab), int(d_model),
                                                 1 if with_backward else 0))


def grpo_lmhead_workspace_bytes_for_chunk(n_tokens: int, vocab: int, d_model: int, chunk_rows: int) -> int:
    """Workspace of the backward when it works through the rows in chunks of ``chunk_rows``."""
    return int(lib().grpo_lmhead_workspace_bytes_for_chunk(int(n_tokens), int(vocab), int(d_model),
                                                           int(chunk_rows)))


def _lmhead_args(hidden, weight):
    for name, t in (("hidden", hidden), ("weight", weight)):
        if t.dim() != 2 or t.stride(1) != 1 or t.dtype != torch.bfloat16 or not t.is_cuda:
            raise ValueError("%s must be a 2-D bfloat16 device tensor with unit stride along d_model" % name)
    n, d = hidden.shape
    v = weight.shape[0]
    if weight.shape[1] != d:
        raise ValueError("hidden is [n_tokens, d_model] and weight [vocab, d_model]: d_model differs")
    hs = hidden.stride(0) if n > 1 else max(hidden.stride(0), d)
    ws = weight.stride(0) if v > 1 else max(weight.stride(0), d)
    return n, v, d, hs, ws


def grpo_lmhead_logprobs_fwd(hidden, weight, tokens, mask=None, temperature=1.0, logprobs_out=None,
                             workspace=None, stream=None):
    """log softmax(hidden @ weight.T / T)[tokens] per row without materialising the logits; see
    grpo_lmhead_logprobs_fwd in grpo.h."""
    n, v, d, hs, ws = _lmhead_args(hidden, weight)
    dev = hidden.device
    _check(tokens, torch.int64, n, "tokens", dev)
    if mask is not None:
        _check(mask, torch.uint8, n, "mask", dev)
    if logprobs_out is None:
        logprobs_out = torch.empty(n, dtype=torch.float32, device=dev)
    if workspace is None:
        workspace = torch.empty(grpo_lmhead_workspace_bytes(n, v, d, False), dtype=torch.uint8, device=dev)
    rc = lib().grpo_lmhead_logprobs_fwd(_ptr(hidden), hs, _ptr(weight), ws, n, v, d, _ptr(tokens),
                                        _ptr(mask), float(temperature), _ptr(logprobs_out),
                                        _ptr(workspace), workspace.numel(), _stream(stream))
    if rc != GRPO_OK:
        raise GrpoError(rc, "grpo_lmhead_logprobs_fwd")
    return logprobs_out


def grpo_lmhead_loss_fwd_bwd(hidden, weight, tokens, old_logprobs, advantages, mask=None, eps_low=0.2,
                             eps_high=0.2, delta=4.0, temperature=1.0, denom=0.0, grad_scale=1.0, *,
                             grad_hidden=None, grad_weight=None, accumulate_grad_weight=False,
                             loss_out=None, logprobs_out=None, counts_out=None, workspace=None,
                             stream=None):
    """Objective on hidden @ weight.T with gradients for both operands; see
    grpo_lmhead_loss_fwd_bwd in grpo.h.  Returns (loss [1], logprobs [n], counts [5],
    grad_hidden bf16 [n, d], grad_weight f32 [vocab, d])."""
    n, v, d, hs, ws = _lmhead_args(hidden, weight)
    dev = hidden.device
    _check(tokens, torch.int64, n, "tokens", dev)
    _check(old_logprobs, torch.float32, n, "old_logprobs", dev)
    _check(advantages, torch.float32, n, "advantages", dev)
    if mask is not None:
        _check(mask, torch.uint8, n, "mask", dev)
    if grad_hidden is None:
        grad_hidden = torch.empty((n, d), dtype=torch.bfloat16, device=dev)
    if grad_weight is None:
        if accumulate_grad_weight:
            raise ValueError("accumulate_grad_weight needs the grad_weight tensor to add to")
        grad_weight = torch.empty((v, d), dtype=torch.float32, device=dev)
    if grad_hidden.dtype != torch.bfloat16 or grad_hidden.shape != (n, d) or grad_hidden.stride(1) != 1:
        raise ValueError("grad_hidden must be bfloat16 [n_tokens, d_model] with unit inner stride")
    if grad_weight.dtype != torch.float32 or grad_weight.shape != (v, d) or grad_weight.stride(1) != 1:
        raise ValueError("grad_weight must be float32 [vocab, d_model] with unit inner stride")
    if loss_out is None:
        loss_out = torch.empty(1, dtype=torch.float32, device=dev)
    if logprobs_out is None:
        logprobs_out = torch.empty(n, dtype=torch.float32, device=dev)
    if counts_out is None:
        counts_out = torch.empty(5, dtype=torch.int64, device=dev)
    if workspace is None:
        workspace = torch.empty(grpo_lmhead_workspace_bytes(n, v, d, True), dtype=torch.uint8, device=dev)
    ghs = grad_hidden.stride(0) if n > 1 else max(grad_hidden.stride(0), d)
    gws = grad_weight.stride(0) if v > 1 else max(grad_weight.stride(0), d)
    rc = lib().grpo_lmhead_loss_fwd_bwd(
        _ptr(hidden), hs, _ptr(weight), ws, n, v, d, _ptr(tokens), _ptr(old_logprobs), _ptr(advantages),
        _ptr(mask), float(eps_low), float(eps_high), float(delta), float(temperature), float(denom),
        float(grad_scale), _ptr(loss_out), _ptr(logprobs_out), _ptr(counts_out), _ptr(grad_hidden), ghs,
        _ptr(grad_weight), gws, 1 if accumulate_grad_weight else 0, _ptr(workspace), workspace.numel(),
        _stream(stream))
    if rc != GRPO_OK:
        raise GrpoError(rc, "grpo_lmhead_loss_fwd_bwd")
    return loss_out, logprobs_out, counts_out, grad_hidden, grad_weight


def grpo_lmhead_loss_aux_fwd_bwd(hidden, weight, tokens, old_logprobs, ref_logprobs, advantages, mask=None,
                                 eps_low=0.2, eps_high=0.2, delta=4.0, temperature=1.0, kl_coef=0.0,
                                 entropy_coef=0.0, denom=0.0, grad_scale=1.0, *, token_weights=None,
                                 grad_hidden=None, grad_weight=None, accumulate_grad_weight=False,
                                 loss_out=None, logprobs_out=None, entropy_out=None, want_entropy=True,
                                 counts_out=None, workspace=None, stream=None):
    """Total objective (policy + KL - entropy bonus, per-token weights) on hidden @ weight.T with
    gradients for both operands; see grpo_lmhead_loss_aux_fwd_bwd in grpo.h.  Returns (loss [4]:
    total, policy, mean kl, mean entropy; logprobs [n]; entropy [n] or None; counts [5];
    grad_hidden bf16 [n, d]; grad_weight f32 [vocab, d])."""
    n, v, d, hs, ws = _lmhead_args(hidden, weight)
    dev = hidden.device
    _check(tokens, torch.int64, n, "tokens", dev)
    _check(old_logprobs, torch.float32, n, "old_logprobs", dev)
    _check(advantages, torch.float32, n, "advantages", dev)
    if ref_logprobs is not None:
        _check(ref_logprobs, torch.float32, n, "ref_logprobs", dev)
    if token_weights is not None:
        _check(token_weights, torch.float32, n, "token_weights", dev)
    if mask is not None:
        _check(mask, torch.uint8, n, "mask", dev)
    if grad_hidden is None:
        grad_hidden = torch.empty((n, d), dtype=torch.bfloat16, device=dev)
    if grad_weight is None:
        if accumulate_grad_weight:
            raise ValueError("accumulate_grad_weight needs the grad_weight tensor to add to")
        grad_weight = torch.empty((v, d), dtype=torch.float32, device=dev)
    if grad_hidden.dtype != torch.bfloat16 or grad_hidden.shape != (n, d) or grad_hidden.stride(1) != 1:
        raise ValueError("grad_hidden must be bfloat16 [n_tokens, d_model] with unit inner stride")
    if grad_weight.dtype != torch.float32 or grad_weight.shape != (v, d) or grad_weight.stride(1) != 1:
        raise ValueError("grad_weight must be float32 [vocab, d_model] with unit inner stride")
    if loss_out is None:
        loss_out = torch.empty(4, dtype=torch.float32, device=dev)
    if logprobs_out is None:
        logprobs_out = torch.empty(n, dtype=torch.float32, device=dev)
    if entropy_out is None and want_entropy:
        entropy_out = torch.empty(n, dtype=torch.float32, device=dev)
    if counts_out is None:
        counts_out = torch.empty(5, dtype=torch.int64, device=dev)
    if workspace is None:
        workspace = torch.empty(grpo_lmhead_workspace_bytes(n, v, d, True), dtype=torch.uint8, device=dev)
    ghs = grad_hidden.stride(0) if n > 1 else max(grad_hidden.stride(0), d)
    gws = grad_weight.stride(0) if v > 1 else max(grad_weight.stride(0), d)
    rc = lib().grpo_lmhead_loss_aux_fwd_bwd(
        _ptr(hidden), hs, _ptr(weight), ws, n, v, d, _ptr(tokens), _ptr(old_logprobs), _ptr(ref_logprobs),
        _ptr(advantages), _ptr(mask), _ptr(token_weights), float(eps_low), float(eps_high), float(delta),
        float(temperature), float(kl_coef), float(entropy_coef), float(denom), float(grad_scale),
        _ptr(loss_out), _ptr(logprobs_out), _ptr(entropy_out), _ptr(counts_out), _ptr(grad_hidden), ghs,
        _ptr(grad_weight), gws, 1 if accumulate_grad_weight else 0, _ptr(workspace), workspace.numel(),
        _stream(stream))
    if rc != GRPO_OK:
        raise GrpoError(rc, "grpo_lmhead_loss_aux_fwd_bwd")
    return loss_out, logprobs_out, entropy_out, counts_out, grad_hidden, grad_weight
