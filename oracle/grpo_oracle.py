"""ctypes front end of the fp64 CPU oracle (``grpo_oracle.c``).

TEST INFRASTRUCTURE ONLY: the tests, the smoke check and the benchmark's
``cpu_baseline`` leg may import this module; the product package never does.
Everything here is argument marshalling for numpy arrays; the arithmetic lives
in the C file next to it, which follows section 3.4 of the paper step by step.

bf16 logits are passed as ``uint16`` arrays holding the raw bit patterns.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "grpo_oracle.c")
_LIB = os.path.join(_HERE, "libgrpo_oracle.so")

F32, BF16, F64 = 0, 1, 2
FLAG_CLIP_HIGH, FLAG_CLIP_LOW, FLAG_DELTA, FLAG_OUT_OF_BAND = 1, 2, 4, 8

_lib = None


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (about a second)."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-std=c99", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
             "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _p(a, ct):
    return None if a is None else a.ctypes.data_as(ctypes.POINTER(ct))


def lib():
    global _lib
    if _lib is None:
        L = ctypes.CDLL(build())
        i64, dbl, i32 = ctypes.c_int64, ctypes.c_double, ctypes.c_int
        vp = ctypes.c_void_p
        L.oracle_group_advantages.restype = i32
        L.oracle_group_advantages.argtypes = [vp, i64, vp, i64, i64, dbl, i32, vp]
        L.oracle_broadcast_advantages.restype = None
        L.oracle_broadcast_advantages.argtypes = [vp, vp, i64, vp]
        L.oracle_row_log_softmax.restype = dbl
        L.oracle_row_log_softmax.argtypes = [vp, i32, i64, dbl, vp]
        L.oracle_logprobs.restype = i32
        L.oracle_logprobs.argtypes = [vp, i32, i64, i64, i64, vp, vp, dbl, vp]
        L.oracle_surrogate_from_ratio.restype = None
        L.oracle_surrogate_from_ratio.argtypes = [dbl, dbl, dbl, dbl, dbl, vp, vp, vp]
        L.oracle_loss_fwd_bwd.restype = i32
        L.oracle_loss_fwd_bwd.argtypes = [vp, i32, i64, i64, i64, vp, vp, vp, vp,
                                          dbl, dbl, dbl, dbl, dbl, dbl,
                                          vp, vp, vp, vp, vp, vp, vp, i64, vp]
        L.oracle_objective_from_logprobs.restype = None
        L.oracle_objective_from_logprobs.argtypes = [i64, vp, vp, vp, vp, dbl, dbl, dbl, dbl, dbl,
                                                     vp, vp, vp, vp, vp]
        L.oracle_grad_rows.restype = None
        L.oracle_grad_rows.argtypes = [vp, i32, i64, i64, vp, vp, dbl, vp, i64, vp]
        L.oracle_row_entropy.restype = dbl
        L.oracle_row_entropy.argtypes = [vp, i32, i64, dbl]
        L.oracle_kl_estimator.restype = None
        L.oracle_kl_estimator.argtypes = [dbl, dbl, vp, vp]
        L.oracle_entropies.restype = i32
        L.oracle_entropies.argtypes = [vp, i32, i64, i64, i64, vp, dbl, vp]
        L.oracle_aux_objective_from_logprobs.restype = None
        L.oracle_aux_objective_from_logprobs.argtypes = [i64, vp, vp, vp, vp, vp, vp, vp, dbl, dbl, dbl,
                                                         dbl, dbl, dbl, dbl, vp, vp, vp, vp, vp]
        L.oracle_packed_layout.restype = i32
        L.oracle_packed_layout.argtypes = [vp, i64, i64, i32, vp, vp]
        L.oracle_aux_grad_rows.restype = None
        L.oracle_aux_grad_rows.argtypes = [vp, i32, i64, i64, vp, vp, vp, dbl, vp, i64, vp]
        L.oracle_total_rewards.restype = None
        L.oracle_total_rewards.argtypes = [vp, vp, vp, i64, dbl, vp]
        L.oracle_filter_groups.restype = i32
        L.oracle_filter_groups.argtypes = [vp, i64, vp, i64, i64, vp, vp, vp, vp]
        L.oracle_lmhead_logits.restype = i32
        L.oracle_lmhead_logits.argtypes = [vp, i32, i64, i64, vp, i32, i64, i64, vp, i64, vp]
        L.oracle_lmhead_grad_hidden.restype = i32
        L.oracle_lmhead_grad_hidden.argtypes = [vp, i64, i64, vp, i32, i64, i64, vp]
        L.oracle_lmhead_grad_weight.restype = i32
        L.oracle_lmhead_grad_weight.argtypes = [vp, i64, i64, vp, i32, i64, i64, vp, i64, vp]
        L.oracle_num_threads.restype = i32
        L.oracle_num_threads.argtypes = []
        L.oracle_set_num_threads.restype = None
        L.oracle_set_num_threads.argtypes = [i32]
        _lib = L
    return _lib


def _ptr(a):
    return None if a is None else ctypes.c_void_p(a.ctypes.data)


def _logits_view(logits):
    """Accept float32, float64 or uint16 (bf16 bit patterns) [N, S] with contiguous rows."""
    a = np.asarray(logits)
    if a.ndim == 1:
        a = a[None, :]
    assert a.ndim == 2 and a.strides[1] == a.itemsize, "rows must be contiguous"
    if a.dtype == np.float32:
        dt = F32
    elif a.dtype == np.uint16:
        dt = BF16
    elif a.dtype == np.float64:
        dt = F64
    else:
        raise TypeError("logits must be float32, float64 or uint16 (bf16 bits), got %s" % a.dtype)
    assert a.strides[0] % a.itemsize == 0
    return a, dt, a.strides[0] // a.itemsize


def num_threads() -> int:
    return int(lib().oracle_num_threads())


def set_num_threads(n: int) -> None:
    """Threads used by the row loops from now on (results do not depend on it)."""
    lib().oracle_set_num_threads(int(n))


def group_advantages(rewards, group_size=None, group_offsets=None, eps_std=1e-6, ddof=0):
    rewards = np.ascontiguousarray(rewards, dtype=np.float32)
    R = rewards.shape[0]
    if group_offsets is not None:
        off = np.ascontiguousarray(group_offsets, dtype=np.int32)
        n_groups, gs = off.shape[0] - 1, 0
    else:
        off = None
        assert group_size and R % group_size == 0
        n_groups, gs = R // group_size, int(group_size)
    out = np.zeros(R, dtype=np.float64)
    rc = lib().oracle_group_advantages(_ptr(rewards), R, _ptr(off), n_groups, gs,
                                       float(eps_std), int(ddof), _ptr(out))
    if rc:
        raise ValueError("oracle_group_advantages: bad group offsets")
    return out


def broadcast_advantages(adv, rollout_of_token):
    adv = np.ascontiguousarray(adv, dtype=np.float64)
    rot = np.ascontiguousarray(rollout_of_token, dtype=np.int32)
    out = np.zeros(rot.shape[0], dtype=np.float64)
    lib().oracle_broadcast_advantages(_ptr(adv), _ptr(rot), rot.shape[0], _ptr(out))
    return out


def row_log_softmax(row, V=None, temperature=1.0):
    a, dt, _ = _logits_view(row)
    V = a.shape[1] if V is None else V
    out = np.zeros(V, dtype=np.float64)
    lse = lib().oracle_row_log_softmax(_ptr(a), dt, V, float(temperature), _ptr(out))
    return out, float(lse)


def logprobs(logits, tokens, mask=None, temperature=1.0, vocab=None):
    a, dt, stride = _logits_view(logits)
    N = a.shape[0]
    V = a.shape[1] if vocab is None else vocab
    tokens = np.ascontiguousarray(tokens, dtype=np.int64)
    m = None if mask is None else np.ascontiguousarray(mask, dtype=np.uint8)
    out = np.zeros(N, dtype=np.float64)
    rc = lib().oracle_logprobs(_ptr(a), dt, N, V, stride, _ptr(tokens), _ptr(m),
                               float(temperature), _ptr(out))
    if rc:
        raise ValueError("oracle_logprobs: token id out of range (rc=%d)" % rc)
    return out


def surrogate_from_ratio(r, A, eps_low, eps_high, delta):
    """Returns (J, dJ/dlogp, flags) for one exact ratio r and advantage A."""
    J, dJ, fl = ctypes.c_double(), ctypes.c_double(), ctypes.c_int()
    lib().oracle_surrogate_from_ratio(float(r), float(A), float(eps_low), float(eps_high),
                                      float(delta), ctypes.byref(J), ctypes.byref(dJ),
                                      ctypes.byref(fl))
    return J.value, dJ.value, fl.value


def loss_fwd_bwd(logits, tokens, old_logprobs, advantages, mask=None, *, eps_low=0.2,
                 eps_high=0.2, delta=4.0, temperature=1.0, denom=0.0, grad_scale=1.0,
                 grad_rows=None, vocab=None):
    """Full objective.  Returns a dict with loss, logprobs, counts, J, coeff, flags and,
    for the row indices in ``grad_rows`` ("all" = every row), dense fp64 gradient rows."""
    a, dt, stride = _logits_view(logits)
    N = a.shape[0]
    V = a.shape[1] if vocab is None else vocab
    tokens = np.ascontiguousarray(tokens, dtype=np.int64)
    old = np.ascontiguousarray(old_logprobs, dtype=np.float32)
    adv = np.ascontiguousarray(advantages, dtype=np.float32)
    m = None if mask is None else np.ascontiguousarray(mask, dtype=np.uint8)
    assert tokens.shape[0] == N and old.shape[0] == N and adv.shape[0] == N
    if isinstance(grad_rows, str) and grad_rows == "all":
        grad_rows = np.arange(N, dtype=np.int64)
    gr = None if grad_rows is None else np.ascontiguousarray(grad_rows, dtype=np.int64)
    n_gr = 0 if gr is None else gr.shape[0]
    grad = None if gr is None else np.zeros((n_gr, V), dtype=np.float64)
    loss = np.zeros(1, dtype=np.float64)
    lp = np.zeros(N, dtype=np.float64)
    counts = np.zeros(5, dtype=np.int64)
    J = np.zeros(N, dtype=np.float64)
    coeff = np.zeros(N, dtype=np.float64)
    flags = np.zeros(N, dtype=np.int32)
    rc = lib().oracle_loss_fwd_bwd(
        _ptr(a), dt, N, V, stride, _ptr(tokens), _ptr(old), _ptr(adv), _ptr(m),
        float(eps_low), float(eps_high), float(delta), float(temperature), float(denom),
        float(grad_scale), _ptr(loss), _ptr(lp), _ptr(counts), _ptr(J), _ptr(coeff),
        _ptr(flags), _ptr(gr), n_gr, _ptr(grad))
    if rc:
        raise ValueError("oracle_loss_fwd_bwd failed (rc=%d)" % rc)
    return dict(loss=float(loss[0]), logprobs=lp, counts=counts, J=J, coeff=coeff,
                flags=flags, grad=grad, grad_rows=gr)


def objective_from_logprobs(logprobs, old_logprobs, advantages, mask=None, *, eps_low=0.2,
                            eps_high=0.2, delta=4.0, denom=0.0, grad_scale=1.0):
    """Ratio, surrogate, masked token mean and counters from per-token log-probs."""
    lp = np.ascontiguousarray(logprobs, dtype=np.float64)
    N = lp.shape[0]
    old = np.ascontiguousarray(old_logprobs, dtype=np.float32)
    adv = np.ascontiguousarray(advantages, dtype=np.float32)
    m = None if mask is None else np.ascontiguousarray(mask, dtype=np.uint8)
    loss = np.zeros(1, dtype=np.float64)
    counts = np.zeros(5, dtype=np.int64)
    J = np.zeros(N, dtype=np.float64)
    coeff = np.zeros(N, dtype=np.float64)
    flags = np.zeros(N, dtype=np.int32)
    lib().oracle_objective_from_logprobs(N, _ptr(lp), _ptr(old), _ptr(adv), _ptr(m),
                                         float(eps_low), float(eps_high), float(delta),
                                         float(denom), float(grad_scale), _ptr(loss),
                                         _ptr(counts), _ptr(J), _ptr(coeff), _ptr(flags))
    return dict(loss=float(loss[0]), counts=counts, J=J, coeff=coeff, flags=flags)


def grad_rows(logits_rows, tokens_rows, coeff_rows, temperature=1.0, vocab=None):
    """Dense fp64 gradient rows for the given logits rows, their sampled tokens and their
    coefficients c_t (from objective_from_logprobs)."""
    a, dt, stride = _logits_view(logits_rows)
    K = a.shape[0]
    V = a.shape[1] if vocab is None else vocab
    tok = np.ascontiguousarray(tokens_rows, dtype=np.int64)
    cf = np.ascontiguousarray(coeff_rows, dtype=np.float64)
    idx = np.arange(K, dtype=np.int64)
    out = np.zeros((K, V), dtype=np.float64)
    lib().oracle_grad_rows(_ptr(a), dt, V, stride, _ptr(tok), _ptr(cf), float(temperature),
                           _ptr(idx), K, _ptr(out))
    return out


# ---------------------------------------------------------------------------
# auxiliary KL and entropy terms
# ---------------------------------------------------------------------------

def row_entropy(row, V=None, temperature=1.0):
    a, dt, _ = _logits_view(row)
    V = a.shape[1] if V is None else V
    return float(lib().oracle_row_entropy(_ptr(a), dt, V, float(temperature)))


def kl_estimator(l, l_ref):
    """(kl, dkl/dl) of the sampled-token estimator exp(d) - d - 1, d = l_ref - l."""
    kl, dkl = ctypes.c_double(), ctypes.c_double()
    lib().oracle_kl_estimator(float(l), float(l_ref), ctypes.byref(kl), ctypes.byref(dkl))
    return kl.value, dkl.value


def entropies(logits, mask=None, temperature=1.0, vocab=None):
    a, dt, stride = _logits_view(logits)
    N = a.shape[0]
    V = a.shape[1] if vocab is None else vocab
    m = None if mask is None else np.ascontiguousarray(mask, dtype=np.uint8)
    out = np.zeros(N, dtype=np.float64)
    lib().oracle_entropies(_ptr(a), dt, N, V, stride, _ptr(m), float(temperature), _ptr(out))
    return out


def packed_layout(cu_seqlens, n_tokens, sample_level):
    """(weights f32 [n_tokens], rollout_of_token i32 [n_tokens]) of a packed batch."""
    cu = np.ascontiguousarray(cu_seqlens, dtype=np.int64)
    w = np.zeros(n_tokens, dtype=np.float32)
    rot = np.zeros(n_tokens, dtype=np.int32)
    rc = lib().oracle_packed_layout(_ptr(cu), cu.shape[0] - 1, int(n_tokens), int(bool(sample_level)),
                                    _ptr(w), _ptr(rot))
    if rc:
        raise ValueError("oracle_packed_layout: bad cu_seqlens")
    return w, rot


def aux_objective_from_logprobs(logprobs, entropies_, old_logprobs, ref_logprobs, advantages,
                                mask=None, *, token_weights=None, eps_low=0.2, eps_high=0.2,
                                delta=4.0, kl_coef=0.0, ent_coef=0.0, denom=0.0, grad_scale=1.0):
    lp = np.ascontiguousarray(logprobs, dtype=np.float64)
    N = lp.shape[0]
    H = np.ascontiguousarray(entropies_, dtype=np.float64)
    old = np.ascontiguousarray(old_logprobs, dtype=np.float32)
    ref = None if ref_logprobs is None else np.ascontiguousarray(ref_logprobs, dtype=np.float32)
    adv = np.ascontiguousarray(advantages, dtype=np.float32)
    m = None if mask is None else np.ascontiguousarray(mask, dtype=np.uint8)
    tw = None if token_weights is None else np.ascontiguousarray(token_weights, dtype=np.float32)
    total = np.zeros(1, dtype=np.float64)
    aux = np.zeros(3, dtype=np.float64)
    counts = np.zeros(5, dtype=np.int64)
    coeff = np.zeros(N, dtype=np.float64)
    ent_coeff = np.zeros(N, dtype=np.float64)
    lib().oracle_aux_objective_from_logprobs(
        N, _ptr(lp), _ptr(H), _ptr(old), _ptr(ref), _ptr(adv), _ptr(m), _ptr(tw), float(eps_low),
        float(eps_high), float(delta), float(kl_coef), float(ent_coef), float(denom),
        float(grad_scale), _ptr(total), _ptr(aux), _ptr(counts), _ptr(coeff), _ptr(ent_coeff))
    return dict(total=float(total[0]), policy=float(aux[0]), kl=float(aux[1]),
                entropy=float(aux[2]), counts=counts, coeff=coeff, ent_coeff=ent_coeff)


def aux_grad_rows(logits_rows, tokens_rows, coeff_rows, ent_coeff_rows, temperature=1.0, vocab=None):
    a, dt, stride = _logits_view(logits_rows)
    K = a.shape[0]
    V = a.shape[1] if vocab is None else vocab
    tok = np.ascontiguousarray(tokens_rows, dtype=np.int64)
    cf = np.ascontiguousarray(coeff_rows, dtype=np.float64)
    ef = np.ascontiguousarray(ent_coeff_rows, dtype=np.float64)
    idx = np.arange(K, dtype=np.int64)
    out = np.zeros((K, V), dtype=np.float64)
    lib().oracle_aux_grad_rows(_ptr(a), dt, V, stride, _ptr(tok), _ptr(cf), _ptr(ef),
                               float(temperature), _ptr(idx), K, _ptr(out))
    return out


def aux_loss_fwd_bwd(logits, tokens, old_logprobs, ref_logprobs, advantages, mask=None, *,
                     token_weights=None, eps_low=0.2, eps_high=0.2, delta=4.0, temperature=1.0,
                     kl_coef=0.0, ent_coef=0.0, denom=0.0, grad_scale=1.0, grad_rows=None, vocab=None):
    """Total objective with the auxiliary terms in one call (composition of the stages)."""
    a, dt, stride = _logits_view(logits)
    N = a.shape[0]
    V = a.shape[1] if vocab is None else vocab
    live = None if mask is None else np.ascontiguousarray(mask, dtype=np.uint8).copy()
    if token_weights is not None:   # a row with zero weight counts as masked: it is never read
        nz = (np.asarray(token_weights, dtype=np.float32) != 0).astype(np.uint8)
        live = nz if live is None else (live & nz)
    lp = logprobs(a, tokens, live, temperature, vocab=V)
    H = entropies(a, live, temperature, vocab=V)
    obj = aux_objective_from_logprobs(lp, H, old_logprobs, ref_logprobs, advantages, mask,
                                      token_weights=token_weights, eps_low=eps_low, eps_high=eps_high, delta=delta,
                                      kl_coef=kl_coef, ent_coef=ent_coef, denom=denom,
                                      grad_scale=grad_scale)
    obj["logprobs"], obj["entropies"] = lp, H
    if grad_rows is not None:
        if isinstance(grad_rows, str):
            grad_rows = np.arange(N)
        gr = np.asarray(grad_rows, dtype=np.int64)
        tok = np.ascontiguousarray(tokens, dtype=np.int64)
        obj["grad"] = aux_grad_rows(a[gr], tok[gr], obj["coeff"][gr], obj["ent_coeff"][gr],
                                    temperature, vocab=V)
    return obj


# ---------------------------------------------------------------------------
# reward shaping and online filtering
# ---------------------------------------------------------------------------

def total_rewards(task_rewards, lengths, target_lengths, alpha):
    tr = np.ascontiguousarray(task_rewards, dtype=np.float32)
    ln = np.ascontiguousarray(lengths, dtype=np.int32)
    tg = np.ascontiguousarray(target_lengths, dtype=np.int32)
    out = np.zeros(tr.shape[0], dtype=np.float64)
    lib().oracle_total_rewards(_ptr(tr), _ptr(ln), _ptr(tg), tr.shape[0], float(alpha), _ptr(out))
    return out


def filter_groups(rewards, group_size=None, group_offsets=None):
    """Returns (keep u8 [n_groups], kept_groups i32 [n_groups], n_kept, rollout_keep u8 [R])."""
    rw = np.ascontiguousarray(rewards, dtype=np.float32)
    R = rw.shape[0]
    if group_offsets is not None:
        off = np.ascontiguousarray(group_offsets, dtype=np.int32)
        n_groups, gs = off.shape[0] - 1, 0
    else:
        off, gs = None, int(group_size)
        n_groups = R // gs
    keep = np.zeros(n_groups, dtype=np.uint8)
    kept = np.zeros(n_groups, dtype=np.int32)
    n_kept = np.zeros(1, dtype=np.int32)
    rk = np.zeros(R, dtype=np.uint8)
    rc = lib().oracle_filter_groups(_ptr(rw), R, _ptr(off), n_groups, gs, _ptr(keep), _ptr(kept),
                                    _ptr(n_kept), _ptr(rk))
    if rc:
        raise ValueError("oracle_filter_groups: bad group offsets")
    return keep, kept, int(n_kept[0]), rk


def lmhead_logits(hidden, weight, rows=None):
    """z = h W^T in fp64 for the token rows in ``rows`` (all rows when None).
    hidden [N, d] and weight [V, d] are float32, float64 or uint16 bf16 bit patterns."""
    h, hdt, hs = _logits_view(hidden)
    w, wdt, ws = _logits_view(weight)
    d = h.shape[1]
    assert w.shape[1] == d
    V = w.shape[0]
    r = None if rows is None else np.ascontiguousarray(rows, dtype=np.int64)
    n = h.shape[0] if r is None else r.shape[0]
    out = np.zeros((n, V), dtype=np.float64)
    rc = lib().oracle_lmhead_logits(_ptr(h), hdt, d, hs, _ptr(w), wdt, V, ws, _ptr(r), n, _ptr(out))
    if rc:
        raise ValueError("oracle_lmhead_logits failed (rc=%d)" % rc)
    return out


def lmhead_grad_hidden(G, weight):
    """dL/dh rows: G [n, V] (fp64 gradient with respect to the logits) times W."""
    G = np.ascontiguousarray(G, dtype=np.float64)
    w, wdt, ws = _logits_view(weight)
    V, d = w.shape
    assert G.ndim == 2 and G.shape[1] == V
    out = np.zeros((G.shape[0], d), dtype=np.float64)
    rc = lib().oracle_lmhead_grad_hidden(_ptr(G), G.shape[0], V, _ptr(w), wdt, d, ws, _ptr(out))
    if rc:
        raise ValueError("oracle_lmhead_grad_hidden failed (rc=%d)" % rc)
    return out


def lmhead_grad_weight(G, hidden, vocab_rows=None):
    """dL/dW rows ``vocab_rows`` (all when None): G^T [V, N] times the hidden states [N, d]."""
    G = np.ascontiguousarray(G, dtype=np.float64)
    h, hdt, hs = _logits_view(hidden)
    N, d = h.shape
    assert G.ndim == 2 and G.shape[0] == N
    V = G.shape[1]
    r = None if vocab_rows is None else np.ascontiguousarray(vocab_rows, dtype=np.int64)
    n = V if r is None else r.shape[0]
    out = np.zeros((n, d), dtype=np.float64)
    rc = lib().oracle_lmhead_grad_weight(_ptr(G), N, V, _ptr(h), hdt, d, hs, _ptr(r), n, _ptr(out))
    if rc:
        raise ValueError("oracle_lmhead_grad_weight failed (rc=%d)" % rc)
    return out


def widen(a):
    """Stored values as fp64, exactly: uint16 arrays are bf16 bit patterns (a bf16 is the upper
    half of a binary32), float32 / float64 arrays are taken as they are."""
    a = np.asarray(a)
    if a.dtype == np.uint16:
        return (a.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    return a.astype(np.float64)


def lmhead_products(products):
    """The three matrix products of the head, z = h W^T, dL/dh = G W, dL/dW = G^T h, either as
    the plain loops of grpo_oracle.c ("loops") or as numpy's fp64 matrix product of the exactly
    widened operands ("library": the same sums, in the order the library picks; what sizes too
    large for the loops are checked with).  Returns (logits, grad_hidden, grad_weight)."""
    if products == "loops":
        return lmhead_logits, lmhead_grad_hidden, lmhead_grad_weight
    if products == "library":
        return (lambda hidden, weight: widen(hidden) @ widen(weight).T,
                lambda G, weight: np.asarray(G, dtype=np.float64) @ widen(weight),
                lambda G, hidden: np.asarray(G, dtype=np.float64).T @ widen(hidden))
    raise ValueError("products must be 'loops' or 'library'")


def lmhead_loss_fwd_bwd(hidden, weight, tokens, old_logprobs, advantages, mask=None, *,
                        eps_low=0.2, eps_high=0.2, delta=4.0, temperature=1.0, denom=0.0,
                        grad_scale=1.0, want_grads=True, products="loops"):
    """The objective of ``loss_fwd_bwd`` on logits z = h W^T that are never rounded,
    and its gradient with respect to the hidden states and the head's weights."""
    logits_of, grad_hidden_of, grad_weight_of = lmhead_products(products)
    z = logits_of(hidden, weight)
    res = loss_fwd_bwd(z, tokens, old_logprobs, advantages, mask, eps_low=eps_low,
                       eps_high=eps_high, delta=delta, temperature=temperature, denom=denom,
                       grad_scale=grad_scale, grad_rows="all" if want_grads else None)
    res["logits"] = z
    if want_grads:
        res["grad_hidden"] = grad_hidden_of(res["grad"], weight)
        res["grad_weight"] = grad_weight_of(res["grad"], hidden)
    return res


def lmhead_aux_loss_fwd_bwd(hidden, weight, tokens, old_logprobs, ref_logprobs, advantages, mask=None, *,
                            token_weights=None, eps_low=0.2, eps_high=0.2, delta=4.0, temperature=1.0,
                            kl_coef=0.0, ent_coef=0.0, denom=0.0, grad_scale=1.0, want_grads=True):
    """The objective of ``aux_loss_fwd_bwd`` (policy term, sampled-token KL against a reference
    policy, entropy bonus, per-token weights) on logits z = h W^T that are never rounded, and
    its gradient with respect to the hidden states and the head's weights (chain rule through
    the same two products as ``lmhead_loss_fwd_bwd``)."""
    z = lmhead_logits(hidden, weight)
    res = aux_loss_fwd_bwd(z, tokens, old_logprobs, ref_logprobs, advantages, mask,
                           token_weights=token_weights, eps_low=eps_low, eps_high=eps_high, delta=delta,
                           temperature=temperature, kl_coef=kl_coef, ent_coef=ent_coef, denom=denom,
                           grad_scale=grad_scale, grad_rows="all" if want_grads else None)
    res["logits"] = z
    if want_grads:
        res["grad_hidden"] = lmhead_grad_hidden(res["grad"], weight)
        res["grad_weight"] = lmhead_grad_weight(res["grad"], hidden)
    return res
