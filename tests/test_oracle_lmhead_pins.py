"""Pins of the oracle's language-model-head functions (logits z = h W^T in front of the
objective of section 3.4, and the chain rule back to h and W), CPU only: library matrix
products, the identity weight matrix, closed forms, autograd, finite differences."""
import math

import numpy as np
import pytest
import torch

from oracle import grpo_oracle as orc
from test_oracle_pins import to_bf16_bits, bf16_bits_to_f64


def _problem(seed, N=6, d=5, V=9, dtype="f64"):
    rng = np.random.default_rng(seed)
    h = rng.standard_normal((N, d))
    w = rng.standard_normal((V, d)) * 0.8
    if dtype == "bf16":
        h, w = to_bf16_bits(h.astype(np.float32)), to_bf16_bits(w.astype(np.float32))
    elif dtype == "f32":
        h, w = h.astype(np.float32), w.astype(np.float32)
    tokens = rng.integers(0, V, N)
    adv = rng.standard_normal(N).astype(np.float32)
    mask = (rng.random(N) < 0.8).astype(np.uint8)
    mask[0] = 1
    return rng, h, w, tokens, adv, mask


def _wide(a):
    return bf16_bits_to_f64(a) if a.dtype == np.uint16 else a.astype(np.float64)


@pytest.mark.parametrize("dtype", ["f64", "f32", "bf16"])
def test_contractions_match_library_products(dtype):
    # non-square everywhere, so a transposed operand or a swapped index cannot pass
    rng, h, w, *_ = _problem(1, N=7, d=13, V=19, dtype=dtype)
    H, W = _wide(h), _wide(w)
    z = orc.lmhead_logits(h, w)
    assert z.shape == (7, 19)
    assert np.abs(z - H @ W.T).max() < 1e-13
    assert np.abs(orc.lmhead_logits(h, w, rows=[5, 0, 5]) - (H @ W.T)[[5, 0, 5]]).max() < 1e-13
    G = rng.standard_normal((7, 19))
    assert np.abs(orc.lmhead_grad_hidden(G, w) - G @ W).max() < 1e-13
    assert np.abs(orc.lmhead_grad_weight(G, h) - G.T @ H).max() < 1e-13
    assert np.abs(orc.lmhead_grad_weight(G, h, [18, 3]) - (G.T @ H)[[18, 3]]).max() < 1e-13


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_composition_with_library_products_equals_the_one_with_plain_loops(dtype):
    """lmhead_loss_fwd_bwd(products="library") swaps the three plain-loop products for numpy's
    fp64 matrix product of the exactly widened operands (what the GPU tests use at sizes the
    loops would take minutes for): every output agrees with the plain-loop composition to
    fp64 rounding, on non-square shapes, with clipped, capped and masked rows present."""
    rng, h, w, tokens, adv, mask = _problem(11, N=23, d=17, V=31, dtype=dtype)
    assert np.array_equal(orc.widen(h), _wide(h)) and orc.widen(h).dtype == np.float64
    lp = orc.logprobs(orc.lmhead_logits(h, w), tokens, mask)
    old = (lp + rng.uniform(-2.0, 2.0, lp.shape)).astype(np.float32)     # ratios e^-2 .. e^2
    kw = dict(eps_low=0.2, eps_high=0.3, delta=3.0, temperature=0.8, denom=7.5, grad_scale=1.7)
    a = orc.lmhead_loss_fwd_bwd(h, w, tokens, old, adv, mask, products="loops", **kw)
    b = orc.lmhead_loss_fwd_bwd(h, w, tokens, old, adv, mask, products="library", **kw)
    assert a["counts"].tolist() == b["counts"].tolist() and min(a["counts"][1:3]) > 0
    assert abs(a["loss"] - b["loss"]) <= 1e-13 * abs(a["loss"])
    for key in ("logits", "logprobs", "grad", "grad_hidden", "grad_weight"):
        scale = np.abs(a[key]).max()
        assert scale > 0 and np.abs(a[key] - b[key]).max() <= 1e-13 * scale, key
    with pytest.raises(ValueError):
        orc.lmhead_loss_fwd_bwd(h, w, tokens, old, adv, mask, products="fast")


def test_row_strides_are_honoured():
    rng = np.random.default_rng(2)
    hb = rng.standard_normal((4, 16)).astype(np.float32)
    wb = rng.standard_normal((6, 24)).astype(np.float32)
    h, w = hb[:, :5], wb[:, :5]          # contiguous rows, row stride larger than d
    z = orc.lmhead_logits(h, w)
    assert np.abs(z - h.astype(np.float64) @ w.astype(np.float64).T).max() < 1e-13
    G = rng.standard_normal((4, 6))
    assert np.abs(orc.lmhead_grad_hidden(G, w) - G @ w.astype(np.float64)).max() < 1e-13
    assert np.abs(orc.lmhead_grad_weight(G, h) - G.T @ h.astype(np.float64)).max() < 1e-13


def test_identity_weight_reduces_to_the_logits_objective():
    # W = I (V = d): z = h, dL/dh = dL/dz, dL/dW = G^T h
    rng, h, _, tokens, adv, mask = _problem(3, N=8, d=12, V=12, dtype="bf16")
    w = to_bf16_bits(np.eye(12, dtype=np.float32))
    old = (rng.standard_normal(8) * 0.3 - 2.5).astype(np.float32)
    a = orc.lmhead_loss_fwd_bwd(h, w, tokens, old, adv, mask, temperature=0.7)
    b = orc.loss_fwd_bwd(h, tokens, old, adv, mask, temperature=0.7, grad_rows="all")
    assert a["loss"] == b["loss"] and np.array_equal(a["logprobs"], b["logprobs"])
    assert np.array_equal(a["counts"], b["counts"])
    assert np.array_equal(a["grad_hidden"], b["grad"])
    assert np.abs(a["grad_weight"] - b["grad"].T @ bf16_bits_to_f64(h)).max() < 1e-15


def test_equal_weight_rows_give_a_uniform_policy():
    # every vocabulary row of W equal: z is constant along the row, pi is uniform,
    # log pi(y) = -ln V, and both gradients vanish (G rows sum to zero)
    rng, h, _, tokens, adv, mask = _problem(4, N=5, d=6, V=10)
    w = np.tile(rng.standard_normal((1, 6)), (10, 1))
    old = np.full(5, -math.log(10), np.float32)
    r = orc.lmhead_loss_fwd_bwd(h, w, tokens, old, adv, mask)
    m = mask.astype(bool)
    assert np.abs(r["logprobs"][m] + math.log(10)).max() < 1e-14
    assert np.abs(r["grad_hidden"]).max() < 1e-15
    assert np.abs(r["grad_weight"].sum(axis=0)).max() < 1e-15


def test_weight_gradient_columns_sum_to_zero_and_masked_rows_vanish():
    rng, h, w, tokens, adv, mask = _problem(5, N=16, d=7, V=33, dtype="bf16")
    mask[3] = 0
    old = (orc.logprobs(orc.lmhead_logits(h, w), tokens) + rng.standard_normal(16) * 0.1)
    r = orc.lmhead_loss_fwd_bwd(h, w, tokens, old.astype(np.float32), adv, mask)
    assert np.abs(r["grad_weight"].sum(axis=0)).max() < 1e-15
    assert np.all(r["grad_hidden"][mask == 0] == 0)
    assert np.abs(r["grad_hidden"][mask == 1]).max() > 0


def _torch_loss(H, W, tokens, old, adv, mask, eps_low, eps_high, delta, T):
    z = H @ W.T / T
    lp = torch.log_softmax(z, dim=-1).gather(1, tokens[:, None])[:, 0]
    r = torch.exp(lp - old)
    J = torch.minimum(torch.clamp(r, max=delta) * adv, torch.clamp(r, 1 - eps_low, 1 + eps_high) * adv)
    return -(J * mask).sum() / mask.sum()


@pytest.mark.parametrize("seed,T", [(11, 1.0), (12, 0.7)])
def test_gradients_match_autograd(seed, T):
    rng, h, w, tokens, adv, mask = _problem(seed, N=24, d=8, V=17)
    new = orc.logprobs(orc.lmhead_logits(h, w), tokens, temperature=T)
    old = (new + rng.uniform(-1.8, 1.8, 24)).astype(np.float32)    # both clip sides and the delta cap
    kw = dict(eps_low=0.2, eps_high=0.3, delta=4.0)
    res = orc.lmhead_loss_fwd_bwd(h, w, tokens, old, adv, mask, temperature=T, **kw)
    H = torch.tensor(h, requires_grad=True)
    W = torch.tensor(w, requires_grad=True)
    loss = _torch_loss(H, W, torch.tensor(tokens), torch.tensor(old, dtype=torch.float64),
                       torch.tensor(adv, dtype=torch.float64), torch.tensor(mask, dtype=torch.float64),
                       T=T, **kw)
    loss.backward()
    assert abs(res["loss"] - loss.item()) < 1e-13
    assert np.abs(res["grad_hidden"] - H.grad.numpy()).max() < 1e-13
    assert np.abs(res["grad_weight"] - W.grad.numpy()).max() < 1e-13
    assert res["counts"][1] > 0 and res["counts"][2] > 0 and res["counts"][3] > 0


def test_gradients_match_central_differences():
    rng, h, w, tokens, adv, mask = _problem(21, N=10, d=4, V=7)
    new = orc.logprobs(orc.lmhead_logits(h, w), tokens)
    # keep every ratio a safe distance inside a smooth region of the surrogate
    old = (new + rng.choice([-0.1, 0.05, 0.12], 10)).astype(np.float32)
    res = orc.lmhead_loss_fwd_bwd(h, w, tokens, old, adv, mask, grad_scale=1.5)
    step = 1e-6

    def loss_at(hh, ww):
        return 1.5 * orc.lmhead_loss_fwd_bwd(hh, ww, tokens, old, adv, mask, want_grads=False)["loss"]

    for (t, k) in [(0, 0), (4, 3), (9, 1)]:
        hp, hm = h.copy(), h.copy()
        hp[t, k] += step
        hm[t, k] -= step
        fd = (loss_at(hp, w) - loss_at(hm, w)) / (2 * step)
        assert abs(fd - res["grad_hidden"][t, k]) < 1e-8, (t, k)
    for (v, k) in [(0, 0), (6, 2), (int(tokens[0]), 1)]:
        wp, wm = w.copy(), w.copy()
        wp[v, k] += step
        wm[v, k] -= step
        fd = (loss_at(h, wp) - loss_at(h, wm)) / (2 * step)
        assert abs(fd - res["grad_weight"][v, k]) < 1e-8, (v, k)


# ---- the head in front of the objective with the auxiliary terms ----

def _torch_total(H, W, tokens, old, ref, adv, mask, tw, eps_low, eps_high, delta, T, klc, enc, denom):
    z = H @ W.T / T
    lp = torch.log_softmax(z, dim=-1).gather(1, tokens[:, None])[:, 0]
    r = torch.exp(lp - old)
    J = torch.minimum(torch.clamp(r, max=delta) * adv, torch.clamp(r, 1 - eps_low, 1 + eps_high) * adv)
    d = ref - lp
    kl = torch.exp(d) - d - 1
    ent = torch.distributions.Categorical(logits=z).entropy()
    w = mask * tw
    D = denom if denom > 0 else mask.sum()
    return (-(J * w).sum() + klc * (kl * w).sum() - enc * (ent * w).sum()) / D


def test_aux_identity_weight_reduces_to_the_logits_objective():
    rng, h, _, tokens, adv, mask = _problem(31, N=8, d=12, V=12, dtype="bf16")
    w = to_bf16_bits(np.eye(12, dtype=np.float32))
    old = (rng.standard_normal(8) * 0.3 - 2.5).astype(np.float32)
    ref = (rng.standard_normal(8) * 0.3 - 2.5).astype(np.float32)
    kw = dict(temperature=0.7, kl_coef=0.05, ent_coef=0.02, grad_scale=1.3)
    a = orc.lmhead_aux_loss_fwd_bwd(h, w, tokens, old, ref, adv, mask, **kw)
    b = orc.aux_loss_fwd_bwd(h, tokens, old, ref, adv, mask, grad_rows="all", **kw)
    for key in ("total", "policy", "kl", "entropy"):
        assert a[key] == b[key], key
    assert np.array_equal(a["logprobs"], b["logprobs"]) and np.array_equal(a["entropies"], b["entropies"])
    assert np.array_equal(a["grad_hidden"], b["grad"])
    assert np.abs(a["grad_weight"] - b["grad"].T @ bf16_bits_to_f64(h)).max() < 1e-15


def test_aux_zero_coefficients_reduce_to_the_plain_head_objective():
    rng, h, w, tokens, adv, mask = _problem(32, N=12, d=6, V=15)
    new = orc.logprobs(orc.lmhead_logits(h, w), tokens)
    old = (new + rng.uniform(-1.5, 1.5, 12)).astype(np.float32)
    a = orc.lmhead_aux_loss_fwd_bwd(h, w, tokens, old, None, adv, mask, grad_scale=0.9)
    b = orc.lmhead_loss_fwd_bwd(h, w, tokens, old, adv, mask, grad_scale=0.9)
    assert abs(a["total"] - b["loss"]) < 1e-15 and a["policy"] == a["total"]
    assert np.abs(a["grad_hidden"] - b["grad_hidden"]).max() < 1e-15
    assert np.abs(a["grad_weight"] - b["grad_weight"]).max() < 1e-15
    assert np.array_equal(a["counts"], b["counts"])


@pytest.mark.parametrize("seed,T,weighted", [(41, 1.0, False), (42, 0.7, True)])
def test_aux_gradients_match_autograd(seed, T, weighted):
    rng, h, w, tokens, adv, mask = _problem(seed, N=24, d=8, V=17)
    new = orc.logprobs(orc.lmhead_logits(h, w), tokens, temperature=T)
    old = (new + rng.uniform(-1.8, 1.8, 24)).astype(np.float32)
    ref = (new + rng.standard_normal(24) * 0.4).astype(np.float32)
    tw = rng.uniform(0.2, 1.5, 24).astype(np.float32) if weighted else None
    if weighted:
        tw[5] = 0.0                                   # a zero weight takes the row out
    kw = dict(eps_low=0.2, eps_high=0.3, delta=4.0)
    res = orc.lmhead_aux_loss_fwd_bwd(h, w, tokens, old, ref, adv, mask, token_weights=tw, temperature=T,
                                      kl_coef=0.07, ent_coef=0.03, denom=13.0, **kw)
    H = torch.tensor(h, requires_grad=True)
    W = torch.tensor(w, requires_grad=True)
    f64 = lambda a: torch.tensor(np.asarray(a), dtype=torch.float64)
    total = _torch_total(H, W, torch.tensor(tokens), f64(old), f64(ref), f64(adv), f64(mask),
                         f64(tw) if weighted else torch.ones(24, dtype=torch.float64),
                         T=T, klc=0.07, enc=0.03, denom=13.0, **kw)
    total.backward()
    assert abs(res["total"] - total.item()) < 1e-13
    assert np.abs(res["grad_hidden"] - H.grad.numpy()).max() < 1e-13
    assert np.abs(res["grad_weight"] - W.grad.numpy()).max() < 1e-13
    assert np.abs(res["grad_weight"].sum(axis=0)).max() < 1e-14      # rows of G still sum to zero
    if weighted:
        assert not res["grad_hidden"][5].any()
    assert res["counts"][1] > 0 and res["counts"][2] > 0


def test_aux_gradients_match_central_differences():
    rng, h, w, tokens, adv, mask = _problem(51, N=10, d=4, V=7)
    new = orc.logprobs(orc.lmhead_logits(h, w), tokens)
    old = (new + rng.choice([-0.1, 0.05, 0.12], 10)).astype(np.float32)
    ref = (new + rng.standard_normal(10) * 0.3).astype(np.float32)
    kw = dict(kl_coef=0.2, ent_coef=0.1)
    res = orc.lmhead_aux_loss_fwd_bwd(h, w, tokens, old, ref, adv, mask, **kw)
    step = 1e-6

    def total_at(hh, ww):
        return orc.lmhead_aux_loss_fwd_bwd(hh, ww, tokens, old, ref, adv, mask, want_grads=False, **kw)["total"]

    for (t, k) in [(0, 0), (4, 3), (9, 1)]:
        hp, hm = h.copy(), h.copy()
        hp[t, k] += step
        hm[t, k] -= step
        assert abs((total_at(hp, w) - total_at(hm, w)) / (2 * step) - res["grad_hidden"][t, k]) < 1e-8, (t, k)
    for (v, k) in [(0, 0), (6, 2), (int(tokens[0]), 1)]:
        wp, wm = w.copy(), w.copy()
        wp[v, k] += step
        wm[v, k] -= step
        assert abs((total_at(h, wp) - total_at(h, wm)) / (2 * step) - res["grad_weight"][v, k]) < 1e-8, (v, k)
