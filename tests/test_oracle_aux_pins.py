"""Pins of the oracle's auxiliary terms (sampled-token KL estimator, entropy bonus), CPU only:
library entropy, closed forms, the identity that makes the estimator a KL, autograd and
finite differences of the total objective."""
import math

import numpy as np
import pytest
import scipy.special
import scipy.stats
import torch

from oracle import grpo_oracle as orc
from test_oracle_pins import to_bf16_bits, bf16_bits_to_f64


@pytest.mark.parametrize("V,T", [(2, 1.0), (7, 0.7), (1000, 1.0), (4096, 2.5)])
def test_entropy_matches_library(V, T):
    rng = np.random.default_rng(V)
    z = (rng.standard_normal(V) * 3).astype(np.float32)
    p = scipy.special.softmax(z.astype(np.float64) / T)
    assert abs(orc.row_entropy(z, temperature=T) - scipy.stats.entropy(p)) < 1e-12
    zb = to_bf16_bits(z)
    pb = scipy.special.softmax(bf16_bits_to_f64(zb) / T)
    assert abs(orc.row_entropy(zb, temperature=T) - scipy.stats.entropy(pb)) < 1e-12


def test_entropy_closed_forms():
    for V in (1, 2, 64, 152064):
        assert abs(orc.row_entropy(np.full(V, -3.25, np.float32)) - math.log(V)) < 1e-11
    # two tokens: binary entropy of the logistic
    for a in (-4.0, -0.5, 0.0, 1.5, 9.0):
        p = 1.0 / (1.0 + math.exp(-a))
        hb = -(p * math.log(p) + (1 - p) * math.log1p(-p))
        assert abs(orc.row_entropy(np.array([a, 0.0], np.float32)) - hb) < 1e-14
    # +40 spike among V-1 zeros: H = -p0 log p0 - (V-1) q log q, q = e^-40 / (1 + (V-1) e^-40)
    V = 152064
    z = np.zeros(V, np.float32)
    z[5] = 40.0
    s = 1 + (V - 1) * math.exp(-40.0)
    q, p0 = math.exp(-40.0) / s, 1.0 / s
    expect = p0 * math.log(s) + (V - 1) * q * (40.0 + math.log(s))
    # log p of the spike is 40 - lse, rounded at an ulp of 40 (7e-15) against 6.5e-13: 1% of a
    # term that is 2.5% of the total
    assert abs(orc.row_entropy(z) - expect) < 1e-3 * expect
    # -inf logits (masked vocabulary entries) contribute nothing
    z2 = np.array([0.0, -np.inf, 0.0, -np.inf], np.float32)
    assert abs(orc.row_entropy(z2) - math.log(2)) < 1e-15


def test_kl_estimator_properties():
    assert orc.kl_estimator(-2.0, -2.0) == (0.0, 0.0)
    rng = np.random.default_rng(3)
    for _ in range(500):
        l, lr = -rng.uniform(0, 12), -rng.uniform(0, 12)
        kl, dkl = orc.kl_estimator(l, lr)
        d = lr - l
        assert kl >= 0.0 and abs(kl - (math.exp(d) - d - 1)) < 1e-12 * max(1.0, math.exp(d))
        assert abs(dkl - (1 - math.exp(d))) < 1e-12 * max(1.0, math.exp(d))
    # small differences: d^2/2 + d^3/6 without cancellation
    d = 2.0 ** -20
    kl, _ = orc.kl_estimator(-3.0, -3.0 + d)
    assert abs(kl - (d * d / 2 + d ** 3 / 6)) < 1e-9 * d * d


def test_kl_estimator_sums_to_the_kl_divergence():
    """sum_y pi(y) [pi_ref/pi - log(pi_ref/pi) - 1] = KL(pi || pi_ref): what makes the
    sampled-token estimator a KL penalty."""
    rng = np.random.default_rng(4)
    V = 50
    lp = scipy.special.log_softmax(rng.standard_normal(V) * 2)
    lr = scipy.special.log_softmax(rng.standard_normal(V) * 2)
    est = sum(math.exp(lp[y]) * orc.kl_estimator(lp[y], lr[y])[0] for y in range(V))
    assert abs(est - scipy.stats.entropy(np.exp(lp), np.exp(lr))) < 1e-13


def _batch(rng, N, V):
    z = (rng.standard_normal((N, V)) * 2).astype(np.float32)
    tokens = rng.integers(0, V, N)
    adv = rng.standard_normal(N).astype(np.float32)
    mask = (rng.random(N) > 0.3).astype(np.uint8)
    mask[0] = 1
    return z, tokens, adv, mask


def test_total_composition_and_zero_coefficients_reduce_to_the_plain_objective():
    rng = np.random.default_rng(5)
    N, V = 40, 23
    z, tokens, adv, mask = _batch(rng, N, V)
    lp = orc.logprobs(z, tokens, mask, temperature=0.9)
    old = (lp + rng.uniform(-2, 2, N)).astype(np.float32)
    ref = (lp + rng.standard_normal(N) * 0.3).astype(np.float32)
    kw = dict(eps_low=0.2, eps_high=0.3, delta=4.0, temperature=0.9, grad_scale=1.3)
    plain = orc.loss_fwd_bwd(z, tokens, old, adv, mask, grad_rows="all", **kw)
    zero = orc.aux_loss_fwd_bwd(z, tokens, old, ref, adv, mask, kl_coef=0.0, ent_coef=0.0,
                                grad_rows="all", **kw)
    assert zero["total"] == plain["loss"] == zero["policy"]
    assert np.array_equal(zero["grad"], plain["grad"])
    full = orc.aux_loss_fwd_bwd(z, tokens, old, ref, adv, mask, kl_coef=0.05, ent_coef=0.01, **kw)
    M = int(mask.sum())
    m = mask == 1
    kl_mean = sum(orc.kl_estimator(lp[t], float(ref[t]))[0] for t in range(N) if m[t]) / M
    h_mean = sum(orc.row_entropy(z[t], temperature=0.9) for t in range(N) if m[t]) / M
    assert abs(full["kl"] - kl_mean) < 1e-14 and abs(full["entropy"] - h_mean) < 1e-13
    assert abs(full["total"] - (plain["loss"] + 0.05 * kl_mean - 0.01 * h_mean)) < 1e-14
    assert np.array_equal(full["counts"], plain["counts"])
    assert not full["entropies"][~m].any()


def _torch_total(z, tokens, old, ref, adv, mask, el, eh, de, T, klc, enc, denom, gs):
    zt = torch.tensor(z, dtype=torch.float64, requires_grad=True)
    logp = torch.log_softmax(zt / T, dim=-1)
    lp = logp.gather(1, torch.as_tensor(tokens)[:, None])[:, 0]
    r = torch.exp(lp - torch.as_tensor(old, dtype=torch.float64))
    A = torch.as_tensor(adv, dtype=torch.float64)
    J = torch.minimum(torch.clamp(r, max=de) * A, torch.clamp(r, 1 - el, 1 + eh) * A)
    d = torch.as_tensor(ref, dtype=torch.float64) - lp
    kl = torch.exp(d) - d - 1
    H = torch.distributions.Categorical(logits=zt / T).entropy()
    m = torch.as_tensor(mask, dtype=torch.float64)
    D = denom if denom > 0 else m.sum()
    total = (-(J * m).sum() + klc * (kl * m).sum() - enc * (H * m).sum()) / D
    (total * gs).backward()
    return float(total.detach()), zt.grad.numpy()


@pytest.mark.parametrize("V,N", [(5, 16), (17, 12), (64, 8)])
def test_total_gradient_against_autograd(V, N):
    rng = np.random.default_rng(60 + V)
    z, tokens, adv, mask = _batch(rng, N, V)
    T, gs = 0.8, 1.7
    lp = orc.logprobs(z, tokens, mask, temperature=T)
    old = (lp + rng.uniform(-2, 2, N)).astype(np.float32)
    ref = (lp + rng.standard_normal(N) * 0.5).astype(np.float32)
    out = orc.aux_loss_fwd_bwd(z, tokens, old, ref, adv, mask, eps_low=0.2, eps_high=0.3, delta=4.0,
                               temperature=T, kl_coef=0.07, ent_coef=0.03, denom=11.0,
                               grad_scale=gs, grad_rows="all")
    tot, grad = _torch_total(z, tokens, old, ref, adv, mask, 0.2, 0.3, 4.0, T, 0.07, 0.03, 11.0, gs)
    assert abs(out["total"] - tot) < 1e-13
    assert np.max(np.abs(out["grad"] - grad)) < 1e-13
    assert np.max(np.abs(out["grad"].sum(axis=1))) < 1e-15     # both terms are orthogonal to 1
    assert not out["grad"][mask == 0].any()


def test_total_gradient_against_finite_differences():
    rng = np.random.default_rng(71)
    N, V = 6, 9
    z = rng.standard_normal((N, V)) * 2                      # fp64 logits
    tokens = rng.integers(0, V, N)
    adv = rng.standard_normal(N).astype(np.float32)
    mask = np.array([1, 1, 0, 1, 1, 1], np.uint8)
    T = 1.2
    lp = orc.logprobs(z, tokens, mask, temperature=T)
    old = (lp + np.array([0.05, -0.1, 0.0, 0.5, -0.6, 1.0])).astype(np.float32)  # away from kinks
    ref = (lp + rng.standard_normal(N) * 0.4).astype(np.float32)
    kw = dict(eps_low=0.2, eps_high=0.2, delta=4.0, temperature=T, kl_coef=0.3, ent_coef=0.2)
    out = orc.aux_loss_fwd_bwd(z, tokens, old, ref, adv, mask, grad_rows="all", **kw)
    h = 1e-6
    fd = np.zeros_like(z)
    for t in range(N):
        for j in range(V):
            zp, zm = z.copy(), z.copy()
            zp[t, j] += h
            zm[t, j] -= h
            fd[t, j] = (orc.aux_loss_fwd_bwd(zp, tokens, old, ref, adv, mask, **kw)["total"] -
                        orc.aux_loss_fwd_bwd(zm, tokens, old, ref, adv, mask, **kw)["total"]) / (2 * h)
    assert np.max(np.abs(out["grad"] - fd)) < 1e-8


def test_entropy_gradient_alone_is_the_textbook_form():
    """Only the entropy term (A = 0, kl_coef = 0): grad = (b/T) p (log p + H)."""
    rng = np.random.default_rng(81)
    V = 31
    z = (rng.standard_normal((1, V)) * 2).astype(np.float32)
    out = orc.aux_loss_fwd_bwd(z, np.array([3]), np.zeros(1, np.float32), None, np.zeros(1, np.float32),
                               None, temperature=2.0, ent_coef=0.5, grad_rows="all")
    lp = scipy.special.log_softmax(z[0].astype(np.float64) / 2.0)
    p = np.exp(lp)
    H = -(p * lp).sum()
    assert abs(out["total"] + 0.5 * H) < 1e-14
    assert np.max(np.abs(out["grad"][0] - 0.5 / 2.0 * p * (lp + H))) < 1e-15


# ----------------------------------------------------------------------------
# packed layout and sample-level normalisation (the objective as printed in section 3.4)
# ----------------------------------------------------------------------------

def test_packed_layout():
    cu = np.array([0, 3, 3, 10, 14])                        # one empty rollout
    w, rot = orc.packed_layout(cu, 16, sample_level=True)
    assert rot.tolist() == [0] * 3 + [2] * 7 + [3] * 4 + [-1, -1]
    assert np.allclose(w, [1 / 3] * 3 + [1 / 7] * 7 + [1 / 4] * 4 + [0, 0], rtol=1e-7)
    w1, _ = orc.packed_layout(cu, 16, sample_level=False)
    assert w1.tolist() == [1.0] * 14 + [0.0, 0.0]
    for bad in ([0, 5, 4], [0, 20], [-1, 4]):
        with pytest.raises(ValueError):
            orc.packed_layout(np.array(bad), 16, True)


def test_sample_level_loss_is_the_printed_objective():
    """1/G sum_i 1/|o_i| sum_t min(...) written out with loops over rollouts, against the
    weighted form (omega = 1/|o_i|, D = number of rollouts)."""
    rng = np.random.default_rng(91)
    lens = [5, 1, 9, 4, 7, 2]
    cu = np.concatenate([[0], np.cumsum(lens)])
    N, V, R = int(cu[-1]), 13, len(lens)
    z = (rng.standard_normal((N, V)) * 2).astype(np.float32)
    tokens = rng.integers(0, V, N)
    lp = orc.logprobs(z, tokens)
    old = (lp + rng.uniform(-2, 2, N)).astype(np.float32)
    adv_r = rng.standard_normal(R).astype(np.float32)
    w, rot = orc.packed_layout(cu, N, sample_level=True)
    adv = adv_r[rot]
    out = orc.aux_loss_fwd_bwd(z, tokens, old, None, adv, None, token_weights=w, denom=float(R),
                               eps_low=0.2, eps_high=0.2, delta=4.0)
    J = 0.0
    for i in range(R):
        inner = 0.0
        for t in range(cu[i], cu[i + 1]):
            r = math.exp(lp[t] - float(old[t]))
            A = float(adv_r[i])
            inner += min(min(r, 4.0) * A, min(max(r, 0.8), 1.2) * A)
        J += inner / lens[i]
    assert abs(out["total"] + J / R) < 1e-7                  # omega is stored in fp32
    # equal lengths: sample-level and token-level coincide
    cu2 = np.arange(0, 25, 6)
    w2, _ = orc.packed_layout(cu2, 24, sample_level=True)
    a = orc.aux_loss_fwd_bwd(z[:24], tokens[:24], old[:24], None, adv[:24], None, token_weights=w2, denom=4.0)
    b = orc.aux_loss_fwd_bwd(z[:24], tokens[:24], old[:24], None, adv[:24], None)
    assert abs(a["total"] - b["total"]) < 1e-7


def test_weighted_total_gradient_against_autograd_and_zero_weight_rows():
    rng = np.random.default_rng(93)
    N, V = 14, 11
    z, tokens, adv, mask = _batch(rng, N, V)
    w = rng.uniform(0.1, 2.0, N).astype(np.float32)
    w[[3, 8]] = 0.0                                            # e.g. prompt tokens of a packed sequence
    T, gs = 0.9, 1.2
    live = (mask == 1) & (w != 0)
    lp = orc.logprobs(z, tokens, live.astype(np.uint8), temperature=T)
    old = (lp + rng.uniform(-1.5, 1.5, N)).astype(np.float32)
    ref = (lp + rng.standard_normal(N) * 0.4).astype(np.float32)
    out = orc.aux_loss_fwd_bwd(z, tokens, old, ref, adv, mask, token_weights=w, temperature=T,
                               kl_coef=0.05, ent_coef=0.02, denom=0.0, grad_scale=gs, grad_rows="all")
    assert out["counts"][0] == int(live.sum())                 # zero-weight rows count as masked
    zt = torch.tensor(z, dtype=torch.float64, requires_grad=True)
    logp = torch.log_softmax(zt / T, dim=-1)
    l = logp.gather(1, torch.as_tensor(tokens)[:, None])[:, 0]
    r = torch.exp(l - torch.as_tensor(old, dtype=torch.float64))
    A = torch.as_tensor(adv, dtype=torch.float64)
    J = torch.minimum(torch.clamp(r, max=4.0) * A, torch.clamp(r, 0.8, 1.2) * A)
    d = torch.as_tensor(ref, dtype=torch.float64) - l
    H = torch.distributions.Categorical(logits=zt / T).entropy()
    wm = torch.as_tensor(w.astype(np.float64) * live)
    total = ((-J + 0.05 * (torch.exp(d) - d - 1) - 0.02 * H) * wm).sum() / float(live.sum())
    (total * gs).backward()
    assert abs(out["total"] - float(total.detach())) < 1e-13
    assert np.max(np.abs(out["grad"] - zt.grad.numpy())) < 1e-13
    assert not out["grad"][~live].any() and not out["logprobs"][~live].any()
