"""Pins of the fp64 oracle against things other than itself (CPU only).

Each test checks the oracle against something the paper or mathematics fixes:
the hand-derived branch table of the two-sided-clipping objective (section 3.4),
closed forms, invariants, library routines for the special cases that reduce to
them (scipy log-softmax, torch cross-entropy and autograd), central finite
differences, and brute force on tiny inputs.
"""
import math
import os

import numpy as np
import pytest
import scipy.special
import torch

from oracle import grpo_oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def to_bf16_bits(x):
    """float array -> uint16 bf16 bit patterns (round to nearest even, via torch)."""
    t = torch.as_tensor(np.asarray(x, dtype=np.float32)).to(torch.bfloat16)
    return t.view(torch.int16).numpy().view(np.uint16).copy()


def bf16_bits_to_f64(bits):
    t = torch.as_tensor(bits.view(np.int16)).view(torch.bfloat16)
    return t.to(torch.float64).numpy()


# ----------------------------------------------------------------------------
# log-softmax / log-probs
# ----------------------------------------------------------------------------

@pytest.mark.parametrize("V", [1, 2, 7, 64, 1000])
@pytest.mark.parametrize("T", [1.0, 0.7, 2.5])
def test_log_softmax_matches_library_and_sums_to_one(V, T):
    rng = np.random.default_rng(V * 131 + int(T * 10))
    z = (rng.standard_normal(V) * 3).astype(np.float32)
    lp, lse = orc.row_log_softmax(z, temperature=T)
    ref = scipy.special.log_softmax(z.astype(np.float64) / T)
    assert np.max(np.abs(lp - ref)) < 1e-12
    assert abs(lse - scipy.special.logsumexp(z.astype(np.float64) / T)) < 1e-12
    assert abs(np.exp(lp).sum() - 1.0) < 1e-12


def test_log_softmax_uniform_row_closed_form():
    for V in (1, 2, 8, 1024, 152064):
        z = np.full(V, 1.75, dtype=np.float32)
        lp, _ = orc.row_log_softmax(z)
        assert np.max(np.abs(lp + math.log(V))) < 1e-12


def test_log_softmax_spike_row_closed_form():
    # one logit at +40, the others at 0: l_y = -log1p((V-1) e^-40), l_j = -40 - log1p(...)
    V, y = 152064, 4711
    z = np.zeros(V, dtype=np.float32)
    z[y] = 40.0
    lp, _ = orc.row_log_softmax(to_bf16_bits(z))
    t = math.log1p((V - 1) * math.exp(-40.0))
    assert abs(lp[y] + t) < 8e-15          # one ulp of 40: lse = 40 + 6.5e-13 is rounded there
    assert abs(lp[0] + 40.0 + t) < 8e-15


def test_log_softmax_shift_and_temperature_scale_invariance():
    rng = np.random.default_rng(5)
    # multiples of 1/8 so that shifting by 16 and scaling by 4 stay exact in fp32
    z = (np.round(rng.standard_normal(333) * 24) / 8).astype(np.float32)
    lp, _ = orc.row_log_softmax(z, temperature=0.5)
    lp_shift, _ = orc.row_log_softmax((z + 16).astype(np.float32), temperature=0.5)
    lp_scale, _ = orc.row_log_softmax((z * 4).astype(np.float32), temperature=2.0)
    assert np.max(np.abs(lp - lp_shift)) < 1e-12
    assert np.max(np.abs(lp - lp_scale)) < 1e-12


def test_bf16_rows_are_widened_exactly():
    rng = np.random.default_rng(6)
    bits = to_bf16_bits(rng.standard_normal(4096) * 5)
    lp, _ = orc.row_log_softmax(bits)
    ref = scipy.special.log_softmax(bf16_bits_to_f64(bits))
    assert np.max(np.abs(lp - ref)) < 1e-12
    # negative zero, large magnitudes and subnormal-free small values survive the widening
    special = np.array([0.0, -0.0, 1.0, -1.0, 3.0e38, -3.0e38, 1e-30, 65280.0], dtype=np.float32)
    sb = to_bf16_bits(special)
    lp2, _ = orc.row_log_softmax(sb, temperature=1e37)  # huge T keeps exp finite
    ref2 = scipy.special.log_softmax(bf16_bits_to_f64(sb) / 1e37)
    assert np.max(np.abs(lp2 - ref2)) < 1e-12


def test_logprobs_gather_stride_and_mask():
    rng = np.random.default_rng(7)
    N, V, S = 9, 50, 64
    buf = np.full((N, S), np.nan, dtype=np.float32)      # padding must never be read
    buf[:, :V] = rng.standard_normal((N, V)) * 2
    tokens = rng.integers(0, V, N)
    mask = np.array([1, 1, 0, 1, 0, 1, 1, 1, 0], dtype=np.uint8)
    buf[mask == 0] = np.nan                                 # masked rows must never be read
    tokens[2] = 10 ** 9                                     # nor their token ids
    lp = orc.logprobs(buf, tokens, mask, temperature=0.9, vocab=V)
    for t in range(N):
        if mask[t]:
            ref = scipy.special.log_softmax(buf[t, :V].astype(np.float64) / 0.9)[tokens[t]]
            assert abs(lp[t] - ref) < 1e-12
        else:
            assert lp[t] == 0.0
    with pytest.raises(ValueError):
        orc.logprobs(buf[:2, :V].copy(), np.array([0, V]), None, vocab=V)
    with pytest.raises(ValueError):
        orc.logprobs(buf[:2, :V].copy(), np.array([-1, 0]), None, vocab=V)


# ----------------------------------------------------------------------------
# the bracketed surrogate term
# ----------------------------------------------------------------------------

def _golden_rows():
    rows = []
    with open(os.path.join(GOLDEN, "surrogate_branch_table.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            el, eh, de, r, A, J, dJ, fl = line.split()
            rows.append((float(el), float(eh), float(de), float(r), float(A), float(J),
                         float(dJ), int(fl)))
    assert len(rows) >= 20
    return rows


def test_surrogate_branch_table_from_paper_formula():
    for el, eh, de, r, A, J, dJ, fl in _golden_rows():
        gJ, gdJ, gfl = orc.surrogate_from_ratio(r, A, el, eh, de)
        assert gJ == J, (el, eh, de, r, A)
        assert gdJ == dJ, (el, eh, de, r, A)
        assert gfl == fl, (el, eh, de, r, A)


def test_surrogate_reduces_to_original_objective_when_delta_is_infinite():
    # first displayed objective of section 3.4: min(r A, clip(r, 1-eps, 1+eps) A)
    rng = np.random.default_rng(11)
    for _ in range(2000):
        r = math.exp(rng.uniform(-4, 4))
        A = rng.standard_normal() * (rng.random() > 0.1)
        eps = rng.uniform(0.05, 0.5)
        J, dJ, fl = orc.surrogate_from_ratio(r, A, eps, eps, math.inf)
        assert J == min(r * A, float(np.clip(r, 1 - eps, 1 + eps)) * A)
        assert not (fl & orc.FLAG_DELTA)
        # the original objective leaves negative advantages unclipped from above
        if A < 0 and r > 1 + eps:
            assert J == r * A and dJ == r * A


def test_surrogate_bounds():
    rng = np.random.default_rng(12)
    el, eh, de = 0.2, 0.28, 4.0
    for _ in range(2000):
        r = math.exp(rng.uniform(-5, 5))
        A = rng.standard_normal()
        J, dJ, fl = orc.surrogate_from_ratio(r, A, el, eh, de)
        s1 = min(r, de) * A
        s2 = min(max(r, 1 - el), 1 + eh) * A
        assert J <= s1 and J <= s2 and (J == s1 or J == s2)
        if A < 0:
            assert J >= de * A                 # the bound delta adds for bad rollouts
            assert (dJ == 0.0) == (r < 1 - el or r > de)
        if A > 0:
            assert J <= (1 + eh) * A
            assert (dJ == 0.0) == (r > 1 + eh)
        if dJ != 0.0:
            assert dJ == r * A


# ----------------------------------------------------------------------------
# loss composition
# ----------------------------------------------------------------------------

def _tiny_batch(rng, N, V, dtype="f32"):
    z = (rng.standard_normal((N, V)) * 2).astype(np.float32)
    if dtype == "bf16":
        z = to_bf16_bits(z)
    tokens = rng.integers(0, V, N)
    adv = rng.standard_normal(N).astype(np.float32)
    mask = (rng.random(N) > 0.3).astype(np.uint8)
    mask[0] = 1
    return z, tokens, adv, mask


def test_ratio_one_gives_masked_mean_of_minus_advantage():
    rng = np.random.default_rng(21)
    z, tokens, adv, mask = _tiny_batch(rng, 40, 33)
    lp = orc.logprobs(z, tokens, mask)
    out = orc.loss_fwd_bwd(z, tokens, lp.astype(np.float32), adv, mask)
    M = int(mask.sum())
    expect = -float(adv.astype(np.float64)[mask == 1].sum()) / M
    assert abs(out["loss"] - expect) < 1e-6 * max(1.0, abs(expect))
    assert out["counts"].tolist() == [M, 0, 0, 0, 0]
    # c_t = -m A r / M with r = 1 up to the fp32 rounding of l_old
    c_expect = -(mask * adv.astype(np.float64)) / M
    assert np.max(np.abs(out["coeff"] - c_expect)) < 1e-6


def test_loss_with_hand_built_ratios_matches_branch_table():
    """Two-token vocabulary: l = -log(1 + e^{-a}) in closed form; l_old = l - ln r_target
    makes the ratio equal r_target, so the loss is the mean of the table's J values.
    Catches a ratio taken the wrong way round and a wrong sign or normalisation."""
    rows = [g for g in _golden_rows() if g[:3] == (0.25, 0.25, 4.0)]
    N = len(rows)
    a = np.linspace(-2.0, 3.0, N)
    z = np.zeros((N, 2), dtype=np.float32)
    z[:, 0] = a.astype(np.float32)
    tokens = np.zeros(N, dtype=np.int64)
    l_closed = -np.log1p(np.exp(-z[:, 0].astype(np.float64)))
    lp = orc.logprobs(z, tokens)
    assert np.max(np.abs(lp - l_closed)) < 1e-14
    r_t = np.array([g[3] for g in rows])
    A = np.array([g[4] for g in rows], dtype=np.float32)
    old = (l_closed - np.log(r_t)).astype(np.float32)
    out = orc.loss_fwd_bwd(z, tokens, old, A, None, eps_low=0.25, eps_high=0.25, delta=4.0)
    # fp32 rounding of l_old moves r by ~1e-7 relative: use rows away from ties for J
    r_real = np.exp(lp - old.astype(np.float64))
    J_expect = []
    for (el, eh, de, r, Av, J, dJ, fl), rr in zip(rows, r_real):
        on_tie = r in (0.75, 1.25, 4.0)
        J_expect.append(orc.surrogate_from_ratio(rr, Av, el, eh, de)[0] if on_tie else
                        (J if dJ == 0 else J * rr / r))
    assert abs(out["loss"] + np.mean(J_expect)) < 1e-12
    # sign and size: table J values are reproduced to fp32-rounding accuracy
    assert np.max(np.abs(out["J"] - np.array([g[5] for g in rows]))) < 1e-5


def test_token_level_normalisation_denominator_and_empty_mask():
    rng = np.random.default_rng(23)
    z, tokens, adv, mask = _tiny_batch(rng, 30, 17)
    old = (orc.logprobs(z, tokens, mask) + rng.standard_normal(30) * 0.3).astype(np.float32)
    out = orc.loss_fwd_bwd(z, tokens, old, adv, mask)
    M = int(mask.sum())
    assert out["counts"][0] == M
    assert abs(out["loss"] + out["J"][mask == 1].sum() / M) < 1e-14
    assert np.all(out["J"][mask == 0] == 0) and np.all(out["coeff"][mask == 0] == 0)
    assert np.all(out["logprobs"][mask == 0] == 0)
    # an imposed global denominator rescales loss and coefficients by M / denom
    out2 = orc.loss_fwd_bwd(z, tokens, old, adv, mask, denom=4.0 * M)
    assert abs(out2["loss"] - out["loss"] / 4.0) < 1e-14
    assert np.max(np.abs(out2["coeff"] - out["coeff"] / 4.0)) < 1e-14
    # mask NULL means all ones
    out3 = orc.loss_fwd_bwd(z, tokens, old, adv, None)
    out4 = orc.loss_fwd_bwd(z, tokens, old, adv, np.ones(30, dtype=np.uint8))
    assert out3["loss"] == out4["loss"] and out3["counts"][0] == 30
    # nothing unmasked: everything is zero
    z0 = orc.loss_fwd_bwd(z, tokens, old, adv, np.zeros(30, dtype=np.uint8), grad_rows="all")
    assert z0["loss"] == 0.0 and z0["counts"].tolist() == [0] * 5 and not z0["grad"].any()


def test_counters_by_brute_force_recount():
    rng = np.random.default_rng(24)
    N, V = 400, 11
    z, tokens, adv, mask = _tiny_batch(rng, N, V)
    adv[rng.random(N) < 0.1] = 0.0
    lp = orc.logprobs(z, tokens, mask)
    old = (lp + rng.uniform(-3, 3, N)).astype(np.float32)
    el, eh, de = 0.2, 0.3, 4.0
    out = orc.loss_fwd_bwd(z, tokens, old, adv, mask, eps_low=el, eps_high=eh, delta=de)
    r = np.exp(lp - old.astype(np.float64))
    m = mask == 1
    A = adv.astype(np.float64)
    hi = int(np.sum(m & (A > 0) & (r > 1 + eh)))
    lo = int(np.sum(m & (A < 0) & (r < 1 - el)))
    dl = int(np.sum(m & (A < 0) & (r > de)))
    oob = int(np.sum(m & ((r < 1 - el) | (r > 1 + eh))))
    assert out["counts"].tolist() == [int(m.sum()), hi, lo, dl, oob]
    assert min(hi, lo, dl, oob) > 0
    # every row whose gradient is cut is counted exactly once among the three clip counters
    cut = m & (A != 0) & (out["coeff"] == 0)
    assert int(cut.sum()) == hi + lo + dl


# ----------------------------------------------------------------------------
# gradient
# ----------------------------------------------------------------------------

def _torch_objective(z, tokens, old, adv, mask, el, eh, de, T, denom, grad_scale):
    """Same objective through torch's library ops in fp64; autograd supplies the gradient."""
    zt = torch.tensor(z, dtype=torch.float64, requires_grad=True)
    lp = torch.log_softmax(zt / T, dim=-1).gather(1, torch.as_tensor(tokens)[:, None])[:, 0]
    r = torch.exp(lp - torch.as_tensor(old, dtype=torch.float64))
    A = torch.as_tensor(adv, dtype=torch.float64)
    J = torch.minimum(torch.clamp(r, max=de) * A, torch.clamp(r, 1 - el, 1 + eh) * A)
    m = torch.as_tensor(mask, dtype=torch.float64)
    D = denom if denom > 0 else m.sum()
    loss = -(J * m).sum() / D
    (loss * grad_scale).backward()
    return float(loss), zt.grad.numpy()


@pytest.mark.parametrize("V,N", [(5, 16), (17, 12), (64, 8)])
def test_gradient_against_autograd_and_row_sums(V, N):
    rng = np.random.default_rng(31 + V)
    z, tokens, adv, mask = _tiny_batch(rng, N, V)
    T, gs = 0.7, 1.7
    lp = orc.logprobs(z, tokens, mask, temperature=T)
    old = (lp + rng.uniform(-2, 2, N)).astype(np.float32)
    out = orc.loss_fwd_bwd(z, tokens, old, adv, mask, eps_low=0.2, eps_high=0.3, delta=4.0,
                           temperature=T, grad_scale=gs, grad_rows="all")
    loss_t, grad_t = _torch_objective(z, tokens, old, adv, mask, 0.2, 0.3, 4.0, T, 0.0, gs)
    assert abs(out["loss"] - loss_t) < 1e-13
    assert np.max(np.abs(out["grad"] - grad_t)) < 1e-13
    assert np.max(np.abs(out["grad"].sum(axis=1))) < 1e-15
    assert not out["grad"][mask == 0].any()
    # the exported per-row coefficient is dloss/dl_t: grad at y is (c/T)(1 - p_y)
    gy = grad_t[np.arange(N), tokens]
    assert np.max(np.abs(out["coeff"] / T * (1 - np.exp(out["logprobs"])) * mask - gy)) < 1e-13


@pytest.mark.parametrize("V,N", [(5, 16), (17, 12), (64, 8)])
def test_gradient_against_central_finite_differences(V, N):
    rng = np.random.default_rng(41 + V)
    z = rng.standard_normal((N, V)) * 2                     # fp64 logits: steps of 1e-6 resolve
    tokens = rng.integers(0, V, N)
    adv = rng.standard_normal(N).astype(np.float32)
    mask = (rng.random(N) > 0.25).astype(np.uint8)
    T, gs, el, eh, de = 1.3, 0.6, 0.2, 0.25, 4.0
    lp = orc.logprobs(z, tokens, mask, temperature=T)
    # keep ratios at least 1e-3 (in log space) away from every kink of the objective
    kinks = np.log([1 - el, 1 + eh, de])
    noise = rng.uniform(-2, 2, N)
    for t in range(N):
        while np.min(np.abs(-noise[t] - kinks)) < 1e-3:
            noise[t] = rng.uniform(-2, 2)
    old = (lp + noise).astype(np.float32)
    kw = dict(eps_low=el, eps_high=eh, delta=de, temperature=T, grad_scale=gs)
    out = orc.loss_fwd_bwd(z, tokens, old, adv, mask, grad_rows="all", **kw)
    h = 1e-6
    fd = np.zeros_like(z)
    for t in range(N):
        for j in range(V):
            zp, zm = z.copy(), z.copy()
            zp[t, j] += h
            zm[t, j] -= h
            fp = orc.loss_fwd_bwd(zp, tokens, old, adv, mask, **kw)["loss"]
            fm = orc.loss_fwd_bwd(zm, tokens, old, adv, mask, **kw)["loss"]
            fd[t, j] = gs * (fp - fm) / (2 * h)
    scale = np.max(np.abs(out["grad"]))
    assert scale > 0
    assert np.max(np.abs(out["grad"] - fd)) < 1e-7 * max(scale, 1e-3) + 1e-9


def test_gradient_reduces_to_cross_entropy():
    """eps_low = 1, eps_high and delta huge, A = 1, l_old = l, mask = 1:
    J = r, loss = -mean r, and at r = 1 the gradient is the mean-NLL gradient."""
    rng = np.random.default_rng(51)
    N, V = 10, 29
    z = (rng.standard_normal((N, V)) * 2).astype(np.float32)
    tokens = rng.integers(0, V, N)
    lp = orc.logprobs(z, tokens)
    out = orc.loss_fwd_bwd(z, tokens, lp.astype(np.float32), np.ones(N, np.float32), None,
                           eps_low=1.0, eps_high=1e30, delta=1e31, grad_rows="all")
    zt = torch.tensor(z, dtype=torch.float64, requires_grad=True)
    torch.nn.functional.cross_entropy(zt, torch.as_tensor(tokens)).backward()
    assert np.max(np.abs(out["grad"] - zt.grad.numpy())) < 1e-7   # r = 1 up to fp32 l_old
    assert abs(out["loss"] + 1.0) < 1e-6


def test_gradient_of_near_one_hot_row():
    """+40 spike on the sampled token: grad at y is (c/T)(1 - p_y) with
    1 - p_y = (V-1)e^-40 / (1 + (V-1)e^-40) in closed form."""
    V, y = 152064, 17
    z = np.zeros((1, V), dtype=np.float32)
    z[0, y] = 40.0
    lp = orc.logprobs(z, np.array([y]))
    out = orc.loss_fwd_bwd(z, np.array([y]), lp.astype(np.float32), np.array([2.0], np.float32),
                           None, grad_rows="all")
    q = (V - 1) * math.exp(-40.0)
    c = out["coeff"][0]
    assert abs(c + 2.0) < 1e-6
    assert abs(out["grad"][0, y] - c * q / (1 + q)) < 1e-12 * abs(c * q)
    assert abs(out["grad"][0, 0] + c * math.exp(-40.0) / (1 + q)) < 1e-12 * abs(c) * math.exp(-40)
    assert abs(out["grad"].sum()) < 1e-25


# ----------------------------------------------------------------------------
# brute force on tiny inputs, written with exact summation (math.fsum)
# ----------------------------------------------------------------------------

def _fsum_reference(z, tokens, old, adv, mask, el, eh, de, T, gs):
    N, V = len(z), len(z[0])
    M = sum(int(m) for m in mask)
    Js, grads = [], []
    for t in range(N):
        if not mask[t]:
            Js.append(0.0)
            grads.append([0.0] * V)
            continue
        u = [float(v) / T for v in z[t]]
        mx = max(u)
        lse = mx + math.log(math.fsum(math.exp(v - mx) for v in u))
        l = u[tokens[t]] - lse
        r = math.exp(l - float(old[t]))
        A = float(adv[t])
        s1 = min(r, de) * A
        s2 = min(max(r, 1 - el), 1 + eh) * A
        Js.append(min(s1, s2))
        if A > 0:
            live = r <= 1 + eh
        elif A < 0:
            live = 1 - el <= r <= de
        else:
            live = False
        c = -gs * (A * r if live else 0.0) / M
        grads.append([(c / T) * ((1.0 if j == tokens[t] else 0.0) - math.exp(u[j] - lse))
                      for j in range(V)])
    return -math.fsum(Js) / M, grads


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_brute_force_tiny(dtype):
    rng = np.random.default_rng(61)
    N, V = 24, 40
    z, tokens, adv, mask = _tiny_batch(rng, N, V, dtype)
    zf = bf16_bits_to_f64(z) if dtype == "bf16" else z.astype(np.float64)
    T = 0.8
    old = (orc.logprobs(z, tokens, mask, temperature=T) + rng.uniform(-2, 2, N)).astype(np.float32)
    out = orc.loss_fwd_bwd(z, tokens, old, adv, mask, eps_low=0.2, eps_high=0.2, delta=4.0,
                           temperature=T, grad_scale=1.0, grad_rows="all")
    loss, grads = _fsum_reference(zf.tolist(), tokens.tolist(), old, adv, mask, 0.2, 0.2, 4.0, T, 1.0)
    assert abs(out["loss"] - loss) < 1e-12
    assert np.max(np.abs(out["grad"] - np.array(grads))) < 1e-12


# ----------------------------------------------------------------------------
# group-relative advantages
# ----------------------------------------------------------------------------

@pytest.mark.parametrize("ddof", [0, 1])
def test_advantages_match_library_std_and_invariants(ddof):
    rng = np.random.default_rng(71 + ddof)
    G, n_groups = 16, 9
    R = rng.random(G * n_groups).astype(np.float32)
    adv = orc.group_advantages(R, group_size=G, eps_std=0.0, ddof=ddof).reshape(n_groups, G)
    Rg = R.astype(np.float64).reshape(n_groups, G)
    ref = (Rg - Rg.mean(axis=1, keepdims=True)) / Rg.std(axis=1, ddof=ddof, keepdims=True)
    assert np.max(np.abs(adv - ref)) < 1e-12
    assert np.max(np.abs(adv.sum(axis=1))) < 1e-12
    assert np.max(np.abs((adv ** 2).sum(axis=1) - (G - ddof))) < 1e-10
    # shift invariance and positive-scale invariance (exact powers of two keep fp32 exact)
    adv_s = orc.group_advantages((R * 4 + 8).astype(np.float32), group_size=G, eps_std=0.0,
                                 ddof=ddof).reshape(n_groups, G)
    assert np.max(np.abs(adv_s - adv)) < 1e-5
    # eps_std enters as sigma + eps_std
    adv_e = orc.group_advantages(R, group_size=G, eps_std=0.5, ddof=ddof).reshape(n_groups, G)
    sig = Rg.std(axis=1, ddof=ddof, keepdims=True)
    assert np.max(np.abs(adv_e - ref * sig / (sig + 0.5))) < 1e-12


def test_advantages_bernoulli_closed_form_ties_and_constant_groups():
    G = 16
    for k in range(1, G):
        R = np.array([1.0] * k + [0.0] * (G - k), dtype=np.float32)
        adv = orc.group_advantages(R, group_size=G, eps_std=0.0, ddof=0)
        assert np.max(np.abs(adv[:k] - math.sqrt((G - k) / k))) < 1e-12
        assert np.max(np.abs(adv[k:] + math.sqrt(k / (G - k)))) < 1e-12
        assert len(set(adv[:k].tolist())) == 1 and len(set(adv[k:].tolist())) == 1
    # all rewards equal: zero advantages (section 3.3), with or without the std guard
    for val in (0.0, 1.0, 0.3):
        R = np.full(G, val, dtype=np.float32)
        assert not orc.group_advantages(R, group_size=G, eps_std=1e-6).any()
        assert not orc.group_advantages(R, group_size=G, eps_std=0.0).any()
        assert not orc.group_advantages(R[:5], group_size=5, eps_std=0.0, ddof=1).any()
    # a single-rollout group has no spread under ddof = 1
    assert orc.group_advantages(np.array([0.7], np.float32), group_size=1, ddof=1)[0] == 0.0


def test_advantages_ragged_groups_and_broadcast():
    rng = np.random.default_rng(73)
    sizes = [3, 1, 16, 7, 0, 5]
    off = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32)
    R = rng.random(off[-1]).astype(np.float32)
    adv = orc.group_advantages(R, group_offsets=off, eps_std=1e-6, ddof=0)
    for g, n in enumerate(sizes):
        if n == 0:
            continue
        seg = R[off[g]:off[g + 1]].astype(np.float64)
        ref = (seg - seg.mean()) / (seg.std() + 1e-6)
        assert np.max(np.abs(adv[off[g]:off[g + 1]] - ref)) < 1e-12
    with pytest.raises(ValueError):
        orc.group_advantages(R, group_offsets=np.array([0, 40], np.int32))
    rot = rng.integers(0, len(R), 200).astype(np.int32)
    assert np.array_equal(orc.broadcast_advantages(adv, rot), adv[rot])


# ----------------------------------------------------------------------------
# the staged entry points are the same computation as the one-call form
# ----------------------------------------------------------------------------

def test_staged_entry_points_agree_with_one_call_form():
    rng = np.random.default_rng(81)
    N, V = 50, 37
    z, tokens, adv, mask = _tiny_batch(rng, N, V, "bf16")
    T = 0.7
    lp = orc.logprobs(z, tokens, mask, temperature=T)
    old = (lp + rng.uniform(-2, 2, N)).astype(np.float32)
    kw = dict(eps_low=0.2, eps_high=0.3, delta=4.0, grad_scale=1.5)
    one = orc.loss_fwd_bwd(z, tokens, old, adv, mask, temperature=T, grad_rows="all", **kw)
    obj = orc.objective_from_logprobs(lp, old, adv, mask, **kw)
    assert obj["loss"] == one["loss"] and np.array_equal(obj["counts"], one["counts"])
    assert np.array_equal(obj["coeff"], one["coeff"]) and np.array_equal(obj["J"], one["J"])
    pick = np.array([3, 0, 17, 49])
    g = orc.grad_rows(z[pick], tokens[pick], obj["coeff"][pick], temperature=T)
    assert np.array_equal(g, one["grad"][pick])


def test_results_do_not_depend_on_the_thread_count():
    """The row loops are the only parallel part and the reductions over rows run in row order:
    one thread, three threads and all of them give the same bits."""
    rng = np.random.default_rng(5)
    N, V = 300, 1000
    z = rng.normal(0, 3, (N, V)).astype(np.float32)
    tok = rng.integers(0, V, N)
    old = rng.normal(-7, 0.3, N).astype(np.float32)
    adv = rng.normal(0, 1, N).astype(np.float32)
    mask = (rng.random(N) > 0.2).astype(np.uint8)
    threads = orc.num_threads()
    outs = []
    try:
        for n in (1, 3, threads):
            orc.set_num_threads(n)
            assert orc.num_threads() == n
            outs.append(orc.loss_fwd_bwd(z, tok, old, adv, mask, eps_low=0.2, eps_high=0.2, delta=4.0,
                                         temperature=1.0, grad_rows="all"))
    finally:
        orc.set_num_threads(threads)
    for o in outs[1:]:
        for k in ("loss", "logprobs", "counts", "J", "coeff", "grad"):
            assert np.array_equal(np.asarray(outs[0][k]), np.asarray(o[k])), k
