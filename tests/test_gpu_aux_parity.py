"""GPU parity of the objective with the auxiliary KL and entropy terms fused in
(grpo_loss_aux_fwd_bwd) against the fp64 oracle.

Same bars as the plain objective: log-probs 2e-4 abs, total / policy loss 1e-4 rel,
gradient 4e-3 x row max, counters exact.  The two new scalars: mean KL estimate
1e-4 rel (+1e-9 abs), mean entropy 1e-4 rel (+2e-7 abs: ln(1 + x) of the fp32
normaliser cannot resolve x below 6e-8, so entropies of that size carry that absolute
error); per-token entropy 2e-4 abs like the log-probs.

One term is added to the gradient bound.  The KL part of a row's coefficient is
kl_coef (1 - exp(l_ref - l)) / D, and l_ref is handed over in fp32: at |l| = 45 its last bit is
3.8e-6, and so is the last bit of the kernel's own l.  A row whose policy part is cut and
whose l_ref - l is a few 1e-4 therefore has a gradient known only to that resolution, however it
is computed.  The bound per element becomes
    4e-3 * row max + |kl_coef grad_scale / (D T)| * 2^-22 * max(|l|, 1)
(two fp32 ulps of l), which is zero without a KL term.  Likewise the entropy part
(b/T) p_j (log p_j + H) is a difference of two numbers of size H; in fp32 it carries an error
of a few 1e-7 of (b/T) p_j H, which only shows where the true value vanishes (a uniform row has
log p_j = -H for every j): the bound gets |ent_coef grad_scale / (D T)| p_max max(H, 1) 2^-20.
Every case also counts the rows whose error exceeds 4e-3 x row max BEFORE the floors are subtracted
and allows only a small share of them (FLOOR_SHARE_MAX): the floors cannot hide a regression.
"""
import numpy as np
import pytest
import torch

import paper_2505_07291_amd as grpo
from paper_2505_07291_amd import workloads as wl
from oracle import grpo_oracle as orc
from helpers import grads_to_f64, logits_to_numpy, oracle_logprobs_blocked
from test_gpu_parity import DEV, REDUCED, TOL_GRAD, TOL_LOGP, TOL_LOSS_REL, f32, say

pytestmark = pytest.mark.gpu

# Rows that meet the gradient bound only thanks to the two floors above: at most this share of a
# case's live rows (or two rows of a small case).  The floors correct for rows whose true gradient
# (nearly) vanishes - uniform rows, rows whose policy part is cut while l_ref is within 1e-4 of l -
# which the recipes hold by the handful (1 % constant rows in numerics_stress); a kernel that needed
# them on ordinary rows would fail here.
FLOOR_SHARE_MAX = 0.02
floor_rows_allowed = 2
floor_rows = []          # (rows that needed a floor, live rows) per case, for the log


def run_aux_case(batch, old, ref, adv_f32, kl_coef, ent_coef, *, denom=0.0, grad_scale=1.0, label="",
                 token_weights=None):
    T = f32(batch["temperature"])
    kw = dict(eps_low=f32(batch["eps_low"]), eps_high=f32(batch["eps_high"]), delta=f32(batch["delta"]))
    N, V = batch["n_tokens"], batch["vocab"]
    z = logits_to_numpy(batch["logits"])
    tokens_np = batch["tokens"].cpu().numpy()
    mask_np = None if batch["mask"] is None else batch["mask"].cpu().numpy()
    ref_np = None if ref is None else ref.numpy()
    tw_np = None if token_weights is None else token_weights.cpu().numpy()
    want = orc.aux_loss_fwd_bwd(z, tokens_np, old.numpy(), ref_np, adv_f32, mask_np, temperature=T,
                                token_weights=tw_np, kl_coef=f32(kl_coef), ent_coef=f32(ent_coef), denom=denom,
                                grad_scale=f32(grad_scale), grad_rows="all", vocab=V, **kw)
    say("[gpu] %s grpo_loss_aux_fwd_bwd N=%d V=%d kl_coef=%g ent_coef=%g" % (label, N, V, kl_coef, ent_coef))
    loss, lp, ent, counts, grad = grpo.grpo_loss_aux_fwd_bwd(
        batch["logits"], batch["tokens"], old.to(DEV), None if ref is None else ref.to(DEV),
        torch.as_tensor(adv_f32, device=DEV), batch["mask"], temperature=T, kl_coef=kl_coef,
        entropy_coef=ent_coef, denom=denom, grad_scale=grad_scale, token_weights=token_weights, **kw)
    torch.cuda.synchronize()
    got = loss.cpu().numpy().astype(np.float64)
    e_lp = np.max(np.abs(lp.cpu().numpy() - want["logprobs"]))
    e_h = np.max(np.abs(ent.cpu().numpy() - want["entropies"]))
    assert e_lp <= TOL_LOGP and e_h <= 2e-4, (e_lp, e_h)
    assert counts.cpu().numpy().tolist() == want["counts"].tolist()
    assert abs(got[0] - want["total"]) <= TOL_LOSS_REL * abs(want["total"]) + 1e-12, (got[0], want["total"])
    assert abs(got[1] - want["policy"]) <= TOL_LOSS_REL * abs(want["policy"]) + 1e-12
    assert abs(got[2] - want["kl"]) <= 1e-4 * want["kl"] + 1e-9, (got[2], want["kl"])
    assert abs(got[3] - want["entropy"]) <= 1e-4 * want["entropy"] + 2e-7, (got[3], want["entropy"])
    g = grads_to_f64(grad)
    rowmax = np.max(np.abs(want["grad"]), axis=1)
    M = int(want["counts"][0])
    D = denom if denom > 0 else float(M)
    wmax = 1.0 if tw_np is None else float(np.max(np.abs(tw_np)))
    kl_floor = (wmax * abs(f32(kl_coef) * f32(grad_scale)) / (D * T) * 2.0 ** -22 *
                np.maximum(np.abs(want["logprobs"]), 1.0)) if ref is not None and D > 0 else np.zeros(N)
    zf = batch["logits"].float().cpu().numpy().astype(np.float64)
    rows = np.arange(N)
    pmax = np.exp(zf.max(axis=1) / T - zf[rows, tokens_np] / T + want["logprobs"])
    ent_floor = (wmax * abs(f32(ent_coef) * f32(grad_scale)) / (D * T) * pmax *
                 np.maximum(want["entropies"], 1.0) * 2.0 ** -20) if D > 0 else np.zeros(N)
    raw = np.max(np.abs(g - want["grad"]), axis=1)
    err = raw - kl_floor - ent_floor
    zero = want["coeff"] == 0
    zero &= want["ent_coeff"] == 0
    assert not g[zero].any(), "a zero-gradient row is not exactly zero"
    live = rowmax > 0
    assert np.all(err[~live & ~zero] <= 0)
    worst = float(np.max(err[live] / rowmax[live])) if live.any() else 0.0
    assert worst <= TOL_GRAD, "grad error %g x row max" % worst
    # the two floors must stay what they are derived as, corrections for rows whose true gradient
    # (nearly) vanishes: the rows that pass only thanks to them are counted, and few are allowed
    n_floor, n_live = int((live & (raw > TOL_GRAD * rowmax)).sum()), int(live.sum())
    floor_rows.append((n_floor, n_live))
    assert n_floor <= max(floor_rows_allowed, FLOOR_SHARE_MAX * n_live), \
        "%d of %d live rows meet the bound only with the floors" % (n_floor, n_live)
    say("      ok: |dl|=%.1e |dH|=%.1e total=%.6g kl=%.4g H=%.6g grad=%.2e x rowmax; floors used on %d of %d rows" %
        (e_lp, e_h, got[0], got[2], got[3], worst, n_floor, n_live))
    return dict(loss=loss, logprobs=lp, grad=grad, counts=counts, want=want)


@pytest.mark.parametrize("name", list(REDUCED))
@pytest.mark.parametrize("coefs", [(0.001, 1e-4), (0.05, 0.02)], ids=["paper_coefs", "large_coefs"])
def test_aux_reduced_configs_every_element(name, coefs):
    """Section 4.1 coefficients (KL 0.001, entropy 1e-4) and larger ones that make the two
    terms a visible part of the gradient, on every config's recipe."""
    cfg = REDUCED[name]
    say("\n[case] aux reduced %s: N=%d V=%d" % (name, cfg.n_tokens, cfg.vocab))
    batch = wl.make_batch(cfg, DEV)
    rewards = batch["rewards"].cpu().numpy()
    adv = orc.group_advantages(rewards, group_size=cfg.group_size, eps_std=f32(1e-6))
    adv_tok = orc.broadcast_advantages(adv, batch["rollout_of_token"].cpu().numpy()).astype(np.float32)
    lp_orc = oracle_logprobs_blocked(batch)
    old = wl.make_old_logprobs(cfg, lp_orc)
    g = torch.Generator().manual_seed(900 + cfg.index)
    ref = (torch.as_tensor(lp_orc) + torch.randn(cfg.n_tokens, generator=g, dtype=torch.float64) * 0.1).float()
    run_aux_case(batch, old, ref, adv_tok, coefs[0], coefs[1], label=name)


def test_aux_with_zero_coefficients_equals_the_plain_objective():
    cfg = REDUCED["qwen_short"]
    batch = wl.make_batch(cfg, DEV)
    lp_orc = oracle_logprobs_blocked(batch)
    old = wl.make_old_logprobs(cfg, lp_orc).to(DEV)
    adv = torch.randn(cfg.n_tokens, generator=torch.Generator().manual_seed(5)).to(DEV)
    a = grpo.grpo_loss_fwd_bwd(batch["logits"], batch["tokens"], old, adv, batch["mask"])
    b = grpo.grpo_loss_aux_fwd_bwd(batch["logits"], batch["tokens"], old, None, adv, batch["mask"])
    torch.cuda.synchronize()
    # the auxiliary kernel takes the accurate ln(1 + x) route for dominant tokens, so the
    # log-probs may differ in the last bits; the bars of the plain objective still hold
    assert torch.equal(a[2], b[3])
    assert abs(float(a[0]) - float(b[0][0])) <= 1e-4 * abs(float(a[0]))
    assert float(b[0][0]) == float(b[0][1]) and float(b[0][2]) == 0.0
    ga, gb = a[3].float(), b[4].float()
    rowmax = ga.abs().amax(dim=1)
    assert bool(((ga - gb).abs().amax(dim=1) <= 4e-3 * rowmax).all())
    assert bool((gb[rowmax == 0] == 0).all())


@pytest.mark.parametrize("dtype,vocab,stride", [("bf16", 5, 8), ("bf16", 2047, 2048), ("bf16", 50257, 50264),
                                                ("bf16", 152069, 152072), ("bf16", 200003, 200008), ("bf16", 600000, 600000),
                                                ("f32", 1000, 1004), ("f32", 100003, 100004)])
def test_aux_ragged_shapes(dtype, vocab, stride):
    run_aux_shape_case(dtype, vocab, stride, 29)


@pytest.mark.parametrize("dtype,vocab,rows", [("bf16", 50304, 600), ("bf16", 65536, 600), ("bf16", 81920, 420), ("bf16", 100352, 420), ("bf16", 128256, 420),
                                              ("bf16", 163840, 420), ("bf16", 204808, 420), ("bf16", 262144, 420),
                                              ("bf16", 278528, 300), ("bf16", 300000, 300), ("f32", 152064, 300)])
def test_aux_wide_rows_several_per_workgroup(dtype, vocab, rows):
    """Every width of the 512-lane instantiations, up to rows whose last slots live in LDS and rows with a streamed
    remainder, with more rows than workgroups; every element compared."""
    run_aux_shape_case(dtype, vocab, vocab, rows)


def run_aux_shape_case(dtype, vocab, stride, N, *, temperature=0.8, eps_low=0.2, eps_high=0.28, delta=3.0,
                       kl_coef=0.04, ent_coef=0.03, denom=40.0, grad_scale=1.5, masked=0.2, weights=False,
                       seed=None):
    say("\n[case] aux shape dtype=%s V=%d stride=%d N=%d T=%g eps=%g/%g delta=%g kl=%g ent=%g denom=%g scale=%g%s"
        % (dtype, vocab, stride, N, temperature, eps_low, eps_high, delta, kl_coef, ent_coef, denom, grad_scale,
           " weights" if weights else ""))
    g = torch.Generator().manual_seed(vocab * 3 + 1 if seed is None else seed)
    dt = torch.bfloat16 if dtype == "bf16" else torch.float32
    store = torch.full((N, stride), 7.0, dtype=dt)
    store[:, :vocab] = (torch.randn((N, vocab), generator=g) * 3).to(dt)
    if vocab > 100 and N > 3:
        store[3, 10:60] = float("-inf")                       # masked vocabulary entries ...
        store[3, vocab - 60:vocab - 10] = float("-inf")       # ... at both ends of the row
    store = store.to(DEV)
    tokens = torch.randint(0, vocab, (N,), generator=g)
    tokens[min(3, N - 1)] = 0
    mask = (torch.rand(N, generator=g) > masked).to(torch.uint8)
    mask[:4] = 1
    batch = dict(logits=store[:, :vocab], tokens=tokens.to(DEV), mask=mask.to(DEV), n_tokens=N,
                 vocab=vocab, temperature=temperature, eps_low=eps_low, eps_high=eps_high, delta=delta)
    lp_orc = oracle_logprobs_blocked(batch)
    noise = torch.rand(N, generator=g, dtype=torch.float64) * 3 - 1.5
    kinks = np.log([1.0 - f32(eps_low), 1.0 + f32(eps_high), f32(delta)])
    for t in range(N):
        while np.min(np.abs(-float(noise[t]) - kinks)) < 1e-3:
            noise[t] = torch.rand(1, generator=g, dtype=torch.float64)[0] * 3 - 1.5
    old = (torch.as_tensor(lp_orc) + noise).float()
    ref = None
    if kl_coef != 0.0:
        ref = (torch.as_tensor(lp_orc) + torch.randn(N, generator=g, dtype=torch.float64) * 0.3).float()
    adv = torch.randn(N, generator=g).numpy().astype(np.float32)
    adv[N // 2] = 0.0
    tw = None
    if weights:                                               # per-token weights, a few of them zero
        tw = (torch.rand(N, generator=g) * 2).float()
        tw[torch.rand(N, generator=g) < 0.1] = 0.0
        tw = tw.to(DEV)
    out = run_aux_case(batch, old, ref, adv, kl_coef, ent_coef, denom=denom, grad_scale=grad_scale, label="shape",
                       token_weights=tw)
    assert bool((store[:, vocab:] == 7.0).all())
    # in place: the gradient over the logits it was computed from, same bits, padding left alone
    store2 = store.clone()
    res = grpo.grpo_loss_aux_fwd_bwd(
        store2[:, :vocab], batch["tokens"], old.to(DEV), None if ref is None else ref.to(DEV),
        torch.as_tensor(adv, device=DEV), batch["mask"], f32(eps_low), f32(eps_high), f32(delta), f32(temperature),
        kl_coef, ent_coef, denom, grad_scale, token_weights=tw, inplace=True)
    torch.cuda.synchronize()
    assert res[4].data_ptr() == store2.data_ptr()
    assert torch.equal(store2[:, :vocab], out["grad"]) and torch.equal(res[0], out["loss"])
    assert bool((store2[:, vocab:] == 7.0).all())


@pytest.mark.parametrize("seed", range(16))
def test_aux_random_shapes_and_parameters(seed):
    """Seeded draws over storage type, vocabulary (half of them ending inside a 16-byte vector), pitch,
    row count, mask share, per-token weights, both coefficients (either may be zero) and every scalar
    parameter; every element compared."""
    rng = np.random.default_rng(9090 + seed)
    dtype = "bf16" if rng.random() < 0.7 else "f32"
    epv = 8 if dtype == "bf16" else 4
    vocab = int(np.exp(rng.uniform(np.log(2), np.log(300000 if dtype == "bf16" else 150000))))
    if rng.random() < 0.5:
        vocab = max(epv, vocab // epv * epv)
    stride = (vocab + epv - 1) // epv * epv + epv * int(rng.integers(0, 3))
    N = int(min(rng.integers(4, 400), max(4, 30_000_000 // vocab)))
    eps_high = float(rng.uniform(0.05, 0.5))
    kl = 0.0 if rng.random() < 0.25 else float(rng.uniform(0.001, 0.1))
    ent = 0.0 if rng.random() < 0.25 else float(rng.uniform(1e-4, 0.05))
    run_aux_shape_case(dtype, vocab, stride, N, temperature=float(rng.uniform(0.5, 1.5)),
                       eps_low=float(rng.uniform(0.05, 0.5)), eps_high=eps_high,
                       delta=1.0 + eps_high + float(rng.uniform(0.2, 4.0)), kl_coef=f32(kl), ent_coef=f32(ent),
                       denom=0.0 if rng.random() < 0.3 else float(rng.uniform(10, 1000)),
                       grad_scale=f32(rng.uniform(0.1, 4.0)), masked=float(rng.uniform(0.0, 0.8)),
                       weights=bool(rng.random() < 0.5), seed=313 * seed + 5)


def test_aux_only_entropy_no_reference():
    """kl_coef = 0 with ref_logprobs = NULL is legal; clipped rows still get the entropy gradient."""
    cfg = REDUCED["numerics_stress"]
    batch = wl.make_batch(cfg, DEV)
    lp_orc = oracle_logprobs_blocked(batch)
    old = wl.make_old_logprobs(cfg, lp_orc)
    adv = np.where(np.arange(cfg.n_tokens) % 3 == 0, 0.0, 1.0).astype(np.float32)
    out = run_aux_case(batch, old, None, adv, 0.0, 0.05, label="entropy only")
    assert out["want"]["kl"] == 0.0


@pytest.mark.parametrize("name", ["qwen_short", "qwen_medium", "long_reasoning", "numerics_stress"])
def test_aux_full_size(name):
    """Benchmark shapes: log-probs, entropies, the four loss scalars and the counters for every
    row; gradients element by element on sampled rows of every class and on the unmasked rows of a
    seeded sample of 8192 rows; masked rows zero throughout."""
    from helpers import sample_rows_by_class
    cfg = wl.CONFIGS[name]
    klc, enc = 0.001, 1e-4                                     # section 4.1
    say("\n[case] aux full size %s: N=%d V=%d" % (name, cfg.n_tokens, cfg.vocab))
    batch = wl.make_batch(cfg, DEV)
    N, V, T = cfg.n_tokens, cfg.vocab, f32(cfg.temperature)
    rewards = batch["rewards"].cpu().numpy()
    adv = orc.group_advantages(rewards, group_size=cfg.group_size, eps_std=f32(1e-6))
    adv_tok = orc.broadcast_advantages(adv, batch["rollout_of_token"].cpu().numpy()).astype(np.float32)
    tokens_np, mask_np = batch["tokens"].cpu().numpy(), batch["mask"].cpu().numpy()
    lp_orc, H_orc = np.zeros(N), np.zeros(N)
    for r0 in range(0, N, 4096):
        r1 = min(N, r0 + 4096)
        if mask_np[r0:r1].any():
            z = logits_to_numpy(batch["logits"][r0:r1])
            lp_orc[r0:r1] = orc.logprobs(z, tokens_np[r0:r1], mask_np[r0:r1], temperature=T)
            H_orc[r0:r1] = orc.entropies(z, mask_np[r0:r1], temperature=T)
        say("    oracle rows done: %d" % r1)
    old = wl.make_old_logprobs(cfg, lp_orc)
    g = torch.Generator().manual_seed(900 + cfg.index)
    ref = (torch.as_tensor(lp_orc) + torch.randn(N, generator=g, dtype=torch.float64) * 0.1).float()
    kw = dict(eps_low=f32(cfg.eps_low), eps_high=f32(cfg.eps_high), delta=f32(cfg.delta))
    want = orc.aux_objective_from_logprobs(lp_orc, H_orc, old.numpy(), ref.numpy(), adv_tok, mask_np,
                                           kl_coef=f32(klc), ent_coef=f32(enc), **kw)
    loss, lp, ent, counts, grad = grpo.grpo_loss_aux_fwd_bwd(
        batch["logits"], batch["tokens"], old.to(DEV), ref.to(DEV), torch.as_tensor(adv_tok, device=DEV),
        batch["mask"], temperature=T, kl_coef=klc, entropy_coef=enc, **kw)
    torch.cuda.synchronize()
    got = loss.cpu().numpy().astype(np.float64)
    assert np.max(np.abs(lp.cpu().numpy() - lp_orc)) <= TOL_LOGP
    assert np.max(np.abs(ent.cpu().numpy() - H_orc)) <= 2e-4
    assert counts.cpu().numpy().tolist() == want["counts"].tolist()
    assert abs(got[0] - want["total"]) <= TOL_LOSS_REL * abs(want["total"])
    assert abs(got[1] - want["policy"]) <= TOL_LOSS_REL * abs(want["policy"])
    assert abs(got[2] - want["kl"]) <= 1e-4 * want["kl"] + 1e-9
    assert abs(got[3] - want["entropy"]) <= 1e-4 * want["entropy"] + 2e-7
    M = int(mask_np.sum())

    def worst_error(rows):
        """Largest gradient error of these rows in units of their row maximum, beyond the floors."""
        rows_t = torch.as_tensor(rows, device=DEV)
        z_rows = logits_to_numpy(batch["logits"][rows_t])
        g_orc = orc.aux_grad_rows(z_rows, tokens_np[rows], want["coeff"][rows], want["ent_coeff"][rows], T, vocab=V)
        g_gpu = grads_to_f64(grad[rows_t])
        zf = batch["logits"][rows_t].float().cpu().numpy().astype(np.float64)
        pmax = np.exp(zf.max(axis=1) / T - zf[np.arange(len(rows)), tokens_np[rows]] / T + lp_orc[rows])
        assert np.all(pmax[mask_np[rows] != 0] <= 1.0 + 1e-9)      # a probability where the row takes part
        floor = (klc / (M * T) * 2.0 ** -22 * np.maximum(np.abs(lp_orc[rows]), 1.0) +
                 enc / (M * T) * pmax * np.maximum(H_orc[rows], 1.0) * 2.0 ** -20)
        rowmax = np.max(np.abs(g_orc), axis=1)
        raw = np.max(np.abs(g_gpu - g_orc), axis=1)
        err = raw - floor
        assert not g_gpu[mask_np[rows] == 0].any()
        live = rowmax > 0
        floored[0] += int((live & (raw > TOL_GRAD * rowmax)).sum())
        floored[1] += int(live.sum())
        return float(np.max(err[live] / rowmax[live])) if live.any() else 0.0

    floored = [0, 0]        # rows that meet the bound only with the floors, live rows compared

    rows = sample_rows_by_class(want["coeff"], mask_np, np.random.default_rng(7), 40)
    worst = worst_error(rows)
    assert worst <= TOL_GRAD, worst
    # ... and on a seeded sample of 8192 rows, in blocks (with an entropy term every unmasked row
    # has a gradient); masked rows of the whole batch must be zero
    sample = np.sort(np.random.default_rng(2000 + cfg.index).choice(N, size=min(N, 8192), replace=False))
    sample = sample[mask_np[sample] != 0]
    for b in range(0, len(sample), 256):
        worst = max(worst, worst_error(sample[b:b + 256]))
    assert worst <= TOL_GRAD, worst
    masked_t = torch.as_tensor(mask_np == 0, device=DEV)
    for r0 in range(0, N, 8192):
        blk = grad[r0:r0 + 8192][masked_t[r0:r0 + 8192]]
        assert not bool(blk.any()), "a masked row is not zero"
    assert floored[0] <= FLOOR_SHARE_MAX * floored[1], "%d of %d live rows meet the bound only with the floors" % tuple(floored)
    say("  ok: total=%.6g policy=%.6g kl=%.4g H=%.5g grad=%.2e x rowmax on %d + %d rows; floors used on %d of %d live rows" %
        (got[0], got[1], got[2], got[3], worst, len(rows), len(sample), floored[0], floored[1]))


@pytest.mark.parametrize("sample_level", [True, False])
def test_packed_batch_with_sample_level_weights(sample_level):
    """Variable-length rollouts packed back to back (no padding rows), advantages broadcast
    through the rollout index the library derives from cu_seqlens, and the objective
    normalised per sample as printed in section 3.4 (or per token), with both auxiliary
    terms.  A few rows before and after the rollouts belong to nobody (weight 0)."""
    g = torch.Generator().manual_seed(17 + sample_level)
    G, n_prompts, V = 4, 3, 50257
    lens = torch.randint(1, 9, (G * n_prompts,), generator=g)
    lens[5] = 0                                               # an empty response
    cu = torch.cat([torch.tensor([2]), 2 + torch.cumsum(lens, 0)])
    N = int(cu[-1]) + 3
    say("\n[case] packed: %d rollouts, N=%d V=%d sample_level=%s" % (len(lens), N, V, sample_level))
    w, rot = grpo.grpo_packed_layout(cu.to(DEV), N, sample_level)
    torch.cuda.synchronize()
    w_ref, rot_ref = orc.packed_layout(cu.numpy(), N, sample_level)
    assert np.array_equal(rot.cpu().numpy(), rot_ref)
    assert np.array_equal(w.cpu().numpy(), w_ref)             # 1/len is correctly rounded on both sides
    rewards = (torch.rand(G * n_prompts, generator=g) < 0.4).float()
    adv = orc.group_advantages(rewards.numpy(), group_size=G, eps_std=f32(1e-6))
    adv_gpu, _ = grpo.grpo_group_advantages(rewards.to(DEV), group_size=G)
    adv_tok = np.where(rot_ref >= 0, adv[np.maximum(rot_ref, 0)], 0.0).astype(np.float32)
    store = torch.full((N, V + 7), 7.0, dtype=torch.bfloat16)
    store[:, :V] = (torch.randn((N, V), generator=g) * 3).to(torch.bfloat16)
    store[:2] = float("nan")                                  # rows nobody owns are never read
    store = store.to(DEV)
    tokens = torch.randint(0, V, (N,), generator=g)
    batch = dict(logits=store[:, :V], tokens=tokens.to(DEV), mask=None, n_tokens=N, vocab=V,
                 temperature=1.0, eps_low=0.2, eps_high=0.2, delta=4.0)
    live = (w_ref != 0).astype(np.uint8)
    lp_orc = orc.logprobs(logits_to_numpy(batch["logits"]), tokens.numpy(), live)
    noise = torch.randn(N, generator=g, dtype=torch.float64) * 0.15
    kinks = np.log([0.8, 1.2, 4.0])
    for t in range(N):                                        # keep the ratios clear of the kinks
        while np.min(np.abs(-float(noise[t]) - kinks)) < 1e-3:
            noise[t] = torch.randn(1, generator=g, dtype=torch.float64)[0] * 0.15
    old = (torch.as_tensor(lp_orc) + noise).float()
    ref = (torch.as_tensor(lp_orc) + torch.randn(N, generator=g, dtype=torch.float64) * 0.1).float()
    denom = float(len(lens)) if sample_level else 0.0
    out = run_aux_case(batch, old, ref, adv_tok, 0.02, 0.01, denom=denom, token_weights=w, label="packed")
    assert int(out["counts"][0]) == int(lens.sum())
