"""GPU parity: the HIP path (through the C ABI) against the fp64 oracle, element by element.

Tolerances are the ones the benchmark definition states for fp32 accumulation:
  per-token log-prob   |dl|    <= 2e-4
  loss                 rel     <= 1e-4
  grad-logits          |dg|    <= 4e-3 * (row max |grad|)   (bf16 rounding alone is 2e-3)
  clip-indicator counts        exact
Rows whose gradient is zero in the oracle (masked, clipped, zero advantage) must be
exactly zero on the GPU: their row max is 0, so the bound above allows nothing else.
"""
import sys

import numpy as np
import pytest
import torch

import paper_2505_07291_amd as grpo
from paper_2505_07291_amd import workloads as wl
from oracle import grpo_oracle as orc
from helpers import (grads_to_f64, logits_to_numpy, oracle_logprobs_blocked,
                     sample_rows_by_class)

pytestmark = pytest.mark.gpu

TOL_LOGP = 2e-4
TOL_LOSS_REL = 1e-4
TOL_GRAD = 4e-3
DEV = "cuda"


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


def f32(x):
    """The python float a C `float` argument will hold: both sides get the same number."""
    return float(np.float32(x))


def oracle_side(batch, ddof=0, eps_std=1e-6):
    """Oracle advantages -> log-probs (blocked) for a batch; returns numpy pieces."""
    rewards = batch["rewards"].cpu().numpy()
    adv = orc.group_advantages(rewards, group_size=batch["group_size"], eps_std=f32(eps_std), ddof=ddof)
    adv_tok = orc.broadcast_advantages(adv, batch["rollout_of_token"].cpu().numpy())
    lp = oracle_logprobs_blocked(batch)
    return adv, adv_tok, lp


def check_against_oracle(batch, old, lp_orc, adv_tok_f32, *, denom=0.0, grad_scale=1.0,
                         grad_rows="all", inplace=False, gpu_adv=None, label=""):
    """Runs grpo_loss_fwd_bwd and compares every output with the oracle."""
    cfg_kw = dict(eps_low=f32(batch["eps_low"]), eps_high=f32(batch["eps_high"]),
                  delta=f32(batch["delta"]))
    T = f32(batch["temperature"])
    N, V = batch["n_tokens"], batch["vocab"]
    mask_np = batch["mask"].cpu().numpy()
    tokens_np = batch["tokens"].cpu().numpy()
    obj = orc.objective_from_logprobs(lp_orc, old.numpy(), adv_tok_f32, mask_np, denom=denom,
                                      grad_scale=f32(grad_scale), **cfg_kw)
    if isinstance(grad_rows, str):
        grad_rows = np.arange(N)
    # the rows' logits must be fetched before an in-place call overwrites them
    rows_t = torch.as_tensor(grad_rows, device=DEV)
    z_rows = logits_to_numpy(batch["logits"][rows_t]) if len(grad_rows) else None

    adv_dev = gpu_adv if gpu_adv is not None else torch.as_tensor(adv_tok_f32, device=DEV)
    say("[gpu] %s grpo_loss_fwd_bwd N=%d V=%d stride=%d dtype=%s inplace=%s" %
        (label, N, V, batch["logits"].stride(0), batch["logits"].dtype, inplace))
    loss, lp, counts, grad = grpo.grpo_loss_fwd_bwd(
        batch["logits"], batch["tokens"], old.to(DEV), adv_dev, batch["mask"],
        temperature=T, denom=denom, grad_scale=grad_scale, inplace=inplace, **cfg_kw)
    torch.cuda.synchronize()

    lp_gpu = lp.cpu().numpy().astype(np.float64)
    err_lp = np.max(np.abs(lp_gpu - lp_orc)) if N else 0.0
    assert err_lp <= TOL_LOGP, "log-prob error %g" % err_lp
    assert np.all(lp_gpu[mask_np == 0] == 0.0)
    assert counts.cpu().numpy().tolist() == obj["counts"].tolist(), "indicator counts differ"
    lg, lo = float(loss.item()), obj["loss"]
    assert abs(lg - lo) <= TOL_LOSS_REL * abs(lo) + 1e-12, "loss %r vs oracle %r" % (lg, lo)

    worst = 0.0
    if len(grad_rows):
        g_gpu = grads_to_f64(grad[rows_t])
        g_orc = orc.grad_rows(z_rows, tokens_np[grad_rows], obj["coeff"][grad_rows], temperature=T, vocab=V)
        rowmax = np.max(np.abs(g_orc), axis=1)
        err = np.max(np.abs(g_gpu - g_orc), axis=1)
        zero = rowmax == 0
        assert not g_gpu[zero].any(), "a zero-gradient row is not exactly zero"
        if (~zero).any():
            worst = float(np.max(err[~zero] / rowmax[~zero]))
        assert worst <= TOL_GRAD, "grad error %g x row max" % worst
    say("      ok: |dl|=%.2e  loss=%.6g (rel %.1e)  grad=%.2e x rowmax  counts=%s" %
        (err_lp, lg, abs(lg - lo) / max(abs(lo), 1e-300), worst, obj["counts"].tolist()))
    return dict(loss=loss, logprobs=lp, counts=counts, grad=grad, obj=obj)


REDUCED = {
    "tiny": wl.CONFIGS["tiny"],
    "qwen_short": wl.CONFIGS["qwen_short"].scaled(n_prompts=2, seq_len=6),
    "qwen_medium": wl.CONFIGS["qwen_medium"].scaled(n_prompts=2, seq_len=6),
    "long_reasoning": wl.CONFIGS["long_reasoning"].scaled(n_prompts=3, seq_len=8),
    "numerics_stress": wl.CONFIGS["numerics_stress"].scaled(n_prompts=2, seq_len=8),
}


@pytest.mark.parametrize("name", list(REDUCED))
def test_reduced_configs_every_element(name):
    """Whole hot path (advantages -> loss -> gradient), every output element, on each
    config's recipe at a row count the oracle finishes in seconds (vocabulary at full size)."""
    cfg = REDUCED[name]
    say("\n[case] reduced %s: N=%d V=%d" % (name, cfg.n_tokens, cfg.vocab))
    batch = wl.make_batch(cfg, DEV)
    adv, adv_tok, lp_orc = oracle_side(batch)
    old = wl.make_old_logprobs(cfg, lp_orc)
    # advantages on the GPU, then fed to the GPU loss: the chain the benchmark times
    adv_gpu, adv_tok_gpu = grpo.grpo_group_advantages(
        batch["rewards"], group_size=cfg.group_size, eps_std=1e-6, ddof=0,
        rollout_of_token=batch["rollout_of_token"])
    torch.cuda.synchronize()
    a = adv_gpu.cpu().numpy().astype(np.float64)
    assert np.max(np.abs(a - adv)) <= 1e-6 * max(1.0, np.max(np.abs(adv)))
    assert np.array_equal(adv_tok_gpu.cpu().numpy(), adv_gpu.cpu().numpy()[batch["rollout_of_token"].cpu().numpy()])
    out = check_against_oracle(batch, old, lp_orc, adv_tok.astype(np.float32), gpu_adv=adv_tok_gpu,
                               label=name)
    # old-policy log-probs entry point on the same rows
    lp_fwd = grpo.grpo_logprobs_fwd(batch["logits"], batch["tokens"], batch["mask"],
                                    temperature=f32(cfg.temperature))
    torch.cuda.synchronize()
    assert np.max(np.abs(lp_fwd.cpu().numpy() - lp_orc)) <= TOL_LOGP
    assert torch.equal(lp_fwd, out["logprobs"])
    # ... and without the row queue (fixed strided assignment): same bits
    lp_strided = grpo.grpo_logprobs_fwd(batch["logits"], batch["tokens"], batch["mask"],
                                        temperature=f32(cfg.temperature), use_queue=False)
    torch.cuda.synchronize()
    assert torch.equal(lp_fwd, lp_strided)
    # every counter the recipe is meant to exercise is exercised
    if name in ("qwen_medium", "numerics_stress"):
        assert min(out["obj"]["counts"][1:].tolist()[0:2]) > 0
    if name == "numerics_stress":
        assert out["obj"]["counts"][3] > 0


RAGGED = [
    # (dtype, vocab, row_stride)   kernels: register-resident at several widths, streamed
    ("bf16", 1, 8), ("bf16", 5, 8), ("bf16", 8, 8), ("bf16", 2047, 2048), ("bf16", 2048, 2048),
    ("bf16", 8200, 8208), ("bf16", 50257, 50264), ("bf16", 81921, 81928),
    ("bf16", 152064, 152064), ("bf16", 152069, 152072), ("bf16", 155649, 155656), ("bf16", 200003, 200008),
    ("bf16", 600000, 600000),                    # too wide to keep half of it resident: streamed
    ("f32", 1, 4), ("f32", 3, 4), ("f32", 1000, 1004), ("f32", 4099, 4100), ("f32", 40001, 40004),
    ("f32", 40000, 40000), ("f32", 77824, 77824), ("f32", 100003, 100004), ("f32", 300000, 300000),
]


def run_shape_case(dtype, vocab, stride, N, grad_rows="all", *, temperature=0.9, eps_low=0.2, eps_high=0.28,
                   delta=3.0, denom=50.0, grad_scale=2.5, masked=0.25, seed=None):
    say("\n[case] shape dtype=%s V=%d stride=%d N=%d T=%g eps=%g/%g delta=%g denom=%g scale=%g" %
        (dtype, vocab, stride, N, temperature, eps_low, eps_high, delta, denom, grad_scale))
    g = torch.Generator().manual_seed(vocab * 7 + (dtype == "f32") if seed is None else seed)
    dt = torch.bfloat16 if dtype == "bf16" else torch.float32
    store = torch.full((N, stride), 7.0, dtype=dt)            # padding holds a sentinel
    store[:, :vocab] = (torch.randn((N, vocab), generator=g) * 3).to(dt)
    store = store.to(DEV)
    logits = store[:, :vocab]
    tokens = torch.randint(0, vocab, (N,), generator=g)
    tokens[0], tokens[-1] = vocab - 1, 0                       # last and first element of a row
    mask = (torch.rand(N, generator=g) > masked).to(torch.uint8)
    mask[:2] = 1
    batch = dict(logits=logits, tokens=tokens.to(DEV), mask=mask.to(DEV), n_tokens=N, vocab=vocab,
                 temperature=temperature, eps_low=eps_low, eps_high=eps_high, delta=delta)
    lp_orc = oracle_logprobs_blocked(batch)
    noise = torch.rand(N, generator=g, dtype=torch.float64) * 4 - 2
    kinks = np.log([1.0 - f32(eps_low), 1.0 + f32(eps_high), f32(delta)]) if eps_low < 1 else \
        np.log([1.0 + f32(eps_high), f32(delta)])
    for t in range(N):                                         # keep clear of the kinks
        while np.min(np.abs(-float(noise[t]) - kinks)) < 1e-3:
            noise[t] = torch.rand(1, generator=g, dtype=torch.float64)[0] * 4 - 2
    old = (torch.as_tensor(lp_orc) + noise).to(torch.float32)
    adv = torch.randn(N, generator=g).numpy().astype(np.float32)
    adv[N // 2] = 0.0
    out = check_against_oracle(batch, old, lp_orc, adv, denom=denom, grad_scale=grad_scale, label="shape",
                               grad_rows=grad_rows)
    pad = store[:, vocab:]
    assert bool((pad == 7.0).all()), "logits padding was written"
    # gradient buffer padding must be left alone too: run into a pre-filled buffer
    gbuf = torch.full((N, stride), 3.0, dtype=dt, device=DEV)
    gview = gbuf[:, :vocab]
    grpo.grpo_loss_fwd_bwd(logits, batch["tokens"], old.to(DEV), torch.as_tensor(adv, device=DEV),
                           batch["mask"], f32(eps_low), f32(eps_high), f32(delta), f32(temperature), denom,
                           grad_scale, grad_logits=gview)
    torch.cuda.synchronize()
    assert bool((gbuf[:, vocab:] == 3.0).all()), "gradient padding was written"
    assert torch.equal(gview, out["grad"])
    lp_fwd = grpo.grpo_logprobs_fwd(logits, batch["tokens"], batch["mask"], temperature=f32(temperature))
    torch.cuda.synchronize()
    assert torch.equal(lp_fwd, out["logprobs"])
    # in place: the gradient over the logits it was computed from, same bits, padding left alone
    store2 = store.clone()
    res = grpo.grpo_loss_fwd_bwd(store2[:, :vocab], batch["tokens"], old.to(DEV), torch.as_tensor(adv, device=DEV),
                                 batch["mask"], f32(eps_low), f32(eps_high), f32(delta), f32(temperature), denom,
                                 grad_scale, inplace=True)
    torch.cuda.synchronize()
    assert res[3].data_ptr() == store2.data_ptr()
    assert torch.equal(store2[:, :vocab], out["grad"]) and torch.equal(res[0], out["loss"])
    assert bool((store2[:, vocab:] == 7.0).all()), "padding was written by the in-place call"


@pytest.mark.parametrize("seed", range(24))
def test_random_shapes_and_parameters(seed):
    """Seeded draws over the whole argument space at once: storage type, vocabulary from a handful of
    entries to 300000 (half of them ending inside a 16-byte vector), padded row pitch, row count,
    share of masked rows, temperature, both clip widths, the cap, denominator and upstream gradient."""
    rng = np.random.default_rng(4242 + seed)
    dtype = "bf16" if rng.random() < 0.7 else "f32"
    epv = 8 if dtype == "bf16" else 4
    vocab = int(np.exp(rng.uniform(np.log(2), np.log(300000 if dtype == "bf16" else 150000))))
    if rng.random() < 0.5:
        vocab = max(epv, vocab // epv * epv)
    stride = (vocab + epv - 1) // epv * epv + epv * int(rng.integers(0, 3))
    N = int(min(rng.integers(2, 700), max(2, 120_000_000 // vocab)))
    eps_high = float(rng.uniform(0.05, 0.5))
    kw = dict(temperature=float(rng.uniform(0.5, 1.5)), eps_low=float(rng.uniform(0.05, 0.5)), eps_high=eps_high,
              delta=1.0 + eps_high + float(rng.uniform(0.2, 4.0)),
              denom=0.0 if rng.random() < 0.3 else float(rng.uniform(10, 1000)),
              grad_scale=f32(rng.uniform(0.1, 4.0)), masked=float(rng.uniform(0.0, 0.9)), seed=977 * seed + 1)
    rows = "all" if N * vocab <= 20_000_000 else np.unique(np.concatenate(
        [[0, 1, N - 1], rng.choice(N, size=min(N, 24), replace=False)]))
    run_shape_case(dtype, vocab, stride, N, grad_rows=rows, **kw)


@pytest.mark.parametrize("dtype,vocab,stride", RAGGED)
def test_ragged_shapes_and_strides(dtype, vocab, stride):
    """Row widths that end inside a 16-byte vector, padded row pitches, a row count that
    does not divide the grid, asymmetric clipping, an imposed denominator and a
    non-unit upstream gradient; every element compared."""
    run_shape_case(dtype, vocab, stride, 37)


WIDE = [
    # (dtype, vocab, row_stride, rows): more rows than workgroups, so that each workgroup takes several
    # in turn and refills its registers and LDS from the next row while it finishes the current one
    ("bf16", 50304, 50304, 900),     # 256 lanes with 256 registers, 26 slots, two workgroups per CU
    ("bf16", 65536, 65536, 900),     # ... 32 slots
    ("f32", 32768, 32768, 900),      # ... the same in fp32
    ("bf16", 65544, 65552, 800),     # the narrowest row on 512 lanes with 256 registers (20 slots)
    ("bf16", 81920, 81920, 800),     # ... and the widest: all 20 slots used, every store behind the loads
    ("bf16", 100352, 100352, 800),   # 26 register slots
    ("bf16", 128256, 128256, 800),   # 32 register slots
    ("bf16", 163840, 163848, 800),   # 44 register slots
    ("bf16", 204808, 204808, 800),   # one lane reaches into the first LDS-resident slot
    ("bf16", 230400, 230400, 700),   # the instantiation with 10 LDS-resident slots
    ("bf16", 262144, 262144, 800),   # 14 of 18 LDS-resident slots used
    ("bf16", 278528, 278528, 600),   # the widest row that is read once
    ("bf16", 270344, 270344, 600),   # one vector beyond registers + LDS of the instantiation with a remainder
    ("bf16", 300000, 300000, 600),   # a streamed remainder of a few slots
    ("bf16", 540672, 540672, 300),   # the widest row with a streamed remainder: half of it
    ("f32", 135172, 135172, 600),    # the same in fp32: one vector of remainder
    ("f32", 152064, 152064, 600),    # the benchmark's vocabulary in fp32: 8 slots of remainder
]


@pytest.mark.parametrize("dtype,vocab,stride,rows", WIDE)
def test_wide_rows_several_per_workgroup(dtype, vocab, stride, rows):
    """Vocabularies beside the benchmark's, each on the instantiation of its width, up to rows wider
    than the registers, whose last slots live in LDS, and rows wider than both, whose remainder is
    streamed.  All log-probs, the loss and the counters; gradients of the first and last rows and
    of a seeded sample in between."""
    rng = np.random.default_rng(vocab)
    pick = np.unique(np.concatenate([np.arange(12), np.arange(rows - 12, rows),
                                     rng.choice(rows, size=100, replace=False)]))
    run_shape_case(dtype, vocab, stride, rows, grad_rows=pick)


# widest vocabulary (bf16) of each instantiation of the row kernel, in dispatch order
WIDTH_LIMITS = [2048, 8192, 32768, 53248, 65536, 81920, 106496, 131072, 155648, 180224, 221184, 245760,
                278528, 540672]


@pytest.mark.parametrize("limit", WIDTH_LIMITS)
def test_both_sides_of_every_width_limit(limit):
    """The last vocabulary an instantiation serves and the first one of the next (one more 16-byte
    vector): a row that fills every slot to the last lane, and one with a single lane in a new slot."""
    for vocab in (limit, limit + 8):
        rows = 300
        rng = np.random.default_rng(vocab)
        pick = np.unique(np.concatenate([np.arange(4), np.arange(rows - 4, rows),
                                         rng.choice(rows, size=24, replace=False)]))
        run_shape_case("bf16", vocab, vocab, rows, grad_rows=pick)


def test_inplace_gradient_and_bitwise_determinism():
    cfg = wl.CONFIGS["qwen_short"].scaled(n_prompts=2, seq_len=5)
    say("\n[case] in-place + determinism: N=%d V=%d" % (cfg.n_tokens, cfg.vocab))
    batch = wl.make_batch(cfg, DEV)
    adv, adv_tok, lp_orc = oracle_side(batch)
    old = wl.make_old_logprobs(cfg, lp_orc)
    a32 = adv_tok.astype(np.float32)
    first = check_against_oracle(batch, old, lp_orc, a32, label="run 1")
    second = check_against_oracle(batch, old, lp_orc, a32, label="run 2")
    for k in ("loss", "logprobs", "counts", "grad"):
        assert torch.equal(first[k], second[k]), k + " differs between two identical runs"
    third = check_against_oracle(batch, old, lp_orc, a32, inplace=True, label="in place")
    assert third["grad"].data_ptr() == batch["logits"].data_ptr()
    for k in ("loss", "logprobs", "counts", "grad"):
        assert torch.equal(first[k], third[k]), k + " differs in place"


def test_the_comparison_rejects_a_wrong_oracle():
    """The comparator itself can fail: with a mistake planted on the oracle's side (never in the
    library) the same check that passes above raises."""
    cfg = wl.CONFIGS["numerics_stress"].scaled(n_prompts=2, seq_len=6)
    batch = wl.make_batch(cfg, DEV)
    adv, adv_tok, lp_orc = oracle_side(batch)
    old = wl.make_old_logprobs(cfg, lp_orc)
    a32 = adv_tok.astype(np.float32)
    check_against_oracle(batch, old, lp_orc, a32, label="as it is")
    live = int(np.flatnonzero(batch["mask"].cpu().numpy())[3])
    wrong_lp = lp_orc.copy()
    wrong_lp[live] += 3e-4                                      # one log-prob off by 1.5 tolerances
    with pytest.raises(AssertionError, match="log-prob error"):
        check_against_oracle(batch, old, wrong_lp, a32, label="log-prob off")
    hot = dict(batch, temperature=batch["temperature"] * 1.001)  # the oracle's softmax at another temperature
    with pytest.raises(AssertionError, match="log-prob error"):
        check_against_oracle(batch, old, oracle_logprobs_blocked(hot), a32, label="temperature off")
    flipped = a32.copy()
    flipped[live] = -flipped[live] if flipped[live] != 0 else 1.0  # the oracle with one advantage of the other sign
    with pytest.raises(AssertionError):
        check_against_oracle(batch, old, lp_orc, flipped, gpu_adv=torch.as_tensor(a32, device=DEV),
                             label="one advantage off")


def test_micro_batches_add_up():
    """A batch cut into micro-batches that all receive the whole batch's token count as `denom`
    (what a trainer with gradient accumulation, or one rank of several, does): per-row outputs
    are the whole batch's bits, losses and counters add up."""
    cfg = wl.CONFIGS["qwen_medium"].scaled(n_prompts=2, seq_len=7)
    batch = wl.make_batch(cfg, DEV)
    N = cfg.n_tokens
    say("\n[case] micro-batches: N=%d V=%d" % (N, cfg.vocab))
    adv, adv_tok, lp_orc = oracle_side(batch)
    old = wl.make_old_logprobs(cfg, lp_orc).to(DEV)
    a_dev = torch.as_tensor(adv_tok.astype(np.float32), device=DEV)
    kw = dict(eps_low=f32(cfg.eps_low), eps_high=f32(cfg.eps_high), delta=f32(cfg.delta),
              temperature=f32(cfg.temperature))
    loss, lp, counts, grad = grpo.grpo_loss_fwd_bwd(batch["logits"], batch["tokens"], old, a_dev, batch["mask"], **kw)
    torch.cuda.synchronize()
    M = int(counts[0].item())
    cuts = [0, N // 5, N // 5 + 1, N // 2, N]                 # uneven pieces, one of a single row
    loss_sum, counts_sum = 0.0, torch.zeros_like(counts)
    for b, e in zip(cuts[:-1], cuts[1:]):
        l_i, lp_i, c_i, g_i = grpo.grpo_loss_fwd_bwd(batch["logits"][b:e], batch["tokens"][b:e], old[b:e],
                                                     a_dev[b:e], batch["mask"][b:e], denom=float(M), **kw)
        torch.cuda.synchronize()
        assert torch.equal(lp_i, lp[b:e]) and torch.equal(g_i, grad[b:e]), (b, e)
        loss_sum += float(l_i.item())
        counts_sum += c_i
    assert torch.equal(counts_sum, counts)
    assert abs(loss_sum - float(loss.item())) <= 1e-6 * abs(float(loss.item())) + 1e-9


@pytest.mark.parametrize("V", [4096, 152064, 262144, 300000, 600000])
def test_edge_cases(V):
    """Degenerate inputs on every kind of row kernel: rows in registers (narrow, and the benchmark's
    width with waiting gradient slots), rows partly in LDS, rows with a streamed remainder, and
    the streaming kernel.  The poisoned entries sit at the far end of the row, i.e. in the LDS-resident
    slots or the remainder where there are such."""
    N = 24
    g = torch.Generator().manual_seed(3)
    logits = (torch.randn((N, V), generator=g) * 2).to(torch.bfloat16).to(DEV)
    tokens = torch.randint(0, V, (N,), generator=g).to(DEV)
    old = torch.full((N,), -8.0, device=DEV)
    adv = torch.randn(N, generator=g).to(DEV)
    ones = torch.ones(N, dtype=torch.uint8, device=DEV)

    say("\n[case] edge: n_tokens = 0")
    e = logits[:0]
    loss, lp, counts, grad = grpo.grpo_loss_fwd_bwd(e, tokens[:0], old[:0], adv[:0], ones[:0])
    torch.cuda.synchronize()
    assert float(loss) == 0.0 and counts.tolist() == [0] * 5
    assert grpo.grpo_logprobs_fwd(e, tokens[:0]).numel() == 0

    say("[case] edge: every row masked, inputs poisoned")
    poison = torch.full_like(logits, float("nan"))
    bad_tok = torch.full_like(tokens, 10 ** 12)
    zeros = torch.zeros_like(ones)
    loss, lp, counts, grad = grpo.grpo_loss_fwd_bwd(poison, bad_tok, old * float("nan"), adv * float("nan"), zeros)
    torch.cuda.synchronize()
    assert float(loss) == 0.0 and counts.tolist() == [0] * 5
    assert not grad.any() and not lp.any()

    say("[case] edge: mask NULL equals mask of ones")
    a = grpo.grpo_loss_fwd_bwd(logits, tokens, old, adv, None)
    b = grpo.grpo_loss_fwd_bwd(logits, tokens, old, adv, ones)
    torch.cuda.synchronize()
    for x, y in zip(a, b):
        assert torch.equal(x, y)
    assert int(a[2][0]) == N

    say("[case] edge: token id out of range -> row behaves as masked, error word set")
    tok2 = tokens.clone()
    tok2[5], tok2[9] = V, -1
    ws = torch.empty(grpo.grpo_workspace_bytes(N), dtype=torch.uint8, device=DEV)
    loss2, lp2, counts2, grad2 = grpo.grpo_loss_fwd_bwd(logits, tok2, old, adv, ones, workspace=ws)
    assert grpo.grpo_workspace_error(ws) == 1
    assert not grad2[5].any() and not grad2[9].any() and float(lp2[5]) == 0.0
    assert int(counts2[0]) == N
    grpo.grpo_loss_fwd_bwd(logits, tokens, old, adv, ones, workspace=ws)
    assert grpo.grpo_workspace_error(ws) == 0                    # the word is reset by every call
    lpf = grpo.grpo_logprobs_fwd(logits, tok2)
    torch.cuda.synchronize()
    assert bool(torch.isnan(lpf[5])) and bool(torch.isnan(lpf[9])) and not bool(torch.isnan(lpf[0]))

    say("[case] edge: NaN in one row's logits reaches that row's outputs and the loss, nothing else")
    z3 = logits.clone()
    z3[7, V - 100] = float("nan")
    loss3, lp3, counts3, grad3 = grpo.grpo_loss_fwd_bwd(z3, tokens, old, adv, ones)
    torch.cuda.synchronize()
    assert bool(torch.isnan(loss3)) and bool(torch.isnan(lp3[7]))
    assert int(torch.isnan(lp3).sum()) == 1 and bool(torch.isnan(grad3[7].float()).all())
    assert not bool(torch.isnan(grad3[6].float()).any())

    say("[case] edge: +inf or NaN at an even or an odd position of the row poisons that row, and only that row")
    # (a bf16 at an odd position is the upper half of a 32-bit word; the position must not matter)
    inf, nan = float("inf"), float("nan")
    for pos, val in ((V - 100, inf), (V - 99, inf), (V - 99, nan), (2, inf), (3, inf), (int(tokens[7]), inf)):
        z5 = logits.clone()
        z5[7, pos] = val
        loss5, lp5, counts5, grad5 = grpo.grpo_loss_fwd_bwd(z5, tokens, old, adv, ones)
        lpf5 = grpo.grpo_logprobs_fwd(z5, tokens)
        torch.cuda.synchronize()
        what = "%s at %d" % (val, pos)
        assert bool(torch.isnan(loss5)) and bool(torch.isnan(lp5[7])) and int(torch.isnan(lp5).sum()) == 1, what
        assert bool(torch.isnan(grad5[7].float()).all()), what
        assert not bool(torch.isnan(grad5[6].float()).any()) and not bool(torch.isnan(grad5[8].float()).any()), what
        assert bool(torch.isnan(lpf5[7])) and int(torch.isnan(lpf5).sum()) == 1, what

    say("[case] edge: -inf logits (vocabulary masking) are legal")
    z4 = logits.clone()
    z4[:, V // 4:3 * V // 4] = float("-inf")
    z4[:, V - V // 50:] = float("-inf")
    tok4 = tokens.clone()
    tok4[((tok4 >= V // 4) & (tok4 < 3 * V // 4)) | (tok4 >= V - V // 50)] = 5
    tok4[1] = V - V // 50 - 1                                   # the last entry that is not masked
    batch = dict(logits=z4, tokens=tok4, mask=ones, n_tokens=N, vocab=V, temperature=1.0,
                 eps_low=0.2, eps_high=0.2, delta=4.0)
    lp_orc = oracle_logprobs_blocked(batch)
    old4 = (torch.as_tensor(lp_orc) + 0.05).to(torch.float32)
    check_against_oracle(batch, old4, lp_orc, adv.cpu().numpy(), label="-inf entries")


@pytest.mark.parametrize("vocab,rows", [(24, 300000), (1000, 100000)])
def test_many_narrow_rows(vocab, rows):
    """Row counts far above the grid with rows of a few bytes: the row queue hands them out in
    chunks over its eight partitions, and every workgroup takes hundreds of rows."""
    run_shape_case("bf16", vocab, vocab, rows)


def test_mask_at_any_alignment_and_length():
    """The unmasked rows are counted 16 mask bytes at a time between the 16-byte boundaries inside the
    mask: every offset of the mask's first byte, lengths around the vector width, any non-zero byte."""
    V = 16
    g = torch.Generator().manual_seed(21)
    for N in (1, 2, 15, 16, 17, 31, 33, 1000, 4099, 70001):
        logits = (torch.randn((N, V), generator=g) * 2).to(torch.bfloat16).to(DEV)
        tokens = torch.randint(0, V, (N,), generator=g).to(DEV)
        old = torch.full((N,), -3.0, device=DEV)
        adv = torch.randn(N, generator=g).to(DEV)
        for offset in (0, 1, 3, 8, 15, 16, 17):
            raw = torch.randint(0, 256, (N + 64,), generator=g).to(torch.uint8)
            raw[torch.rand(N + 64, generator=g) < 0.4] = 0
            buf = raw.to(DEV)
            mask = buf[offset:offset + N]
            assert mask.data_ptr() % 16 == offset % 16
            counts = grpo.grpo_loss_fwd_bwd(logits, tokens, old, adv, mask)[2]
            torch.cuda.synchronize()
            assert int(counts[0]) == int((raw[offset:offset + N] != 0).sum()), (N, offset)


def test_maximum_vocabulary():
    """The widest row the library accepts, 2^28 entries (512 MB in bf16): three rows, one of them
    masked; log-probs, loss and counters of all, the gradient of one row element by element."""
    V, N = 1 << 28, 3
    say("\n[case] maximum vocabulary: N=%d V=%d" % (N, V))
    g = torch.Generator(device=DEV).manual_seed(99)
    logits = torch.empty((N, V), dtype=torch.bfloat16, device=DEV)
    for r in range(N):
        for c0 in range(0, V, 1 << 26):
            logits[r, c0:c0 + (1 << 26)] = (torch.randn(1 << 26, generator=g, device=DEV) * 3).to(torch.bfloat16)
    tokens = torch.tensor([V - 1, 12345, 7], device=DEV)
    mask = torch.tensor([1, 0, 1], dtype=torch.uint8, device=DEV)
    batch = dict(logits=logits, tokens=tokens, mask=mask, n_tokens=N, vocab=V, temperature=1.0,
                 eps_low=0.2, eps_high=0.2, delta=4.0)
    lp_orc = oracle_logprobs_blocked(batch)
    old = (torch.as_tensor(lp_orc) + torch.tensor([0.05, 0.0, -0.1], dtype=torch.float64)).to(torch.float32)
    adv = np.array([1.0, 1.0, -0.5], dtype=np.float32)
    check_against_oracle(batch, old, lp_orc, adv, grad_rows=np.array([0]), label="maximum vocabulary")
    assert grpo.lib().grpo_workspace_bytes(N) > 0


@pytest.mark.parametrize("ddof", [0, 1])
def test_group_advantages(ddof):
    say("\n[case] group advantages ddof=%d" % ddof)
    g = torch.Generator().manual_seed(11 + ddof)
    for G, n_groups in ((1, 3), (4, 2), (16, 256), (64, 5), (100, 7), (1000, 2)):
        R = torch.rand(G * n_groups, generator=g)
        R[:G] = 0.25                                            # a group without signal
        for eps in (1e-6, 0.0):
            adv, _ = grpo.grpo_group_advantages(R.to(DEV), group_size=G, eps_std=eps, ddof=ddof)
            ref = orc.group_advantages(R.numpy(), group_size=G, eps_std=f32(eps), ddof=ddof)
            got = adv.cpu().numpy().astype(np.float64)
            assert np.max(np.abs(got - ref)) <= 2e-6 * max(1.0, np.max(np.abs(ref))), (G, eps)
            assert not got[:G].any()
    sizes = [3, 1, 16, 0, 70, 5]
    off = torch.tensor(np.concatenate([[0], np.cumsum(sizes)]), dtype=torch.int32)
    R = torch.randint(0, 3, (int(off[-1]),), generator=g).float() * 0.5    # ties
    rot = torch.randint(0, int(off[-1]), (1000,), generator=g, dtype=torch.int32)
    adv, adv_tok = grpo.grpo_group_advantages(R.to(DEV), group_offsets=off.to(DEV), eps_std=1e-6,
                                              ddof=ddof, rollout_of_token=rot.to(DEV))
    ref = orc.group_advantages(R.numpy(), group_offsets=off.numpy(), eps_std=f32(1e-6), ddof=ddof)
    got = adv.cpu().numpy().astype(np.float64)
    assert np.max(np.abs(got - ref)) <= 2e-6 * max(1.0, np.max(np.abs(ref)))
    assert np.array_equal(adv_tok.cpu().numpy(), adv.cpu().numpy()[rot.numpy()])
    bad = rot.clone()
    bad[0] = 10 ** 6
    _, t2 = grpo.grpo_group_advantages(R.to(DEV), group_offsets=off.to(DEV), rollout_of_token=bad.to(DEV))
    assert bool(torch.isnan(t2[0])) and not bool(torch.isnan(t2[1:]).any())


FULL = ["qwen_short", "qwen_medium", "long_reasoning", "numerics_stress"]


@pytest.mark.parametrize("name", FULL)
def test_full_size_configs(name):
    """The benchmark's own shapes and launch configuration.  Log-probs, loss and counters
    are compared for every row (the oracle streams the logits in blocks); gradients are
    compared element by element on sampled rows of every row class and on a seeded sample of
    8192 rows, and for all rows
    through two properties that hold at any size: rows with zero coefficient are exactly
    zero, and the largest |gradient| of a row sits on the sampled token, where it equals
    (c/T)(1 - p_y)."""
    cfg = wl.CONFIGS[name]
    say("\n[case] full size %s: N=%d V=%d (%.1f GB of logits)" %
        (name, cfg.n_tokens, cfg.vocab, cfg.n_tokens * cfg.vocab * 2 / 1e9))
    batch = wl.make_batch(cfg, DEV)
    say("  inputs generated; oracle log-probs for %d unmasked rows ..." % int(batch["mask"].sum()))
    rewards = batch["rewards"].cpu().numpy()
    adv = orc.group_advantages(rewards, group_size=cfg.group_size, eps_std=f32(1e-6), ddof=0)
    adv_tok = orc.broadcast_advantages(adv, batch["rollout_of_token"].cpu().numpy()).astype(np.float32)
    lp_orc = oracle_logprobs_blocked(batch, progress=lambda r: say("    oracle rows done: %d" % r)
                                     if r % 16384 == 0 else None)
    old = wl.make_old_logprobs(cfg, lp_orc)
    mask_np = batch["mask"].cpu().numpy()
    T = f32(cfg.temperature)
    pre = orc.objective_from_logprobs(lp_orc, old.numpy(), adv_tok, mask_np, eps_low=f32(cfg.eps_low),
                                      eps_high=f32(cfg.eps_high), delta=f32(cfg.delta))
    rows = sample_rows_by_class(pre["coeff"], mask_np, np.random.default_rng(cfg.index), 40)
    out = check_against_oracle(batch, old, lp_orc, adv_tok, grad_rows=rows, label=name)
    say("  classes: masked=%d zero-coefficient=%d live=%d" %
        (int((mask_np == 0).sum()), int(((mask_np == 1) & (pre["coeff"] == 0)).sum()),
         int((pre["coeff"] != 0).sum())))

    grad, N = out["grad"], cfg.n_tokens
    coeff = torch.as_tensor(pre["coeff"], device=DEV)
    rowmax = torch.empty(N, dtype=torch.float32, device=DEV)
    for r0 in range(0, N, 8192):
        rowmax[r0:r0 + 8192] = grad[r0:r0 + 8192].abs().amax(dim=1).float()
    zero_rows = coeff == 0
    assert float(rowmax[zero_rows].max() if bool(zero_rows.any()) else 0.0) == 0.0
    g_y = grad[torch.arange(N, device=DEV), batch["tokens"]].double()
    expect = coeff / T * (-torch.expm1(torch.as_tensor(lp_orc, device=DEV)))
    live = ~zero_rows
    scale = expect[live].abs()
    # 1 - p_y is taken from the oracle's l = z_y/T - lse, whose last bit is an ulp of lse
    # (1.4e-14 below 64); on near-one-hot rows (1 - p_y ~ 1e-10) that is 1e-4 of the value,
    # more than the 9e-5 the bound leaves beside bf16 rounding (2^-8): allow for it here.
    # The element-by-element comparison above has no such term.
    slack = (coeff[live] / T).abs() * 1.5e-14
    assert bool(((g_y[live] - expect[live]).abs() <= TOL_GRAD * scale + slack).all())
    assert bool(((rowmax[live].double() - scale).abs() <= TOL_GRAD * scale + slack).all())
    # element by element on a seeded sample of 8192 rows of the batch.  Every class occurs in it;
    # its rows with a zero coefficient were compared exactly above (all of them are zero), the
    # live ones go through the oracle in blocks
    sample = np.sort(np.random.default_rng(1000 + cfg.index).choice(N, size=min(N, 8192), replace=False))
    live_s = sample[pre["coeff"][sample] != 0]
    tokens_np = batch["tokens"].cpu().numpy()
    worst = 0.0
    for b in range(0, len(live_s), 256):
        rows_b = live_s[b:b + 256]
        rt = torch.as_tensor(rows_b, device=DEV)
        g_orc = orc.grad_rows(logits_to_numpy(batch["logits"][rt]), tokens_np[rows_b], pre["coeff"][rows_b],
                              temperature=T, vocab=cfg.vocab)
        top = np.abs(g_orc).max(axis=1)
        assert (top > 0).all()
        worst = max(worst, float((np.abs(grads_to_f64(grad[rt]) - g_orc).max(axis=1) / top).max()))
    say("  sample of %d rows (%d live): grad=%.2e x rowmax" % (len(sample), len(live_s), worst))
    assert worst <= TOL_GRAD, "grad error %g x row max on the large sample" % worst
    del batch, out, grad
    torch.cuda.empty_cache()
