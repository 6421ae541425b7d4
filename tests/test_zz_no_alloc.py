"""grpo_loss_fwd_bwd_noalloc (scratch built into the library, no workspace argument) against
grpo_loss_fwd_bwd (caller's workspace) through the C ABI.

Both run the same kernels in the same launch shapes, so the bar is the strictest one: every
output bit-identical (which implies the oracle tolerances the workspace variant is held to in
test_gpu_parity.py).  Two calls in a row share the library's scratch array, the second on a
smaller batch, so anything the first call left behind there (per-row terms, indicator bits,
queue counters, the error word) would show in the second.
"""
import sys

import numpy as np
import pytest
import torch

import paper_2505_07291_amd as grpo
from paper_2505_07291_amd import workloads as wl

pytestmark = pytest.mark.gpu
DEV = "cuda"


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


def f32(x):
    return float(np.float32(x))


def both_ways(cfg, bad_token_row=None, seed=None):
    """One batch of the recipe through both entry points; returns nothing, asserts equality."""
    batch = wl.make_batch(cfg, DEV, seed=seed)
    N = batch["n_tokens"]
    tokens = batch["tokens"].clone()
    if bad_token_row is not None:                   # a data error: must reach error_out, and only this call's
        row = int(torch.nonzero(batch["mask"])[bad_token_row])
        tokens[row] = cfg.vocab + 5
    new_lp = grpo.grpo_logprobs_fwd(batch["logits"], batch["tokens"], None, f32(cfg.temperature))
    torch.cuda.synchronize()
    old = wl.make_old_logprobs(cfg, new_lp).to(DEV)
    _, adv_tok = grpo.grpo_group_advantages(batch["rewards"], group_size=cfg.group_size,
                                            rollout_of_token=batch["rollout_of_token"])
    kw = (f32(cfg.eps_low), f32(cfg.eps_high), f32(cfg.delta), f32(cfg.temperature), 0.0, 1.0)

    # reference: the workspace variant
    loss_a, lp_a, counts_a, grad_a = grpo.grpo_loss_fwd_bwd(batch["logits"], tokens, old, adv_tok,
                                                            batch["mask"], *kw)
    # the variant under test: every output pre-allocated, poisoned first
    grad_b = torch.full_like(batch["logits"], 7.0)
    loss_b = torch.full((1,), 7.0, dtype=torch.float32, device=DEV)
    lp_b = torch.full((N,), 7.0, dtype=torch.float32, device=DEV)
    counts_b = torch.full((5,), 7, dtype=torch.int64, device=DEV)
    err_b = torch.full((1,), 7, dtype=torch.int32, device=DEV)
    say("[gpu] grpo_loss_fwd_bwd_noalloc %s N=%d V=%d %s bad_token=%s" %
        (cfg.name, N, cfg.vocab, cfg.dtype, bad_token_row is not None))
    grpo.grpo_loss_fwd_bwd_noalloc(batch["logits"], tokens, old, adv_tok, batch["mask"], *kw,
                                   grad_logits=grad_b, loss_out=loss_b, logprobs_out=lp_b,
                                   counts_out=counts_b, error_out=err_b)
    torch.cuda.synchronize()
    assert torch.equal(loss_a.view(torch.int32), loss_b.view(torch.int32)), (loss_a, loss_b)
    assert torch.equal(lp_a.view(torch.int32), lp_b.view(torch.int32))
    assert torch.equal(counts_a, counts_b), (counts_a, counts_b)
    ia = grad_a.view(torch.int16) if grad_a.dtype == torch.bfloat16 else grad_a.view(torch.int32)
    ib = grad_b.view(torch.int16) if grad_b.dtype == torch.bfloat16 else grad_b.view(torch.int32)
    assert torch.equal(ia, ib), "gradients differ"
    assert int(err_b) == (1 if bad_token_row is not None else 0)
    assert int(counts_b[0]) == int(batch["mask"].sum())
    say("      ok: loss=%.6g counts=%s error=%d" % (float(loss_b), counts_b.tolist(), int(err_b)))


def test_noalloc_matches_workspace_variant_twice_in_a_row():
    # first call: the wider batch, with a token id outside the vocabulary (sets the error word)
    big = wl.CONFIGS["numerics_stress"].scaled(n_prompts=2, seq_len=24)      # 768 rows x 152064 bf16
    both_ways(big, bad_token_row=11)
    # second call: fewer rows, another recipe (masked tails), no data error: the error word, the
    # queue counters and the per-row arrays of the first call must not leak into it
    small = wl.CONFIGS["qwen_short"].scaled(n_prompts=1, seq_len=9)          # 144 rows
    both_ways(small)
    # and once more on narrow fp32 rows (another row-kernel instantiation, eight queue partitions)
    both_ways(wl.CONFIGS["tiny"])
