"""Shared test plumbing: tensor <-> numpy views and block-wise oracle evaluation."""
import numpy as np
import torch

from oracle import grpo_oracle as orc


def logits_to_numpy(t):
    """torch [n, V] float32 or bfloat16 (any device, row-strided) -> numpy the oracle accepts."""
    t = t.detach().cpu()
    if t.dtype == torch.bfloat16:
        return t.contiguous().view(torch.int16).numpy().view(np.uint16)
    return t.contiguous().numpy()


def grads_to_f64(t):
    return t.detach().cpu().to(torch.float64).numpy()


def oracle_logprobs_blocked(batch, block_rows=4096, progress=None):
    """Oracle log-probs for every row of a (possibly device-resident) batch, streaming
    the logits to the host in row blocks so that they never sit there as a whole."""
    N = batch["n_tokens"]
    lp = np.zeros(N, dtype=np.float64)
    tokens = batch["tokens"].cpu().numpy()
    mask = batch["mask"].cpu().numpy()
    for r0 in range(0, N, block_rows):
        r1 = min(N, r0 + block_rows)
        if not mask[r0:r1].any():
            continue
        z = logits_to_numpy(batch["logits"][r0:r1])
        lp[r0:r1] = orc.logprobs(z, tokens[r0:r1], mask[r0:r1], temperature=batch["temperature"])
        if progress:
            progress(r1)
    return lp


def sample_rows_by_class(coeff, mask, rng, per_class):
    """Row indices covering every row class: masked, zero-coefficient, live."""
    masked = np.flatnonzero(mask == 0)
    zero_c = np.flatnonzero((mask == 1) & (coeff == 0))
    live = np.flatnonzero((mask == 1) & (coeff != 0))
    pick = []
    for cls in (masked, zero_c, live):
        if len(cls):
            pick.append(rng.choice(cls, size=min(per_class, len(cls)), replace=False))
    return np.sort(np.concatenate(pick)) if pick else np.zeros(0, dtype=np.int64)
