"""Seeded synthetic inputs for the GRPO-loss hot path.

This module only draws random inputs of the right shape and distribution; it
contains none of the method's arithmetic (no softmax, no ratio, no clipping) and
is the one piece of code the HIP path's callers and the CPU oracle's callers
share.  The paper's real workload (policy logits of a 32B Qwen-family model on
its RL dataset, section 4.1) needs weights and data that are not available here;
these batches stand in for it: Qwen-sized vocabulary, 16 responses per prompt
(section 4.1), binary task rewards (section 3.1), old log-probs that differ from
the new ones as they do under multi-step asynchrony (section 3.2).

Everything is generated with torch generators on the device the caller names, in
row chunks, so that a 40 GB logits tensor never needs an fp32 staging copy.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, replace

import torch

BASE_SEED = 20250507


@dataclass(frozen=True)
class Workload:
    name: str
    index: int              # position in the benchmark's config list (seed offset)
    n_prompts: int
    group_size: int
    seq_len: int            # tokens per rollout (rows = n_prompts * group_size * seq_len)
    vocab: int
    dtype: str              # "f32" | "bf16"
    logits: str             # "normal" | "normal_boost" | "zipf_gumbel" | "spike"
    logit_std: float
    len_dist: str           # "uniform" | "lognormal" | "full"
    len_lo: int
    len_hi: int
    reward: str             # "bernoulli" | "uniform" | "ternary"
    reward_p: float
    old_noise: str          # "normal" | "uniform"
    old_noise_scale: float
    forced_zero_groups: int = 0
    eps_low: float = 0.2
    eps_high: float = 0.2
    delta: float = 4.0
    temperature: float = 1.0

    @property
    def n_rollouts(self) -> int:
        return self.n_prompts * self.group_size

    @property
    def n_tokens(self) -> int:
        return self.n_rollouts * self.seq_len

    def scaled(self, n_prompts=None, seq_len=None, vocab=None, group_size=None) -> "Workload":
        """Same recipe at another shape, e.g. one the oracle finishes quickly; response
        lengths scale with the sequence length."""
        L = self.seq_len if seq_len is None else seq_len
        f = L / self.seq_len
        return replace(self,
                       n_prompts=self.n_prompts if n_prompts is None else n_prompts,
                       seq_len=L,
                       vocab=self.vocab if vocab is None else vocab,
                       group_size=self.group_size if group_size is None else group_size,
                       len_lo=max(1, min(L, round(self.len_lo * f))),
                       len_hi=max(1, min(L, round(self.len_hi * f))))


QWEN_VOCAB = 152064

CONFIGS = {
    "tiny": Workload("tiny", 0, 2, 4, 64, 1024, "f32", "normal", 2.0, "uniform", 16, 64,
                     "bernoulli", 0.5, "normal", 0.05),
    "qwen_short": Workload("qwen_short", 1, 4, 16, 256, QWEN_VOCAB, "bf16", "normal_boost", 3.0,
                           "uniform", 64, 256, "bernoulli", 0.3, "normal", 0.1),
    "qwen_medium": Workload("qwen_medium", 2, 8, 16, 512, QWEN_VOCAB, "bf16", "zipf_gumbel", 1.0,
                            "uniform", 128, 512, "uniform", 0.0, "normal", 0.2, temperature=0.7),
    "long_reasoning": Workload("long_reasoning", 3, 8, 16, 1024, QWEN_VOCAB, "bf16", "normal", 3.0,
                               "lognormal", 1, 1024, "bernoulli", 0.2, "normal", 0.1,
                               forced_zero_groups=2),
    "numerics_stress": Workload("numerics_stress", 4, 8, 16, 256, QWEN_VOCAB, "bf16", "spike", 3.0,
                                "full", 256, 256, "ternary", 0.0, "uniform", 3.0),
}
CONFIG_ORDER = ["tiny", "qwen_short", "qwen_medium", "long_reasoning", "numerics_stress"]


def _gen(device, seed):
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def _torch_dtype(name):
    return torch.float32 if name == "f32" else torch.bfloat16


def make_batch(cfg: Workload, device="cpu", seed=None, chunk_rows=1024, row_stride=None):
    """Draws one batch.  Returns a dict of tensors on ``device``:

    logits [N, vocab] (a view of a [N, row_stride] buffer when row_stride is given),
    tokens i64 [N], mask u8 [N], rewards f32 [R], rollout_of_token i32 [N],
    lengths i64 [R], plus the python scalars of the config.
    """
    device = torch.device(device)
    seed = BASE_SEED + cfg.index if seed is None else seed
    N, V, R, L = cfg.n_tokens, cfg.vocab, cfg.n_rollouts, cfg.seq_len
    small = _gen("cpu", seed)               # small arrays: always the CPU generator
    big = _gen(device, seed + 1000)         # logits: generated where they live

    # ---- response lengths and mask: the tail of every rollout is masked ----
    if cfg.len_dist == "uniform":
        lengths = torch.randint(cfg.len_lo, cfg.len_hi + 1, (R,), generator=small)
    elif cfg.len_dist == "lognormal":
        z = torch.randn(R, generator=small, dtype=torch.float64)
        # median 300 of 1024 positions (scaled with the sequence length for reduced shapes),
        # heavy right tail cut at the sequence length: about 60% of positions end up masked
        lengths = torch.exp(math.log(300.0 * L / 1024.0) + 0.8 * z).round().clamp(1, L).to(torch.int64)
    elif cfg.len_dist == "full":
        lengths = torch.full((R,), L, dtype=torch.int64)
    else:
        raise ValueError(cfg.len_dist)
    lengths = lengths.clamp(max=L)
    pos = torch.arange(L).expand(R, L)
    mask = (pos < lengths[:, None]).to(torch.uint8).reshape(N)
    rollout_of_token = torch.arange(R, dtype=torch.int32)[:, None].expand(R, L).reshape(N).contiguous()

    # ---- rewards per rollout ----
    if cfg.reward == "bernoulli":
        rewards = (torch.rand(R, generator=small) < cfg.reward_p).to(torch.float32)
    elif cfg.reward == "uniform":
        rewards = torch.rand(R, generator=small)
    elif cfg.reward == "ternary":       # ties inside groups
        rewards = torch.randint(0, 3, (R,), generator=small).to(torch.float32) * 0.5
    else:
        raise ValueError(cfg.reward)
    if cfg.forced_zero_groups:          # groups without any reward signal
        for g in range(min(cfg.forced_zero_groups, cfg.n_prompts)):
            rewards[g * cfg.group_size:(g + 1) * cfg.group_size] = 0.0

    # ---- sampled tokens (overwritten below for the Zipf config) ----
    tokens = torch.randint(0, V, (N,), generator=small, dtype=torch.int64)
    spike_other = torch.randint(1, max(V, 2), (N,), generator=small, dtype=torch.int64)
    const_rows = torch.rand(N, generator=small) < 0.01

    # ---- logits, chunk by chunk ----
    S = V if row_stride is None else int(row_stride)
    assert S >= V
    dt = _torch_dtype(cfg.dtype)
    store = torch.zeros((N, S), dtype=dt, device=device)
    logits = store[:, :V]
    tokens_d = tokens.to(device)
    if cfg.logits == "zipf_gumbel":
        perm = torch.randperm(V, generator=small)
        ranks = torch.empty(V, dtype=torch.float64)
        ranks[perm] = torch.arange(1, V + 1, dtype=torch.float64)
        logfreq = -1.1 * torch.log(ranks)
        logfreq = (logfreq - torch.logsumexp(logfreq, 0)).to(torch.float32).to(device)
    for r0 in range(0, N, chunk_rows):
        r1 = min(N, r0 + chunk_rows)
        n = r1 - r0
        rows = torch.arange(n, device=device)
        if cfg.logits in ("normal", "normal_boost", "spike"):
            x = torch.randn((n, V), generator=big, device=device, dtype=torch.float32) * cfg.logit_std
            if cfg.logits == "normal_boost":
                x[rows, tokens_d[r0:r1]] += 8.0
            if cfg.logits == "spike":
                y = tokens_d[r0:r1]
                other = (y + spike_other[r0:r1].to(device)) % V
                on_y = (torch.arange(r0, r1, device=device) % 2) == 0
                x[rows, torch.where(on_y, y, other)] += 40.0
                x[const_rows[r0:r1].to(device)] = 1.5
        elif cfg.logits == "zipf_gumbel":
            u = torch.rand((n, V), generator=big, device=device, dtype=torch.float32)
            u = u.clamp_(1e-20, 1.0 - 1e-7)
            x = logfreq[None, :] - torch.log(-torch.log(u))
            x = x.to(dt)
            # Gumbel-max: the arg max of the perturbed log-frequencies is a sample of the law
            tokens_d[r0:r1] = torch.argmax(x.float(), dim=1)
        else:
            raise ValueError(cfg.logits)
        logits[r0:r1] = x.to(dt)
        del x
    return dict(cfg=cfg, logits=logits, logits_storage=store, row_stride=S,
                tokens=tokens_d, mask=mask.to(device), rewards=rewards.to(device),
                rollout_of_token=rollout_of_token.to(device), lengths=lengths,
                n_tokens=N, vocab=V, n_rollouts=R, group_size=cfg.group_size,
                eps_low=cfg.eps_low, eps_high=cfg.eps_high, delta=cfg.delta,
                temperature=cfg.temperature, seed=seed)


def make_old_logprobs(cfg: Workload, new_logprobs, seed=None, guard=1e-3):
    """old = new + noise (fp32), the staleness of the rollout policy.

    ``new_logprobs`` is supplied by the caller (the oracle's in tests, the library's in
    the benchmark).  log r = -noise, so noise is re-drawn while -noise lies within
    ``guard`` of a kink of the objective (log(1-eps_low), log(1+eps_high), log delta):
    then fp32 and fp64 evaluations take the same branch and indicator counts are exact.
    """
    seed = BASE_SEED + cfg.index + 500 if seed is None else seed
    g = _gen("cpu", seed)
    new = torch.as_tensor(new_logprobs).detach().to("cpu", torch.float64)
    n = new.shape[0]

    def draw(k):
        if cfg.old_noise == "normal":
            return torch.randn(k, generator=g, dtype=torch.float64) * cfg.old_noise_scale
        return (torch.rand(k, generator=g, dtype=torch.float64) * 2 - 1) * cfg.old_noise_scale

    kinks = torch.tensor([math.log(1 - cfg.eps_low) if cfg.eps_low < 1 else -1e30,
                          math.log(1 + cfg.eps_high), math.log(cfg.delta)], dtype=torch.float64)
    noise = draw(n)
    for _ in range(100):
        bad = ((-noise[:, None] - kinks[None, :]).abs() < guard).any(dim=1)
        k = int(bad.sum())
        if k == 0:
            break
        noise[bad] = draw(k)
    return (new + noise).to(torch.float32)


def make_lmhead_batch(cfg: Workload, d_model: int, device="cpu", seed=None, chunk_rows=4096):
    """The inputs of the fused language-model-head path for the recipe of ``cfg``: final
    hidden states [N, d_model] and head weights [vocab, d_model] in bf16 instead of logits.
    Tokens (Zipf recipe aside), mask, rewards and lengths are the ones ``make_batch`` draws for
    the same seed.  Logits cannot be set element by element here, only through h and W:

    normal / normal_boost: hidden ~ N(0, 1), weight ~ N(0, logit_std^2 / d_model), so the logits
        h W^T have the configured standard deviation; for "normal_boost" each row's hidden
        state is moved along its sampled token's weight row so that this one logit rises by 8
        (the other logits move by 8 cos(w_v, w_y), a few tenths).
    spike: as normal, then every row's hidden state is moved along ONE weight row so that this
        logit rises by 40 (near-one-hot softmax): the sampled token's on even rows, another
        entry's on odd rows; 1 % of the rows get h = 0, i.e. all logits equal.
    zipf_gumbel: the last coordinate of every weight row holds the log-frequency of its entry
        under Zipf(1.1) over a random permutation of ranks and every hidden state has 1 there, so
        z = log-frequency + Gaussian noise of unit standard deviation from the other coordinates
        (Gaussian where ``make_batch`` has Gumbel noise: a product cannot carry element-wise
        noise of another law); tokens are drawn from that Zipf law; stored unscaled, the
        recipe's temperature is applied by the kernel.
    """
    if cfg.logits not in ("normal", "normal_boost", "spike", "zipf_gumbel"):
        raise ValueError("unknown logits recipe %r" % cfg.logits)
    device = torch.device(device)
    seed = BASE_SEED + cfg.index if seed is None else seed
    N, V, R, L = cfg.n_tokens, cfg.vocab, cfg.n_rollouts, cfg.seq_len
    small = _gen("cpu", seed)
    big = _gen(device, seed + 2000)
    if cfg.len_dist == "uniform":
        lengths = torch.randint(cfg.len_lo, cfg.len_hi + 1, (R,), generator=small)
    elif cfg.len_dist == "lognormal":
        z = torch.randn(R, generator=small, dtype=torch.float64)
        lengths = torch.exp(math.log(300.0 * L / 1024.0) + 0.8 * z).round().clamp(1, L).to(torch.int64)
    else:
        lengths = torch.full((R,), L, dtype=torch.int64)
    lengths = lengths.clamp(max=L)
    pos = torch.arange(L).expand(R, L)
    mask = (pos < lengths[:, None]).to(torch.uint8).reshape(N)
    rollout_of_token = torch.arange(R, dtype=torch.int32)[:, None].expand(R, L).reshape(N).contiguous()
    if cfg.reward == "bernoulli":
        rewards = (torch.rand(R, generator=small) < cfg.reward_p).to(torch.float32)
    elif cfg.reward == "uniform":
        rewards = torch.rand(R, generator=small)
    else:
        rewards = torch.randint(0, 3, (R,), generator=small).to(torch.float32) * 0.5
    for g in range(min(cfg.forced_zero_groups, cfg.n_prompts)):
        rewards[g * cfg.group_size:(g + 1) * cfg.group_size] = 0.0
    tokens_cpu = torch.randint(0, V, (N,), generator=small, dtype=torch.int64)
    spike_other = torch.randint(1, max(V, 2), (N,), generator=small, dtype=torch.int64)
    const_rows = torch.rand(N, generator=small) < 0.01
    logfreq = None
    if cfg.logits == "zipf_gumbel":
        perm = torch.randperm(V, generator=small)
        ranks = torch.empty(V, dtype=torch.float64)
        ranks[perm] = torch.arange(1, V + 1, dtype=torch.float64)
        logfreq = -1.1 * torch.log(ranks)
        logfreq = logfreq - torch.logsumexp(logfreq, 0)
        tokens_cpu = torch.multinomial(torch.exp(logfreq), N, replacement=True, generator=small)
    tokens = tokens_cpu.to(device)

    noise_dims = d_model - 1 if cfg.logits == "zipf_gumbel" else d_model
    w_std = cfg.logit_std / math.sqrt(max(noise_dims, 1))
    weight = torch.empty((V, d_model), dtype=torch.bfloat16, device=device)
    for v0 in range(0, V, chunk_rows):
        v1 = min(V, v0 + chunk_rows)
        w = torch.randn((v1 - v0, d_model), generator=big, device=device, dtype=torch.float32) * w_std
        if logfreq is not None:
            w[:, d_model - 1] = logfreq[v0:v1].to(torch.float32).to(device)
        weight[v0:v1] = w.to(torch.bfloat16)
    hidden = torch.empty((N, d_model), dtype=torch.bfloat16, device=device)
    for r0 in range(0, N, chunk_rows):
        r1 = min(N, r0 + chunk_rows)
        h = torch.randn((r1 - r0, d_model), generator=big, device=device, dtype=torch.float32)
        if cfg.logits == "normal_boost":
            wy = weight[tokens[r0:r1]].to(torch.float32)
            h += 8.0 * wy / (wy * wy).sum(dim=1, keepdim=True).clamp_min(1e-20)
        elif cfg.logits == "spike":
            y = tokens[r0:r1]
            other = (y + spike_other[r0:r1].to(device)) % V
            on_y = (torch.arange(r0, r1, device=device) % 2) == 0
            wt = weight[torch.where(on_y, y, other)].to(torch.float32)
            h += 40.0 * wt / (wt * wt).sum(dim=1, keepdim=True).clamp_min(1e-20)
            h[const_rows[r0:r1].to(device)] = 0.0
        elif cfg.logits == "zipf_gumbel":
            h[:, d_model - 1] = 1.0
        hidden[r0:r1] = h.to(torch.bfloat16)
    return dict(cfg=cfg, hidden=hidden, weight=weight, d_model=d_model, tokens=tokens,
                mask=mask.to(device), rewards=rewards.to(device),
                rollout_of_token=rollout_of_token.to(device), lengths=lengths,
                n_tokens=N, vocab=V, n_rollouts=R, group_size=cfg.group_size,
                eps_low=cfg.eps_low, eps_high=cfg.eps_high, delta=cfg.delta,
                temperature=cfg.temperature, seed=seed)
