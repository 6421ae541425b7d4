"""The seeded input generators (CPU, reduced shapes): shapes, determinism, recipe properties."""
import math

import numpy as np
import torch

from paper_2505_07291_amd import workloads as wl


def test_config_table_matches_the_benchmark_shapes():
    sizes = {k: (c.n_tokens, c.vocab, c.dtype) for k, c in wl.CONFIGS.items()}
    assert sizes == {"tiny": (512, 1024, "f32"), "qwen_short": (16384, 152064, "bf16"),
                     "qwen_medium": (65536, 152064, "bf16"),
                     "long_reasoning": (131072, 152064, "bf16"),
                     "numerics_stress": (32768, 152064, "bf16")}
    assert [wl.CONFIGS[n].index for n in wl.CONFIG_ORDER] == [0, 1, 2, 3, 4]


def test_batches_are_seeded_and_shaped():
    cfg = wl.CONFIGS["tiny"]
    a, b = wl.make_batch(cfg), wl.make_batch(cfg)
    assert torch.equal(a["logits"], b["logits"]) and torch.equal(a["tokens"], b["tokens"])
    assert torch.equal(a["mask"], b["mask"]) and torch.equal(a["rewards"], b["rewards"])
    c = wl.make_batch(cfg, seed=1)
    assert not torch.equal(a["logits"], c["logits"])
    assert a["logits"].shape == (512, 1024) and a["logits"].dtype == torch.float32
    assert a["mask"].dtype == torch.uint8 and a["tokens"].dtype == torch.int64
    # the tail of each rollout is masked, lengths within [16, 64]
    m = a["mask"].reshape(8, 64)
    assert torch.equal(m.sum(1), a["lengths"]) and int(a["lengths"].min()) >= 16
    assert bool((m[:, :-1] >= m[:, 1:]).all())
    assert set(a["rewards"].tolist()) <= {0.0, 1.0}
    assert torch.equal(a["rollout_of_token"].reshape(8, 64)[:, 0], torch.arange(8, dtype=torch.int32))


def test_row_stride_padding_is_outside_the_view():
    cfg = wl.CONFIGS["tiny"].scaled(vocab=1000)
    b = wl.make_batch(cfg, row_stride=1008)
    assert b["logits"].shape == (512, 1000) and b["logits"].stride(0) == 1008


def test_reduced_recipes():
    short = wl.make_batch(wl.CONFIGS["qwen_short"].scaled(n_prompts=1, seq_len=4, vocab=4096))
    z = short["logits"].float()
    rows = torch.arange(z.shape[0])
    assert float((z[rows, short["tokens"]] - 8).mean()) > -1.0           # boosted sampled token
    med = wl.make_batch(wl.CONFIGS["qwen_medium"].scaled(n_prompts=1, seq_len=4, vocab=4096))
    assert torch.equal(med["tokens"], med["logits"].float().argmax(1))    # Gumbel-max sample
    assert med["temperature"] == 0.7 and float(med["rewards"].max()) <= 1.0
    lng = wl.make_batch(wl.CONFIGS["long_reasoning"].scaled(n_prompts=4, seq_len=64, vocab=512))
    frac_masked = 1.0 - float(lng["mask"].float().mean())
    assert 0.35 < frac_masked < 0.8
    assert not lng["rewards"][:32].any()                                    # two all-zero groups
    st = wl.make_batch(wl.CONFIGS["numerics_stress"].scaled(n_prompts=2, seq_len=16, vocab=2048))
    zs = st["logits"].float()
    const = (zs.max(1).values == zs.min(1).values)
    spike = zs.max(1).values > 25
    assert bool((const | spike).all()) and bool(st["mask"].all())
    on_y = zs[torch.arange(zs.shape[0]), st["tokens"]] > 25
    assert 0.3 < float(on_y.float().mean()) < 0.7
    assert set(st["rewards"].tolist()) <= {0.0, 0.5, 1.0}


def test_old_logprobs_keep_clear_of_the_kinks():
    for name in ("qwen_medium", "numerics_stress"):
        cfg = wl.CONFIGS[name]
        new = torch.linspace(-12, 0, 20000, dtype=torch.float64)
        old = wl.make_old_logprobs(cfg, new)
        assert old.dtype == torch.float32
        logr = (new - old.double()).numpy()
        for b in (math.log(0.8), math.log(1.2), math.log(4.0)):
            assert np.min(np.abs(logr - b)) > 0.9e-3
        assert torch.equal(old, wl.make_old_logprobs(cfg, new))
    spread = (new - wl.make_old_logprobs(wl.CONFIGS["numerics_stress"], new).double())
    assert float(spread.max()) > 2.9 and float(spread.min()) < -2.9
