#!/usr/bin/env python3
"""Benchmark of the GRPO-loss hot path on one MI355X.

One "step" is the whole hot path over one synthetic batch that is already resident
in HBM: group advantages (+ broadcast to tokens), then the objective forward and the
fused backward over the full vocabulary (grpo_group_advantages + grpo_loss_fwd_bwd).
Prints ONE JSON line: whole-job tokens/s, the HBM roofline of the dominant (row)
kernel measured with events on the launch stream, and the fp64 CPU oracle timed on a
bounded sample of the same batch as a reported baseline.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0  # MI355X published HBM3E peak, 8 TB/s


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def traffic_from_profiles(workload):
    """Measured HBM bytes per row-kernel launch, if a counter summary was committed for
    this workload (profiles/hbm_traffic_<workload>.txt, line 'traffic_bytes_per_launch = N')."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic_%s.txt" % workload)
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch"):
                return float(line.split("=")[1])
    except OSError:
        pass
    return None


def cpu_baseline(batch, old, adv_tok, budget_s=10.0, block=512):
    """fp64 oracle, forward + backward, over the rows of the same batch in blocks (wrapping
    around if the batch is finished early) until the time budget is used; tokens/s of that."""
    import numpy as np
    import torch
    from oracle import grpo_oracle as orc
    cfg = batch["cfg"]
    N = batch["n_tokens"]
    done, live, t_used, r0 = 0, 0, 0.0, 0
    tokens = batch["tokens"].cpu().numpy()
    mask = batch["mask"].cpu().numpy()
    oldn, advn = old.cpu().numpy(), adv_tok.cpu().numpy()
    while t_used < budget_s:
        r1 = min(r0 + block, N)
        z = batch["logits"][r0:r1].cpu()
        z = z.view(torch.int16).numpy().view(np.uint16) if z.dtype == torch.bfloat16 else z.numpy()
        t0 = time.perf_counter()
        orc.loss_fwd_bwd(z, tokens[r0:r1], oldn[r0:r1], advn[r0:r1], mask[r0:r1],
                         eps_low=cfg.eps_low, eps_high=cfg.eps_high, delta=cfg.delta,
                         temperature=cfg.temperature, grad_rows="all")
        t_used += time.perf_counter() - t0
        done += r1 - r0
        live += int(mask[r0:r1].sum())
        r0 = r1 % N
    # the same on one thread, on the first rows of the batch (about a second)
    threads = orc.num_threads()
    n1 = min(N, 256)
    z = batch["logits"][:n1].cpu()
    z = z.view(torch.int16).numpy().view(np.uint16) if z.dtype == torch.bfloat16 else z.numpy()
    orc.set_num_threads(1)
    try:
        t0 = time.perf_counter()
        orc.loss_fwd_bwd(z, tokens[:n1], oldn[:n1], advn[:n1], mask[:n1], eps_low=cfg.eps_low,
                         eps_high=cfg.eps_high, delta=cfg.delta, temperature=cfg.temperature, grad_rows="all")
        t1 = time.perf_counter() - t0
    finally:
        orc.set_num_threads(threads)
    return dict(value=done / t_used, unit="tokens/s", cores=threads, kind="oracle",
                sample="%d rows of the batch in order from row 0, wrapping (%d unmasked), fp64 "
                       "forward+backward in blocks of %d rows, %.1f s" % (done, live, block, t_used),
                single_thread_value=n1 / t1, single_thread_sample="the first %d rows, %.1f s" % (n1, t1))


def lmhead_leg(grpo, wl, cfg, d_model, dev, stream, reps):
    """The fused language-model-head path on the same recipe: hidden states [N, d_model] and head
    weights [V, d_model] instead of logits.  A dense contraction, so its roofline is the bf16
    matrix-core peak; flops are the algorithmic 2 N V d per product (one product forward,
    three with the backward)."""
    import torch
    N, V = cfg.n_tokens, cfg.vocab
    log("[bench] language-model-head leg: N=%d V=%d d=%d" % (N, V, d_model))
    b = wl.make_lmhead_batch(cfg, d_model, dev)
    lp = torch.empty(N, dtype=torch.float32, device=dev)
    ws_f = torch.empty(grpo.grpo_lmhead_workspace_bytes(N, V, d_model, False), dtype=torch.uint8, device=dev)
    ws_b = torch.empty(grpo.grpo_lmhead_workspace_bytes(N, V, d_model, True), dtype=torch.uint8, device=dev)
    dH = torch.empty((N, d_model), dtype=torch.bfloat16, device=dev)
    dW = torch.empty((V, d_model), dtype=torch.float32, device=dev)
    loss = torch.empty(1, dtype=torch.float32, device=dev)
    counts = torch.empty(5, dtype=torch.int64, device=dev)
    adv, adv_tok = grpo.grpo_group_advantages(b["rewards"], group_size=cfg.group_size,
                                              rollout_of_token=b["rollout_of_token"], stream=stream)

    def fwd():
        grpo.grpo_lmhead_logprobs_fwd(b["hidden"], b["weight"], b["tokens"], b["mask"], cfg.temperature,
                                      logprobs_out=lp, workspace=ws_f, stream=stream)
    fwd()
    torch.cuda.synchronize()
    old = wl.make_old_logprobs(cfg, lp).to(dev)

    def fwd_bwd():
        grpo.grpo_lmhead_loss_fwd_bwd(b["hidden"], b["weight"], b["tokens"], old, adv_tok, b["mask"],
                                      cfg.eps_low, cfg.eps_high, cfg.delta, cfg.temperature, 0.0, 1.0,
                                      grad_hidden=dH, grad_weight=dW, loss_out=loss, logprobs_out=lp,
                                      counts_out=counts, workspace=ws_b, stream=stream)

    def timed(fn):
        fn()
        evs = []
        for _ in range(reps):
            a, e = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record(stream)
            fn()
            e.record(stream)
            evs.append((a, e))
        torch.cuda.synchronize()
        return sum(a.elapsed_time(e) for a, e in evs) / reps
    ref = wl.make_old_logprobs(cfg, lp, seed=cfg.index + 77).to(dev)
    loss4 = torch.empty(4, dtype=torch.float32, device=dev)

    def fwd_bwd_aux():   # the coefficients of section 4.1
        grpo.grpo_lmhead_loss_aux_fwd_bwd(b["hidden"], b["weight"], b["tokens"], old, ref, adv_tok, b["mask"],
                                          cfg.eps_low, cfg.eps_high, cfg.delta, cfg.temperature, 0.001, 1e-4,
                                          0.0, 1.0, grad_hidden=dH, grad_weight=dW, loss_out=loss4,
                                          logprobs_out=lp, want_entropy=False, counts_out=counts,
                                          workspace=ws_b, stream=stream)
    ms_f = timed(fwd)
    ms_x = timed(fwd_bwd_aux)
    aux_vals = loss4.cpu().tolist()
    ms_b = timed(fwd_bwd)
    c = counts.cpu().tolist()
    n_unmasked = c[0]
    zero_adv = int(((adv_tok == 0) & (b["mask"] != 0)).sum())
    n_grad = n_unmasked - (c[1] + c[2] + c[3] + zero_adv)   # rows whose objective has a gradient
    # algorithmic flops: rows that take no part need none (2 V d per unmasked row for the logits,
    # twice that again per row with a gradient for dL/dH and dL/dW)
    flops_f = 2.0 * n_unmasked * V * d_model
    flops_b = flops_f + 4.0 * n_grad * V * d_model
    return {"note": "grpo_lmhead_logprobs_fwd / grpo_lmhead_loss_fwd_bwd: hidden [N, d] and head "
                    "weights [V, d] in bf16, logits formed on the matrix cores; tokens/s count all N rows, "
                    "flops only the rows that take part",
            "d_model": d_model, "rows": N, "rows_unmasked": n_unmasked, "rows_with_gradient": n_grad,
            "fwd_ms": ms_f, "fwd_tokens_per_s": N / (ms_f * 1e-3),
            "fwd_bwd_ms": ms_b, "fwd_bwd_tokens_per_s": N / (ms_b * 1e-3), "loss": float(loss.cpu()),
            "aux": {"note": "grpo_lmhead_loss_aux_fwd_bwd, KL 0.001 and entropy 1e-4: every unmasked row has a "
                            "gradient", "fwd_bwd_ms": ms_x, "fwd_bwd_tokens_per_s": N / (ms_x * 1e-3),
                    "tflops": (flops_f + 4.0 * n_unmasked * V * d_model) / (ms_x * 1e-3) / 1e12,
                    "total": aux_vals[0], "policy": aux_vals[1], "mean_kl": aux_vals[2],
                    "mean_entropy": aux_vals[3]},
            "roofline": {"bound": "mfma", "achieved": flops_f / (ms_f * 1e-3) / 1e12, "peak": 2500.0,
                         "unit": "TFLOP/s", "frac": flops_f / (ms_f * 1e-3) / 1e12 / 2500.0,
                         "kernel": "lm_gemm_nt (forward: logits + softmax partials)",
                         "algorithmic_flops": flops_f, "traffic": None},
            "roofline_fwd_bwd": {"bound": "mfma", "achieved": flops_b / (ms_b * 1e-3) / 1e12,
                                 "peak": 2500.0, "unit": "TFLOP/s",
                                 "frac": flops_b / (ms_b * 1e-3) / 1e12 / 2500.0,
                                 "algorithmic_flops": flops_b}}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="qwen_short")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-lmhead", action="store_true",
                    help="skip the fused language-model-head leg (hidden states and head weights in)")
    ap.add_argument("--d-model", type=int, default=5120,
                    help="hidden size of the language-model-head leg (5120: a 32B Qwen-family model)")
    ap.add_argument("--vocab", type=int, default=0,
                    help="another vocabulary size for the workload's recipe (rows scaled to keep the "
                         "bytes of logits); not the headline configuration, no language-model-head leg")
    ap.add_argument("--logits-dtype", choices=["bf16", "f32"], default=None,
                    help="another storage type for the logits, as --vocab")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run plain 1 GiB device copies (reference for HBM counters)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (rows are independent; a multi-GPU run "
              "would be this same kernel per rank plus a 40-byte all-reduce); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2505_07291_amd as grpo
    from paper_2505_07291_amd import workloads as wl

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    dev = "cuda:0"
    cfg = wl.CONFIGS[args.workload]
    variant = ""
    if args.vocab or args.logits_dtype:
        # the same recipe at another row width: the sequence length takes up the difference
        import dataclasses
        esz0 = 2 if cfg.dtype == "bf16" else 4
        dt = args.logits_dtype or cfg.dtype
        vocab = args.vocab or cfg.vocab
        L = max(1, round(cfg.seq_len * cfg.vocab * esz0 / (vocab * (2 if dt == "bf16" else 4))))
        cfg = dataclasses.replace(cfg.scaled(seq_len=L, vocab=vocab), dtype=dt)
        variant = "@V=%d,%s" % (vocab, dt)
        args.no_lmhead = True
    N, V = cfg.n_tokens, cfg.vocab
    log("[bench] generating %s: N=%d V=%d %s (%.2f GB of logits)" %
        (cfg.name, N, V, cfg.dtype, N * V * (2 if cfg.dtype == "bf16" else 4) / 1e9))
    batch = wl.make_batch(cfg, dev)
    esz = batch["logits"].element_size()
    # old-policy log-probs: the library's own forward pass plus the recipe's staleness noise
    new_lp = grpo.grpo_logprobs_fwd(batch["logits"], batch["tokens"], None, cfg.temperature)
    torch.cuda.synchronize()
    old = wl.make_old_logprobs(cfg, new_lp).to(dev)

    adv = torch.empty(cfg.n_rollouts, dtype=torch.float32, device=dev)
    adv_tok = torch.empty(N, dtype=torch.float32, device=dev)
    grad = torch.empty_like(batch["logits"])
    loss = torch.empty(1, dtype=torch.float32, device=dev)
    lp = torch.empty(N, dtype=torch.float32, device=dev)
    counts = torch.empty(5, dtype=torch.int64, device=dev)
    ws = torch.empty(grpo.grpo_workspace_bytes(N), dtype=torch.uint8, device=dev)
    stream = torch.cuda.current_stream()

    def step(ev=None, mask=batch["mask"], oldlp=old, advantages=None):
        a_tok = adv_tok
        if advantages is None:
            grpo.grpo_group_advantages(batch["rewards"], group_size=cfg.group_size, eps_std=1e-6,
                                       ddof=0, rollout_of_token=batch["rollout_of_token"],
                                       adv_out=adv, adv_tok_out=adv_tok, stream=stream)
        else:
            a_tok = advantages
        if ev:
            ev[0].record(stream)
        grpo.grpo_loss_fwd_bwd(batch["logits"], batch["tokens"], oldlp, a_tok, mask,
                               cfg.eps_low, cfg.eps_high, cfg.delta, cfg.temperature, 0.0, 1.0,
                               grad_logits=grad, loss_out=loss, logprobs_out=lp,
                               counts_out=counts, workspace=ws, stream=stream)
        if ev:
            ev[1].record(stream)

    def timed(K, W, **kw):
        for _ in range(W):
            step(**kw)
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
               for _ in range(K)]
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(K):
            step(ev=evs[i], **kw)
        torch.cuda.synchronize()
        wall = (time.perf_counter() - t0) / K
        per_step = sorted(a.elapsed_time(b) for a, b in evs)
        timed.last = {"median": per_step[len(per_step) // 2], "min": per_step[0], "max": per_step[-1]}
        kern = sum(per_step) / K * 1e-3
        return wall, kern

    log("[bench] timing %d steps after %d warm-up steps" % (args.steps, args.warmup))
    wall, kern = timed(args.steps, args.warmup)
    kern_spread = dict(timed.last)
    assert grpo.grpo_workspace_error(ws) == 0
    c = counts.cpu().tolist()
    loss_value = float(loss.cpu())
    M = c[0]
    zero_adv = int(((adv_tok == 0) & (batch["mask"] != 0)).sum())
    n_zero_coeff = c[1] + c[2] + c[3] + zero_adv
    n_full, n_masked = M - n_zero_coeff, N - M
    row_bytes = V * esz
    # algorithmic bytes by row class: live rows 2 reads + 1 write, rows whose gradient is
    # cut 1 read + 1 zero-fill, masked rows 1 zero-fill; plus 29 B of per-token scalars
    alg_bytes = row_bytes * (3 * n_full + 2 * n_zero_coeff + 1 * n_masked) + 29 * N
    conv_bytes = 3 * N * row_bytes
    # what this design has to move through HBM: live rows are read once (kept in registers)
    design_bytes = row_bytes * (2 * n_full + 2 * n_zero_coeff + 1 * n_masked) + 29 * N

    # worst case for the kernel: every row unmasked and live (ratio 1, non-zero advantage)
    ones = torch.ones(N, dtype=torch.uint8, device=dev)
    adv_ones = torch.full((N,), 0.5, dtype=torch.float32, device=dev)
    wall_full, kern_full = timed(max(5, args.steps // 3), 2, mask=ones, oldlp=new_lp, advantages=adv_ones)
    full_counts = counts.cpu().tolist()

    # the old-policy log-probs pass (one read of the logits), every row unmasked
    fwd_ws = torch.empty(grpo.grpo_workspace_bytes(0), dtype=torch.uint8, device=dev)
    fwd_evs = []
    for i in range(3 + max(5, args.steps // 3)):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record(stream)
        grpo.grpo_logprobs_fwd(batch["logits"], batch["tokens"], ones, cfg.temperature,
                               logprobs_out=lp, workspace=fwd_ws, stream=stream)
        b.record(stream)
        fwd_evs.append((a, b))
    torch.cuda.synchronize()
    fwd_ms = sum(a.elapsed_time(b) for a, b in fwd_evs[3:]) / len(fwd_evs[3:])

    # the objective with the KL and entropy terms fused in (section 4.1 coefficients),
    # on the benchmark's own batch
    ref = wl.make_old_logprobs(cfg, new_lp, seed=cfg.index + 77).to(dev)
    loss4 = torch.empty(4, dtype=torch.float32, device=dev)
    ent = torch.empty(N, dtype=torch.float32, device=dev)
    aux_evs = []
    for i in range(3 + max(5, args.steps // 3)):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record(stream)
        grpo.grpo_loss_aux_fwd_bwd(batch["logits"], batch["tokens"], old, ref, adv_tok, batch["mask"],
                                   cfg.eps_low, cfg.eps_high, cfg.delta, cfg.temperature, 0.001, 1e-4,
                                   0.0, 1.0, grad_logits=grad, loss_out=loss4, logprobs_out=lp,
                                   entropy_out=ent, counts_out=counts, workspace=ws, stream=stream)
        b.record(stream)
        aux_evs.append((a, b))
    torch.cuda.synchronize()
    aux_ms = sum(a.elapsed_time(b) for a, b in aux_evs[3:]) / len(aux_evs[3:])
    aux_vals = loss4.cpu().tolist()
    # with an entropy term every unmasked row gets a gradient: 2 reads + 1 write each
    aux_alg = row_bytes * (3 * M + 1 * n_masked) + 37 * N

    if args.copy_calibration:
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()

    out = {
        "metric": "GRPO loss fwd+bwd tokens/s (V=152064 bf16)" if V == 152064 and cfg.dtype == "bf16" else
                  "GRPO loss fwd+bwd tokens/s (V=%d %s)" % (V, cfg.dtype),
        "value": N / wall, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": wall * 1e3, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": cfg.name + variant, "n_tokens": N, "vocab": V, "logits_dtype": cfg.dtype,
                   "group_size": cfg.group_size, "n_rollouts": cfg.n_rollouts,
                   "rows_live": n_full, "rows_zero_coeff": n_zero_coeff, "rows_masked": n_masked,
                   "eps_low": cfg.eps_low, "eps_high": cfg.eps_high, "delta": cfg.delta,
                   "temperature": cfg.temperature,
                   "row_kernel": grpo.grpo_row_kernel_plan(grpo.GRPO_BF16 if cfg.dtype == "bf16" else grpo.GRPO_F32, V)},
        "counts": dict(zip(grpo.COUNT_NAMES, c)), "loss": loss_value,
        "roofline": {"bound": "hbm", "achieved": alg_bytes / kern / 1e9, "peak": HBM_PEAK_GBPS,
                     "unit": "GB/s", "frac": alg_bytes / kern / 1e9 / HBM_PEAK_GBPS,
                     "traffic": None if variant else traffic_from_profiles(cfg.name),
                     "kernel": "grpo_rows_cached (inside grpo_loss_fwd_bwd)",
                     "kernel_ms": kern * 1e3, "kernel_ms_median": kern_spread["median"],
                     "kernel_ms_min": kern_spread["min"], "kernel_ms_max": kern_spread["max"],
                     "algorithmic_bytes": alg_bytes,
                     "gbps_2r1w_all_rows_convention": conv_bytes / kern / 1e9,
                     "gbps_design_traffic_1r1w": design_bytes / kern / 1e9},
        "full_rows": {"note": "same logits, every row unmasked and live: the kernel's worst case",
                      "tokens_per_s": N / wall_full, "kernel_ms": kern_full * 1e3,
                      "gbps_2r1w": conv_bytes / kern_full / 1e9,
                      "frac_2r1w": conv_bytes / kern_full / 1e9 / HBM_PEAK_GBPS,
                      "gbps_design_traffic_1r1w": 2 * N * row_bytes / kern_full / 1e9,
                      "rows_live": full_counts[0]},
        "aux_loss": {"note": "grpo_loss_aux_fwd_bwd on the same batch, KL 0.001 and entropy 1e-4 fused in",
                     "tokens_per_s": N / (aux_ms * 1e-3), "kernel_ms": aux_ms,
                     "achieved_gbps": aux_alg / (aux_ms * 1e-3) / 1e9,
                     "frac": aux_alg / (aux_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS,
                     "total": aux_vals[0], "policy": aux_vals[1], "mean_kl": aux_vals[2],
                     "mean_entropy": aux_vals[3]},
        "logprobs_fwd": {"note": "grpo_logprobs_fwd, every row unmasked: one read of the logits",
                         "tokens_per_s": N / (fwd_ms * 1e-3), "kernel_ms": fwd_ms,
                         "gbps": N * row_bytes / (fwd_ms * 1e-3) / 1e9,
                         "frac": N * row_bytes / (fwd_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS},
    }
    if not args.no_lmhead and cfg.logits in ("normal", "normal_boost") and cfg.dtype == "bf16":
        # the leg needs its own operands, gradients and two workspaces next to the batch
        need = (grpo.grpo_lmhead_workspace_bytes(N, V, args.d_model, True) +
                grpo.grpo_lmhead_workspace_bytes(N, V, args.d_model, False) +
                6 * V * args.d_model + 4 * N * args.d_model)
        free = torch.cuda.mem_get_info()[0]
        if need < 0.9 * free:
            out["lmhead"] = lmhead_leg(grpo, wl, cfg, args.d_model, dev, stream, max(3, args.steps // 6))
        else:
            out["lmhead"] = {"skipped": "needs %.0f GB of device memory, %.0f GB free" % (need / 1e9, free / 1e9)}
    if not args.no_cpu_baseline:
        log("[bench] timing the fp64 oracle on a sample of the batch (about 12 s)")
        step()
        torch.cuda.synchronize()
        out["cpu_baseline"] = cpu_baseline(batch, old, adv_tok)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
