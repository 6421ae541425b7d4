#!/usr/bin/env python3
"""Benchmark of the GRPO-loss hot path on one MI355X.

One "step" is the whole hot path over one synthetic batch that is already resident
in HBM: group advantages (+ broadcast to tokens), then the objective forward and the
fused backward over the full vocabulary (grpo_group_advantages + grpo_loss_fwd_bwd).
Prints ONE JSON line.  The headline (`value`, `roofline`) is the qwen_short batch; the
`workloads` object carries the same measurement for every 152064-vocabulary batch
(qwen_short, qwen_medium, long_reasoning, numerics_stress), each generated, timed and
freed in turn; the fp64 CPU oracle is timed on a bounded sample of the headline batch
as a reported baseline.

Two bandwidth figures per workload, both from the row kernel's event-bracketed time:
  frac        algorithmic bytes (2 reads + 1 write of a live row, 1 read + 1 zero-fill of a
              row whose gradient is cut, 1 zero-fill of a masked row) / time / 8 TB/s;
  frac_moved  bytes this design moves through HBM (live rows are read ONCE: 1 read +
              1 write) / time / 8 TB/s: the physical share of the peak.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME|all]
"""
import argparse
import gc
import hashlib
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0  # MI355X published HBM3E peak, 8 TB/s
BF16_MFMA_PEAK_TFLOPS = 2500.0
QWEN_WORKLOADS = ["qwen_short", "qwen_medium", "long_reasoning", "numerics_stress"]
KERNEL_SOURCES = {"grpo_rows_cached": "paper_2505_07291_amd/csrc/grpo.hip",
                  "lm_gemm_nt": "paper_2505_07291_amd/csrc/lmhead.hpp"}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def source_hash(kernel):
    """First 16 hex digits of the SHA-256 of the source file that holds a kernel."""
    with open(os.path.join(ROOT, KERNEL_SOURCES[kernel]), "rb") as f:
        return hashlib.sha256(f.read()).hexdigest()[:16]


def traffic_from_profile(name, kernel):
    """Measured HBM bytes per launch from a committed counter summary, profiles/<name>.txt
    (lines 'traffic_bytes_per_launch = N', 'kernel_source_sha256 = H', 'git_commit = C').
    The figure is only handed on when the summary was taken with the kernel source that is
    in the tree now; otherwise the traffic is reported as unmeasured."""
    path = os.path.join(ROOT, "profiles", name + ".txt")
    found = {}
    try:
        for line in open(path):
            m = re.match(r"\s*(traffic_bytes_per_launch|kernel_source_sha256|git_commit)\s*=\s*(\S+)", line)
            if m:
                found[m.group(1)] = m.group(2)
    except OSError:
        return None, {"profile": None}
    stamp = {"profile": "profiles/%s.txt" % name, "profile_git_commit": found.get("git_commit"),
             "profile_kernel_source_sha256": found.get("kernel_source_sha256"),
             "current_kernel_source_sha256": source_hash(kernel)}
    stamp["current"] = stamp["profile_kernel_source_sha256"] == stamp["current_kernel_source_sha256"]
    if not stamp["current"] or "traffic_bytes_per_launch" not in found:
        return None, stamp
    return float(found["traffic_bytes_per_launch"]), stamp


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


def timed_calls(fn, stream, reps, warmup):
    """Mean / median / min / max milliseconds of `reps` calls of fn after `warmup` untimed ones,
    each bracketed by events on the launch stream."""
    import torch
    for _ in range(warmup):
        fn()
    evs = []
    for _ in range(reps):
        a, e = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record(stream)
        fn()
        e.record(stream)
        evs.append((a, e))
    torch.cuda.synchronize()
    ms = sorted(a.elapsed_time(e) for a, e in evs)
    return {"mean": sum(ms) / len(ms), "median": ms[len(ms) // 2], "min": ms[0], "max": ms[-1]}


def lmhead_leg(grpo, wl, cfg, d_model, dev, stream, reps, warmup):
    """The fused language-model-head path on the same recipe: hidden states [N, d_model] and head
    weights [V, d_model] instead of logits.  A dense contraction, so its roofline is the bf16
    matrix-core peak; flops are the algorithmic 2 N V d per product (one product forward,
    three with the backward)."""
    import torch
    N, V = cfg.n_tokens, cfg.vocab
    log("[bench] language-model-head leg: N=%d V=%d d=%d" % (N, V, d_model))
    b = wl.make_lmhead_batch(cfg, d_model, dev)
    lp = torch.empty(N, dtype=torch.float32, device=dev)
    ws_f_bytes = grpo.grpo_lmhead_workspace_bytes(N, V, d_model, False)
    ws_b_bytes = grpo.grpo_lmhead_workspace_bytes(N, V, d_model, True)
    ws_f = torch.empty(ws_f_bytes, dtype=torch.uint8, device=dev)
    ws_b = torch.empty(ws_b_bytes, dtype=torch.uint8, device=dev)
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

    ref = wl.make_old_logprobs(cfg, lp, seed=cfg.index + 77).to(dev)
    loss4 = torch.empty(4, dtype=torch.float32, device=dev)

    def fwd_bwd_aux():   # the coefficients of section 4.1
        grpo.grpo_lmhead_loss_aux_fwd_bwd(b["hidden"], b["weight"], b["tokens"], old, ref, adv_tok, b["mask"],
                                          cfg.eps_low, cfg.eps_high, cfg.delta, cfg.temperature, 0.001, 1e-4,
                                          0.0, 1.0, grad_hidden=dH, grad_weight=dW, loss_out=loss4,
                                          logprobs_out=lp, want_entropy=False, counts_out=counts,
                                          workspace=ws_b, stream=stream)
    ms_f = timed_calls(fwd, stream, reps, warmup)["mean"]
    ms_x = timed_calls(fwd_bwd_aux, stream, reps, max(2, warmup // 2))["mean"]
    aux_vals = loss4.cpu().tolist()
    ms_b = timed_calls(fwd_bwd, stream, reps, max(2, warmup // 2))["mean"]
    c = counts.cpu().tolist()
    # the same call with a workspace for chunks of half the default (the default workspace bounds the
    # chunk at 10240 rows, whatever N): what working through the rows in more, smaller chunks costs
    half_rows = 5120
    ws_h_bytes = grpo.grpo_lmhead_workspace_bytes_for_chunk(N, V, d_model, half_rows)
    ws_b = torch.empty(ws_h_bytes, dtype=torch.uint8, device=dev)
    ms_h = timed_calls(fwd_bwd, stream, reps, max(2, warmup // 2))["mean"]
    half = {"chunk_rows": half_rows, "fwd_bwd_ms": ms_h, "workspace_bytes": ws_h_bytes,
            "workspace_bytes_per_logit": ws_h_bytes / (float(N) * V)}
    n_unmasked = c[0]
    zero_adv = int(((adv_tok == 0) & (b["mask"] != 0)).sum())
    n_grad = n_unmasked - (c[1] + c[2] + c[3] + zero_adv)   # rows whose objective has a gradient
    # algorithmic flops: rows that take no part need none (2 V d per unmasked row for the logits,
    # twice that again per row with a gradient for dL/dH and dL/dW)
    flops_f = 2.0 * n_unmasked * V * d_model
    flops_b = flops_f + 4.0 * n_grad * V * d_model
    traffic, stamp = traffic_from_profile("lm_gemm_nt_%s_hbm_traffic" % cfg.name, "lm_gemm_nt")
    return {"note": "grpo_lmhead_logprobs_fwd / grpo_lmhead_loss_fwd_bwd: hidden [N, d] and head "
                    "weights [V, d] in bf16, logits formed on the matrix cores; tokens/s count all N rows, "
                    "flops only the rows that take part",
            "d_model": d_model, "rows": N, "rows_unmasked": n_unmasked, "rows_with_gradient": n_grad,
            "workspace_bytes_fwd": ws_f_bytes, "workspace_bytes_fwd_bwd": ws_b_bytes,
            "workspace_bytes_per_logit_fwd_bwd": ws_b_bytes / (float(N) * V),
            "fwd_ms": ms_f, "fwd_tokens_per_s": N / (ms_f * 1e-3),
            "fwd_bwd_ms": ms_b, "fwd_bwd_tokens_per_s": N / (ms_b * 1e-3), "loss": float(loss.cpu()),
            "fwd_bwd_half_chunks": half,
            "aux": {"note": "grpo_lmhead_loss_aux_fwd_bwd, KL 0.001 and entropy 1e-4: every unmasked row has a "
                            "gradient", "fwd_bwd_ms": ms_x, "fwd_bwd_tokens_per_s": N / (ms_x * 1e-3),
                    "tflops": (flops_f + 4.0 * n_unmasked * V * d_model) / (ms_x * 1e-3) / 1e12,
                    "total": aux_vals[0], "policy": aux_vals[1], "mean_kl": aux_vals[2],
                    "mean_entropy": aux_vals[3]},
            "roofline": {"bound": "mfma", "achieved": flops_f / (ms_f * 1e-3) / 1e12,
                         "peak": BF16_MFMA_PEAK_TFLOPS, "unit": "TFLOP/s",
                         "frac": flops_f / (ms_f * 1e-3) / 1e12 / BF16_MFMA_PEAK_TFLOPS,
                         "kernel": "lm_gemm_nt (forward: logits + softmax partials)",
                         "algorithmic_flops": flops_f, "traffic": traffic, "traffic_profile": stamp},
            "roofline_fwd_bwd": {"bound": "mfma", "achieved": flops_b / (ms_b * 1e-3) / 1e12,
                                 "peak": BF16_MFMA_PEAK_TFLOPS, "unit": "TFLOP/s",
                                 "frac": flops_b / (ms_b * 1e-3) / 1e12 / BF16_MFMA_PEAK_TFLOPS,
                                 "algorithmic_flops": flops_b}}


def run_workload(grpo, wl, cfg, args, dev, variant="", headline=False):
    """Generates one batch, times the whole step and the side legs on it, frees it.
    Returns (record, headline extras)."""
    import torch
    N, V = cfg.n_tokens, cfg.vocab
    log("[bench] generating %s: N=%d V=%d %s (%.2f GB of logits)" %
        (cfg.name, N, V, cfg.dtype, N * V * (2 if cfg.dtype == "bf16" else 4) / 1e9))
    batch = wl.make_batch(cfg, dev)
    esz = batch["logits"].element_size()
    stream = torch.cuda.current_stream()
    lp_ws = torch.empty(grpo.grpo_workspace_bytes(0), dtype=torch.uint8, device=dev)
    # old-policy log-probs: the library's own forward pass plus the recipe's staleness noise
    new_lp = grpo.grpo_logprobs_fwd(batch["logits"], batch["tokens"], None, cfg.temperature, workspace=lp_ws)
    torch.cuda.synchronize()
    old = wl.make_old_logprobs(cfg, new_lp).to(dev)

    adv = torch.empty(cfg.n_rollouts, dtype=torch.float32, device=dev)
    adv_tok = torch.empty(N, dtype=torch.float32, device=dev)
    grad = torch.empty_like(batch["logits"])
    loss = torch.empty(1, dtype=torch.float32, device=dev)
    lp = torch.empty(N, dtype=torch.float32, device=dev)
    counts = torch.empty(5, dtype=torch.int64, device=dev)
    ws = torch.empty(grpo.grpo_workspace_bytes(N), dtype=torch.uint8, device=dev)

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
        spread = {"median": per_step[len(per_step) // 2], "min": per_step[0], "max": per_step[-1]}
        return wall, sum(per_step) / K * 1e-3, spread

    log("[bench] %s: timing %d steps after %d warm-up steps" % (cfg.name, args.steps, args.warmup))
    wall, kern, kern_spread = timed(args.steps, args.warmup)
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
    # what this design moves through HBM: live rows are read once (kept in registers)
    moved_bytes = row_bytes * (2 * n_full + 2 * n_zero_coeff + 1 * n_masked) + 29 * N

    side_reps, side_warm = max(10, args.steps // 2), max(6, args.warmup)
    # worst case for the kernel: every row unmasked and live (ratio 1, non-zero advantage)
    ones = torch.ones(N, dtype=torch.uint8, device=dev)
    adv_ones = torch.full((N,), 0.5, dtype=torch.float32, device=dev)
    wall_full, kern_full, full_spread = timed(side_reps, side_warm, mask=ones, oldlp=new_lp, advantages=adv_ones)
    full_counts = counts.cpu().tolist()

    # the old-policy log-probs pass (one read of the logits), every row unmasked
    fwd = timed_calls(lambda: grpo.grpo_logprobs_fwd(batch["logits"], batch["tokens"], ones, cfg.temperature,
                                                     logprobs_out=lp, workspace=lp_ws, stream=stream),
                      stream, side_reps, side_warm)

    # the objective with the KL and entropy terms fused in (section 4.1 coefficients), same batch
    ref = wl.make_old_logprobs(cfg, new_lp, seed=cfg.index + 77).to(dev)
    loss4 = torch.empty(4, dtype=torch.float32, device=dev)
    ent = torch.empty(N, dtype=torch.float32, device=dev)
    aux = timed_calls(lambda: grpo.grpo_loss_aux_fwd_bwd(
        batch["logits"], batch["tokens"], old, ref, adv_tok, batch["mask"], cfg.eps_low, cfg.eps_high,
        cfg.delta, cfg.temperature, 0.001, 1e-4, 0.0, 1.0, grad_logits=grad, loss_out=loss4,
        logprobs_out=lp, entropy_out=ent, counts_out=counts, workspace=ws, stream=stream),
        stream, side_reps, side_warm)
    aux_vals = loss4.cpu().tolist()
    # with an entropy term every unmasked row gets a gradient: 2 reads + 1 write each
    aux_alg = row_bytes * (3 * M + 1 * n_masked) + 37 * N
    aux_moved = row_bytes * (2 * M + 1 * n_masked) + 37 * N

    traffic, stamp = (None, {"profile": None}) if variant else \
        traffic_from_profile("hbm_traffic_%s" % cfg.name, "grpo_rows_cached")
    gb = lambda nbytes, sec: nbytes / sec / 1e9
    rec = {
        "workload": cfg.name + variant, "n_tokens": N, "vocab": V, "logits_dtype": cfg.dtype,
        "rows_live": n_full, "rows_zero_coeff": n_zero_coeff, "rows_masked": n_masked,
        "ms_per_step": wall * 1e3, "tokens_per_s": N / wall, "tokens_per_s_unmasked": M / wall,
        "kernel_ms": kern * 1e3, "kernel_ms_median": kern_spread["median"],
        "kernel_ms_min": kern_spread["min"], "kernel_ms_max": kern_spread["max"],
        "algorithmic_bytes": alg_bytes, "achieved_gbps": gb(alg_bytes, kern),
        "frac": gb(alg_bytes, kern) / HBM_PEAK_GBPS,
        "moved_bytes": moved_bytes, "moved_gbps": gb(moved_bytes, kern),
        "frac_moved": gb(moved_bytes, kern) / HBM_PEAK_GBPS,
        "gbps_2r1w_all_rows_convention": gb(conv_bytes, kern),
        "traffic": traffic, "traffic_profile": stamp,
        # launches of the row kernel in this workload's part of the run, in order (for reading a kernel trace)
        "row_kernel_launches": [["grpo_logprobs_fwd (setup)", 1], ["workload", args.warmup + args.steps],
                                ["every row live", side_warm + side_reps], ["grpo_logprobs_fwd", side_warm + side_reps],
                                ["grpo_loss_aux_fwd_bwd (its own instantiation)", side_warm + side_reps]],
        "counts": dict(zip(grpo.COUNT_NAMES, c)), "loss": loss_value,
        "full_rows": {"note": "same logits, every row unmasked and live: the kernel's worst case",
                      "tokens_per_s": N / wall_full, "kernel_ms": kern_full * 1e3,
                      "kernel_ms_median": full_spread["median"], "kernel_ms_min": full_spread["min"],
                      "kernel_ms_max": full_spread["max"],
                      "frac": gb(conv_bytes, kern_full) / HBM_PEAK_GBPS,
                      "moved_gbps": gb(2 * N * row_bytes, kern_full),
                      "frac_moved": gb(2 * N * row_bytes, kern_full) / HBM_PEAK_GBPS,
                      "rows_live": full_counts[0]},
        "logprobs_fwd": {"note": "grpo_logprobs_fwd, every row unmasked: one read of the logits",
                         "tokens_per_s": N / (fwd["mean"] * 1e-3), "kernel_ms": fwd["mean"],
                         "kernel_ms_median": fwd["median"], "kernel_ms_min": fwd["min"],
                         "moved_gbps": gb(N * row_bytes, fwd["mean"] * 1e-3),
                         "frac_moved": gb(N * row_bytes, fwd["mean"] * 1e-3) / HBM_PEAK_GBPS},
        "aux_loss": {"note": "grpo_loss_aux_fwd_bwd on the same batch, KL 0.001 and entropy 1e-4 fused in",
                     "tokens_per_s": N / (aux["mean"] * 1e-3), "kernel_ms": aux["mean"],
                     "frac": gb(aux_alg, aux["mean"] * 1e-3) / HBM_PEAK_GBPS,
                     "frac_moved": gb(aux_moved, aux["mean"] * 1e-3) / HBM_PEAK_GBPS,
                     "total": aux_vals[0], "policy": aux_vals[1], "mean_kl": aux_vals[2],
                     "mean_entropy": aux_vals[3]},
    }
    extras = {}
    if headline:
        extras["row_kernel"] = grpo.grpo_row_kernel_plan(
            grpo.GRPO_BF16 if cfg.dtype == "bf16" else grpo.GRPO_F32, V)
        if not args.no_lmhead and cfg.logits in ("normal", "normal_boost") and cfg.dtype == "bf16":
            # the leg needs its own operands, gradients and two workspaces next to the batch
            need = (grpo.grpo_lmhead_workspace_bytes(N, V, args.d_model, True) +
                    grpo.grpo_lmhead_workspace_bytes(N, V, args.d_model, False) +
                    6 * V * args.d_model + 4 * N * args.d_model)
            free = torch.cuda.mem_get_info()[0]
            if need < 0.9 * free:
                extras["lmhead"] = lmhead_leg(grpo, wl, cfg, args.d_model, dev, stream,
                                              max(3, args.steps // 6), max(5, args.warmup))
            else:
                extras["lmhead"] = {"skipped": "needs %.0f GB of device memory, %.0f GB free" % (need / 1e9, free / 1e9)}
        if not args.no_cpu_baseline:
            log("[bench] timing the fp64 oracle on a sample of the batch (about 12 s)")
            step()
            torch.cuda.synchronize()
            extras["cpu_baseline"] = cpu_baseline(batch, old, adv_tok)
    if args.copy_calibration:
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    return rec, extras


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="all",
                    help="all (default): qwen_short as the headline plus the other three 152064-vocabulary "
                         "batches; or one workload by name")
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
    names = QWEN_WORKLOADS if args.workload == "all" else [args.workload]
    variant = ""
    if args.vocab or args.logits_dtype:
        if args.workload == "all":
            names = ["qwen_short"]
        args.no_lmhead = True

    records, head, head_extras, head_cfg = {}, None, {}, None
    for i, name in enumerate(names):
        cfg = wl.CONFIGS[name]
        if args.vocab or args.logits_dtype:
            # the same recipe at another row width: the sequence length takes up the difference
            import dataclasses
            esz0 = 2 if cfg.dtype == "bf16" else 4
            dt = args.logits_dtype or cfg.dtype
            vocab = args.vocab or cfg.vocab
            L = max(1, round(cfg.seq_len * cfg.vocab * esz0 / (vocab * (2 if dt == "bf16" else 4))))
            cfg = dataclasses.replace(cfg.scaled(seq_len=L, vocab=vocab), dtype=dt)
            variant = "@V=%d,%s" % (vocab, dt)
        rec, extras = run_workload(grpo, wl, cfg, args, dev, variant, headline=(i == 0))
        gc.collect()                 # the batch died with run_workload's frame: hand its memory back
        torch.cuda.empty_cache()
        records[name] = rec
        if i == 0:
            head, head_extras, head_cfg = rec, extras, cfg

    V = head["vocab"]
    worst = min(records.values(), key=lambda r: r["frac"])
    worst_moved = min(records.values(), key=lambda r: r["frac_moved"])
    worst_full = min(records.values(), key=lambda r: r["full_rows"]["frac_moved"])
    out = {
        "metric": "GRPO loss fwd+bwd tokens/s (V=152064 bf16)" if V == 152064 and head["logits_dtype"] == "bf16" else
                  "GRPO loss fwd+bwd tokens/s (V=%d %s)" % (V, head["logits_dtype"]),
        "value": head["tokens_per_s"], "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": head["ms_per_step"], "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": head["workload"], "n_tokens": head["n_tokens"], "vocab": V,
                   "logits_dtype": head["logits_dtype"], "group_size": head_cfg.group_size,
                   "n_rollouts": head_cfg.n_rollouts, "rows_live": head["rows_live"],
                   "rows_zero_coeff": head["rows_zero_coeff"], "rows_masked": head["rows_masked"],
                   "eps_low": head_cfg.eps_low, "eps_high": head_cfg.eps_high, "delta": head_cfg.delta,
                   "temperature": head_cfg.temperature, "row_kernel": head_extras.get("row_kernel"),
                   "also_timed": [n for n in names[1:]]},
        "value_unmasked_tokens_per_s": head["tokens_per_s_unmasked"],
        "counts": head["counts"], "loss": head["loss"],
        "roofline": {"bound": "hbm", "achieved": head["achieved_gbps"], "peak": HBM_PEAK_GBPS,
                     "unit": "GB/s", "frac": head["frac"],
                     "traffic": head["traffic"], "traffic_profile": head["traffic_profile"],
                     "kernel": "grpo_rows_cached (inside grpo_loss_fwd_bwd)",
                     "kernel_ms": head["kernel_ms"], "kernel_ms_median": head["kernel_ms_median"],
                     "kernel_ms_min": head["kernel_ms_min"], "kernel_ms_max": head["kernel_ms_max"],
                     "algorithmic_bytes": head["algorithmic_bytes"],
                     "note": "achieved/frac count ALGORITHMIC bytes (a live row 2 reads + 1 write); the kernel "
                             "keeps a row in registers and moves 1 read + 1 write: achieved_moved/frac_moved "
                             "are the physical share of the 8 TB/s peak",
                     "moved_bytes": head["moved_bytes"], "achieved_moved": head["moved_gbps"],
                     "frac_moved": head["frac_moved"],
                     "effective_gbps_2r1w_all_rows_convention": head["gbps_2r1w_all_rows_convention"],
                     "worst_frac": worst["frac"], "worst_frac_workload": worst["workload"],
                     "worst_frac_moved": worst_moved["frac_moved"],
                     "worst_frac_moved_workload": worst_moved["workload"],
                     "worst_full_rows_frac_moved": worst_full["full_rows"]["frac_moved"],
                     "worst_full_rows_frac_moved_workload": worst_full["workload"]},
        "workloads": records,
    }
    for key in ("lmhead", "cpu_baseline"):
        if key in head_extras:
            out[key] = head_extras[key]
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
