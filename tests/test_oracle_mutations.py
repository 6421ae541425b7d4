"""The pins must be able to fail: each planted mistake below is put into a private copy of the
oracle's C source, and the pin tests, run against that copy in a child process, have to reject
it.  A pin file that still passes with a wrong sign, a dropped 1/T or a reversed ratio in the
oracle would pin nothing.  Everything here runs on the CPU; the GPU path is not involved.
"""
import concurrent.futures
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CORE, AUX, REW, LMH = ("test_oracle_pins.py", "test_oracle_aux_pins.py", "test_oracle_rewards_pins.py",
                       "test_oracle_lmhead_pins.py")

# (what is planted, text in grpo_oracle.c, its replacement, which occurrence, pin file that must object)
MUTATIONS = [
    ("advantages: ddof ignored", "sqrt(ss / (double)(G - ddof))", "sqrt(ss / (double)G)", 0, CORE),
    ("advantages: mean over G + 1", "double mu = sum / (double)G;", "double mu = sum / (double)(G + 1);", 0, CORE),
    ("advantages: divided by the variance", "adv_out[i] = (den > 0.0) ? d / den : 0.0;",
     "adv_out[i] = (den > 0.0) ? d / (den * den) : 0.0;", 0, CORE),
    ("softmax: 1/T dropped in the sum", "csum_add(&acc, exp(logit_at(row, dtype, j) / T - mx));",
     "csum_add(&acc, exp(logit_at(row, dtype, j) - mx));", 0, CORE),
    ("log-prob: 1/T dropped at the sampled token", "logprobs_out[t] = logit_at(row, dtype, y) / T - lse;",
     "logprobs_out[t] = logit_at(row, dtype, y) - lse;", 0, CORE),
    ("surrogate: delta cap dropped", "double r_capped = (r < delta) ? r : delta;", "double r_capped = r;", 0, CORE),
    ("surrogate: eps_low and eps_high swapped", "double lo = 1.0 - eps_low, hi = 1.0 + eps_high;",
     "double lo = 1.0 - eps_high, hi = 1.0 + eps_low;", 0, CORE),
    ("surrogate: outer max instead of min", "if (s1 <= s2) {", "if (s1 >= s2) {", 0, CORE),
    ("surrogate: gradient flows through the cap", "dJ_dr = (r <= delta) ? A : 0.0;", "dJ_dr = A;", 0, CORE),
    ("surrogate: gradient flows through the clip", "dJ_dr = (r >= lo && r <= hi) ? A : 0.0;", "dJ_dr = A;", 0, CORE),
    ("surrogate: dr/dl dropped", "*dJ_dlogp_out = dJ_dr * r;", "*dJ_dlogp_out = dJ_dr;", 0, CORE),
    ("counter: clip_high regardless of the advantage's sign", "if (A > 0.0 && r > hi)", "if (r > hi)", 0, CORE),
    ("counter: delta regardless of the advantage's sign", "if (A < 0.0 && r > delta)", "if (r > delta)", 0, CORE),
    ("objective: ratio reversed", "double r = exp(logprobs[t] - (double)old_logprobs[t]);",
     "double r = exp((double)old_logprobs[t] - logprobs[t]);", 0, CORE),
    ("objective: sign of the loss", "*loss_out = (D > 0.0) ? -csum_value(&sumJ) / D : 0.0;",
     "*loss_out = (D > 0.0) ? csum_value(&sumJ) / D : 0.0;", 0, CORE),
    ("objective: grad_scale dropped", "coeff_out[t] = (D > 0.0) ? -grad_scale * dJ / D : 0.0;",
     "coeff_out[t] = (D > 0.0) ? -dJ / D : 0.0;", 0, CORE),
    ("objective: mean over all rows instead of the unmasked ones", "double D = (denom > 0.0) ? denom : (double)M;",
     "double D = (denom > 0.0) ? denom : (double)n_tokens;", 0, CORE),
    ("gradient: 1/T dropped", "g[j] = -(c / T) * p;", "g[j] = -c * p;", 0, CORE),
    ("gradient: sign at the sampled token", "g[y] = (c / T) * csum_value(&others);",
     "g[y] = -(c / T) * csum_value(&others);", 0, CORE),
    ("KL: difference reversed", "double d = l_ref - l;", "double d = l - l_ref;", 0, AUX),
    ("KL: sign of the derivative", "*dkl_dl_out = -expm1(d);", "*dkl_dl_out = expm1(d);", 0, AUX),
    ("entropy: sign", "csum_add(&h, -p * lp);", "csum_add(&h, p * lp);", 0, AUX),
    ("total: entropy added instead of subtracted", "*total_out = policy + kl_coef * klm - ent_coef * hm;",
     "*total_out = policy + kl_coef * klm + ent_coef * hm;", 0, AUX),
    ("coefficient: sign of the KL part", "c = grad_scale * w * (-dJ + kl_coef * dkl) / D;",
     "c = grad_scale * w * (-dJ - kl_coef * dkl) / D;", 0, AUX),
    ("entropy gradient: log p - H", "g[j] += (b / T) * p * (lp + H);", "g[j] += (b / T) * p * (lp - H);", 0, AUX),
    ("aux objective: ratio reversed", "double r = exp(logprobs[t] - (double)old_logprobs[t]);",
     "double r = exp((double)old_logprobs[t] - logprobs[t]);", 1, AUX),
    ("packed layout: sample-level weight 1/(len + 1)", "(float)(1.0 / (double)(e - b))", "(float)(1.0 / (double)(e - b + 1))",
     0, AUX),
    ("length reward: penalty added", "rewards_out[i] = (double)task_rewards[i] - alpha * fabs(diff);",
     "rewards_out[i] = (double)task_rewards[i] + alpha * fabs(diff);", 0, REW),
    ("filter: only larger rewards count as different", "if (rewards[i] != rewards[b])", "if (rewards[i] > rewards[b])", 0, REW),
    ("LM head: logits without the weights", "acc += h[k] * logit_at(weight, w_dtype, v * w_stride + k);", "acc += h[k];", 0, LMH),
    ("LM head: dL/dH without the weights", "out[k] += g * logit_at(weight, w_dtype, v * w_stride + k);", "out[k] += g;", 0, LMH),
    ("LM head: dL/dW without the hidden states", "acc += G[t * V + v] * logit_at(hidden, h_dtype, t * h_stride + k);",
     "acc += G[t * V + v];", 0, LMH),
]


def _replace_nth(text, old, new, n):
    at = -1
    for _ in range(n + 1):
        at = text.find(old, at + 1)
        assert at >= 0, "mutation target not found: %r" % old
    return text[:at] + new + text[at + len(old):]


def _run_pins(workdir, index, old, new, occurrence, pin_files):
    """Private copy of oracle/ and of the pin tests, optionally mutated, compiled, and run."""
    tmp = os.path.join(workdir, "m%02d" % index)
    os.makedirs(os.path.join(tmp, "tests"))
    shutil.copytree(os.path.join(ROOT, "oracle"), os.path.join(tmp, "oracle"),
                    ignore=shutil.ignore_patterns("*.so", "*.tmp.*", "__pycache__"))
    shutil.copytree(os.path.join(ROOT, "tests", "golden"), os.path.join(tmp, "tests", "golden"))
    for f in ("conftest.py", CORE, AUX, REW, LMH):
        shutil.copy(os.path.join(ROOT, "tests", f), os.path.join(tmp, "tests", f))
    src = os.path.join(tmp, "oracle", "grpo_oracle.c")
    text = open(src).read()
    if old is not None:
        text = _replace_nth(text, old, new, occurrence)
        open(src, "w").write(text)
    # compiled here, so that a mutation that does not compile is told apart from one the pins reject
    lib = os.path.join(tmp, "oracle", "libgrpo_oracle.so")
    cc = subprocess.run(["gcc", "-O2", "-std=c99", "-fopenmp", "-fPIC", "-shared", "-o", lib, src, "-lm"],
                        capture_output=True, text=True)
    assert cc.returncode == 0, cc.stderr
    env = dict(os.environ, PYTHONPATH=tmp, OMP_NUM_THREADS="2", PYTHONDONTWRITEBYTECODE="1")
    run = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider"] +
                         [os.path.join("tests", f) for f in pin_files], cwd=tmp, env=env, capture_output=True, text=True)
    return run.returncode, run.stdout[-2000:]


def test_every_planted_mistake_is_rejected_by_the_pins(tmp_path):
    jobs = [(0, None, None, 0, [CORE, AUX, REW, LMH])]             # control: the oracle as it is passes
    jobs += [(i + 1, old, new, occ, [pins]) for i, (_, old, new, occ, pins) in enumerate(MUTATIONS)]
    with concurrent.futures.ThreadPoolExecutor(max_workers=min(6, os.cpu_count() or 2)) as pool:
        results = list(pool.map(lambda j: _run_pins(str(tmp_path), *j), jobs))
    rc, out = results[0]
    assert rc == 0, "the unmodified copy does not pass its pins:\n" + out
    survivors = []
    for (what, *_), (rc, out) in zip(MUTATIONS, results[1:]):
        # 1 = some test failed; anything else (0 = passed, 2+ = collection or usage error) is a miss
        if rc != 1 or " failed" not in out:
            survivors.append("%s (exit %d)\n%s" % (what, rc, out[-400:]))
    assert not survivors, "planted mistakes the pins did not reject:\n" + "\n".join(survivors)
