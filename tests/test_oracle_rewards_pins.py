"""Pins of the oracle's reward shaping (section 3.1) and online filtering (section 3.3)."""
import numpy as np

from oracle import grpo_oracle as orc


def test_total_reward_worked_values():
    # alpha = 3e-4 (section 4.1), targets from the discrete sets of section 4.2
    task = [1.0, 1.0, 0.0, 1.0, 0.0]
    length = [2500, 1500, 2000, 2000, 9000]
    target = [2000, 2000, 2000, 2000, 6000]
    out = orc.total_rewards(task, length, target, 3e-4)
    expect = [1 - 3e-4 * 500, 1 - 3e-4 * 500, 0.0, 1.0, -3e-4 * 3000]      # symmetric in the sign
    assert np.max(np.abs(out - expect)) < 1e-15
    assert np.array_equal(orc.total_rewards(task, length, target, 0.0), np.array(task))


def test_filter_keeps_exactly_the_groups_with_signal():
    rng = np.random.default_rng(1)
    G, n = 16, 40
    R = (rng.random(G * n) < 0.2).astype(np.float32)
    R[:G] = 0.0
    R[G:2 * G] = 1.0
    keep, kept, n_kept, rk = orc.filter_groups(R, group_size=G)
    brute = [int(len(set(R[g * G:(g + 1) * G].tolist())) > 1) for g in range(n)]
    assert keep.tolist() == brute and keep[0] == 0 and keep[1] == 0
    assert n_kept == sum(brute)
    assert kept[:n_kept].tolist() == [g for g in range(n) if brute[g]]
    assert (kept[n_kept:] == -1).all()
    assert rk.tolist() == np.repeat(brute, G).tolist()
    # kept <=> some advantage is non-zero (section 3.3: equal rewards give zero advantages)
    adv = orc.group_advantages(R, group_size=G, eps_std=1e-6).reshape(n, G)
    assert (np.any(adv != 0, axis=1).astype(int)).tolist() == brute
    # ragged groups, continuous rewards with ties
    off = np.array([0, 1, 4, 4, 9], np.int32)
    R2 = np.array([0.3, 0.5, 0.5, 0.5, 0.1, 0.1, 0.2, 0.1, 0.1], np.float32)
    keep2, kept2, n2, _ = orc.filter_groups(R2, group_offsets=off)
    assert keep2.tolist() == [0, 0, 0, 1] and n2 == 1 and kept2.tolist() == [3, -1, -1, -1]
