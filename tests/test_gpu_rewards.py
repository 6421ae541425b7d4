"""GPU parity of the reward shaping and online filter kernels (sections 3.1, 3.3)."""
import numpy as np
import pytest
import torch

import paper_2505_07291_amd as grpo
from oracle import grpo_oracle as orc

pytestmark = pytest.mark.gpu
DEV = "cuda"


def test_total_rewards():
    g = torch.Generator().manual_seed(2)
    for R in (1, 63, 4096, 100001):
        task = (torch.rand(R, generator=g) < 0.3).float()
        target = torch.tensor([1000, 2000, 3000, 4000], dtype=torch.int32)[torch.randint(0, 4, (R,), generator=g)]
        length = torch.randint(1, 32769, (R,), generator=g, dtype=torch.int32)
        out = grpo.grpo_total_rewards(task.to(DEV), length.to(DEV), target.to(DEV), 3e-4)
        ref = orc.total_rewards(task.numpy(), length.numpy(), target.numpy(), float(np.float32(3e-4)))
        got = out.cpu().numpy().astype(np.float64)
        # one product and one difference in fp32 against fp64
        assert np.max(np.abs(got - ref)) <= 2.0 ** -22 * np.maximum(1.0, np.abs(ref)).max()
    assert grpo.grpo_total_rewards(task[:0].to(DEV), length[:0].to(DEV), target[:0].to(DEV), 3e-4).numel() == 0


def test_filter_groups_bit_exact():
    g = torch.Generator().manual_seed(3)
    for G, n in ((16, 256), (4, 5000), (64, 33), (1, 10), (100, 1500)):
        R = (torch.rand(G * n, generator=g) < 0.15).float()
        R[:G] = 1.0
        keep, kept, n_kept, rk = grpo.grpo_filter_groups(R.to(DEV), group_size=G)
        torch.cuda.synchronize()
        rkeep, rkept, rn, rrk = orc.filter_groups(R.numpy(), group_size=G)
        assert np.array_equal(keep.cpu().numpy(), rkeep) and int(n_kept) == rn
        assert np.array_equal(kept.cpu().numpy(), rkept)
        assert np.array_equal(rk.cpu().numpy(), rrk)
    sizes = [3, 1, 16, 0, 70, 5, 2]
    off = torch.tensor(np.concatenate([[0], np.cumsum(sizes)]), dtype=torch.int32)
    R = torch.randint(0, 3, (int(off[-1]),), generator=g).float() * 0.5
    R[off[5]:off[6]] = 0.5                                    # a constant group
    keep, kept, n_kept, rk = grpo.grpo_filter_groups(R.to(DEV), group_offsets=off.to(DEV))
    rkeep, rkept, rn, rrk = orc.filter_groups(R.numpy(), group_offsets=off.numpy())
    assert np.array_equal(keep.cpu().numpy(), rkeep) and int(n_kept) == rn
    assert np.array_equal(kept.cpu().numpy(), rkept) and np.array_equal(rk.cpu().numpy(), rrk)
    # no groups at all
    keep, kept, n_kept, rk = grpo.grpo_filter_groups(R[:0].to(DEV), group_size=4)
    assert int(n_kept) == 0


def test_reward_chain_feeds_the_advantages():
    """total reward -> filter -> advantages of the kept groups, as the trainer would chain them."""
    g = torch.Generator().manual_seed(4)
    G, n = 16, 64
    task = (torch.rand(G * n, generator=g) < 0.2).float()
    target = torch.full((G * n,), 2000, dtype=torch.int32)
    length = torch.randint(500, 4000, (G * n,), generator=g, dtype=torch.int32)
    length[:G] = 2000
    task[:G] = 0.0                                            # equal total rewards: filtered out
    rew = grpo.grpo_total_rewards(task.to(DEV), length.to(DEV), target.to(DEV), 3e-4)
    keep, kept, n_kept, _ = grpo.grpo_filter_groups(rew, group_size=G)
    adv, _ = grpo.grpo_group_advantages(rew, group_size=G)
    torch.cuda.synchronize()
    assert int(keep[0]) == 0 and int(n_kept) == n - 1
    a = adv.cpu().numpy().reshape(n, G)
    assert not a[0].any() and np.all(np.any(a[1:] != 0, axis=1))
