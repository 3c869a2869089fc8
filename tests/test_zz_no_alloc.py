"""The allocation-free variant of the policy-gradient loss (sr_grpo_loss_static) against sr_grpo_loss.

Both run the same kernel; the variant keeps the per-group shares in the library's fixed device array instead
of a caller-provided workspace.  Two calls in a row, the second on a smaller input, each compared bit for bit
with the workspace variant: the second call must not see anything the first one left in the shared array.
"""
import ctypes

import numpy as np
import pytest
import torch

import paper_2605_05802_amd as sr

pytestmark = pytest.mark.gpu


def _case(n_groups, G, seed):
    rng = np.random.default_rng(seed)
    r = rng.integers(0, 2, size=(n_groups, G)).astype(np.float32)      # success / failure rewards
    r[::3] = r[::3, :1]                                                 # a third of the groups: zero variance
    lp = -rng.uniform(5.0, 400.0, size=(n_groups, G))
    return torch.from_numpy(lp).cuda(), torch.from_numpy(r).cuda()


def _both(n_groups, G, seed):
    lp, r = _case(n_groups, G, seed)
    adv_a = torch.full((n_groups, G), 7.0, dtype=torch.float32, device="cuda")
    adv_b = torch.full((n_groups, G), 9.0, dtype=torch.float32, device="cuda")
    loss_a = torch.zeros(1, dtype=torch.float64, device="cuda")
    loss_b = torch.ones(1, dtype=torch.float64, device="cuda")
    scratch = torch.empty(n_groups, dtype=torch.float64, device="cuda")
    sr.sr_grpo_loss(lp, r, G, 1e-6, adv_a, scratch, loss_a)
    before = torch.cuda.memory_allocated()
    sr.sr_grpo_loss_static(lp, r, G, 1e-6, adv_b, loss_b)
    assert torch.cuda.memory_allocated() == before
    torch.cuda.synchronize()
    assert np.isfinite(loss_a.item()) and loss_a.item() != 0.0
    assert loss_b.cpu().numpy().tobytes() == loss_a.cpu().numpy().tobytes()
    assert np.array_equal(adv_b.cpu().numpy(), adv_a.cpu().numpy())
    assert np.all(adv_b.cpu().numpy()[::3] == 0.0)
    return loss_b.item()


def test_static_scratch_variant_matches_the_workspace_variant_twice():
    big = _both(4096, 8, seed=1)
    small = _both(37, 16, seed=2)          # a smaller input right after: the array still holds 4096 old shares
    assert big != small
    again = _both(4096, 8, seed=1)
    assert again == big


def test_limit_and_argument_checks():
    L = sr.lib()
    fake = ctypes.c_void_p(4096)            # never dereferenced: validation fails first
    n_max = sr.GRPO_STATIC_MAX_GROUPS
    assert L.sr_grpo_loss_static(fake, fake, n_max + 1, 8, 1e-6, None, fake, None) == sr.SR_E_LIMIT
    assert "capacity" in sr.strerror(sr.SR_E_LIMIT)
    assert L.sr_grpo_loss_static(None, fake, 4, 8, 1e-6, None, fake, None) == sr.SR_E_ARG
    assert L.sr_grpo_loss_static(fake, fake, 0, 8, 1e-6, None, fake, None) == sr.SR_E_ARG
    # exactly at the limit is accepted and correct
    _both(n_max, 2, seed=3)
