"""lsgd_select_pull_static (the entry point for callers that cannot allocate) against lsgd_step on an
external batch with a full refresh: same kernels, so the results must be identical bit for bit.  Two calls
in a row, the second on a smaller population, so that whatever the first left in the static array would show."""
import numpy as np
import pytest
import torch

import workloads as wl
import paper_1905_10395_amd as L
from gpu_util import DEV, dev

pytestmark = pytest.mark.gpu


def both_ways(W, G, P, ld, off, mu, flags, wd, seed, step_t):
    x0, g0, _ = wl.stress_state(W, P, ld, seed=seed)
    m0 = (wl.stress_grad(W, P, ld, 77, seed=seed) * np.float32(3.0)).astype(np.float32) if mu else None
    losses = dev(wl.stress_losses(W, step_t, seed=seed))
    eta, lamL, lamG = 0.05, 0.1, 0.05
    # existing entry point: handle + workspace
    xa, ga = dev(x0), dev(g0)
    ma = dev(m0) if mu else None
    pop = L.Population(xa, ga, G, m=ma, P=P, group_offsets=None if off is None else list(off), momentum=mu, flags=flags,
                       weight_decay=wd)
    pop.step(L.ExternalBatch(losses), eta, lamL, lamG)
    lead, gl = pop.get_leaders()
    # static entry point: buffers preallocated, then the call itself
    xb, gb = dev(x0), dev(g0)
    mb = dev(m0) if mu else None
    leaders = torch.full((G + 1,), -7, dtype=torch.int32, device=DEV)
    torch.cuda.synchronize()
    before = torch.cuda.memory_stats(DEV)["allocation.all.allocated"]
    L.select_pull_static(xb, gb, losses, G, eta, lamL, lamG, m=mb, P=P, group_offsets=None if off is None else list(off),
                         momentum=mu, weight_decay=wd, flags=flags, leaders=leaders)
    torch.cuda.synchronize()
    assert torch.cuda.memory_stats(DEV)["allocation.all.allocated"] == before        # torch's allocator was not touched
    assert leaders.cpu().tolist() == lead + [gl]
    assert torch.equal(xa, xb)
    if mu:
        assert torch.equal(ma, mb)
    return xb


def test_static_entry_matches_step_twice_second_smaller():
    both_ways(32, 4, 300_003, 300_032, None, 0.9, 0, 0.0, seed=5, step_t=0)
    both_ways(7, 3, 3003, 3004, np.array([0, 2, 3, 7], dtype=np.int32), 0.5, L.MOMENTUM_GRAD_ONLY | L.NESTEROV, 1e-3, seed=6, step_t=1)
    both_ways(5, 5, 515, 516, None, 0.0, L.PULL_UNSCALED_BY_ETA, 0.0, seed=7, step_t=2)
    both_ways(70, 6, 1030, 1032, np.array([0, 5, 20, 21, 40, 64, 70], dtype=np.int32), 0.9, L.LEADER_EXEMPT, 0.0, seed=8, step_t=3)


def test_static_entry_rejects_sizes_beyond_its_scratch():
    x = torch.zeros((4, 64), device=DEV); g = torch.zeros_like(x); lo = torch.zeros(4, device=DEV)
    big = torch.zeros((L.binding.STATIC_MAX_WORKERS + 1, 4), device=DEV)
    with pytest.raises(L.LsgdError, match="SHAPE.*static scratch"):
        L.select_pull_static(big, torch.zeros_like(big), torch.zeros(big.shape[0], device=DEV), 1, 0.1, 0.1, 0.1)
    wide = torch.zeros((130, 4), device=DEV)
    with pytest.raises(L.LsgdError, match="SHAPE.*static scratch"):
        L.select_pull_static(wide, torch.zeros_like(wide), torch.zeros(130, device=DEV), 65, 0.1, 0.1, 0.1)
    with pytest.raises(L.LsgdError, match="m buffer"):
        L.select_pull_static(x, g, lo, 2, 0.1, 0.1, 0.1, momentum=0.9)
    with pytest.raises(L.LsgdError, match="not available"):
        L.select_pull_static(x, g, lo, 2, 0.1, 0.1, 0.1, flags=L.WRITE_BF16_SHADOW)
    with pytest.raises(L.LsgdError, match="group_offsets"):
        L.select_pull_static(x, g, lo, 2, 0.1, 0.1, 0.1, group_offsets=[0, 2, 3])
    torch.cuda.synchronize()
    assert torch.count_nonzero(x) == 0
