"""Checkpoint / resume: the state of a run is x, m, the kept leader copies and the G+1 leader indices, all
visible to the caller.  2k steps in one go against k steps, a new handle over copies of the buffers with the
leaders restored, and k more steps: bit-identical on the paths whose kernels are deterministic (caller-supplied
gradients, MLP); the matrix-completion gradient kernels sum a row's contributions in an order that varies from
run to run, so that path is held to rounding level instead."""
import numpy as np
import pytest
import torch

import workloads as wl
import paper_1905_10395_amd as L
from gpu_util import DEV, dev, rel_l2_rows

pytestmark = pytest.mark.gpu


def run_with_resume(make_pop, step, k, resume):
    """make_pop(x, m, Z) -> population; step(pop, t).  Returns final (x, m, Z, leaders)."""
    x, m, Z, pop = make_pop(None)
    for t in range(k):
        step(pop, t)
    if resume:
        lead, gl = pop.get_leaders()
        torch.cuda.synchronize()
        saved = (x.clone(), m.clone(), Z.clone())
        pop.close()
        del pop
        x.fill_(float("nan")); m.fill_(float("nan")); Z.fill_(float("nan"))      # the old buffers are gone
        x, m, Z, pop = make_pop(saved)
        pop.set_leaders(lead, gl)
    for t in range(k, 2 * k):
        step(pop, t)
    out = (x.clone(), m.clone(), Z.clone(), pop.get_leaders())
    torch.cuda.synchronize()
    return out


def test_resume_external_gradients_bit_identical():
    W, G, P, k, tau = 8, 2, 5003, 4, 3
    ld = wl.padded_ld(P)
    x0, _, _ = wl.stress_state(W, P, ld, seed=9)
    grads = [dev(wl.stress_grad(W, P, ld, t, seed=9)) for t in range(2 * k)]
    losses = [dev(wl.stress_losses(W, t, seed=9)) for t in range(2 * k)]
    g = torch.zeros((W, ld), device=DEV)

    def make_pop(saved):
        x, m, Z = (dev(x0), torch.zeros((W, ld), device=DEV), torch.zeros((G + 1, ld), device=DEV)) if saved is None else saved
        return x, m, Z, L.Population(x, g, G, m=m, z_snapshot=Z, P=P, momentum=0.9, flags=L.NESTEROV, weight_decay=1e-4)

    def step(pop, t):
        g.copy_(grads[t])
        rl, rg = wl.refresh_masks(t, tau, G, staggered=True, tau_G=2 * tau)
        pop.step(L.ExternalBatch(losses[t]), 0.05, 0.1, 0.05, rl, rg)

    a = run_with_resume(make_pop, step, k, resume=False)
    b = run_with_resume(make_pop, step, k, resume=True)
    assert a[3] == b[3]
    for u, v in zip(a[:3], b[:3]):
        assert torch.equal(u, v)


@pytest.mark.parametrize("fused", [False, True])
def test_resume_mlp_bit_identical(fused):
    dims, W, G, B, k, tau = [192, 256, 10], 8, 2, 128, 3, 4
    P = wl.mlp_param_count(dims)
    ld = wl.padded_ld(P)
    x0 = wl.mlp_init(W, dims, ld=ld, seed=21, bias_std=0.05)
    means = wl.gmm_means(dims[0], dims[-1], seed=21)
    batches = []
    for t in range(2 * k):
        Xb, y = wl.gmm_batch(W, B, means, t, seed=21)
        batches.append(L.MLPBatch(dims, dev(Xb.view(np.int16)).view(torch.bfloat16), dev(y)))
    g = torch.zeros((W, ld), device=DEV)

    def make_pop(saved):
        x, m, Z = (dev(x0), torch.zeros((W, ld), device=DEV), torch.zeros((G + 1, ld), device=DEV)) if saved is None else saved
        xb = torch.zeros((W, ld), dtype=torch.bfloat16, device=DEV)             # rebuilt from x by the first gradient call
        flags = L.FUSED_MLP_UPDATE if fused else L.WRITE_BF16_SHADOW
        return x, m, Z, L.Population(x, g, G, m=m, z_snapshot=Z, x_bf16=xb, P=P, momentum=0.9, flags=flags, largest_batch=batches[0])

    def step(pop, t):
        rl, rg = wl.refresh_masks(t, tau, G, staggered=True)
        pop.step(batches[t], 0.01, 0.1, 0.05, rl, rg)

    a = run_with_resume(make_pop, step, k, resume=False)
    b = run_with_resume(make_pop, step, k, resume=True)
    assert a[3] == b[3]
    for u, v in zip(a[:3], b[:3]):
        assert torch.equal(u, v)


def test_resume_matrix_completion_to_rounding():
    W, G, k, tau = 8, 2, 3, 4
    prob = wl.mc_problem(600, 500, 32, 0.05, 32 ** -0.5, noise_std=0.01, seed=23)
    P, ld = prob.P, wl.padded_ld(prob.P)
    x0 = wl.mc_init(W, prob, 32 ** -0.5, ld=ld, seed=3)
    rows, cols, vals = dev(prob.rows), dev(prob.cols), dev(prob.vals)
    B = 2048
    idx = wl.mc_batches(W, B, prob.n_obs, 2 * k, seed=5)
    batches = [L.MCBatch(prob.m, prob.n, prob.r, rows, cols, vals, dev(idx[t]), 0.5 * prob.n_obs / B) for t in range(2 * k)]
    g = torch.zeros((W, ld), device=DEV)

    def make_pop(saved):
        x, m, Z = (dev(x0), torch.zeros((W, ld), device=DEV), torch.zeros((G + 1, ld), device=DEV)) if saved is None else saved
        return x, m, Z, L.Population(x, g, G, m=m, z_snapshot=Z, P=P, momentum=0.9, largest_batch=batches[0])

    def step(pop, t):
        rl, rg = wl.refresh_masks(t, tau, G, staggered=True)
        pop.step(batches[t], 0.005, 0.1, 0.05, rl, rg)

    a = run_with_resume(make_pop, step, k, resume=False)
    b = run_with_resume(make_pop, step, k, resume=True)
    assert a[3] == b[3]
    for u, v in zip(a[:3], b[:3]):
        assert rel_l2_rows(u.cpu().numpy()[:, :P], v.cpu().numpy()[:, :P]).max() < 1e-6


def test_call_order_errors():
    W, P = 4, 64
    x0, g0, _ = wl.stress_state(W, P, P, seed=1)
    x, g = dev(x0), dev(g0)
    Z = torch.zeros((3, P), device=DEV)
    pop = L.Population(x, g, 2, z_snapshot=Z, P=P)
    with pytest.raises(L.LsgdError, match="STATE.*never written"):
        pop.select_leaders()                                     # the population's own losses were never produced
    win = torch.zeros((3, W), device=DEV)
    with pytest.raises(L.LsgdError, match="STATE.*never written"):
        pop.smooth_losses(win, 0)
    lo = dev(wl.stress_losses(W, 0))
    pop.grad_loss(L.ExternalBatch(lo))
    pop.select_leaders()                                         # fine now
    pop.pull_update(0.1, 0.1, 0.1)
    # a re-selection consumed by an update that skips the local term leaves that group's old copy invalid
    pop.select_leaders(lo)
    pop.pull_update(0.1, 0.0, 0.1)
    with pytest.raises(L.LsgdError, match="STATE.*no selected leader copy"):
        pop.pull_update(0.1, 0.1, 0.1)
    before = x.clone()
    with pytest.raises(L.LsgdError, match="not a row of group"):
        pop.set_leaders([0, 1], 0)
    pop.set_leaders([1, 2], 2)
    assert pop.get_leaders() == ([1, 2], 2)
    pop.pull_update(0.1, 0.1, 0.1)                               # restored leaders make the kept copies usable again
    torch.cuda.synchronize()
    assert not torch.equal(before, x)
