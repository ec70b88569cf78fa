"""GPU parity for lsgd_loss, the objective-only evaluation that leader selection needs (Section 3.1.3,
Algorithm 1: the best workers are determined after the local step), against the CPU oracle's losses, and
Algorithm 1 in its printed order composed from the separate calls."""
import numpy as np
import pytest
import torch

import workloads as wl
import paper_1905_10395_amd as L
from gpu_util import DEV, Pair, dev
from test_gpu_alg1 import alg1_oracle_iteration
from test_gpu_mc import mc_batch, upload
from test_gpu_mlp import make

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("packed", [False, True])
@pytest.mark.parametrize("m,n,r,frac,W,B", [
    (100, 100, 5, 0.30, 4, None),          # every observed entry, odd rank
    (300, 200, 32, 0.10, 3, 5000),         # the shape whose gradient takes the binned path
    (257, 129, 7, 0.20, 2, 1111),
    (40, 30, 100, 0.50, 2, 300),           # rank above a wavefront
    (64, 64, 1, 0.50, 2, 100),
    (128, 96, 8, 0.90, 8, 300_000),        # hundreds of partial sums per worker
])
def test_mc_loss_matches_oracle_and_leaves_g_alone(m, n, r, frac, W, B, packed):
    prob = upload(wl.mc_problem(m, n, r, frac, 1.0, noise_std=0.01, seed=m + r))
    ld = wl.padded_ld(prob.P, 4)
    x0 = wl.mc_init(W, prob, 0.7, ld=ld, seed=r)
    idx = None if B is None else wl.mc_batches(W, B, prob.n_obs, 1, seed=m)[0]
    c = 0.5 if B is None else 0.5 * prob.n_obs / B
    batch = mc_batch(prob, None if idx is None else dev(idx), c, packed)
    pr = Pair(x0, np.array([0, W], dtype=np.int32), P=prob.P, largest_batch=batch)
    pr.g.fill_(123.0)
    pr.ora.grad_loss_mc(m, n, r, prob.rows, prob.cols, prob.vals, idx, c)
    pr.pop.loss(batch)
    torch.cuda.synchronize()
    assert bool((pr.g == 123.0).all())                      # g is not an output
    assert np.array_equal(pr.x.cpu().numpy(), x0)
    np.testing.assert_allclose(pr.pop.get_losses(), pr.ora.losses, rtol=1e-5)
    out = torch.full((W,), -1.0, device=DEV)                # caller's buffer instead of the population's
    pr.pop.loss(batch, out)
    np.testing.assert_allclose(out.cpu().numpy(), pr.ora.losses, rtol=1e-5)
    pr.pop.grad_loss(batch)                                 # the gradient pass agrees up to the order of its sum
    np.testing.assert_allclose(pr.pop.get_losses(), out.cpu().numpy(), rtol=2e-6)


def test_mc_loss_of_an_empty_batch_is_zero():
    prob = upload(wl.mc_problem(40, 30, 8, 0.5, 1.0, seed=1))
    W = 3
    x0 = wl.mc_init(W, prob, 0.7, ld=wl.padded_ld(prob.P, 4), seed=2)
    batch = mc_batch(prob, torch.zeros((W, 0), dtype=torch.int32, device=DEV), 1.0, False)   # B = 0
    pr = Pair(x0, np.array([0, W], dtype=np.int32), P=prob.P, largest_batch=batch)
    pr.pop.loss(batch)
    assert pr.pop.get_losses() == [0.0] * W


@pytest.mark.parametrize("dims,W,B", [
    ([12, 16, 5], 2, 9),                      # vector-ALU path
    ([192, 256, 128, 10], 3, 128),            # MFMA tiles
    ([64, 512, 10], 64, 256),                 # whole batch per tile
    ([3072, 512, 512, 10], 4, 256),
])
def test_mlp_loss_is_the_forward_pass(dims, W, B):
    pr, batch, Xb, y, P, _ = make(dims, W, B, seed=len(dims) * 10 + W)
    pr.g.fill_(7.0)
    pr.ora.grad_loss_mlp(dims, Xb, y)
    pr.pop.loss(batch)
    torch.cuda.synchronize()
    assert bool((pr.g == 7.0).all())
    lo = np.array(pr.pop.get_losses(), dtype=np.float32)
    np.testing.assert_allclose(lo, pr.ora.losses, rtol=1e-4)
    pr.pop.grad_loss(batch)
    assert np.array_equal(np.array(pr.pop.get_losses(), dtype=np.float32), lo)      # same kernels, same bits


def test_external_loss_copies():
    W, P = 5, 64
    x0, _, _ = wl.stress_state(W, P, P, seed=3)
    pr = Pair(x0, wl.equal_group_offsets(W, 1), P=P)
    lo = wl.stress_losses(W, 4)
    pr.pop.loss(L.ExternalBatch(dev(lo)))
    assert np.array_equal(np.array(pr.pop.get_losses(), dtype=np.float32), lo)
    pr.pop.select_leaders()                                 # the population's buffer now counts as written
    assert pr.pop.get_leaders()[1] == int(np.argmin(lo))


def test_alg1_in_printed_order_with_reevaluated_losses():
    """Algorithm 1 as printed: local step on sample t, then at a communication the best workers are determined
    from the objective on sample t+1 at the parameters the step produced, then the pull."""
    W, G = 8, 2
    prob = wl.mc_problem(600, 500, 32, 0.05, 32 ** -0.5, noise_std=0.01, seed=29)
    m, n, r, P = prob.m, prob.n, prob.r, prob.P
    ld = wl.padded_ld(P)
    x0 = wl.mc_init(W, prob, 32 ** -0.5, ld=ld, seed=4)
    rows, cols, vals = dev(prob.rows), dev(prob.cols), dev(prob.vals)
    B = 2048
    c = 0.5 * prob.n_obs / B
    idx = wl.mc_batches(W, B, prob.n_obs, 11, seed=6)      # [steps, W, B]
    mk = lambda t: L.MCBatch(m, n, r, rows, cols, vals, dev(idx[t]), c)
    pr = Pair(x0, wl.equal_group_offsets(W, G), P=P, largest_batch=mk(0))
    eta, tau = 0.005, 3
    gamL, gamG, lamL, lamG = 0.02, 0.01, 0.3, 0.1
    none = np.zeros(G, dtype=np.uint8)
    pr.ora.grad_loss_mc(m, n, r, prob.rows, prob.cols, prob.vals, idx[0], c)
    pr.ora.select(); pr.ora.leader_pull(0.0, 0.0)
    pr.pop.loss(mk(0)); pr.pop.select_leaders(); pr.pop.leader_pull(0.0, 0.0)
    assert pr.check_leaders()
    comms = 0
    for t in range(1, 10):
        rl, rg = wl.refresh_masks(t, tau, G, tau_G=2 * tau)
        pr.ora.grad_loss_mc(m, n, r, prob.rows, prob.cols, prob.vals, idx[t], c)
        alg1_oracle_iteration(pr.ora, eta, gamL, gamG, lamL, lamG, none, 0)      # local step only
        pr.pop.step_alg1(mk(t), eta, gamL, gamG, lamL, lamG, 0)
        if rl.any() or rg:
            comms += 1
            pr.ora.grad_loss_mc(m, n, r, prob.rows, prob.cols, prob.vals, idx[t + 1], c)   # its losses; g is recomputed next iteration
            pr.ora.select(rl, rg); pr.ora.leader_pull(lamL, lamG, rl, rg)
            pr.pop.loss(mk(t + 1))
            lo = np.array(pr.pop.get_losses())
            assert np.abs(lo - pr.ora.losses).max() <= 1e-4 * np.abs(pr.ora.losses).max()
            pr.pop.select_leaders(None, rl, rg)
            pr.pop.leader_pull(lamL, lamG)
            if not pr.check_leaders(rl, rg):
                pr.resync_from_oracle()
        pr.check_state(3e-4, f"iteration {t}")
    assert comms >= 3
