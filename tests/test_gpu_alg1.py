"""GPU parity for Algorithm 1's communication schedule, the smoothed selection loss and the
center variable (Section 4.1), each against the CPU oracle through the C boundary."""
import numpy as np
import pytest
import torch

import oracle
import workloads as wl
import paper_1905_10395_amd as L
from gpu_util import DEV, Pair, assert_update_elementwise, dev, rel_l2_rows
from test_gpu_select_update import random_offsets

pytestmark = pytest.mark.gpu

PULL_CASES = [
    # W, G, P, ld
    (4, 1, 1000, 1000),
    (16, 4, 4099, 4160),            # ragged P, padded rows
    (8, 2, 5000, 5001),             # ld % 4 != 0: scalar path
    (7, 3, 3003, 3004),             # unequal groups
    (5, 5, 515, 516),               # every worker its own group
    (70, 6, 1030, 1032),            # W > 64
    (6, 2, 1_300_003, 1_300_032),   # more than one column chunk
]


@pytest.mark.parametrize("W,G,P,ld", PULL_CASES)
def test_leader_pull_matches_oracle(W, G, P, ld):
    """Random communication masks and coefficients; both sides restart each trial from the same
    x, so captured leader copies must be bit-exact and pulled rows equal up to fp32 rounding."""
    r = wl.stream("gpu_leader_pull", W, G, P)
    off = random_offsets(r, W, G) if W % G else wl.equal_group_offsets(W, G)
    x0, _, _ = wl.stress_state(W, P, ld, seed=W * 31 + G)
    pr = Pair(x0, off, P=P, flags=L.WRITE_BF16_SHADOW, shadow=True)
    pr.pop.sync_shadow()
    lams = [(0.1, 0.05), (0.0, 0.0), (1.0, 0.0), (0.25, 1.0), (0.0, 0.3), (0.7, 0.0), (0.5, 0.5), (0.3, 0.2)]
    for trial, (lamL, lamG) in enumerate(lams):
        losses = wl.stress_losses(W, trial, seed=W + G)
        rl = np.ones(G, dtype=np.uint8) if trial in (0, 3) else (r.random(G) < 0.5).astype(np.uint8)
        rg = 1 if trial in (0, 3) else int(r.random() < 0.5)
        if not rl.any() and not rg:
            rl[int(r.integers(0, G))] = 1
        pr.ora.losses[:] = losses
        x_before = pr.ora.x.copy()
        pr.ora.select(rl, rg); pr.ora.leader_pull(lamL, lamG, rl, rg)
        pr.pop.select_leaders(dev(losses), rl, rg)
        pr.pop.leader_pull(lamL, lamG)
        assert pr.check_leaders(rl, rg)
        torch.cuda.synchronize()
        assert_update_elementwise(pr.x.cpu().numpy()[:, :P], pr.ora.x[:, :P], x_before[:, :P], f"trial {trial}")
        Zg = pr.Z.cpu().numpy()
        for j in list(np.nonzero(rl)[0]) + ([G] if rg else []):
            np.testing.assert_array_equal(Zg[j, :P], pr.ora.Z[j, :P])
        # bf16 operand copy follows every changed row
        assert torch.equal(pr.xb[:, :P], pr.x[:, :P].to(torch.bfloat16))
        if lamL == 1.0 and rl.all():          # full local pull: every worker lands on its group's leader
            xg = pr.x.cpu().numpy()            # (x - (x - z) is z up to the rounding of the difference)
            for j in range(G):
                assert rel_l2_rows(xg[off[j]:off[j + 1], :P], Zg[j:j + 1, :P]).max() < 2e-7
        if ld > P:
            assert np.array_equal(pr.x.cpu().numpy()[:, P:], x0[:, P:])
        pr.resync_from_oracle()
        pr.pop.sync_shadow()


def test_leader_pull_state_errors():
    W, P = 4, 64
    x0, g0, _ = wl.stress_state(W, P, P, seed=2)
    pr = Pair(x0, wl.equal_group_offsets(W, 2), P=P)
    with pytest.raises(L.LsgdError, match="re-selected"):
        pr.pop.leader_pull(0.1, 0.1)
    pr.pop.select_leaders(dev(wl.stress_losses(W, 0)))
    pr.pop.leader_pull(0.0, 0.0)                            # initialisation: capture only
    torch.cuda.synchronize()
    assert np.array_equal(pr.x.cpu().numpy(), x0)
    with pytest.raises(L.LsgdError, match="re-selected"):
        pr.pop.leader_pull(0.1, 0.1)
    with pytest.raises(L.LsgdError, match="finite"):
        pr.pop.leader_pull(float("inf"), 0.1)
    pr2 = Pair(x0, wl.equal_group_offsets(W, 2), P=P, snapshot=False)
    pr2.set_grad(g0, wl.stress_losses(W, 0))
    with pytest.raises(L.LsgdError, match="z_snapshot"):
        pr2.pop.step_alg1(L.ExternalBatch(pr2.losses_dev), 0.1, 0.01, 0.01, 0.1, 0.1, L.COMM_LOCAL)
    with pytest.raises(L.LsgdError, match="comm bits"):
        pr.pop.step_alg1(L.ExternalBatch(dev(wl.stress_losses(W, 0))), 0.1, 0.01, 0.01, 0.1, 0.1, 4)


def alg1_oracle_iteration(ora, eta, gamL, gamG, lamL, lamG, rl, rg):
    """The oracle's pieces in Algorithm 1's order: local step with the small pulls to the kept
    copies, then (at a communication) selection from this iteration's losses and the pull."""
    none = np.zeros(ora.G, dtype=np.uint8)
    flags = ora.flags
    ora.flags = flags | oracle.PULL_UNSCALED_BY_ETA
    ora.update(eta, gamL, gamG, none, 0)
    ora.flags = flags
    if rl.any() or rg:
        ora.select(rl, rg)
        ora.leader_pull(lamL, lamG, rl, rg)


@pytest.mark.parametrize("W,G,P,ld,mu,staggered", [
    (8, 2, 4099, 4160, 0.0, False),
    (12, 3, 2050, 2052, 0.9, True),
    (7, 3, 3003, 3003, 0.0, True),
])
def test_step_alg1_external_gradients(W, G, P, ld, mu, staggered):
    r = wl.stream("gpu_alg1", W, G, P)
    off = random_offsets(r, W, G) if W % G else wl.equal_group_offsets(W, G)
    x0, _, _ = wl.stress_state(W, P, ld, seed=W * 7 + G)
    pr = Pair(x0, off, P=P, momentum=mu)
    eta, tau, tauG = 0.05, 3, 6
    gamL, gamG, lamL, lamG = 0.1 / tau, 0.05 / tauG, 0.2, 0.1
    # initialisation: all leaders from the first losses, captured without moving anyone
    l0 = wl.stress_losses(W, 1000, seed=W + G)
    pr.ora.losses[:] = l0; pr.ora.select(); pr.ora.leader_pull(0.0, 0.0)
    pr.pop.select_leaders(dev(l0)); pr.pop.leader_pull(0.0, 0.0)
    for t in range(1, 14):
        g = wl.stress_grad(W, P, ld, t, seed=W)
        losses = wl.stress_losses(W, t, seed=W + G)
        pr.set_grad(g, losses)
        rl, rg = wl.refresh_masks(t, tau, G, staggered=staggered, tau_G=tauG)
        before = pr.follow_gpu()            # identical pre-iteration states: element-wise comparison
        alg1_oracle_iteration(pr.ora, eta, gamL, gamG, lamL, lamG, rl, rg)
        comm = (L.COMM_LOCAL if rl.any() else 0) | (L.COMM_GLOBAL if rg else 0)
        pr.pop.step_alg1(L.ExternalBatch(pr.losses_dev), eta, gamL, gamG, lamL, lamG, comm, rl)
        lead, gl = pr.pop.get_leaders()
        assert lead == pr.ora.lead.tolist() and gl == int(pr.ora.glead[0])
        # two or three chained fp32 updates per iteration (local step, local pull, global pull), each reading the
        # previous one's rounded result: a few ulps of the value itself
        pr.check_step_elementwise(before, f"iteration {t}", k_self=6.0)
        # copies are taken after the local step, whose result differs in its last bits between the two sides
        assert np.abs(pr.Z.cpu().numpy()[:, :P] - pr.ora.Z[:, :P]).max() <= 4 * np.finfo(np.float32).eps * np.abs(pr.ora.Z[:, :P]).max() + \
            16 * np.finfo(np.float32).eps * np.abs(pr.ora.x[:, :P] - before[0][:, :P]).max()


def test_step_alg1_matrix_completion():
    """Whole path: gradient kernels, small pulls, communication every tau iterations."""
    W, G = 8, 2
    prob = wl.mc_problem(600, 500, 32, 0.05, 32 ** -0.5, noise_std=0.01, seed=23)
    m, n, r, P = prob.m, prob.n, prob.r, prob.P
    ld = wl.padded_ld(P)
    x0 = wl.mc_init(W, prob, 32 ** -0.5, ld=ld, seed=3)
    rows, cols, vals = dev(prob.rows), dev(prob.cols), dev(prob.vals)
    B = 2048
    c = 0.5 * prob.n_obs / B
    idx = wl.mc_batches(W, B, prob.n_obs, 9, seed=5)      # [steps, W, B]
    big = L.MCBatch(m, n, r, rows, cols, vals, dev(idx[0]), c)
    pr = Pair(x0, wl.equal_group_offsets(W, G), P=P, largest_batch=big)
    eta, tau = 0.005, 4
    gamL, gamG, lamL, lamG = 0.02, 0.01, 0.3, 0.1
    pr.ora.grad_loss_mc(m, n, r, prob.rows, prob.cols, prob.vals, idx[0], c)
    pr.ora.select(); pr.ora.leader_pull(0.0, 0.0)
    pr.pop.grad_loss(big); pr.pop.select_leaders(); pr.pop.leader_pull(0.0, 0.0)
    assert pr.check_leaders()
    for t in range(1, 9):
        b = L.MCBatch(m, n, r, rows, cols, vals, dev(idx[t]), c)
        rl, rg = wl.refresh_masks(t, tau, G, tau_G=2 * tau)
        pr.ora.grad_loss_mc(m, n, r, prob.rows, prob.cols, prob.vals, idx[t], c)
        alg1_oracle_iteration(pr.ora, eta, gamL, gamG, lamL, lamG, rl, rg)
        comm = (L.COMM_LOCAL if rl.any() else 0) | (L.COMM_GLOBAL if rg else 0)
        pr.pop.step_alg1(b, eta, gamL, gamG, lamL, lamG, comm, rl)
        if not pr.check_leaders(rl, rg):
            pr.resync_from_oracle()
        pr.check_state(3e-4, f"iteration {t}")
        lo = np.array(pr.pop.get_losses())
        assert np.abs(lo - pr.ora.losses).max() <= 1e-4 * np.abs(pr.ora.losses).max()


@pytest.mark.parametrize("W,K", [(5, 1), (16, 10), (300, 64), (33, 3)])
def test_smooth_losses_bit_exact(W, K):
    x0 = np.zeros((W, 8), dtype=np.float32)
    G = 1 if W < 16 else 4
    off = wl.equal_group_offsets(W, G) if W % G == 0 else np.array([0, 7, 15, 20, W], dtype=np.int32)
    pr = Pair(x0, off)
    win_o = np.full((K, W), np.nan, dtype=np.float32)          # unfilled slots must never be read
    win_g = torch.full((K, W), float("nan"), device=DEV)
    out_o = np.zeros(W, dtype=np.float32)
    out_g = torch.zeros(W, device=DEV)
    for t in range(2 * K + 3):
        losses = (wl.stress_losses(W, t, seed=K) * np.float32(3.0) + np.float32(1e-3 * t)).astype(np.float32)
        oracle.smooth_losses(win_o, t, losses, out_o)
        if t % 2:
            pr.pop.smooth_losses(win_g, t, dev(losses), out_g)
            got = out_g
        else:                                                 # in place on the population's own buffer
            pr.pop.grad_loss(L.ExternalBatch(dev(losses)))
            pr.pop.smooth_losses(win_g, t)
            got = torch.tensor(pr.pop.get_losses())
        np.testing.assert_array_equal(got.cpu().numpy(), out_o)
        np.testing.assert_array_equal(win_g.cpu().numpy(), win_o)
        pr.ora.losses[:] = out_o
        pr.ora.select()
        pr.pop.select_leaders(dev(out_o) if t % 2 else None)
        lead, gl = pr.pop.get_leaders()
        assert lead == pr.ora.lead.tolist() and gl == int(pr.ora.glead[0])


@pytest.mark.parametrize("W,P,ld", [(1, 100, 100), (4, 1000, 1000), (16, 4099, 4160), (13, 5000, 5001), (70, 2051, 2052),
                                    (8, 300_001, 300_032)])
def test_center_bit_exact(W, P, ld):
    x0, _, _ = wl.stress_state(W, P, ld, x_std=1.0, seed=W + P)
    x0[:, :P] += np.float32(0.3)                                # a mean that does not cancel
    pr = Pair(x0, np.array([0, W], dtype=np.int32), P=P)
    out = torch.full((ld,), float("nan"), device=DEV)
    pr.pop.center(out)
    want = np.zeros(P, dtype=np.float32)
    oracle.center(pr.ora.x, P, want)
    got = out.cpu().numpy()
    np.testing.assert_array_equal(got[:P], want)
    assert np.isnan(got[P:]).all()                              # nothing written past P


def test_center_full_size_sampled_columns():
    """The matrix-completion headline shape; columns sampled across tiles and the tail."""
    W, P = 16, 4_194_304
    x = torch.empty((W, P), device=DEV).normal_(generator=torch.Generator(device=DEV).manual_seed(7))
    pop = L.Population(x, torch.zeros_like(x), 1, P=P)
    out = torch.empty(P, device=DEV)
    pop.center(out)
    cols = np.unique(np.concatenate([np.arange(0, 2048), np.arange(P - 2048, P),
                                     wl.stream("center_cols").integers(0, P, size=4096)]))
    xs = np.ascontiguousarray(x[:, torch.from_numpy(cols).to(DEV)].cpu().numpy())
    want = np.zeros(len(cols), dtype=np.float32)
    oracle.center(xs, len(cols), want)
    np.testing.assert_array_equal(out.cpu().numpy()[cols], want)
