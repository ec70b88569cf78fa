"""GPU parity: leader selection and the fused pull update against the CPU oracle."""
import numpy as np
import pytest
import torch

import oracle
import workloads as wl
import paper_1905_10395_amd as L
from gpu_util import DEV, Pair, assert_update_elementwise, dev, rel_l2_rows

pytestmark = pytest.mark.gpu


def random_offsets(r, W, G):
    cuts = np.sort(r.choice(np.arange(1, W), size=G - 1, replace=False)) if G > 1 else np.array([], dtype=int)
    return np.concatenate([[0], cuts, [W]]).astype(np.int32)


# ---------------------------------------------------------------------------
@pytest.mark.parametrize("W,G", [(1, 1), (4, 1), (16, 4), (32, 4), (64, 7), (63, 5), (65, 3), (200, 9), (1000, 64)])
def test_select_leaders_bit_exact(W, G):
    r = wl.stream("gpu_sel", W, G)
    off = random_offsets(r, W, G)
    x0 = np.zeros((W, 8), dtype=np.float32)
    pr = Pair(x0, off)
    pool = np.array([0.0, -0.0, np.inf, -np.inf, np.nan, 1.0, 1.0, -2.5], dtype=np.float32)
    for trial in range(12):
        losses = r.standard_normal(W).astype(np.float32)
        if trial % 3 == 1:
            k = int(r.integers(1, W + 1)); pos = r.choice(W, size=k, replace=False)
            losses[pos] = pool[r.integers(0, len(pool), size=k)]
        if trial % 3 == 2:
            losses[:] = np.float32(r.choice(pool))          # everything tied (or all NaN / inf)
        rl = (r.random(G) < 0.6).astype(np.uint8) if trial % 2 else None
        rg = int(trial % 4 != 3)
        if trial == 0:
            rl, rg = None, 1
        pr.ora.losses[:] = losses
        pr.ora.select(rl, rg)
        pr.pop.select_leaders(dev(losses), rl, rg)
        lead, gl = pr.pop.get_leaders()
        assert lead == pr.ora.lead.tolist(), (trial, losses, off)
        assert gl == int(pr.ora.glead[0])


# ---------------------------------------------------------------------------
CASES = [
    # W, G, P, ld, mu, flags, wd
    (4, 1, 1000, 1000, 0.0, 0, 0.0),
    (16, 4, 4099, 4160, 0.9, 0, 0.0),                       # ragged P, padded rows
    (32, 4, 70001, 70004, 0.9, L.NESTEROV, 1e-4),
    (8, 2, 5000, 5001, 0.9, 0, 0.0),                        # ld % 4 != 0: scalar path
    (7, 3, 3003, 3004, 0.5, L.MOMENTUM_GRAD_ONLY, 0.0),     # unequal groups
    (7, 3, 3003, 3004, 0.5, L.MOMENTUM_GRAD_ONLY | L.NESTEROV, 1e-3),
    (12, 3, 2048, 2048, 0.0, L.PULL_UNSCALED_BY_ETA, 0.0),
    (12, 3, 2050, 2052, 0.9, L.LEADER_EXEMPT, 0.0),
    (5, 5, 515, 516, 0.9, 0, 0.0),                          # every worker its own group
    (70, 6, 1030, 1032, 0.9, 0, 0.0),                       # W > 64
    (6, 2, 2_500_003, 2_500_032, 0.9, 0, 0.0),              # several column chunks, ragged last chunk and tail
    (5, 2, 1_100_000, 1_100_000, 0.0, 0, 0.0),              # unequal groups across a chunk boundary
]


@pytest.mark.parametrize("W,G,P,ld,mu,flags,wd", CASES)
def test_pull_update_one_step_and_stale_periods(W, G, P, ld, mu, flags, wd):
    """Every step is compared element by element: before it, the oracle takes over the GPU's state (x, m, kept
    copies), so both sides update identical values and only fp32 rounding of the expression may differ."""
    r = wl.stream("gpu_pull", W, G, P)
    off = random_offsets(r, W, G) if W % G else wl.equal_group_offsets(W, G)
    x0, g0, _ = wl.stress_state(W, P, ld, seed=W * 1000 + G)
    pr = Pair(x0, off, P=P, momentum=mu, flags=flags, weight_decay=wd)
    eta, lamL, lamG = 0.05, 0.1, 0.05
    tau = 3
    for t in range(7):
        g = wl.stress_grad(W, P, ld, t, seed=W)
        losses = wl.stress_losses(W, t, seed=W + G)
        pr.set_grad(g, losses)
        rl, rg = wl.refresh_masks(t, tau, G, staggered=(G > 1), tau_G=2 * tau)
        before = pr.follow_gpu()
        pr.ora.select(rl, rg); pr.ora.update(eta, lamL, lamG, rl, rg)
        pr.pop.select_leaders(pr.losses_dev, rl, rg)
        pr.pop.pull_update(eta, lamL, lamG)
        lead, gl = pr.pop.get_leaders()
        assert lead == pr.ora.lead.tolist() and gl == int(pr.ora.glead[0])
        pr.check_step_elementwise(before, f"step {t}")
        # kept leader copies are pure copies of rows of identical states
        np.testing.assert_array_equal(pr.Z.cpu().numpy()[:, :P], pr.ora.Z[:, :P])


@pytest.mark.parametrize("W,G,P,ld,mu,flags,wd", CASES[:4] + CASES[6:8])
def test_pull_update_drift_over_steps(W, G, P, ld, mu, flags, wd):
    """The same schedule with each side keeping its own state: per-row relative L2 after several fp32 steps."""
    off = wl.equal_group_offsets(W, G)
    x0, g0, _ = wl.stress_state(W, P, ld, seed=W * 1000 + G)
    pr = Pair(x0, off, P=P, momentum=mu, flags=flags, weight_decay=wd)
    for t in range(7):
        pr.set_grad(wl.stress_grad(W, P, ld, t, seed=W), wl.stress_losses(W, t, seed=W + G))
        rl, rg = wl.refresh_masks(t, 3, G, staggered=(G > 1), tau_G=6)
        pr.ora.select(rl, rg); pr.ora.update(0.05, 0.1, 0.05, rl, rg)
        pr.pop.select_leaders(pr.losses_dev, rl, rg)
        pr.pop.pull_update(0.05, 0.1, 0.05)
        assert pr.check_leaders(rl, rg)
        pr.check_state(1e-6 if t == 0 else 1e-5, f"step {t}")
    assert rel_l2_rows(pr.Z.cpu().numpy()[:, :P], pr.ora.Z[:, :P]).max() < 1e-5
    if ld > P:
        assert np.array_equal(pr.x.cpu().numpy()[:, P:], x0[:, P:])


KEPT_LEADER_CASES = [(0.0, 0), (0.9, 0), (0.9, L.NESTEROV), (0.5, L.MOMENTUM_GRAD_ONLY), (0.0, L.PULL_UNSCALED_BY_ETA),
                     (0.9, L.LEADER_EXEMPT)]


@pytest.mark.parametrize("mu,flags", KEPT_LEADER_CASES)
@pytest.mark.parametrize("P,ld", [(4099, 4160), (3001, 3001)])
def test_fresh_global_leader_is_kept_local_leader(mu, flags, P, ld):
    """Step 0 refreshes everything (leaders 0 and 3, global 3).  Step 1 re-selects group 0 and the global
    leader while group 1 keeps worker 3: the global leader is then also the *kept* leader of its own group,
    and its local pull goes to the copy of itself taken at step 0 (leader copies change only at the start of a
    period: Section 3.1.2, supplement B.1), not to its current row."""
    W, G = 4, 2
    off = wl.equal_group_offsets(W, G)
    x0, _, _ = wl.stress_state(W, P, ld, seed=41)
    pr = Pair(x0, off, P=P, momentum=mu, flags=flags)
    eta, lamL, lamG = 0.05, 0.1, 0.05
    sched = [(np.array([0.5, 0.9, 0.8, 0.1], np.float32), np.array([1, 1], np.uint8), 1),
             (np.array([0.6, 0.4, 0.9, 0.2], np.float32), np.array([1, 0], np.uint8), 1),
             (np.array([0.3, 0.4, 0.1, 0.2], np.float32), np.array([0, 0], np.uint8), 1),   # global moves to 2, group 1 keeps 3
             (np.array([0.3, 0.4, 0.5, 0.2], np.float32), np.array([0, 0], np.uint8), 1)]   # global back to 3, still kept locally
    want = [([0, 3], 3), ([1, 3], 3), ([1, 3], 2), ([1, 3], 3)]
    for t, (losses, rl, rg) in enumerate(sched):
        pr.set_grad(wl.stress_grad(W, P, ld, t, seed=41), losses)
        before = pr.follow_gpu()
        pr.ora.select(rl, rg); pr.ora.update(eta, lamL, lamG, rl, rg)
        pr.pop.select_leaders(pr.losses_dev, rl, rg)
        pr.pop.pull_update(eta, lamL, lamG)
        lead, gl = pr.pop.get_leaders()
        assert (lead, gl) == want[t] == (pr.ora.lead.tolist(), int(pr.ora.glead[0]))
        pr.check_step_elementwise(before, f"step {t}")
        np.testing.assert_array_equal(pr.Z.cpu().numpy()[:, :P], pr.ora.Z[:, :P])


def test_in_place_equals_out_of_place_bitwise():
    """The leader rows are read by every other row's update while being updated themselves:
    capturing them first must make the in-place result identical to one computed from copies."""
    W, G, P = 16, 4, 9001
    ld = wl.padded_ld(P, 4)
    x0, g0, _ = wl.stress_state(W, P, ld, seed=3)
    losses = wl.stress_losses(W, 0, seed=3)
    off = wl.equal_group_offsets(W, G)
    a = Pair(x0, off, P=P, momentum=0.9)
    a.set_grad(g0, losses)
    a.pop.select_leaders(a.losses_dev); a.pop.pull_update(0.1, 0.3, 0.2)
    lead, gl = a.pop.get_leaders()
    # second population: same inputs, but leaders supplied as kept copies (no aliasing with x)
    b = Pair(x0, off, P=P, momentum=0.9)
    b.set_grad(g0, losses)
    b.pop.select_leaders(b.losses_dev); b.pop.pull_update(0.0, 0.0, 0.0)     # consumes the refresh, moves nothing
    b.m.zero_()
    Z = np.concatenate([x0[lead], x0[[gl]]]); b.Z.copy_(dev(Z))
    with pytest.raises(L.LsgdError):           # copies were never captured (coefficients were zero)
        b.pop.pull_update(0.1, 0.3, 0.2)
    c = Pair(x0, off, P=P, momentum=0.9)
    c.set_grad(g0, losses)
    c.pop.select_leaders(c.losses_dev); c.pop.pull_update(0.0, 1e-30, 1e-30)  # captures copies, moves nothing
    c.x.copy_(dev(x0)); c.m.zero_()
    c.pop.pull_update(0.1, 0.3, 0.2)
    torch.cuda.synchronize()
    assert torch.equal(a.x, c.x) and torch.equal(a.m, c.m)


def test_state_errors_and_no_side_effects():
    W, P = 4, 64
    x0, g0, _ = wl.stress_state(W, P, P, seed=1)
    pr = Pair(x0, wl.equal_group_offsets(W, 2), P=P, snapshot=False)
    with pytest.raises(L.LsgdError, match="STATE"):
        pr.pop.pull_update(0.1, 0.1, 0.0)                  # nothing selected yet
    pr.set_grad(g0, wl.stress_losses(W, 0))
    pr.pop.select_leaders(pr.losses_dev)
    pr.pop.pull_update(0.1, 0.1, 0.1)                      # fine: full refresh, no kept copies needed
    with pytest.raises(L.LsgdError, match="z_snapshot"):
        pr.pop.pull_update(0.1, 0.1, 0.1)                  # stale step without a snapshot buffer
    with pytest.raises(L.LsgdError, match="finite"):
        pr.pop.pull_update(float("nan"), 0.1, 0.1)
    before = pr.x.clone()
    with pytest.raises(L.LsgdError):
        pr.pop.step(L.ExternalBatch(pr.losses_dev), 0.1, 0.1, 0.1, [0, 0], 0)
    torch.cuda.synchronize()
    assert torch.equal(before, pr.x)
    pr.pop.pull_update(0.1, 0.0, 0.0)                      # zero pulls never need leaders


def test_zero_pulls_is_sgd_on_gpu():
    W, P = 6, 777
    ld = 780
    x0, g0, _ = wl.stress_state(W, P, ld, seed=5)
    pr = Pair(x0, wl.equal_group_offsets(W, 3), P=P, momentum=0.9, flags=L.NESTEROV, snapshot=False)
    tx = torch.tensor(x0[:, :P], dtype=torch.float64, requires_grad=True)
    opt = torch.optim.SGD([tx], lr=0.05, momentum=0.9, nesterov=True)
    for t in range(3):
        g = wl.stress_grad(W, P, ld, t, seed=5)
        pr.set_grad(g, wl.stress_losses(W, t))
        pr.pop.pull_update(0.05, 0.0, 0.0)
        tx.grad = torch.tensor(g[:, :P], dtype=torch.float64); opt.step()
    torch.cuda.synchronize()
    assert rel_l2_rows(pr.x.cpu().numpy()[:, :P], tx.detach().numpy()).max() < 1e-6


def test_hundred_steps_external_quadratic():
    """100 fp32 steps with leader flips: diagonal quadratic, gradient computed on the host from
    the GPU's own iterates would hide drift, so both sides get the gradient of their own state."""
    W, G, P = 8, 2, 4096
    r = wl.stream("gpu_quad")
    A = np.linspace(0.5, 4.0, P).astype(np.float32)
    x0 = (r.standard_normal((W, P)) * 2).astype(np.float32)
    pr = Pair(x0, wl.equal_group_offsets(W, G), momentum=0.9)
    Ad = dev(A)
    flips = 0
    for t in range(100):
        # oracle side
        xo = pr.ora.x.astype(np.float64)
        pr.ora.g[:] = (A * xo).astype(np.float32)
        pr.ora.losses[:] = (0.5 * np.sum(A * xo * xo, axis=1)).astype(np.float32)
        # GPU side: gradient of its own state (torch elementwise, caller-supplied gradient)
        pr.g.copy_(Ad * pr.x)
        losses_dev = (0.5 * (Ad.double() * pr.x.double() * pr.x.double()).sum(1)).float()
        rl, rg = wl.refresh_masks(t, 4, G)
        pr.ora.select(rl, rg); pr.ora.update(0.05, 0.1, 0.05, rl, rg)
        pr.pop.select_leaders(losses_dev, rl, rg); pr.pop.pull_update(0.05, 0.1, 0.05)
        if not pr.check_leaders(rl, rg):
            flips += 1; pr.resync_from_oracle()
    pr.check_state(1e-3, "after 100 steps")
    assert flips <= 2


def test_full_size_stress_sampled_columns():
    """W=32 x P=11,689,512 in 4 groups of 8, momentum 0.9, in the launch configuration the benchmark times.
    The update is independent per column, so the oracle recomputes a sample of column blocks (first, last
    ragged one, chunk boundaries, random ones) from the same pre-update values."""
    W, G, P = 32, 4, 11_689_512
    ld = wl.padded_ld(P)
    gen = torch.Generator(device=DEV); gen.manual_seed(1234)
    x = torch.randn((W, ld), device=DEV, generator=gen) * 0.05
    g = torch.randn((W, ld), device=DEV, generator=gen) * 1e-2
    m = torch.randn((W, ld), device=DEV, generator=gen) * 1e-2
    pop = L.Population(x, g, G, m=m, P=P, momentum=0.9)
    r = wl.stream("full_stress")
    starts = [0, 1024 * 1024 - 512, 4 * 1024 * 1024 - 100, P - 1000] + [int(v) for v in r.integers(0, P - 2048, size=24)]
    cols = np.unique(np.concatenate([np.arange(s0, min(s0 + 1024, P)) for s0 in starts]))
    ct = torch.from_numpy(cols).to(DEV)
    off = wl.equal_group_offsets(W, G)
    pad_before = x[:, P:].clone()
    for t in range(2):
        # both sides update the same pre-step values of the sampled columns
        x_old = x[:, ct].cpu().numpy(); m_old = m[:, ct].cpu().numpy()
        ora = oracle.Population(x_old, off, momentum=0.9)
        ora.m[:] = m_old
        losses = wl.stress_losses(W, t, seed=99)
        ora.g[:] = g[:, ct].cpu().numpy(); ora.losses[:] = losses
        ora.select(); ora.update(0.01, 0.1, 0.05)
        pop.select_leaders(dev(losses)); pop.pull_update(0.01, 0.1, 0.05)
        lead, gl = pop.get_leaders()
        assert lead == ora.lead.tolist() and gl == int(ora.glead[0])
        assert_update_elementwise(x[:, ct].cpu().numpy(), ora.x, x_old, f"step {t} x")
        assert_update_elementwise(m[:, ct].cpu().numpy(), ora.m, np.zeros_like(m_old), f"step {t} m")
    # columns outside [0, P) were not touched
    assert torch.equal(x[:, P:], pad_before)
