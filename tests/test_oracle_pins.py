"""Pins for the CPU oracle: each test checks it against something the paper or
the mathematics fixes, not against itself.  CPU only."""
import os

import numpy as np
import pytest
import torch

import oracle
import workloads as wl

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def one_group(W):
    return np.array([0, W], dtype=np.int32)


# ----------------------------------------------------------------------------
# Leader selection: argmin definitions under Eq. 1 / Eq. 2
# ----------------------------------------------------------------------------
def brute_argmin(vals):
    """O(W^2): index i such that no j beats it and no lower j ties it."""
    v = [np.inf if np.isnan(a) else float(a) for a in vals]
    for i in range(len(v)):
        if all(v[i] <= v[j] for j in range(len(v))) and all(v[j] != v[i] for j in range(i)):
            return i
    raise AssertionError


@pytest.mark.parametrize("seed", range(20))
def test_select_matches_brute_force_and_sort(seed):
    r = wl.stream("sel_pin", seed)
    W = int(r.integers(1, 70))
    G = int(r.integers(1, min(W, 8) + 1))
    cuts = np.sort(r.choice(np.arange(1, W), size=G - 1, replace=False)) if G > 1 else np.array([], dtype=int)
    off = np.concatenate([[0], cuts, [W]]).astype(np.int32)
    losses = r.standard_normal(W).astype(np.float32)
    # adversarial values: ties, signed zeros, infinities, NaN
    pool = np.array([0.0, -0.0, np.inf, -np.inf, np.nan, 1.0, 1.0, -2.5], dtype=np.float32)
    k = int(r.integers(0, W + 1))
    pos = r.choice(W, size=k, replace=False)
    losses[pos] = pool[r.integers(0, len(pool), size=k)]
    lead = np.full(G, -1, dtype=np.int32)
    glead = np.full(1, -1, dtype=np.int32)
    oracle.select_leaders(losses, off, lead, glead)
    for j in range(G):
        seg = losses[off[j]:off[j + 1]]
        assert lead[j] == off[j] + brute_argmin(seg)
        # stable sort of (value, index) pairs gives the same winner
        key = np.where(np.isnan(seg), np.inf, seg).astype(np.float64)
        assert lead[j] == off[j] + int(np.argsort(key, kind="stable")[0])
    assert glead[0] == brute_argmin(losses)
    # Eq. 2: the global leader is the best worker among the local leaders
    best_local = min(lead, key=lambda i: (np.inf if np.isnan(losses[i]) else losses[i], i))
    assert glead[0] == best_local


def test_select_honours_refresh_mask():
    losses = np.array([3, 1, 2, 0.5, 9, 8], dtype=np.float32)
    off = np.array([0, 3, 6], dtype=np.int32)
    lead = np.array([2, 5], dtype=np.int32)
    glead = np.array([4], dtype=np.int32)
    oracle.select_leaders(losses, off, lead, glead, np.array([0, 1], dtype=np.uint8), 0)
    assert lead.tolist() == [2, 3] and glead[0] == 4
    oracle.select_leaders(losses, off, lead, glead, np.array([1, 0], dtype=np.uint8), 1)
    assert lead.tolist() == [1, 3] and glead[0] == 3


def test_gap_values_by_hand():
    """The relative gap (second best - best)/|best| that the parity tests use to recognise a near-tie, on
    losses whose gaps are known by hand.  Row G of the output is the global selection's gap."""
    f = lambda *v: np.array(v, dtype=np.float32)
    two = np.array([0, 2, 4], dtype=np.int32)

    def gaps(losses, off, rl=None, rg=1):
        G = len(off) - 1
        return oracle.select_leaders(losses, off, np.zeros(G, np.int32), np.zeros(1, np.int32), rl, rg)

    # plain positive losses: (3-2)/2 and (5-4)/4; globally (3-2)/2 again (best 2, second 3)
    np.testing.assert_allclose(gaps(f(2, 3, 5, 4), two), [0.5, 0.25, 0.5], rtol=1e-12)
    # negative best: (-1 - -2)/|-2| = 0.5, positive, not -0.5
    np.testing.assert_allclose(gaps(f(-2, -1, -8, 0), two), [0.5, 1.0, 0.75], rtol=1e-12)
    # exact ties (also -0 against +0) have gap 0
    assert gaps(f(1, 1, -0.0, 0.0), two)[:2].tolist() == [0.0, 0.0]
    # two losses one fp32 ulp apart: a near-tie far below the 1e-6 protocol threshold, but not zero
    a = np.float32(1.0); b = np.nextafter(a, np.float32(2.0))
    g = gaps(f(a, b, b, a), two)
    np.testing.assert_allclose(g[:2], [float(b) - 1.0, float(b) - 1.0], rtol=1e-12)
    assert 0.0 < g[0] < 1e-6 and g[2] == 0.0                    # globally, workers 0 and 3 tie exactly
    # 1e-7 apart on a larger scale
    np.testing.assert_allclose(gaps(f(100.0, 100.0 + 1e-5), one_group(2))[0], (float(np.float32(100.0 + 1e-5)) - 100.0) / 100.0, rtol=1e-12)
    # a single finite member (NaN counts as +inf): nobody is close, gap is infinite
    g = gaps(f(np.inf, 2, np.nan, 7), two)
    assert g[0] == np.inf and g[1] == np.inf and np.isclose(g[2], 2.5)
    # a group of infinities and NaN: every member ties
    assert gaps(f(np.inf, np.nan, np.nan, np.nan), two).tolist() == [0.0, 0.0, 0.0]
    # -inf best: |best| is infinite, a finite runner-up is infinitely far; two -inf tie
    g = gaps(f(-np.inf, 1, -np.inf, -np.inf), two, rg=0)
    assert g[0] == np.inf and g[1] == 0.0 and np.isnan(g[2])     # no global refresh: its gap is not reported
    # a group of one worker has no runner-up
    assert gaps(f(3), one_group(1)).tolist() == [np.inf, np.inf]
    assert gaps(f(np.nan), one_group(1)).tolist() == [0.0, 0.0]
    # best exactly zero: the denominator falls back to 1e-30, so any positive runner-up is far
    g = gaps(f(0, 1e-3), one_group(2))
    assert g[0] > 1e20
    # groups left out of a refresh report nothing
    g = gaps(f(2, 3, 5, 4), two, rl=np.array([0, 1], dtype=np.uint8), rg=0)
    assert np.isnan(g[0]) and g[1] == 0.25 and np.isnan(g[2])


# ----------------------------------------------------------------------------
# Update: reductions to SGD (Eq. 3 with zero pulls) against torch.optim.SGD
# ----------------------------------------------------------------------------
@pytest.mark.parametrize("mu,nesterov,wd,grad_only", [
    (0.0, False, 0.0, False), (0.9, False, 0.0, False), (0.9, True, 0.0, False),
    (0.9, True, 1e-4, False), (0.9, False, 1e-2, True), (0.5, True, 0.0, True)])
def test_zero_pull_is_per_worker_sgd(mu, nesterov, wd, grad_only):
    W, P = 5, 37
    r = wl.stream("sgd_pin", int(mu * 10), int(nesterov))
    x0 = r.standard_normal((W, P)).astype(np.float32)
    flags = (oracle.NESTEROV if nesterov else 0) | (oracle.MOMENTUM_GRAD_ONLY if grad_only else 0)
    pop = oracle.Population(x0, np.array([0, 2, 5], dtype=np.int32), momentum=mu, flags=flags, weight_decay=wd)
    pop.Z[:] = 1e6  # garbage: must not matter
    tx = torch.tensor(x0, dtype=torch.float64, requires_grad=True)
    opt = torch.optim.SGD([tx], lr=0.05, momentum=mu, nesterov=nesterov, weight_decay=wd)
    for t in range(4):
        g = r.standard_normal((W, P)).astype(np.float32)
        pop.g[:] = g
        pop.losses[:] = r.random(W, dtype=np.float32)
        pop.select()
        pop.update(0.05, 0.0, 0.0)
        tx.grad = torch.tensor(g, dtype=torch.float64)
        opt.step()
    np.testing.assert_allclose(pop.x, tx.detach().numpy(), rtol=2e-6, atol=2e-7)


@pytest.mark.parametrize("mu,nesterov,wd,grad_only", [
    (0.9, False, 0.0, False), (0.9, True, 0.0, False), (0.7, True, 1e-2, False),
    (0.9, False, 0.0, True), (0.5, True, 1e-2, True)])
def test_momentum_with_pulls_is_momentum_sgd_on_the_pulled_objective(mu, nesterov, wd, grad_only):
    """Heavy ball on the full direction is momentum-SGD applied to the objective of Eq. 2 with the leader
    copies held fixed: feed torch.optim.SGD the augmented gradient g + lam_L (x - z_L) + lam_G (x - z_G).
    With the pulls outside the buffer (grad-only mode) the optimizer sees g alone and the pulls, taken at the
    pre-update point, are a plain step beside it.  Leaders, copies and refresh periods are tracked here
    independently: refresh every 3 steps, global every 6, so stale copies (former leaders pulled to their own
    old parameters) are covered."""
    W, P = 6, 23
    off = np.array([0, 2, 6], dtype=np.int32)
    r = wl.stream("mom_pull_pin", int(mu * 10), int(nesterov), int(grad_only))
    x0 = r.standard_normal((W, P)).astype(np.float32)
    flags = (oracle.NESTEROV if nesterov else 0) | (oracle.MOMENTUM_GRAD_ONLY if grad_only else 0)
    pop = oracle.Population(x0, off, momentum=mu, flags=flags, weight_decay=wd)
    lr, lamL, lamG = 0.05, 0.3, 0.2
    e, lL, lG = (float(np.float32(v)) for v in (lr, lamL, lamG))
    tx = torch.tensor(x0, dtype=torch.float64, requires_grad=True)
    opt = torch.optim.SGD([tx], lr=e, momentum=float(np.float32(mu)), nesterov=nesterov, weight_decay=float(np.float32(wd)))
    zL = np.zeros((2, P)); zG = np.zeros(P)
    group = np.array([0, 0, 1, 1, 1, 1])
    for t in range(8):
        g = r.standard_normal((W, P)).astype(np.float32)
        losses = r.random(W, dtype=np.float32)
        rl = np.array([t % 3 == 0, t % 3 == 0], dtype=np.uint8)
        rg = int(t % 6 == 0)
        pop.g[:] = g; pop.losses[:] = losses
        pop.select(rl, rg); pop.update(lr, lamL, lamG, rl, rg)
        # independent bookkeeping of leaders and their kept copies
        xt = tx.detach().numpy().copy()
        if rl[0]:
            zL[0] = xt[int(np.argmin(losses[0:2]))]; zL[1] = xt[2 + int(np.argmin(losses[2:6]))]
        if rg:
            zG = xt[int(np.argmin(losses))].copy()
        pulls = lL * (xt - zL[group]) + lG * (xt - zG)
        if grad_only:
            tx.grad = torch.tensor(g, dtype=torch.float64)
            opt.step()
            with torch.no_grad():
                tx -= e * torch.tensor(pulls)
        else:
            tx.grad = torch.tensor(g + pulls, dtype=torch.float64)
            opt.step()
    np.testing.assert_allclose(pop.x, tx.detach().numpy(), rtol=2e-5, atol=2e-6)
    # the pulls did something: the same run without them ends elsewhere
    assert np.abs(pop.x - x0).max() > 0.1


def test_leader_row_takes_a_pure_gradient_step():
    """Supplement B.1: the update reduces to a (S)GD step for the leader."""
    W, P = 8, 50
    r = wl.stream("leader_pin")
    x0 = r.standard_normal((W, P)).astype(np.float32)
    off = np.array([0, 4, 8], dtype=np.int32)
    pop = oracle.Population(x0, off)
    pop.g[:] = r.standard_normal((W, P)).astype(np.float32)
    pop.losses[:] = np.array([5, 4, 1, 6, 0.5, 7, 8, 9], dtype=np.float32)
    pop.select()
    assert pop.lead.tolist() == [2, 4] and pop.glead[0] == 4
    pop.update(0.1, 0.3, 0.2)
    sgd = lambda i: (x0[i].astype(np.float64) - np.float32(0.1).astype(np.float64) * pop.g[i]).astype(np.float32)
    # global leader (also its group's leader): both pulls vanish, bit-exact SGD
    np.testing.assert_array_equal(pop.x[4], sgd(4))
    # local leader of group 0 feels only the global pull
    e, lg = float(np.float32(0.1)), float(np.float32(0.2))
    want = x0[2].astype(np.float64) - e * (pop.g[2] + lg * (x0[2].astype(np.float64) - x0[4]))
    np.testing.assert_allclose(pop.x[2], want, rtol=1e-6, atol=1e-7)
    # a follower moved towards its leaders relative to plain SGD
    assert np.linalg.norm(pop.x[0] - x0[2]) < np.linalg.norm(sgd(0) - x0[2])
    # snapshots are the pre-update leader rows
    np.testing.assert_array_equal(pop.Z[0], x0[2]); np.testing.assert_array_equal(pop.Z[2], x0[4])


def test_affine_form_of_the_update():
    """Matrix-completion supplement: X+ = (1 - eta*lam) X + eta*lam Z - eta*grad."""
    W, P = 6, 64
    r = wl.stream("affine_pin")
    x0 = r.standard_normal((W, P)).astype(np.float32)
    pop = oracle.Population(x0, one_group(W))
    pop.g[:] = r.standard_normal((W, P)).astype(np.float32)
    pop.losses[:] = r.random(W, dtype=np.float32)
    pop.select()
    z = x0[pop.lead[0]].astype(np.float64)
    eta, lam = float(np.float32(5e-4)), float(np.float32(0.2))
    want = (1 - eta * lam) * x0.astype(np.float64) + eta * lam * z - eta * pop.g.astype(np.float64)
    pop.update(5e-4, 0.2, 0.0)
    np.testing.assert_allclose(pop.x, want, rtol=1e-6, atol=1e-7)


def test_eq3_as_printed_leaves_pulls_unscaled():
    """Eq. 3: x - eta*g - lam*(x - z_local) - lam_G*(x - z_global)."""
    W, P = 4, 16
    r = wl.stream("eq3_pin")
    x0 = r.standard_normal((W, P)).astype(np.float32)
    pop = oracle.Population(x0, np.array([0, 2, 4], dtype=np.int32), flags=oracle.PULL_UNSCALED_BY_ETA)
    pop.g[:] = r.standard_normal((W, P)).astype(np.float32)
    pop.losses[:] = np.array([2, 1, 0.5, 3], dtype=np.float32)
    pop.select()
    e, l, lg = (float(np.float32(v)) for v in (0.1, 0.25, 0.125))
    zl = np.stack([x0[1], x0[1], x0[2], x0[2]]).astype(np.float64)
    xd = x0.astype(np.float64)
    want = xd - e * pop.g - l * (xd - zl) - lg * (xd - xd[2])
    pop.update(0.1, 0.25, 0.125)
    np.testing.assert_allclose(pop.x, want, rtol=2e-6, atol=1e-6)


def test_two_leaders_collapse_to_one_guiding_point():
    """Section 3: pulls (lam_i, z_i) equal one pull Lam = sum lam_i to z~ = sum lam_i z_i / Lam."""
    W, P = 4, 40
    r = wl.stream("collapse_pin")
    x0 = r.standard_normal((W, P)).astype(np.float32)
    g = r.standard_normal((W, P)).astype(np.float32)
    off = np.array([0, 2, 4], dtype=np.int32)
    zL = r.standard_normal((2, P)).astype(np.float32)
    zG = r.standard_normal(P).astype(np.float32)
    none = np.zeros(2, dtype=np.uint8)
    a = oracle.Population(x0, off)
    a.g[:] = g; a.Z[:2] = zL; a.Z[2] = zG
    a.update(0.05, 0.5, 0.25, refresh_local=none, refresh_global=0)
    # one leader per group at Lam = 0.75, z~_j = (0.5 zL_j + 0.25 zG) / 0.75 (kept in fp64 via two half-pulls)
    xd = x0.astype(np.float64)
    zt = (0.5 * zL.astype(np.float64) + 0.25 * zG.astype(np.float64)) / 0.75
    want = xd - float(np.float32(0.05)) * (g + 0.75 * (xd - np.repeat(zt, 2, axis=0)))
    np.testing.assert_allclose(a.x, want, rtol=1e-6, atol=1e-7)


def test_stationary_points_do_not_move():
    """Theorem (stationary points): zero gradient at a consensus point is a fixed point; a
    leader with zero gradient does not move whatever the others do."""
    W, P = 6, 33
    r = wl.stream("stat_pin")
    row = r.standard_normal(P).astype(np.float32)
    pop = oracle.Population(np.tile(row, (W, 1)), np.array([0, 3, 6], dtype=np.int32), momentum=0.9)
    pop.losses[:] = 1.0
    pop.select(); pop.update(0.1, 0.3, 0.2)
    np.testing.assert_array_equal(pop.x, np.tile(row, (W, 1)))
    assert pop.lead.tolist() == [0, 3] and pop.glead[0] == 0   # all tied: lowest index
    x0 = r.standard_normal((W, P)).astype(np.float32)
    pop = oracle.Population(x0, np.array([0, 3, 6], dtype=np.int32))
    pop.g[:] = r.standard_normal((W, P)).astype(np.float32); pop.g[1] = 0
    pop.losses[:] = np.array([3, 0, 2, 4, 5, 6], dtype=np.float32)
    pop.select(); pop.update(0.1, 0.3, 0.2)
    np.testing.assert_array_equal(pop.x[1], x0[1])
    assert not np.array_equal(pop.x[0], x0[0])


def test_fixed_leader_limit_on_a_diagonal_quadratic():
    """Section 3.1.2: with z held, the iterates converge to the minimiser w of
    f + lam/2 |x - z|^2; for f = 1/2 x'Ax, w = lam (A + lam I)^-1 z, and Theorem 2:
    f(w) - f* <= lam/(m + lam) (f(z) - f*)."""
    P = 24
    r = wl.stream("quad_pin")
    A = np.linspace(0.5, 8.0, P)
    z = r.standard_normal(P).astype(np.float32)
    x0 = r.standard_normal((3, P)).astype(np.float32) * 3
    pop = oracle.Population(x0, one_group(3))
    pop.Z[0] = z
    none = np.zeros(1, dtype=np.uint8)
    lam = 0.7
    for _ in range(4000):
        pop.g[:] = (A * pop.x.astype(np.float64)).astype(np.float32)
        pop.update(0.05, lam, 0.0, refresh_local=none, refresh_global=0)
    lamf = float(np.float32(lam))
    w = lamf * z.astype(np.float64) / (A + lamf)
    np.testing.assert_allclose(pop.x, np.tile(w, (3, 1)), rtol=0, atol=2e-6)
    f = lambda v: 0.5 * np.sum(A * v * v, axis=-1)
    assert f(pop.x[0].astype(np.float64)) <= lamf / (A.min() + lamf) * f(z.astype(np.float64)) + 1e-9
    np.testing.assert_array_equal(pop.Z[0], z)          # a kept leader copy is never rewritten


def test_leader_exempt_flag_and_monotone_leader_value():
    """Lemma 'leader_descent': with full gradients and eta < 2/M the leader's value at the
    start of each period is non-increasing (the leader takes pure gradient steps all period)."""
    P = 12
    r = wl.stream("mono_pin")
    A = np.linspace(1.0, 10.0, P)
    f = lambda v: 0.5 * np.sum(A * v.astype(np.float64) ** 2, axis=-1)
    x0 = (r.standard_normal((5, P)) * 2).astype(np.float32)
    pop = oracle.Population(x0, one_group(5), flags=oracle.LEADER_EXEMPT)
    tau, prev = 7, np.inf
    for t in range(70):
        pop.g[:] = (A * pop.x.astype(np.float64)).astype(np.float32)
        pop.losses[:] = f(pop.x).astype(np.float32)
        rl, rg = wl.refresh_masks(t, tau, 1)
        if rl[0]:
            pop.select(rl, rg)
            cur = float(f(pop.x[pop.lead[0]]))
            assert cur <= prev * (1 + 1e-6)
            prev = cur
        before = pop.x[pop.lead[0]].copy()
        pop.update(0.15, 0.5, 0.0, refresh_local=rl, refresh_global=rg)
        # exempt leader: pure gradient step even against a stale copy of itself
        want = (before.astype(np.float64) - float(np.float32(0.15)) * pop.g[pop.lead[0]].astype(np.float64)).astype(np.float32)
        np.testing.assert_array_equal(pop.x[pop.lead[0]], want)


def test_stale_leader_copy_is_used_between_refreshes():
    """Communication periods (supplement B.1): z changes only at the start of a period."""
    r = wl.stream("stale_pin")
    x0 = r.standard_normal((4, 10)).astype(np.float32)
    pop = oracle.Population(x0, np.array([0, 2, 4], dtype=np.int32))
    pop.losses[:] = np.array([1, 2, 0.5, 3], dtype=np.float32)
    pop.select(); pop.update(0.1, 0.2, 0.1)
    Z0 = pop.Z.copy()
    np.testing.assert_array_equal(Z0, x0[[0, 2, 2]])
    pop.losses[:] = np.array([9, 0, 9, 0.1], dtype=np.float32)     # would elect others
    x1 = pop.x.copy()
    none = np.zeros(2, dtype=np.uint8)
    pop.update(0.1, 0.2, 0.1, refresh_local=none, refresh_global=0)
    np.testing.assert_array_equal(pop.Z, Z0)
    e, l, lg = (float(np.float32(v)) for v in (0.1, 0.2, 0.1))
    xd = x1.astype(np.float64)
    want = xd - e * (l * (xd - Z0[[0, 0, 1, 1]]) + lg * (xd - Z0[2]))
    np.testing.assert_allclose(pop.x, want, rtol=1e-6, atol=1e-7)
    # staggered: only group 1 refreshes; group 0 keeps its copy, the global one is kept too
    pop.select(np.array([0, 1], dtype=np.uint8), 0)
    assert pop.lead.tolist() == [0, 3] and pop.glead[0] == 2
    x2 = pop.x.copy()
    pop.update(0.1, 0.2, 0.1, refresh_local=np.array([0, 1], dtype=np.uint8), refresh_global=0)
    np.testing.assert_array_equal(pop.Z[0], Z0[0]); np.testing.assert_array_equal(pop.Z[2], Z0[2])
    np.testing.assert_array_equal(pop.Z[1], x2[3])


# ----------------------------------------------------------------------------
# The paper's printed worked example
# ----------------------------------------------------------------------------
def _sinc(p):
    r = np.sqrt((p ** 2).sum(-1))
    return np.sin(np.pi * r) / (np.pi * r)


def _sinc_grad(p):
    r = np.sqrt((p ** 2).sum(-1, keepdims=True))
    u = np.pi * r
    return np.pi * (np.cos(u) * u - np.sin(u)) / u ** 2 * p / r


@pytest.mark.parametrize("flags", [0, oracle.PULL_UNSCALED_BY_ETA])
def test_sinc_example_reaches_the_printed_optimum(flags):
    with open(os.path.join(GOLD, "sinc_table1.txt")) as fh:
        gold = {ln.split()[0]: float(ln.split()[1]) for ln in fh if ln.strip() and not ln.startswith("#")}
    x0 = np.array([[-6, -4], [-15, -18], [20, 11], [17, 8]], dtype=np.float32)
    pop = oracle.Population(x0, one_group(4), flags=flags)
    for _ in range(3000):
        xd = pop.x.astype(np.float64)
        pop.g[:] = _sinc_grad(xd).astype(np.float32)
        pop.losses[:] = _sinc(xd).astype(np.float32)
        pop.select()
        pop.update(0.1, 0.1, 0.0)
    best = float(_sinc(pop.x.astype(np.float64)).min())
    assert abs(best - gold["LGD"]) < 5e-5
    # it is the global minimum of sin(u)/u: tan(u) = u at u = 4.4934..., value cos(u)
    u = 4.493409457909064
    assert abs(best - np.cos(u)) < 1e-6
    rbest = np.linalg.norm(pop.x[pop.lead[0]].astype(np.float64))
    assert abs(rbest - u / np.pi) < 1e-3


# ----------------------------------------------------------------------------
# Elastic averaging (the comparison method), as the supplement writes it beside LGD
# ----------------------------------------------------------------------------
@pytest.mark.parametrize("center0", ["mean", "origin"])
def test_sinc_example_eagd_reaches_its_printed_optimum(center0):
    """Table 1 of the supplement prints -0.0912 for EAGD with beta = 0.43.  beta is the moving rate of the
    center, p*eta*lam in the matrix-completion supplement's center update, so lam = beta/(p*eta) = 1.075.
    The run ends on the second ring of sin(u)/u (tan u = u at u = 10.9041, value cos u = -0.09132): every
    worker and the center.  The paper does not say where the center starts; the mean of the starts and the
    origin both end there."""
    with open(os.path.join(GOLD, "sinc_table1.txt")) as fh:
        gold = {ln.split()[0]: float(ln.split()[1]) for ln in fh if ln.strip() and not ln.startswith("#")}
    x0 = np.array([[-6, -4], [-15, -18], [20, 11], [17, 8]], dtype=np.float32)
    pop = oracle.Population(x0, one_group(4))
    center = x0.mean(0).astype(np.float32) if center0 == "mean" else np.full(2, 1e-6, dtype=np.float32)
    lam = 0.43 / (4 * 0.1)
    for _ in range(6000):
        pop.g[:] = _sinc_grad(pop.x.astype(np.float64)).astype(np.float32)
        pop.easgd_update(center, 0.1, lam)
    vals = _sinc(pop.x.astype(np.float64))
    u2 = 10.904121659428899
    assert abs(np.tan(u2) - u2) < 1e-9
    assert np.abs(vals - np.cos(u2)).max() < 1e-5 and abs(float(_sinc(center.astype(np.float64))) - np.cos(u2)) < 1e-5
    assert abs(vals.min() - gold["EAGD"]) < 2e-4            # printed to four digits, presumably short of full convergence
    # and it is NOT the global ring LGD reaches
    assert vals.min() > gold["LGD"] + 0.1


def test_eagd_formulas_and_conserved_sum():
    """X+ = (1 - eta lam) X + eta lam Xc - eta grad and Xc+ = (1 - p eta lam) Xc + p eta lam mean(X), both from
    pre-update values; with zero gradients the elastic forces are internal, so sum_i X^i + Xc is conserved."""
    W, P = 5, 31
    r = wl.stream("eagd_pin")
    x0 = r.standard_normal((W, P)).astype(np.float32)
    c0 = r.standard_normal(P).astype(np.float32)
    g = r.standard_normal((W, P)).astype(np.float32)
    pop = oracle.Population(x0, np.array([0, 2, 5], dtype=np.int32))
    pop.g[:] = g
    center = c0.copy()
    pop.easgd_update(center, 0.05, 0.3)
    e, l = float(np.float32(0.05)), float(np.float32(0.3))
    xd, cd = x0.astype(np.float64), c0.astype(np.float64)
    np.testing.assert_allclose(pop.x, (1 - e * l) * xd + e * l * cd - e * g, rtol=1e-6, atol=1e-7)
    np.testing.assert_allclose(center, (1 - W * e * l) * cd + W * e * l * xd.mean(0), rtol=1e-6, atol=1e-7)
    # conservation with zero gradients, over several steps
    pop = oracle.Population(x0, one_group(W)); center = c0.copy()
    total = x0.astype(np.float64).sum(0) + c0
    for _ in range(20):
        pop.easgd_update(center, 0.05, 0.3)
    np.testing.assert_allclose(pop.x.astype(np.float64).sum(0) + center, total, rtol=0, atol=2e-5)
    # and everyone has contracted towards the common point total/(W+1)
    assert np.abs(pop.x - total / (W + 1)).max() < np.abs(x0 - total / (W + 1)).max()


def test_eagd_spurious_stationary_point_of_the_supplement():
    """Supplement, stationary points of EASGD: for f with f'(x) = -exp(-x+1) (x >= 1), f'(x) = exp(x+1) (x <= -1)
    and 0 < lam <= 1 there is y >= 1 with lam*y + f'(y) = 0; then (-y, y, center 0) is stationary for EASGD
    although f'(+-y) != 0.  The elastic-averaging step must leave it where it is; the LSGD step from the same
    point (leader = either worker, equal losses) must not."""
    lam = 0.5
    y = 1.0
    for _ in range(200):                                    # Newton on lam*y - exp(1-y)
        y -= (lam * y - np.exp(1 - y)) / (lam + np.exp(1 - y))
    assert y >= 1 and abs(lam * y - np.exp(1 - y)) < 1e-14
    fp = lambda v: np.where(v >= 1, -np.exp(-v + 1), np.exp(v + 1))
    x0 = np.array([[-y], [y]], dtype=np.float32)
    pop = oracle.Population(x0, one_group(2))
    center = np.zeros(1, dtype=np.float32)
    for _ in range(50):
        pop.g[:] = fp(pop.x.astype(np.float64)).astype(np.float32)
        pop.easgd_update(center, 0.1, lam)
    np.testing.assert_allclose(pop.x, x0, rtol=0, atol=1e-5)
    assert abs(float(center[0])) < 1e-6 and abs(float(fp(np.float64(y)))) > 0.1
    lsgd = oracle.Population(x0, one_group(2))
    lsgd.g[:] = fp(x0.astype(np.float64)).astype(np.float32)
    lsgd.losses[:] = 0.0
    lsgd.select(); lsgd.update(0.1, lam, 0.0)
    assert abs(lsgd.x[0, 0] - x0[0, 0]) > 1e-2              # the leader takes a plain gradient step: it moves


# ----------------------------------------------------------------------------
# Matrix completion workload
# ----------------------------------------------------------------------------
def test_mc_gradient_reduces_to_dense_psd_formula():
    """Supplement: F(X) = 1/4 |M - XX'|_F^2 has grad F = (XX' - M) X.  With every entry
    observed, U = V = X and c = 1/4, dU + dV is that gradient and the loss is F."""
    d, r = 17, 3
    s = wl.stream("psd_pin")
    Ut = s.standard_normal((d, r)); M = (Ut @ Ut.T)
    X = s.standard_normal((d, r)).astype(np.float32)
    rows, cols = np.divmod(np.arange(d * d, dtype=np.int32), np.int32(d))
    rows = rows.astype(np.int32); cols = cols.astype(np.int32)
    vals = M.reshape(-1).astype(np.float32)
    x = np.concatenate([X.reshape(-1), X.reshape(-1)])[None, :].copy()
    g = np.zeros_like(x); losses = np.zeros(1, dtype=np.float32)
    oracle.mc_grad_loss(x, d, d, r, rows, cols, vals, None, 0.25, g, losses)
    Xd = X.astype(np.float64); Md = vals.astype(np.float64).reshape(d, d)
    want = (Xd @ Xd.T - Md) @ Xd
    # M is symmetric, so dU = dV = half the PSD gradient each
    np.testing.assert_allclose(g[0, :d * r].reshape(d, r) + g[0, d * r:].reshape(d, r), want, rtol=2e-6, atol=1e-6)
    np.testing.assert_allclose(g[0, :d * r], g[0, d * r:], rtol=2e-6, atol=1e-6)
    np.testing.assert_allclose(losses[0], 0.25 * np.sum((Md - Xd @ Xd.T) ** 2), rtol=1e-6)


def test_mc_gradient_rectangular_against_dense_matmul_and_duplicates():
    """Masked dense form: dU = 2c (E .* N) V, dV = 2c (E .* N)' U with N the multiplicity
    of each entry in the batch (duplicates count multiply)."""
    prob = wl.mc_problem(13, 9, 4, 0.6, 1.0, seed=7)
    W, B = 3, 50
    x = wl.mc_init(W, prob, 1.0, ld=wl.padded_ld(prob.P, 8), seed=7)
    idx = wl.mc_batches(W, B, prob.n_obs, 1, seed=7)[0]
    idx[:, :5] = idx[:, 5:10]                     # force duplicates
    g = np.full_like(x, 7.0); losses = np.zeros(W, dtype=np.float32)
    c = 0.5 * prob.n_obs / B
    oracle.mc_grad_loss(x, prob.m, prob.n, prob.r, prob.rows, prob.cols, prob.vals, idx, c, g, losses)
    for i in range(W):
        U = x[i, :prob.m * prob.r].reshape(prob.m, prob.r).astype(np.float64)
        V = x[i, prob.m * prob.r:prob.P].reshape(prob.n, prob.r).astype(np.float64)
        N = np.zeros((prob.m, prob.n)); Mv = np.zeros((prob.m, prob.n))
        for s_ in idx[i]:
            N[prob.rows[s_], prob.cols[s_]] += 1; Mv[prob.rows[s_], prob.cols[s_]] = prob.vals[s_]
        E = (U @ V.T - Mv) * N
        cf = float(np.float32(c))
        np.testing.assert_allclose(g[i, :prob.m * prob.r].reshape(prob.m, prob.r), 2 * cf * E @ V, rtol=1e-5, atol=1e-5)
        np.testing.assert_allclose(g[i, prob.m * prob.r:prob.P].reshape(prob.n, prob.r), 2 * cf * E.T @ U, rtol=1e-5, atol=1e-5)
        np.testing.assert_allclose(losses[i], cf * np.sum((U @ V.T - Mv) ** 2 * N), rtol=1e-6)
        assert np.all(g[i, prob.P:] == 0)


def test_mc_gradient_against_central_differences():
    prob = wl.mc_problem(6, 5, 2, 0.8, 1.0, seed=3)
    x = wl.mc_init(1, prob, 0.5, seed=3)
    x = (np.round(x * 64) / 64).astype(np.float32)       # exactly representable +- h
    g = np.zeros_like(x); l0 = np.zeros(1, dtype=np.float32)
    oracle.mc_grad_loss(x, prob.m, prob.n, prob.r, prob.rows, prob.cols, prob.vals, None, 0.5, g, l0)
    h = 1.0 / 64
    lp = np.zeros(1, dtype=np.float32); lm = np.zeros(1, dtype=np.float32); junk = np.zeros_like(x)
    for p in range(prob.P):
        xp = x.copy(); xp[0, p] += h
        xm = x.copy(); xm[0, p] -= h
        oracle.mc_grad_loss(xp, prob.m, prob.n, prob.r, prob.rows, prob.cols, prob.vals, None, 0.5, junk, lp)
        oracle.mc_grad_loss(xm, prob.m, prob.n, prob.r, prob.rows, prob.cols, prob.vals, None, 0.5, junk, lm)
        # the loss is quadratic in any single coordinate, so central differences are exact
        fd = (float(lp[0]) - float(lm[0])) / (2 * h)
        assert abs(fd - g[0, p]) <= 2e-4 * max(1.0, abs(g[0, p]))


def test_tiny_low_rank_matrix_is_recovered_by_lgd():
    """Motivating example: every local minimiser of low-rank completion is global, and LGD
    reaches one.  Full-batch LGD on a 100x100 rank-5 instance with 30% observed."""
    prob = wl.mc_problem(100, 100, 5, 0.30, 1.0, seed=11)
    W = 4
    pop = oracle.Population(wl.mc_init(W, prob, 1.0, seed=11), one_group(W))
    best = []
    for t in range(200):
        pop.grad_loss_mc(prob.m, prob.n, prob.r, prob.rows, prob.cols, prob.vals, None, 0.5)
        pop.select(); best.append(float(pop.losses.min()))
        pop.update(0.01, 0.1, 0.0)
    assert best[-1] < 1e-3 * best[0]
    i = int(pop.lead[0])
    U = pop.x[i, :500].reshape(100, 5).astype(np.float64); V = pop.x[i, 500:].reshape(100, 5).astype(np.float64)
    Mtrue = prob.U_true.astype(np.float64) @ prob.V_true.astype(np.float64).T
    mask = np.ones((100, 100), bool); mask[prob.rows, prob.cols] = False
    rel = np.linalg.norm((U @ V.T - Mtrue)[mask]) / np.linalg.norm(Mtrue[mask])
    assert rel < 0.05, rel


# ----------------------------------------------------------------------------
# MLP workload against an independent derivation: fp64 autograd with the same
# rounding points expressed through torch's own bf16 casts
# ----------------------------------------------------------------------------
class _RoundGrad(torch.autograd.Function):
    @staticmethod
    def forward(ctx, a):
        return a.clone()

    @staticmethod
    def backward(ctx, ga):
        return ga.to(torch.float32).to(torch.bfloat16).to(torch.float64)


def _rf(a):      # forward rounding, straight-through gradient
    return a + (a.detach().to(torch.float32).to(torch.bfloat16).to(torch.float64) - a.detach())


def _torch_mlp(xrow, dims, Xb, y):
    params, off = [], 0
    for k in range(len(dims) - 1):
        nw = dims[k + 1] * dims[k]
        Wk = torch.tensor(xrow[off:off + nw].reshape(dims[k + 1], dims[k]), dtype=torch.float64, requires_grad=True)
        bk = torch.tensor(xrow[off + nw:off + nw + dims[k + 1]], dtype=torch.float64, requires_grad=True)
        params += [Wk, bk]; off += nw + dims[k + 1]
    h = torch.tensor(wl.bf16_bits_to_f32(Xb), dtype=torch.float64)
    L = len(dims) - 1
    for k in range(L):
        z = h @ _rf(params[2 * k]).T + params[2 * k + 1]
        z = z.to(torch.float32).to(torch.float64)            # stored fp32
        z = _RoundGrad.apply(z)
        h = _rf(torch.relu(z)) if k + 1 < L else z
    loss = torch.nn.functional.cross_entropy(h, torch.tensor(y, dtype=torch.long))
    loss.backward()
    return float(loss.detach()), np.concatenate([p.grad.reshape(-1).numpy() for p in params])


@pytest.mark.parametrize("dims,B", [([12, 16, 5], 9), ([20, 24, 16, 8, 4], 13)])
def test_mlp_gradient_matches_fp64_autograd_with_same_rounding(dims, B):
    W = 2
    P = wl.mlp_param_count(dims)
    x = wl.mlp_init(W, dims, ld=wl.padded_ld(P, 8), seed=5, bias_std=0.1)
    means = wl.gmm_means(dims[0], dims[-1], seed=5)
    Xb, y = wl.gmm_batch(W, B, means, 0, seed=5)
    g = np.full_like(x, 3.0); losses = np.zeros(W, dtype=np.float32)
    oracle.mlp_grad_loss(x, dims, Xb, y, g, losses)
    for i in range(W):
        loss, grad = _torch_mlp(x[i], dims, Xb[i], y[i])
        np.testing.assert_allclose(losses[i], loss, rtol=1e-6)
        # a delta that lands on a bf16 rounding boundary may round either way: allow a
        # handful of elements at bf16 resolution, everything else to fp32 resolution
        err = np.abs(g[i, :P] - grad)
        tol = 1e-6 + 2e-6 * np.abs(grad)
        assert np.mean(err > tol) < 0.01, np.mean(err > tol)
        assert np.linalg.norm(err) <= 1e-4 * np.linalg.norm(grad)
        assert np.all(g[i, P:] == 0)


def test_mlp_first_layer_is_a_softmax_regression_closed_form():
    """One layer: dW = (softmax - onehot)' X / B, db = column sums; textbook softmax regression."""
    dims, B = [7, 4], 6
    x = wl.mlp_init(1, dims, seed=9, bias_std=0.2)
    means = wl.gmm_means(7, 4, seed=9)
    Xb, y = wl.gmm_batch(1, B, means, 0, seed=9)
    g = np.zeros_like(x); losses = np.zeros(1, dtype=np.float32)
    oracle.mlp_grad_loss(x, dims, Xb, y, g, losses)
    Wq = torch.tensor(x[0, :28].reshape(4, 7)).to(torch.bfloat16).to(torch.float64).numpy()
    Xd = wl.bf16_bits_to_f32(Xb[0]).astype(np.float64)
    z = (Xd @ Wq.T + x[0, 28:32]).astype(np.float32).astype(np.float64)
    p = np.exp(z - z.max(1, keepdims=True)); p /= p.sum(1, keepdims=True)
    d = p.copy(); d[np.arange(B), y[0]] -= 1; d /= B
    np.testing.assert_allclose(losses[0], -np.mean(np.log(p[np.arange(B), y[0]])), rtol=1e-6)
    np.testing.assert_allclose(g[0, :28].reshape(4, 7), d.T @ Xd, rtol=2e-2, atol=2e-3)   # delta is bf16-rounded
    dq = torch.tensor(d, dtype=torch.float32).to(torch.bfloat16).to(torch.float64).numpy()
    np.testing.assert_allclose(g[0, :28].reshape(4, 7), dq.T @ Xd, rtol=1e-6, atol=1e-7)
    np.testing.assert_allclose(g[0, 28:32], dq.sum(0), rtol=1e-6, atol=1e-7)


# ----------------------------------------------------------------------------
# Algorithm 1's communication pull, smoothed selection loss, center variable
# ----------------------------------------------------------------------------
def test_leader_pull_is_two_successive_interpolations():
    """Algorithm 1: x <- x - lam (x - x~^j), then x <- x - lam_G (x - x~); leaders' own pulls vanish."""
    r = wl.stream("alg1_pin")
    W, P = 6, 21
    x0 = r.standard_normal((W, P)).astype(np.float32)
    off = np.array([0, 3, 6], dtype=np.int32)
    pop = oracle.Population(x0, off)
    pop.losses[:] = np.array([3, 1, 2, 0.5, 4, 5], dtype=np.float32)
    pop.select()
    assert pop.lead.tolist() == [1, 3] and pop.glead[0] == 3
    pop.leader_pull(0.25, 0.125)
    lam, lg = float(np.float32(0.25)), float(np.float32(0.125))
    xd = x0.astype(np.float64)
    zl = xd[[1, 1, 1, 3, 3, 3]]
    y = xd - lam * (xd - zl)                      # phase 1 leaves both local leaders where they are
    np.testing.assert_array_equal(y[[1, 3]], xd[[1, 3]])
    want = y - lg * (y - xd[3])                   # phase 2 pulls to the (unmoved) global leader
    np.testing.assert_allclose(pop.x, want, rtol=1e-6, atol=1e-7)
    np.testing.assert_array_equal(pop.x[3], x0[3])          # the global leader does not move at all
    np.testing.assert_array_equal(pop.Z, x0[[1, 3, 3]])
    # lam = 1 puts every follower exactly on its leader; lam_G = 1 puts everybody on the global leader
    pop = oracle.Population(x0, off); pop.losses[:] = np.array([3, 1, 2, 0.5, 4, 5], dtype=np.float32); pop.select()
    pop.leader_pull(1.0, 0.0)
    np.testing.assert_array_equal(pop.x, x0[[1, 1, 1, 3, 3, 3]])
    pop.select(); pop.leader_pull(0.0, 1.0)
    np.testing.assert_array_equal(pop.x, np.tile(x0[3], (W, 1)))
    # only refreshed groups are pulled locally; without a global refresh there is no global pull
    pop = oracle.Population(x0, off); pop.losses[:] = np.array([3, 1, 2, 0.5, 4, 5], dtype=np.float32)
    m = np.array([0, 1], dtype=np.uint8)
    pop.select(m, 0); pop.leader_pull(0.5, 0.5, m, 0)
    np.testing.assert_array_equal(pop.x[:3], x0[:3])
    np.testing.assert_allclose(pop.x[3:], 0.5 * (xd[3:] + xd[3]), rtol=1e-6, atol=1e-7)


def test_smoothed_loss_is_the_mean_of_the_last_k_batches():
    r = wl.stream("smooth_pin")
    W, K = 5, 4
    window = np.zeros((K, W), dtype=np.float32)
    hist = []
    out = np.zeros(W, dtype=np.float32)
    for t in range(11):
        l = r.random(W, dtype=np.float32); hist.append(l)
        oracle.smooth_losses(window, t, l, out)
        np.testing.assert_allclose(out, np.mean(np.array(hist[-K:], dtype=np.float64), axis=0), rtol=1e-6)


def test_center_variable_is_the_column_mean():
    r = wl.stream("center_pin")
    x = r.standard_normal((7, 40)).astype(np.float32)
    out = np.zeros(33, dtype=np.float32)
    oracle.center(x, 33, out)
    np.testing.assert_allclose(out, x[:, :33].astype(np.float64).mean(0), rtol=1e-6, atol=1e-7)
