"""GPU parity: MLP gradients (MFMA and vector-ALU paths) and whole LSGD steps with momentum and the
bf16 shadow, against the CPU oracle."""
import numpy as np
import pytest
import torch

import oracle
import workloads as wl
import paper_1905_10395_amd as L
from gpu_util import DEV, Pair, dev, rel_l2_rows

pytestmark = pytest.mark.gpu


def make(dims, W, B, seed, momentum=0.0, flags=0, G=1, bias_std=0.05):
    P = wl.mlp_param_count(dims)
    ld = wl.padded_ld(P)
    x0 = wl.mlp_init(W, dims, ld=ld, seed=seed, bias_std=bias_std)
    means = wl.gmm_means(dims[0], dims[-1], seed=seed)
    Xb, y = wl.gmm_batch(W, B, means, 0, seed=seed)
    Xd = dev(Xb.view(np.int16)).view(torch.bfloat16)
    yd = dev(y)
    batch = L.MLPBatch(dims, Xd, yd)
    pr = Pair(x0, wl.equal_group_offsets(W, G), P=P, momentum=momentum, flags=flags, shadow=True, largest_batch=batch)
    return pr, batch, Xb, y, P, means


# Gradient tolerance.  Activations and deltas are quantised to bf16 (8 significant bits) and the ReLU mask is a
# sign decision; the GPU takes those decisions on fp32-accumulated sums, the oracle on fp64-accumulated ones, so
# a value that lies within fp32 rounding of a bf16 tie or of zero may legitimately fall the other way.  One such
# event moves one activation by one bf16 ulp (2^-8 relative) or switches one unit of one sample on or off, which
# shows as an isolated deviation in one worker.  Hence: the typical (median) worker must agree to 1e-4, and no
# worker may deviate by more than 2e-3 (half a bf16 ulp of the operands) in relative L2.
# With more than one quantised hidden layer a second mechanism appears.  The matrix cores' fp32 accumulation
# over K = 3072 leaves about 1e-4 of the first hidden layer's activations one bf16 ulp away from the oracle's.
# One such activation shifts all pre-activations of that sample in the next layer by ~1e-4, and a unit whose
# pre-activation lies that close to zero switches its ReLU mask.  Measured on 3072-512-512-10, batch 256: h_1
# differs in 13 of 131072 values (one ulp each), h_2 in 0.16 % (one ulp each), and exactly ONE unit of one sample
# has the opposite mask; that single back-propagated value (2.4x the rms) alone is 6.6e-3 of delta_2 in relative
# L2 and spreads to every earlier layer.  Both results are correct roundings of the same network; what is
# unique is the forward loss (agrees to 4e-7) and everything before the first switched mask.  Deep nets are
# therefore held to DEEP_TOL for every worker and block; parameters after a step still agree to 1e-4.
DEEP_TOL = 2e-2
GRAD_TOL_MEDIAN, GRAD_TOL_MAX = 1e-4, 2e-3


def per_layer_errors(g_gpu, g_ora, dims):
    """(median, max) over workers of the relative L2 error, per parameter block (W_k, b_k)"""
    med, mx, off = [], [], 0
    for k in range(len(dims) - 1):
        for n in (dims[k + 1] * dims[k], dims[k + 1]):
            e = rel_l2_rows(g_gpu[:, off:off + n], g_ora[:, off:off + n])
            med.append(np.median(e)); mx.append(e.max()); off += n
    return med, mx


def check_grads(g_gpu, g_ora, dims):
    med, mx = per_layer_errors(g_gpu, g_ora, dims)
    if len(dims) <= 3:                       # one quantised hidden layer
        assert max(med) < GRAD_TOL_MEDIAN, med
        assert max(mx) < GRAD_TOL_MAX, mx
    else:
        assert max(mx) < DEEP_TOL, mx


SHAPES = [
    ([12, 16, 5], 2, 9),                      # tiny, vector-ALU path everywhere
    ([20, 24, 16, 8, 4], 3, 13),              # 4 layers, ragged
    ([192, 256, 128, 10], 3, 128),            # MFMA 128x64 tiles: forward, d-input, d-weight
    ([512, 1024, 10], 8, 128),                # d-weight on 128x128 tiles
    ([64, 512, 256, 10], 64, 128),            # forward and d-input on 128x128 tiles
    ([128, 128, 10], 2, 256),                 # two M tiles, K = 256 for d-weight
    ([512, 1024, 10], 32, 128),               # d-weight on 256x256 tiles (8 wavefronts)
    ([64, 1024, 10], 64, 256),                # forward on 256x256 tiles
    ([64, 1024, 256, 10], 64, 256),           # forward and d-input on 256x256 tiles
    ([64, 512, 10], 64, 256),                 # forward on the 256x128 tile (whole batch per tile)
    ([64, 512, 128, 10], 64, 256),            # d-input on the 256x128 tile
]


@pytest.mark.parametrize("dims,W,B", SHAPES)
def test_mlp_grad_loss_matches_oracle(dims, W, B):
    pr, batch, Xb, y, P, _ = make(dims, W, B, seed=len(dims) * 100 + W)
    pr.g.fill_(7.0)
    pr.ora.grad_loss_mlp(dims, Xb, y)
    pr.pop.grad_loss(batch)
    torch.cuda.synchronize()
    g = pr.g.cpu().numpy()
    np.testing.assert_allclose(pr.pop.get_losses(), pr.ora.losses, rtol=1e-4)
    check_grads(g[:, :P], pr.ora.g[:, :P], dims)
    assert np.all(g[:, P:] == 0)


@pytest.mark.parametrize("dims,W,B", [([12, 16, 5], 2, 9), ([192, 256, 128, 10], 3, 128)])
def test_mlp_fp32_inputs_are_rounded_to_bf16_on_load(dims, W, B):
    """X given as fp32: h_0 = bf16(X), to nearest even, is the first rounding point of the forward pass.  The oracle
    gets the bits torch's CPU conversion produces; the GPU gets the fp32 values and must behave exactly as when it
    is handed those bits."""
    P = wl.mlp_param_count(dims)
    ld = wl.padded_ld(P)
    x0 = wl.mlp_init(W, dims, ld=ld, seed=77)
    Xb, y = wl.gmm_batch(W, B, wl.gmm_means(dims[0], dims[-1], seed=77), 0, seed=77)
    r = wl.stream("mlp_fp32_inputs", W, B)
    X32 = (Xb.view(np.uint16).astype(np.uint32) << 16).view(np.float32) * (1.0 + 3e-3 * r.standard_normal(Xb.shape, dtype=np.float32))
    bits = torch.from_numpy(X32).to(torch.bfloat16).view(torch.int16).numpy()
    assert (bits != Xb.view(np.int16)).any()                  # the perturbation crosses rounding boundaries
    b32 = L.MLPBatch(dims, dev(X32), dev(y))
    b16 = L.MLPBatch(dims, dev(bits).view(torch.bfloat16), dev(y))
    pr = Pair(x0, wl.equal_group_offsets(W, 1), P=P, shadow=True, largest_batch=b32)
    pr.ora.grad_loss_mlp(dims, bits.view(Xb.dtype), y)
    pr.pop.grad_loss(b32)
    torch.cuda.synchronize()
    g32 = pr.g.clone()
    l32 = pr.pop.get_losses()
    np.testing.assert_allclose(l32, pr.ora.losses, rtol=1e-4)
    check_grads(g32.cpu().numpy()[:, :P], pr.ora.g[:, :P], dims)
    pr.pop.grad_loss(b16)
    torch.cuda.synchronize()
    assert torch.equal(pr.g, g32) and pr.pop.get_losses() == l32
    # the bf16 copy lives in the workspace: a population sized for bf16 batches says so instead of overrunning it
    if L.workspace_bytes(W, P, ld, 1, batch=b32) > L.workspace_bytes(W, P, ld, 1, batch=b16):
        small = Pair(x0, wl.equal_group_offsets(W, 1), P=P, shadow=True, largest_batch=b16)
        with pytest.raises(L.LsgdError, match="workspace"):
            small.pop.grad_loss(b32)
    else:
        assert B * dims[0] * 2 < 256                          # only a copy that fits the rounding slack is free


def later_layer_wmax(x, dims):
    """largest |weight| of the layers that read a quantised activation (all but the first)"""
    off, w = dims[0] * dims[1] + dims[1], 0.0
    for k in range(1, len(dims) - 1):
        n = dims[k] * dims[k + 1]
        w = max(w, float(np.abs(x[:, off:off + n]).max()))
        off += n + dims[k + 1]
    return w


def margin_safe_batch(pr, dims, W, B, means, seed, oversample=4):
    """A batch made of the samples that are farthest from a ReLU mask switch.  The oracle's forward pass over
    oversample*B candidates per worker reports, per sample, the smallest |pre-activation| over all hidden units
    (a sample's pre-activations do not depend on which other samples share its batch); the B candidates with
    the largest such margin are kept.  Returns (X bits, y, smallest kept margin)."""
    Xc, yc = wl.gmm_batch(W, oversample * B, means, 900, seed=seed)
    margins = np.zeros((W, oversample * B), dtype=np.float32)
    pr.ora.grad_loss_mlp(dims, Xc, yc, margins)
    keep = np.sort(np.argsort(-margins, axis=1, kind="stable")[:, :B], axis=1)
    rows = np.arange(W)[:, None]
    return np.ascontiguousarray(Xc[rows, keep]), np.ascontiguousarray(yc[rows, keep]), float(margins[rows, keep].min())


DEEP_SHAPES = [(d, W, B) for d, W, B in SHAPES if len(d) > 3] + [
    ([3072, 512, 512, 10], 4, 256),           # K = 3072 first layer, then d-input at K = 512
    ([3072, 512, 512, 512, 10], 4, 256),      # the 4-layer configuration's depth at width 512
]


@pytest.mark.parametrize("dims,W,B", DEEP_SHAPES)
def test_deep_mlp_grads_tight_on_margin_safe_batches(dims, W, B):
    """Nets with several hidden layers held to the single-hidden-layer bar.  What separates the two sides on a
    deep net is a ReLU unit whose pre-activation lies so close to zero that an upstream activation differing by
    one bf16 ulp (2^-8 of a value of order one) times a weight flips its sign.  The batch is therefore built
    from samples the oracle certifies to be farther than that from any switch: every kept sample has
    min |z| >= 2^-8 * max|w| over all hidden units.  On such a batch both sides take the same mask decisions and
    what is left is the rounding of bf16 operands, as with one hidden layer: median worker 1e-4 (per
    requantisation of the deltas on their way back), every worker 2e-3 per parameter block.  Every deep-only code path (d-input products, transposed delta copies at
    K = hidden width, the 256x128 tile) is in these shapes."""
    pr, _, _, _, P, means = make(dims, W, B, seed=len(dims) * 100 + W)
    Xb, y, margin = margin_safe_batch(pr, dims, W, B, means, seed=len(dims) * 100 + W, oversample=6 if dims[0] > 1000 else 4)
    assert margin >= later_layer_wmax(pr.ora.x, dims) / 256.0, margin
    batch = L.MLPBatch(dims, dev(Xb.view(np.int16)).view(torch.bfloat16), dev(y))
    pr.g.fill_(7.0)
    pr.ora.grad_loss_mlp(dims, Xb, y)
    pr.pop.grad_loss(batch)
    torch.cuda.synchronize()
    g = pr.g.cpu().numpy()
    np.testing.assert_allclose(pr.pop.get_losses(), pr.ora.losses, rtol=1e-4)
    med, mx = per_layer_errors(g[:, :P], pr.ora.g[:, :P], dims)
    # each requantisation of the back-propagated deltas adds its own share of values that round to the other
    # bf16 neighbour (measured: 6e-5 median with two hidden layers, 1.2e-4 with three): 1e-4 per requantisation
    requant = max(1, len(dims) - 3)
    assert max(med) < GRAD_TOL_MEDIAN * requant, [float(f"{v:.2e}") for v in med]
    assert max(mx) < GRAD_TOL_MAX, [float(f"{v:.2e}") for v in mx]
    assert np.all(g[:, P:] == 0)


def check_m_like_gradient(pr, dims):
    """After one step from m = 0 the momentum buffer is the gradient plus the pulls: the gradient's bar."""
    P = pr.P
    med, mx = per_layer_errors(pr.m.cpu().numpy()[:, :P], pr.ora.m[:, :P], dims)
    assert max(med) < GRAD_TOL_MEDIAN, med
    assert max(mx) < GRAD_TOL_MAX, mx


def test_mlp_lsgd_steps_with_momentum_and_shadow():
    """16 workers in 4 groups, momentum 0.9, lam_L 0.1, lam_G 0.05, leaders every step; the bf16 operands
    of step t+1 come from the shadow written by the update of step t."""
    dims, W, G, B = [192, 256, 10], 16, 4, 128
    pr, _, _, _, P, means = make(dims, W, B, seed=77, momentum=0.9, flags=L.WRITE_BF16_SHADOW, G=G)
    steps = 12
    for t in range(steps):
        Xb, y = wl.gmm_batch(W, B, means, t, seed=77)
        batch = L.MLPBatch(dims, dev(Xb.view(np.int16)).view(torch.bfloat16), dev(y))
        pr.ora.grad_loss_mlp(dims, Xb, y)
        pr.ora.select(); pr.ora.update(0.01, 0.1, 0.05)
        pr.pop.step(batch, 0.01, 0.1, 0.05)
        if not pr.check_leaders():
            pr.resync_from_oracle()
        if t == 0:
            np.testing.assert_allclose(pr.pop.get_losses(), pr.ora.losses, rtol=1e-4)
            pr.check_state(1e-4, "step 0", tol_m=GRAD_TOL_MAX)
    np.testing.assert_allclose(pr.pop.get_losses(), pr.ora.losses, rtol=1e-3)
    pr.check_state(1e-3, f"after {steps} steps", tol_m=GRAD_TOL_MAX)
    # the shadow is exactly bf16(x) of the GPU's own master weights
    xb = pr.xb.view(torch.int16).cpu().numpy().view(np.uint16)
    assert np.array_equal(xb[:, :P], wl.to_bf16_bits(pr.x.cpu().numpy()[:, :P]))


def test_mlp_two_layer_config_full_size_one_step():
    """2-layer MLP 3072-1024-10, W=16 in 4 groups, batch 128, momentum 0.9, lam_L 0.1, lam_G 0.05: one whole
    step at full size against the oracle."""
    dims, W, G, B = [3072, 1024, 10], 16, 4, 128
    pr, batch, Xb, y, P, _ = make(dims, W, B, seed=3, momentum=0.9, flags=L.WRITE_BF16_SHADOW, G=G, bias_std=0.0)
    pr.ora.grad_loss_mlp(dims, Xb, y)
    pr.ora.select(); pr.ora.update(0.01, 0.1, 0.05)
    pr.pop.step(batch, 0.01, 0.1, 0.05)
    assert pr.check_leaders()
    np.testing.assert_allclose(pr.pop.get_losses(), pr.ora.losses, rtol=1e-4)
    check_grads(pr.g.cpu().numpy()[:, :P], pr.ora.g[:, :P], dims)
    # parameters to 1e-4; the momentum buffer after one step is the gradient plus pulls, so it
    # is held to the gradient's own bar (typical worker 1e-4, no worker beyond 2e-3), block by block
    pr.check_state(1e-4, "full-size step", tol_m=GRAD_TOL_MAX)
    check_m_like_gradient(pr, dims)


def test_mlp_four_layer_staggered_refresh_steps():
    """The 4-layer configuration at reduced width (3072-512-512-512-10 instead of hidden 4096, which the
    oracle cannot finish in seconds): W=8 in 2 groups of 4, batch 256, momentum 0.9, lam_L 0.1, lam_G 0.02,
    leaders kept for tau steps with the groups refreshing at staggered phases."""
    dims, W, G, B, tau = [3072, 512, 512, 512, 10], 8, 2, 256, 4
    pr, _, _, _, P, means = make(dims, W, B, seed=55, momentum=0.9, flags=L.WRITE_BF16_SHADOW, G=G, bias_std=0.0)
    steps = 7
    for t in range(steps):
        Xb, y = wl.gmm_batch(W, B, means, t, seed=55)
        batch = L.MLPBatch(dims, dev(Xb.view(np.int16)).view(torch.bfloat16), dev(y))
        rl, rg = wl.refresh_masks(t, tau, G, staggered=True)
        pr.ora.grad_loss_mlp(dims, Xb, y)
        pr.ora.select(rl, rg); pr.ora.update(0.01, 0.1, 0.02, rl, rg)
        pr.pop.step(batch, 0.01, 0.1, 0.02, rl, rg)
        if not pr.check_leaders(rl, rg):
            pr.resync_from_oracle()
        if t == 0:
            np.testing.assert_allclose(pr.pop.get_losses(), pr.ora.losses, rtol=1e-4)
            check_grads(pr.g.cpu().numpy()[:, :P], pr.ora.g[:, :P], dims)
            pr.check_state(1e-4, "step 0", tol_m=DEEP_TOL)
    np.testing.assert_allclose(pr.pop.get_losses(), pr.ora.losses, rtol=1e-3)
    pr.check_state(1e-3, f"after {steps} steps", tol_m=DEEP_TOL)


# ---------------------------------------------------------------------------
# Update applied inside the backward kernels (LSGD_FUSED_MLP_UPDATE): same oracle sequence
# (gradient, selection, update), the gradient never stored.
FUSED_CASES = [
    # dims, W, G, B, mu, flags, wd
    ([192, 256, 10], 16, 4, 128, 0.9, 0, 0.0),                                  # 128x64 MFMA tiles + narrow layer
    ([192, 256, 10], 16, 4, 128, 0.0, 0, 0.0),                                  # no momentum buffer
    ([192, 256, 10], 8, 2, 128, 0.9, L.NESTEROV, 1e-4),
    ([192, 256, 10], 8, 2, 128, 0.5, L.MOMENTUM_GRAD_ONLY | L.NESTEROV, 1e-3),
    ([192, 256, 10], 8, 2, 128, 0.9, L.LEADER_EXEMPT, 0.0),
    ([192, 256, 10], 8, 2, 128, 0.0, L.PULL_UNSCALED_BY_ETA, 0.0),
    ([100, 70, 10], 6, 3, 50, 0.9, 0, 0.0),                                     # vector-ALU kernels only
    ([512, 512, 10], 64, 8, 64, 0.9, 0, 0.0),                                   # 256x256 tiles
    ([256, 128, 128, 10], 8, 2, 64, 0.9, 0, 0.0),                               # two hidden layers
]


@pytest.mark.parametrize("dims,W,G,B,mu,flags,wd", FUSED_CASES)
def test_fused_update_steps(dims, W, G, B, mu, flags, wd):
    P = wl.mlp_param_count(dims)
    ld = wl.padded_ld(P)
    x0 = wl.mlp_init(W, dims, ld=ld, seed=91, bias_std=0.05)
    means = wl.gmm_means(dims[0], dims[-1], seed=91)
    Xb0, y0 = wl.gmm_batch(W, B, means, 0, seed=91)
    b0 = L.MLPBatch(dims, dev(Xb0.view(np.int16)).view(torch.bfloat16), dev(y0))
    pr = Pair(x0, wl.equal_group_offsets(W, G), P=P, momentum=mu, flags=flags | L.FUSED_MLP_UPDATE, weight_decay=wd,
              shadow=True, largest_batch=b0)
    pr.g.fill_(7.0)
    deep = len(dims) > 3
    eta, lamL, lamG, tau = 0.01, 0.1, 0.05, 3
    for t in range(6):
        Xb, y = wl.gmm_batch(W, B, means, t, seed=91)
        batch = L.MLPBatch(dims, dev(Xb.view(np.int16)).view(torch.bfloat16), dev(y))
        rl, rg = wl.refresh_masks(t, tau, G, staggered=True, tau_G=2 * tau)
        pr.ora.grad_loss_mlp(dims, Xb, y)
        pr.ora.select(rl, rg); pr.ora.update(eta, lamL, lamG, rl, rg)
        pr.pop.step(batch, eta, lamL, lamG, rl, rg)
        if not pr.check_leaders(rl, rg):
            pr.resync_from_oracle()
            pr.pop.sync_shadow()
        np.testing.assert_allclose(pr.pop.get_losses(), pr.ora.losses, rtol=1e-4 if t == 0 else 1e-3)
        # the momentum buffer carries the gradient's own tolerance (one switched ReLU unit per worker, see above);
        # from the second step on the two sides start from states up to 1e-3 apart, so allow a few such units
        pr.check_state(1e-4 if t == 0 else 1e-3, f"step {t}",
                       tol_m=DEEP_TOL if deep else (GRAD_TOL_MAX if t == 0 else 3 * GRAD_TOL_MAX))
        xb = pr.xb.view(torch.int16).cpu().numpy().view(np.uint16)
        assert np.array_equal(xb[:, :P], wl.to_bf16_bits(pr.x.cpu().numpy()[:, :P])), f"shadow at step {t}"
    # padding untouched, kept copies are the oracle's up to the state tolerance
    assert np.array_equal(pr.x.cpu().numpy()[:, P:], x0[:, P:])
    assert rel_l2_rows(pr.Z.cpu().numpy()[:, :P], pr.ora.Z[:, :P]).max() < 1e-3


def test_fused_update_equals_three_call_sequence():
    """Same population stepped with and without the fused flag: identical leaders, states equal up to the
    rounding order of the update expression."""
    dims, W, G, B = [192, 256, 10], 8, 2, 128
    P = wl.mlp_param_count(dims)
    ld = wl.padded_ld(P)
    x0 = wl.mlp_init(W, dims, ld=ld, seed=5, bias_std=0.05)
    means = wl.gmm_means(dims[0], dims[-1], seed=5)
    Xb, y = wl.gmm_batch(W, B, means, 0, seed=5)
    batch = L.MLPBatch(dims, dev(Xb.view(np.int16)).view(torch.bfloat16), dev(y))
    a = Pair(x0, wl.equal_group_offsets(W, G), P=P, momentum=0.9, flags=L.WRITE_BF16_SHADOW, shadow=True, largest_batch=batch)
    b = Pair(x0, wl.equal_group_offsets(W, G), P=P, momentum=0.9, flags=L.FUSED_MLP_UPDATE, shadow=True, largest_batch=batch)
    for t in range(3):
        a.pop.step(batch, 0.01, 0.1, 0.05)
        b.pop.step(batch, 0.01, 0.1, 0.05)
        assert a.pop.get_leaders() == b.pop.get_leaders()
        torch.cuda.synchronize()
        assert rel_l2_rows(b.x.cpu().numpy()[:, :P], a.x.cpu().numpy()[:, :P]).max() < 1e-6
        assert rel_l2_rows(b.m.cpu().numpy()[:, :P], a.m.cpu().numpy()[:, :P]).max() < 1e-5


def test_fused_update_needs_snapshot_buffer():
    dims, W, B = [64, 32, 10], 2, 16
    P = wl.mlp_param_count(dims)
    x0 = wl.mlp_init(W, dims, ld=wl.padded_ld(P), seed=1)
    means = wl.gmm_means(dims[0], dims[-1], seed=1)
    Xb, y = wl.gmm_batch(W, B, means, 0, seed=1)
    batch = L.MLPBatch(dims, dev(Xb.view(np.int16)).view(torch.bfloat16), dev(y))
    pr = Pair(x0, np.array([0, W], dtype=np.int32), P=P, flags=L.FUSED_MLP_UPDATE, shadow=True, snapshot=False, largest_batch=batch)
    before = pr.x.clone()
    with pytest.raises(L.LsgdError, match="z_snapshot"):
        pr.pop.step(batch, 0.01, 0.1, 0.0)
    torch.cuda.synchronize()
    assert torch.equal(before, pr.x)
    pr.pop.step(batch, 0.01, 0.0, 0.0)                      # plain SGD needs no leader copies


def test_fused_update_two_layer_config_full_size_one_step():
    dims, W, G, B = [3072, 1024, 10], 16, 4, 128
    pr, batch, Xb, y, P, _ = make(dims, W, B, seed=3, momentum=0.9, flags=L.FUSED_MLP_UPDATE, G=G, bias_std=0.0)
    pr.ora.grad_loss_mlp(dims, Xb, y)
    pr.ora.select(); pr.ora.update(0.01, 0.1, 0.05)
    pr.pop.step(batch, 0.01, 0.1, 0.05)
    assert pr.check_leaders()
    np.testing.assert_allclose(pr.pop.get_losses(), pr.ora.losses, rtol=1e-4)
    pr.check_state(1e-4, "full-size fused step", tol_m=GRAD_TOL_MAX)
    check_m_like_gradient(pr, dims)


def test_four_layer_config_full_size_two_workers_against_oracle():
    """3072-4096-4096-4096-10, W=8 in 2 groups of 4, batch 256, momentum 0.9, lam_L 0.1, lam_G 0.02 at full
    size on the GPU.  Gradients are independent per worker, so the oracle (64.5 GFLOP per worker) runs two of
    the eight workers, one from each group: their losses to 1e-4, their gradients per parameter block at the
    deep-net bar (this batch is the configuration's own, not selected for margins), and their rows after the
    whole fused step against the oracle's update fed the same leader rows."""
    dims, W, G, B = [3072, 4096, 4096, 4096, 10], 8, 2, 256
    P = wl.mlp_param_count(dims)
    ld = wl.padded_ld(P)
    gen = torch.Generator(device=DEV).manual_seed(17)
    x = torch.empty((W, ld), device=DEV)
    off = 0
    for k in range(len(dims) - 1):                          # U(+-fan_in^-1/2) weights, zero biases, as in the workload recipe
        n = dims[k + 1] * dims[k]
        x[:, off:off + n].uniform_(-dims[k] ** -0.5, dims[k] ** -0.5, generator=gen)
        x[:, off + n:off + n + dims[k + 1]] = 0
        off += n + dims[k + 1]
    x[:, P:] = 0
    means = wl.gmm_means(dims[0], dims[-1], seed=17)
    Xb, y = wl.gmm_batch(W, B, means, 0, seed=17)
    batch = L.MLPBatch(dims, dev(Xb.view(np.int16)).view(torch.bfloat16), dev(y))
    g = torch.zeros_like(x); m = torch.zeros_like(x)
    Z = torch.zeros((G + 1, ld), device=DEV)
    xb = torch.zeros((W, ld), dtype=torch.bfloat16, device=DEV)
    pop = L.Population(x, g, G, m=m, z_snapshot=Z, x_bf16=xb, P=P, momentum=0.9, flags=L.FUSED_MLP_UPDATE, largest_batch=batch)
    sample = [1, 6]
    x_old = x[sample].cpu().numpy()
    ora = oracle.Population(x_old, np.array([0, 1, 2], dtype=np.int32), momentum=0.9, P=P)
    ora.grad_loss_mlp(dims, np.ascontiguousarray(Xb[sample]), np.ascontiguousarray(y[sample]))
    # gradients and losses through the separate call
    pop.grad_loss(batch)
    losses = np.array(pop.get_losses())
    np.testing.assert_allclose(losses[sample], ora.losses, rtol=1e-4)
    med, mx = per_layer_errors(g[sample].cpu().numpy()[:, :P], ora.g[:, :P], dims)
    assert max(mx) < DEEP_TOL, mx
    assert torch.count_nonzero(g[:, P:]) == 0
    # the whole step with the update applied inside the backward kernels
    lead_want = [int(np.argmin(losses[0:4])), 4 + int(np.argmin(losses[4:8]))]
    gl_want = int(np.argmin(losses))
    z_rows = x[lead_want + [gl_want]].cpu().numpy()          # the leaders' parameters before the step
    pop.step(batch, 0.01, 0.1, 0.02)
    lead, gl = pop.get_leaders()
    assert lead == lead_want and gl == gl_want
    np.testing.assert_allclose(np.array(pop.get_losses())[sample], ora.losses, rtol=1e-4)
    ora.Z[:] = z_rows                                       # worker 1 pulls to Z[0] and Z[2], worker 6 to Z[1] and Z[2]
    ora.lead[:] = [-1, -1]; ora.glead[0] = -1               # (indices only matter to the leader-exempt flag)
    none = np.zeros(2, dtype=np.uint8)
    ora.update(0.01, 0.1, 0.02, none, 0)
    torch.cuda.synchronize()
    ex = rel_l2_rows(x[sample].cpu().numpy()[:, :P], ora.x[:, :P])
    assert ex.max() <= 1e-4, ex
    em = rel_l2_rows(m[sample].cpu().numpy()[:, :P], ora.m[:, :P])
    assert em.max() <= DEEP_TOL, em
    np.testing.assert_array_equal(Z.cpu().numpy()[:, :P], z_rows[:, :P])
    assert torch.equal(xb[:, :P], x[:, :P].to(torch.bfloat16))


def test_fused_update_four_layer_full_size_matches_three_call_step():
    """3072-4096-4096-4096-10, W=8 in 2 groups, batch 256: too large for the oracle (its parity case is the same
    network at width 512, above), so at full size the fused step is held against the three-call step of the same
    library in the launch shape the benchmark times: same leaders and losses, x within 1e-6, m within 1e-5."""
    dims, W, G, B = [3072, 4096, 4096, 4096, 10], 8, 2, 256
    P = wl.mlp_param_count(dims)
    ld = wl.padded_ld(P)
    gen = torch.Generator(device=DEV).manual_seed(11)
    x0 = torch.empty((W, ld), device=DEV)
    off = 0
    for k in range(len(dims) - 1):                          # U(+-fan_in^-1/2) weights, zero biases, as in the workload recipe
        n = dims[k + 1] * dims[k]
        x0[:, off:off + n].uniform_(-dims[k] ** -0.5, dims[k] ** -0.5, generator=gen)
        x0[:, off + n:off + n + dims[k + 1]] = 0
        off += n + dims[k + 1]
    x0[:, P:] = 0
    means = wl.gmm_means(dims[0], dims[-1], seed=11)
    Xb, y = wl.gmm_batch(W, B, means, 0, seed=11)
    batch = L.MLPBatch(dims, dev(Xb.view(np.int16)).view(torch.bfloat16), dev(y))
    pops = []
    for flags in (L.WRITE_BF16_SHADOW, L.FUSED_MLP_UPDATE):
        x = x0.clone(); g = torch.zeros_like(x); m = torch.zeros_like(x)
        Z = torch.zeros((G + 1, ld), device=DEV)
        xb = torch.zeros((W, ld), dtype=torch.bfloat16, device=DEV)
        pops.append((L.Population(x, g, G, m=m, z_snapshot=Z, x_bf16=xb, P=P, momentum=0.9, flags=flags, largest_batch=batch),
                     x, m, xb, g, Z))
    (pa, xa, ma, xba, _, _), (pb, xf, mf, xbf, _, _) = pops

    def rel(a, b):
        return max((torch.linalg.vector_norm((a[i, :P] - b[i, :P]).double()) / torch.linalg.vector_norm(b[i, :P].double())).item()
                   for i in range(W))

    # step 1 from identical states: same gradient bits, so only the rounding order of the update differs
    pa.step(batch, 0.01, 0.1, 0.02); pb.step(batch, 0.01, 0.1, 0.02)
    torch.cuda.synchronize()
    assert pa.get_leaders() == pb.get_leaders()
    np.testing.assert_allclose(pb.get_losses(), pa.get_losses(), rtol=1e-6)
    assert rel(xf, xa) < 1e-6 and rel(mf, ma) < 1e-5
    assert torch.equal(xbf[:, :P], xf[:, :P].to(torch.bfloat16))
    # step 2 (one group keeps its leader, the global leader is kept): the two x differ in their last bits, a few
    # bf16 weights round differently, and the gradients then differ like two correct roundings of a deep net do
    pa.step(batch, 0.01, 0.1, 0.02, [0, 1], 0); pb.step(batch, 0.01, 0.1, 0.02, [0, 1], 0)
    torch.cuda.synchronize()
    assert pa.get_leaders() == pb.get_leaders()
    np.testing.assert_allclose(pb.get_losses(), pa.get_losses(), rtol=1e-4)
    assert rel(xf, xa) < 1e-5 and rel(mf, ma) < DEEP_TOL
    assert torch.equal(xbf[:, :P], xf[:, :P].to(torch.bfloat16))
