"""Seeded synthetic inputs for the batched LSGD step.

This module only *draws inputs* (matrices, index lists, batches, initial
points, refresh masks).  It contains none of the method's arithmetic: no
gradients, no losses, no leader selection, no updates.  Both the CPU oracle's
tests and the HIP path's tests feed on the same bytes produced here.

Shapes follow the paper's workloads: low-rank Gaussian factors for matrix
completion (supplement, "Low-Rank Matrix Completion Experiments"), 3x32x32
= 3072-dimensional 10-class inputs in batches of 128 (supplement, "Data
preprocessing"), and n groups of l workers (Eq. 2).
"""
from __future__ import annotations

import zlib
from dataclasses import dataclass

import numpy as np

MASTER_SEED = 190510395


def stream(purpose: str, *ids: int, seed: int = MASTER_SEED) -> np.random.Generator:
    """Independent counter-based (Philox) stream keyed by (seed, purpose, ids)."""
    tag = zlib.crc32(purpose.encode())
    ss = np.random.SeedSequence([int(seed), int(tag), *[int(i) for i in ids]])
    return np.random.Generator(np.random.Philox(ss))


def padded_ld(P: int, align: int = 64) -> int:
    """Row stride (in floats) that keeps every row 256-byte aligned."""
    return (int(P) + align - 1) // align * align


def equal_group_offsets(W: int, G: int) -> np.ndarray:
    assert W % G == 0
    return (np.arange(G + 1, dtype=np.int32) * (W // G)).astype(np.int32)


def to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """fp32 -> bf16 bit patterns (round to nearest even), used to store inputs."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


# --------------------------------------------------------------------------
# Matrix completion
# --------------------------------------------------------------------------
@dataclass
class MCProblem:
    m: int
    n: int
    r: int
    rows: np.ndarray   # int32 [n_obs]
    cols: np.ndarray   # int32 [n_obs]
    vals: np.ndarray   # fp32  [n_obs]
    U_true: np.ndarray  # fp32 [m, r]
    V_true: np.ndarray  # fp32 [n, r]

    @property
    def n_obs(self) -> int:
        return int(self.rows.shape[0])

    @property
    def P(self) -> int:
        return (self.m + self.n) * self.r


def mc_problem(m: int, n: int, r: int, frac: float, factor_std: float,
               noise_std: float = 0.0, seed: int = MASTER_SEED) -> MCProblem:
    """M = U V^T observed on floor(frac*m*n) distinct uniform entries (+ noise)."""
    g = stream("mc_factors", m, n, r, seed=seed)
    U = (g.standard_normal((m, r)) * factor_std).astype(np.float32)
    V = (g.standard_normal((n, r)) * factor_std).astype(np.float32)
    n_obs = int(np.floor(frac * m * n))
    go = stream("mc_omega", m, n, seed=seed)
    total = m * n
    if n_obs * 4 >= total:
        flat = go.permutation(total)[:n_obs]
    else:
        # oversample with replacement, keep the first n_obs distinct draws
        have = np.empty(0, dtype=np.int64)
        while have.shape[0] < n_obs:
            draw = go.integers(0, total, size=int((n_obs - have.shape[0]) * 1.1) + 16)
            cat = np.concatenate([have, draw])
            _, first = np.unique(cat, return_index=True)
            have = cat[np.sort(first)]
        flat = have[:n_obs]
    rows = (flat // n).astype(np.int32)
    cols = (flat % n).astype(np.int32)
    vals = np.einsum("kr,kr->k", U[rows].astype(np.float64), V[cols].astype(np.float64))
    if noise_std > 0:
        vals = vals + stream("mc_noise", m, n, seed=seed).standard_normal(n_obs) * noise_std
    return MCProblem(m, n, r, rows, cols, vals.astype(np.float32), U, V)


def mc_init(W: int, prob: MCProblem, std: float, ld: int | None = None,
            seed: int = MASTER_SEED) -> np.ndarray:
    """Per-worker start [U_i (m*r) | V_i (n*r)], entries N(0, std^2); pad = 0."""
    P = prob.P
    ld = P if ld is None else ld
    x = np.zeros((W, ld), dtype=np.float32)
    for i in range(W):
        x[i, :P] = (stream("mc_init", i, seed=seed).standard_normal(P) * std).astype(np.float32)
    return x


def mc_batches(W: int, B: int, n_obs: int, steps: int, seed: int = MASTER_SEED) -> np.ndarray:
    """int32 [steps, W, B]: i.i.d. uniform draws with replacement from the observed list."""
    out = np.empty((steps, W, B), dtype=np.int32)
    for t in range(steps):
        out[t] = stream("mc_batch", t, seed=seed).integers(0, n_obs, size=(W, B), dtype=np.int32)
    return out


# --------------------------------------------------------------------------
# Gaussian-mixture classification batches + MLP starts
# --------------------------------------------------------------------------
def mlp_param_count(dims) -> int:
    return int(sum(dims[k + 1] * dims[k] + dims[k + 1] for k in range(len(dims) - 1)))


def gmm_means(d: int, classes: int, seed: int = MASTER_SEED) -> np.ndarray:
    return stream("gmm_means", d, classes, seed=seed).standard_normal((classes, d)).astype(np.float32)


def gmm_batch(W: int, B: int, means: np.ndarray, step: int, seed: int = MASTER_SEED):
    """X: bf16 bit patterns uint16 [W,B,d]; y: int32 [W,B].  x = mean[y] + N(0, I)."""
    classes, d = means.shape
    g = stream("gmm_batch", step, seed=seed)
    y = g.integers(0, classes, size=(W, B), dtype=np.int32)
    X = means[y] + g.standard_normal((W, B, d), dtype=np.float32)
    return to_bf16_bits(X), y


def mlp_init(W: int, dims, ld: int | None = None, seed: int = MASTER_SEED,
             bias_std: float = 0.0) -> np.ndarray:
    """Row = [W_1 (out x in, row-major) | b_1 | W_2 | b_2 ...]; W_k ~ U(+-fan_in^-1/2)."""
    P = mlp_param_count(dims)
    ld = P if ld is None else ld
    x = np.zeros((W, ld), dtype=np.float32)
    for i in range(W):
        g = stream("mlp_init", i, seed=seed)
        off = 0
        for k in range(len(dims) - 1):
            fin, fout = dims[k], dims[k + 1]
            a = fin ** -0.5
            x[i, off:off + fin * fout] = g.uniform(-a, a, size=fin * fout).astype(np.float32)
            off += fin * fout
            if bias_std > 0:
                x[i, off:off + fout] = (g.standard_normal(fout) * bias_std).astype(np.float32)
            off += fout
    return x


# --------------------------------------------------------------------------
# Pull-update stress tensors
# --------------------------------------------------------------------------
def stress_state(W: int, P: int, ld: int | None = None, x_std: float = 0.05,
                 g_std: float = 1e-2, seed: int = MASTER_SEED):
    """x ~ N(0, x_std^2), g ~ N(0, g_std^2), m = 0; padding columns are zero."""
    ld = P if ld is None else ld
    x = np.zeros((W, ld), dtype=np.float32)
    g = np.zeros((W, ld), dtype=np.float32)
    for i in range(W):
        s = stream("stress", i, seed=seed)
        x[i, :P] = s.standard_normal(P, dtype=np.float32) * np.float32(x_std)
        g[i, :P] = s.standard_normal(P, dtype=np.float32) * np.float32(g_std)
    m = np.zeros((W, ld), dtype=np.float32)
    return x, g, m


def stress_grad(W: int, P: int, ld: int, step: int, g_std: float = 1e-2,
                seed: int = MASTER_SEED) -> np.ndarray:
    g = np.zeros((W, ld), dtype=np.float32)
    for i in range(W):
        s = stream("stress_grad", i, step, seed=seed)
        g[i, :P] = s.standard_normal(P, dtype=np.float32) * np.float32(g_std)
    return g


def stress_losses(W: int, step: int, seed: int = MASTER_SEED) -> np.ndarray:
    return stream("stress_loss", step, seed=seed).random(W, dtype=np.float32)


# --------------------------------------------------------------------------
# Refresh masks (caller policy: which leaders are re-selected at step t)
# --------------------------------------------------------------------------
def refresh_masks(t: int, tau: int, G: int, staggered: bool = False, tau_G: int | None = None):
    """(uint8[G] local mask, int global flag) for lock-step workers.

    Synchronous: every group refreshes when t % tau == 0.  Staggered: group j
    refreshes when (t - floor(j*tau/G)) % tau == 0.  The global leader is
    refreshed when t % tau_G == 0 (tau_G defaults to tau).  Step 0 refreshes
    everything (the algorithm's initialisation picks all leaders).
    """
    tau_G = tau if tau_G is None else tau_G
    mask = np.zeros(G, dtype=np.uint8)
    if t == 0:
        mask[:] = 1
        return mask, 1
    for j in range(G):
        phase = (j * tau) // G if staggered else 0
        mask[j] = 1 if (t - phase) % tau == 0 else 0
    return mask, int(t % tau_G == 0)
