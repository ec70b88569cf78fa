"""Helpers for the GPU parity tests: run the same seeded inputs through the HIP
library (via its C boundary) and through the CPU oracle, and compare."""
import numpy as np
import torch

import oracle
import paper_1905_10395_amd as L

DEV = "cuda:0"


def dev(a, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(a))
    if dtype is not None:
        t = t.to(dtype)
    return t.to(DEV)


EPS32 = float(np.finfo(np.float32).eps)


def assert_update_elementwise(new_gpu, new_ora, old, what="", k_self=2.0, k_row=16.0):
    """One update from identical pre-update values `old`: every element of the GPU result must equal the
    oracle's up to fp32 rounding of the update expression.  The oracle evaluates the expression in fp64 and
    rounds once; the GPU chains fp32 operations whose individual roundings are relative to the terms of the
    expression (which may cancel), so the bound per element is k_self ulps of the value itself plus k_row ulps
    of the largest displacement in its row.  A missing pull term, a wrong leader copy or a skipped element is
    orders of magnitude above this."""
    new_gpu = np.asarray(new_gpu, dtype=np.float64); new_ora = np.asarray(new_ora, dtype=np.float64)
    old = np.asarray(old, dtype=np.float64)
    disp = np.abs(new_ora - old)
    bound = k_self * EPS32 * np.abs(new_ora) + k_row * EPS32 * disp.max(axis=-1, keepdims=True) + 1e-37
    err = np.abs(new_gpu - new_ora)
    bad = err > bound
    if bad.any():
        i = np.unravel_index(np.argmax(err / bound), err.shape)
        raise AssertionError(f"{what}: {int(bad.sum())} elements beyond fp32 rounding; worst at {i}: gpu {new_gpu[i]!r} "
                             f"oracle {new_ora[i]!r} old {old[i]!r} err {err[i]:.3e} bound {bound[i]:.3e}")


def rel_l2_rows(a, b):
    """Per-row relative L2 error of a against b (b is the oracle)."""
    a = np.asarray(a, dtype=np.float64); b = np.asarray(b, dtype=np.float64)
    num = np.linalg.norm(a - b, axis=-1)
    den = np.maximum(np.linalg.norm(b, axis=-1), 1e-30)
    return num / den


class Pair:
    """One population on the GPU and its oracle twin, built from the same host arrays."""

    def __init__(self, x0, off, P=None, momentum=0.0, flags=0, weight_decay=0.0, snapshot=True,
                 shadow=False, largest_batch=None):
        W, ld = x0.shape
        self.W, self.ld = W, ld
        self.P = ld if P is None else P
        self.off = np.ascontiguousarray(off, dtype=np.int32)
        self.G = len(off) - 1
        self.ora = oracle.Population(x0, self.off, momentum=momentum, flags=flags & 15, weight_decay=weight_decay, P=self.P)
        self.x = dev(x0)
        self.g = torch.zeros_like(self.x)
        self.m = torch.zeros_like(self.x) if momentum != 0.0 else None
        self.Z = torch.full((self.G + 1, ld), float("nan"), device=DEV) if snapshot else None
        self.xb = torch.zeros((W, ld), dtype=torch.bfloat16, device=DEV) if shadow else None
        self.pop = L.Population(self.x, self.g, self.G, m=self.m, z_snapshot=self.Z, x_bf16=self.xb, P=self.P,
                                group_offsets=list(off), momentum=momentum, flags=flags, weight_decay=weight_decay,
                                largest_batch=largest_batch)

    def set_grad(self, g, losses):
        self.ora.g[:] = g; self.ora.losses[:] = losses
        self.g.copy_(dev(g))
        self.losses_dev = dev(losses)

    def check_leaders(self, rl=None, rg=1, gap_tol=1e-6):
        """Exact agreement, except where the oracle's own gap says it is a near-tie."""
        lead, gl = self.pop.get_leaders()
        ok = True
        for j in range(self.G):
            if (rl is None or rl[j]) and lead[j] != self.ora.lead[j]:
                assert self.ora.gaps[j] < gap_tol, (j, lead, self.ora.lead, self.ora.gaps)
                ok = False
        if rg and gl != self.ora.glead[0]:
            assert self.ora.gaps[self.G] < gap_tol, (gl, self.ora.glead, self.ora.gaps)
            ok = False
        return ok

    def follow_gpu(self):
        """Make the oracle's state the GPU's (x, m, kept copies), so that the next step on both sides starts
        from identical values and can be compared element by element; returns the pre-step (x, m)."""
        torch.cuda.synchronize()
        self.ora.x[:] = self.x.cpu().numpy()
        if self.m is not None:
            self.ora.m[:] = self.m.cpu().numpy()
        if self.Z is not None:
            Z = self.Z.cpu().numpy()
            ok = ~np.isnan(Z)
            self.ora.Z[ok] = Z[ok]
        return self.ora.x.copy(), (None if self.m is None else self.ora.m.copy())

    def check_step_elementwise(self, before, what="", k_self=2.0):
        """After one update from the state `before` = follow_gpu(): x and m element by element."""
        torch.cuda.synchronize()
        P = self.P
        x_old, m_old = before
        assert_update_elementwise(self.x.cpu().numpy()[:, :P], self.ora.x[:, :P], x_old[:, :P], f"{what} x", k_self=k_self)
        if self.m is not None:
            # m+ = mu m + d: the displacement scale of m is |m+| itself
            assert_update_elementwise(self.m.cpu().numpy()[:, :P], self.ora.m[:, :P], np.zeros_like(m_old[:, :P]), f"{what} m")
        if self.ld > P:
            assert np.array_equal(self.x.cpu().numpy()[:, P:], x_old[:, P:]), f"{what}: padding columns of x changed"

    def check_state(self, tol, what="", tol_m=None):
        torch.cuda.synchronize()
        P = self.P
        ex = rel_l2_rows(self.x.cpu().numpy()[:, :P], self.ora.x[:, :P])
        assert ex.max() <= tol, f"{what} x rel-L2 {ex.max():.3e} > {tol}"
        if self.m is not None:
            em = rel_l2_rows(self.m.cpu().numpy()[:, :P], self.ora.m[:, :P])
            tm = tol if tol_m is None else tol_m
            assert em.max() <= tm, f"{what} m rel-L2 {em.max():.3e} > {tm}"
        return ex.max()

    def resync_from_oracle(self):
        """Near-tie protocol: after a tolerated leader flip, continue from the oracle's state."""
        self.x.copy_(dev(self.ora.x))
        if self.m is not None:
            self.m.copy_(dev(self.ora.m))
        if self.Z is not None:
            self.Z.copy_(dev(self.ora.Z))
        if self.xb is not None:
            self.pop.sync_shadow()
