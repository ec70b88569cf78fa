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
