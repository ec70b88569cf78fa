"""ctypes front for the CPU oracle (oracle/lsgd_oracle.c).  TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's CPU-baseline leg may import
this package.  It does not import, and is not imported by, the HIP library's
Python binding.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "lsgd_oracle.c")
_LIB = os.path.join(_HERE, "liblsgd_oracle.so")

NESTEROV = 1
LEADER_EXEMPT = 2
PULL_UNSCALED_BY_ETA = 4
MOMENTUM_GRAD_ONLY = 8


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (no FMA contraction, OpenMP over workers)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c99", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
               "-Wall", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.lsgd_oracle_bf16_round.restype = C.c_float
        _lib.lsgd_oracle_bf16_round.argtypes = [C.c_float]
    return _lib


def _p(a, ct):
    return None if a is None else a.ctypes.data_as(C.POINTER(ct))


def _f32(a):
    assert a.dtype == np.float32 and a.flags.c_contiguous
    return _p(a, C.c_float)


def _i32(a):
    assert a.dtype == np.int32 and a.flags.c_contiguous
    return _p(a, C.c_int32)


def _u8(a):
    if a is None:
        return None
    assert a.dtype == np.uint8 and a.flags.c_contiguous
    return _p(a, C.c_uint8)


def select_leaders(losses, off, lead, glead, refresh_local=None, refresh_global=1):
    """In place on lead[G] (int32) and glead[1] (int32); returns gaps[G+1] (nan = not refreshed)."""
    W = int(losses.shape[0])
    G = int(off.shape[0]) - 1
    gaps = np.full(G + 1, np.nan, dtype=np.float64)
    lib().lsgd_oracle_select_leaders(_f32(losses), C.c_int(W), C.c_int(G), _i32(off),
                                     _u8(refresh_local), C.c_int(int(refresh_global)),
                                     _i32(lead), _i32(glead), _p(gaps, C.c_double))
    return gaps


def pull_update(x, m, g, Z, P, off, lead, glead, eta, lam_L, lam_G, mu=0.0,
                refresh_local=None, refresh_global=1, flags=0, weight_decay=0.0):
    """In place on x, m (None if mu == 0), Z[(G+1), ld]."""
    W, ld = x.shape
    G = int(off.shape[0]) - 1
    assert Z.shape == (G + 1, ld) and g.shape == x.shape
    if mu != 0.0:
        assert m is not None and m.shape == x.shape
    lib().lsgd_oracle_pull_update(_f32(x), None if m is None else _f32(m), _f32(g), _f32(Z),
                                  C.c_int(W), C.c_int64(int(P)), C.c_int64(int(ld)), C.c_int(G), _i32(off),
                                  _i32(lead), C.c_int32(int(glead[0])), _u8(refresh_local),
                                  C.c_int(int(refresh_global)), C.c_float(eta), C.c_float(lam_L),
                                  C.c_float(lam_G), C.c_float(mu), C.c_int(int(flags)),
                                  C.c_float(weight_decay))


def leader_pull(x, Z, P, off, lead, glead, lam_L, lam_G, refresh_local=None, refresh_global=1):
    """Algorithm 1's communication pull, in place on x and Z[(G+1), ld]."""
    W, ld = x.shape
    G = int(off.shape[0]) - 1
    lib().lsgd_oracle_leader_pull(_f32(x), _f32(Z), C.c_int(W), C.c_int64(int(P)), C.c_int64(int(ld)), C.c_int(G), _i32(off),
                                  _i32(lead), C.c_int32(int(glead[0])), _u8(refresh_local), C.c_int(int(refresh_global)),
                                  C.c_float(lam_L), C.c_float(lam_G))


def smooth_losses(window, t, losses, out):
    """window: float32 [K, W] ring (in place); out: float32 [W]."""
    K, W = window.shape
    lib().lsgd_oracle_smooth_losses(_f32(window), C.c_int(K), C.c_int64(int(t)), _f32(losses), C.c_int(W), _f32(out))


def center(x, P, out):
    W, ld = x.shape
    lib().lsgd_oracle_center(_f32(x), C.c_int(W), C.c_int64(int(P)), C.c_int64(int(ld)), _f32(out))


def easgd_center(x, P, center, old_center, eta, lam):
    """Elastic-averaging center update from the workers' current (pre-update) parameters, in place on
    center[ld]; old_center[ld] receives the center as it was."""
    W, ld = x.shape
    lib().lsgd_oracle_easgd_center(_f32(x), C.c_int(W), C.c_int64(int(P)), C.c_int64(int(ld)), _f32(center), _f32(old_center),
                                   C.c_float(eta), C.c_float(lam))


def mc_grad_loss(x, m, n, r, rows, cols, vals, batch_idx, c, g, losses):
    """batch_idx: int32 [W,B] or None (every observed entry, for every worker)."""
    W, ld = x.shape
    B = 0 if batch_idx is None else int(batch_idx.shape[1])
    if batch_idx is not None:
        assert batch_idx.shape[0] == W
    lib().lsgd_oracle_mc_grad_loss(_f32(x), C.c_int(W), C.c_int64(int(ld)), C.c_int(m), C.c_int(n), C.c_int(r),
                                   _i32(rows), _i32(cols), _f32(vals), C.c_int64(int(rows.shape[0])),
                                   None if batch_idx is None else _i32(batch_idx), C.c_int64(B),
                                   C.c_float(c), _f32(g), _f32(losses))


def mlp_grad_loss(x, dims, X_bf16, y, g, losses, min_abs_preact=None):
    """X_bf16: uint16 [W,B,d0] bf16 bit patterns; y: int32 [W,B]; min_abs_preact: optional float32 [W,B] output,
    per sample the smallest |pre-activation| over all hidden units (distance from a ReLU mask switch)."""
    W, ld = x.shape
    dims = np.ascontiguousarray(dims, dtype=np.int32)
    B = int(y.shape[1])
    assert X_bf16.dtype == np.uint16 and X_bf16.shape == (W, B, int(dims[0])) and X_bf16.flags.c_contiguous
    lib().lsgd_oracle_mlp_grad_loss(_f32(x), C.c_int(W), C.c_int64(int(ld)), C.c_int(len(dims) - 1), _i32(dims),
                                    _p(X_bf16, C.c_uint16), _i32(y), C.c_int(B), _f32(g), _f32(losses),
                                    None if min_abs_preact is None else _f32(min_abs_preact))


class Population:
    """Oracle-side state of one population and the step that advances it.

    step(): gradient and loss at the current point on each worker's own batch,
    leaders from those losses, then every worker updated from pre-update values.
    """

    def __init__(self, x, off, momentum=0.0, flags=0, weight_decay=0.0, P=None):
        self.x = np.ascontiguousarray(x, dtype=np.float32).copy()
        self.W, self.ld = self.x.shape
        self.P = self.ld if P is None else int(P)
        self.off = np.ascontiguousarray(off, dtype=np.int32)
        self.G = len(self.off) - 1
        self.mu = float(momentum)
        self.flags = int(flags)
        self.wd = float(weight_decay)
        self.g = np.zeros_like(self.x)
        self.m = np.zeros_like(self.x) if self.mu != 0.0 else None
        self.Z = np.zeros((self.G + 1, self.ld), dtype=np.float32)
        self.losses = np.zeros(self.W, dtype=np.float32)
        self.lead = np.zeros(self.G, dtype=np.int32)
        self.glead = np.zeros(1, dtype=np.int32)
        self.gaps = np.full(self.G + 1, np.nan)

    def grad_loss_mc(self, prob_m, prob_n, r, rows, cols, vals, batch_idx, c):
        mc_grad_loss(self.x, prob_m, prob_n, r, rows, cols, vals, batch_idx, c, self.g, self.losses)

    def grad_loss_mlp(self, dims, X_bf16, y, min_abs_preact=None):
        mlp_grad_loss(self.x, dims, X_bf16, y, self.g, self.losses, min_abs_preact)

    def select(self, refresh_local=None, refresh_global=1):
        self.gaps = select_leaders(self.losses, self.off, self.lead, self.glead, refresh_local, refresh_global)

    def leader_pull(self, lam_L, lam_G, refresh_local=None, refresh_global=1):
        leader_pull(self.x, self.Z, self.P, self.off, self.lead, self.glead, lam_L, lam_G, refresh_local, refresh_global)

    def easgd_update(self, center, eta, lam):
        """Elastic averaging: center (float32 [ld], in place) moves towards the workers' mean, every worker
        takes the pulled step towards the center as it was (the global row of Z is used for it)."""
        easgd_center(self.x, self.P, center, self.Z[self.G], eta, lam)
        none = np.zeros(self.G, dtype=np.uint8)
        pull_update(self.x, self.m, self.g, self.Z, self.P, self.off, np.full(self.G, -1, np.int32), np.full(1, -1, np.int32),
                    eta, 0.0, lam, self.mu, none, 0, self.flags & ~LEADER_EXEMPT, self.wd)

    def update(self, eta, lam_L, lam_G, refresh_local=None, refresh_global=1):
        pull_update(self.x, self.m, self.g, self.Z, self.P, self.off, self.lead, self.glead,
                    eta, lam_L, lam_G, self.mu, refresh_local, refresh_global, self.flags, self.wd)
