"""ctypes marshalling for include/lsgd.h.  Same names as the C entry points:
lsgd_create_population, lsgd_grad_loss, lsgd_select_leaders, lsgd_pull_update,
lsgd_step (+ helpers).  No arithmetic of the method happens in Python."""
from __future__ import annotations

import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))

NESTEROV = 1
LEADER_EXEMPT = 2
PULL_UNSCALED_BY_ETA = 4
MOMENTUM_GRAD_ONLY = 8
WRITE_BF16_SHADOW = 16
FUSED_MLP_UPDATE = 32
COMM_LOCAL = 1
COMM_GLOBAL = 2

BATCH_EXTERNAL, BATCH_MC, BATCH_MLP = 0, 1, 2

_STATUS = {0: "OK", 1: "INVALID_ARG", 2: "SHAPE", 3: "STATE", 4: "UNSUPPORTED", 5: "HIP", 6: "NOMEM"}


class LsgdError(RuntimeError):
    def __init__(self, status, msg):
        super().__init__(f"LSGD_ERR_{_STATUS.get(status, status)}: {msg}")
        self.status = status


class _Config(C.Structure):
    _fields_ = [("W", C.c_int32), ("P", C.c_int64), ("ld", C.c_int64), ("n_groups", C.c_int32),
                ("group_offsets", C.POINTER(C.c_int32)), ("momentum", C.c_float), ("flags", C.c_int32),
                ("weight_decay", C.c_float)]


class _External(C.Structure):
    _fields_ = [("losses", C.c_void_p)]


class _MC(C.Structure):
    _fields_ = [("m", C.c_int32), ("n", C.c_int32), ("r", C.c_int32), ("rows", C.c_void_p), ("cols", C.c_void_p),
                ("vals", C.c_void_p), ("n_obs", C.c_int64), ("batch_idx", C.c_void_p), ("B", C.c_int64),
                ("c", C.c_float), ("entries", C.c_void_p)]


class _MLP(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("dims", C.POINTER(C.c_int32)), ("X", C.c_void_p), ("y", C.c_void_p),
                ("B", C.c_int32), ("x_is_fp32", C.c_int32)]


class _Batch(C.Structure):
    _fields_ = [("kind", C.c_int32), ("desc", C.c_void_p)]


def lib_path() -> str:
    return os.path.join(_HERE, "liblsgd.so")


_lib = None


def lib():
    """Loads liblsgd.so; raises if it has not been built (there is no fallback)."""
    global _lib
    if _lib is None:
        path = lib_path()
        if not os.path.exists(path):
            raise ImportError(f"{path} is missing: run `python -m paper_1905_10395_amd.build` "
                              "(or __graft_entry__.build()) first")
        L = C.CDLL(path)
        L.lsgd_last_error.restype = C.c_char_p
        L.lsgd_workspace_bytes.restype = C.c_size_t
        L.lsgd_workspace_bytes.argtypes = [C.POINTER(_Config), C.POINTER(_Batch)]
        L.lsgd_create_population.argtypes = [C.POINTER(_Config), C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                             C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p, C.POINTER(C.c_void_p)]
        L.lsgd_destroy_population.argtypes = [C.c_void_p]
        L.lsgd_grad_loss.argtypes = [C.c_void_p, C.POINTER(_Batch), C.c_void_p]
        L.lsgd_select_leaders.argtypes = [C.c_void_p, C.c_void_p, C.POINTER(C.c_uint8), C.c_int]
        L.lsgd_pull_update.argtypes = [C.c_void_p, C.c_float, C.c_float, C.c_float]
        L.lsgd_step.argtypes = [C.c_void_p, C.POINTER(_Batch), C.c_float, C.c_float, C.c_float,
                                C.POINTER(C.c_uint8), C.c_int]
        L.lsgd_leader_pull.argtypes = [C.c_void_p, C.c_float, C.c_float]
        L.lsgd_step_alg1.argtypes = [C.c_void_p, C.POINTER(_Batch), C.c_float, C.c_float, C.c_float, C.c_float, C.c_float,
                                     C.c_int, C.POINTER(C.c_uint8)]
        L.lsgd_smooth_losses.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int64, C.c_void_p, C.c_void_p]
        L.lsgd_center.argtypes = [C.c_void_p, C.c_void_p]
        L.lsgd_easgd_update.argtypes = [C.c_void_p, C.c_void_p, C.c_float, C.c_float]
        L.lsgd_easgd_step.argtypes = [C.c_void_p, C.POINTER(_Batch), C.c_void_p, C.c_float, C.c_float]
        L.lsgd_sync_shadow.argtypes = [C.c_void_p]
        L.lsgd_mc_pack_entries.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p]
        L.lsgd_select_pull_static.argtypes = [C.c_int32, C.c_int64, C.c_int64, C.c_int32, C.POINTER(C.c_int32), C.c_void_p,
                                              C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_float, C.c_float,
                                              C.c_float, C.c_float, C.c_float, C.c_int32, C.c_void_p]
        L.lsgd_stream_probe.argtypes = [C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p]
        L.lsgd_get_leaders.argtypes = [C.c_void_p, C.POINTER(C.c_int32), C.POINTER(C.c_int32)]
        L.lsgd_get_losses.argtypes = [C.c_void_p, C.POINTER(C.c_float)]
        L.lsgd_set_leaders.argtypes = [C.c_void_p, C.POINTER(C.c_int32), C.c_int32]
        _lib = L
    return _lib


def _check(status):
    if status != 0:
        raise LsgdError(status, lib().lsgd_last_error().decode())


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


class ExternalBatch:
    """Gradient already in g; losses: device float32 [W]."""

    def __init__(self, losses):
        self.losses = losses
        self._d = _External(losses.data_ptr())
        self.c = _Batch(BATCH_EXTERNAL, C.cast(C.pointer(self._d), C.c_void_p))


class MCBatch:
    """rows, cols: int32 [n_obs]; vals: float32 [n_obs]; batch_idx: int32 [W,B] or None (all entries);
    entries: optional int32 [n_obs, 4] from mc_pack_entries (read instead of rows/cols/vals)."""

    def __init__(self, m, n, r, rows, cols, vals, batch_idx, c, entries=None):
        B = 0 if batch_idx is None else int(batch_idx.shape[-1])
        idx_ptr = None
        if batch_idx is not None:
            # an empty tensor has a NULL data pointer, which the C side reads as "all entries"
            anchor = batch_idx if batch_idx.numel() else torch.zeros(1, dtype=torch.int32, device=rows.device)
            idx_ptr = anchor.data_ptr()
            batch_idx = anchor
        self.keep = (rows, cols, vals, batch_idx, entries)
        self._d = _MC(m, n, r, rows.data_ptr(), cols.data_ptr(), vals.data_ptr(), int(rows.numel()),
                      idx_ptr, B, float(c), None if entries is None else entries.data_ptr())
        self.c = _Batch(BATCH_MC, C.cast(C.pointer(self._d), C.c_void_p))


class MLPBatch:
    """dims: [d0..dL]; X: bfloat16 (or int16/uint16 bit patterns) or float32 [W,B,d0]; y: int32 [W,B]."""

    def __init__(self, dims, X, y):
        self.keep = (X, y)
        self._dims = (C.c_int32 * len(dims))(*[int(d) for d in dims])
        self._d = _MLP(len(dims) - 1, self._dims, X.data_ptr(), y.data_ptr(), int(y.shape[-1]),
                       1 if X.dtype == torch.float32 else 0)
        self.c = _Batch(BATCH_MLP, C.cast(C.pointer(self._d), C.c_void_p))


def mc_pack_entries(rows, cols, vals, stream=None):
    """lsgd_mc_pack_entries: returns an int32 [n_obs, 4] tensor of 16-byte records {row, col, val bits, 0}."""
    n = int(rows.numel())
    out = torch.empty((n, 4), dtype=torch.int32, device=rows.device)
    st = torch.cuda.current_stream(rows.device) if stream is None else stream
    _check(lib().lsgd_mc_pack_entries(_ptr(rows), _ptr(cols), _ptr(vals), n, _ptr(out), C.c_void_p(st.cuda_stream)))
    return out


def _config(W, P, ld, n_groups, group_offsets, momentum, flags, weight_decay):
    off = None
    if group_offsets is not None:
        off = (C.c_int32 * len(group_offsets))(*[int(v) for v in group_offsets])
    cfg = _Config(W, P, ld, n_groups, off, momentum, flags, weight_decay)
    return cfg, off


def workspace_bytes(W, P, ld, n_groups, group_offsets=None, momentum=0.0, flags=0, weight_decay=0.0, batch=None):
    cfg, _keep = _config(W, P, ld, n_groups, group_offsets, momentum, flags, weight_decay)
    n = lib().lsgd_workspace_bytes(C.byref(cfg), None if batch is None else C.byref(batch.c))
    if n == 0:
        raise LsgdError(-1, lib().lsgd_last_error().decode())
    return n


PROBE_READ, PROBE_COPY, PROBE_UPDATE = 0, 1, 2


def stream_probe(kind, a, b, c=None, stream=None):
    """lsgd_stream_probe over the whole of the (contiguous, equally sized) float32 tensors a, b, c."""
    assert a.is_contiguous() and b.is_contiguous() and a.numel() == b.numel() and (c is None or c.numel() == a.numel())
    st = torch.cuda.current_stream(a.device) if stream is None else stream
    _check(lib().lsgd_stream_probe(int(kind), _ptr(a), _ptr(b), _ptr(c), a.numel(), C.c_void_p(st.cuda_stream)))


STATIC_MAX_WORKERS, STATIC_MAX_GROUPS = 1024, 64


def select_pull_static(x, g, losses, n_groups, eta, lambda_L, lambda_G, m=None, P=None, group_offsets=None, momentum=0.0,
                       weight_decay=0.0, flags=0, leaders=None, stream=None):
    """lsgd_select_pull_static: selection over all groups + pull update with no handle, workspace or allocation.
    x, g, m: float32 [W, ld]; losses: float32 [W]; leaders: optional int32 [n_groups+1] output."""
    W, ld = x.shape
    off = None if group_offsets is None else (C.c_int32 * len(group_offsets))(*[int(v) for v in group_offsets])
    st = torch.cuda.current_stream(x.device) if stream is None else stream
    _check(lib().lsgd_select_pull_static(W, ld if P is None else int(P), ld, int(n_groups), off, _ptr(x), _ptr(g), _ptr(m),
                                         _ptr(losses), _ptr(leaders), eta, lambda_L, lambda_G, momentum, weight_decay,
                                         int(flags), C.c_void_p(st.cuda_stream)))


class Population:
    """Handle over caller-owned torch CUDA tensors (lsgd_create_population).

    x, g: float32 [W, ld]; m: float32 [W, ld] or None; z_snapshot: float32 [G+1, ld] or None;
    x_bf16: bfloat16 [W, ld] or None.  P defaults to ld.
    """

    def __init__(self, x, g, n_groups, m=None, z_snapshot=None, x_bf16=None, P=None, group_offsets=None,
                 momentum=0.0, flags=0, weight_decay=0.0, largest_batch=None, stream=None, workspace=None):
        assert x.is_cuda and x.dtype == torch.float32 and x.dim() == 2 and x.is_contiguous()
        W, ld = x.shape
        self.W, self.ld, self.P, self.G = W, ld, (ld if P is None else int(P)), int(n_groups)
        self.x, self.g, self.m, self.Z, self.xb = x, g, m, z_snapshot, x_bf16
        cfg, self._off = _config(W, self.P, ld, n_groups, group_offsets, momentum, flags, weight_decay)
        if workspace is None:
            nbytes = lib().lsgd_workspace_bytes(C.byref(cfg), None if largest_batch is None else C.byref(largest_batch.c))
            if nbytes == 0:
                raise LsgdError(-1, lib().lsgd_last_error().decode())
            workspace = torch.empty(nbytes, dtype=torch.uint8, device=x.device)
        self.workspace = workspace
        self.stream = torch.cuda.current_stream(x.device) if stream is None else stream
        h = C.c_void_p()
        _check(lib().lsgd_create_population(C.byref(cfg), _ptr(x), _ptr(g), _ptr(m), _ptr(z_snapshot), _ptr(x_bf16),
                                            _ptr(workspace), workspace.numel(), C.c_void_p(self.stream.cuda_stream),
                                            C.byref(h)))
        self._h = h

    def close(self):
        if getattr(self, "_h", None):
            lib().lsgd_destroy_population(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    @staticmethod
    def _mask(refresh_local):
        if refresh_local is None:
            return None
        return (C.c_uint8 * len(refresh_local))(*[int(v) for v in refresh_local])

    def grad_loss(self, batch, losses=None):
        _check(lib().lsgd_grad_loss(self._h, C.byref(batch.c), _ptr(losses)))

    def loss(self, batch, losses=None):
        _check(lib().lsgd_loss(self._h, C.byref(batch.c), _ptr(losses)))

    def select_leaders(self, losses=None, refresh_local=None, refresh_global=1):
        _check(lib().lsgd_select_leaders(self._h, _ptr(losses), self._mask(refresh_local), int(refresh_global)))

    def pull_update(self, eta, lambda_L, lambda_G):
        _check(lib().lsgd_pull_update(self._h, eta, lambda_L, lambda_G))

    def step(self, batch, eta, lambda_L, lambda_G, refresh_local=None, refresh_global=1):
        _check(lib().lsgd_step(self._h, C.byref(batch.c), eta, lambda_L, lambda_G, self._mask(refresh_local),
                               int(refresh_global)))

    def leader_pull(self, lambda_L, lambda_G):
        _check(lib().lsgd_leader_pull(self._h, lambda_L, lambda_G))

    def step_alg1(self, batch, eta, gamma_L, gamma_G, lambda_L, lambda_G, comm=0, comm_local_mask=None):
        _check(lib().lsgd_step_alg1(self._h, C.byref(batch.c), eta, gamma_L, gamma_G, lambda_L, lambda_G, int(comm),
                                    self._mask(comm_local_mask)))

    def smooth_losses(self, window, t, losses=None, out=None):
        """window: device float32 [K, W] ring."""
        assert window.dtype == torch.float32 and window.is_contiguous() and window.shape[1] == self.W
        _check(lib().lsgd_smooth_losses(self._h, _ptr(window), int(window.shape[0]), int(t), _ptr(losses), _ptr(out)))

    def center(self, out):
        assert out.dtype == torch.float32 and out.is_contiguous() and out.numel() >= self.P
        _check(lib().lsgd_center(self._h, _ptr(out)))

    def easgd_update(self, center, eta, lam):
        assert center.dtype == torch.float32 and center.is_contiguous() and center.numel() >= self.ld
        _check(lib().lsgd_easgd_update(self._h, _ptr(center), eta, lam))

    def easgd_step(self, batch, center, eta, lam):
        assert center.dtype == torch.float32 and center.is_contiguous() and center.numel() >= self.ld
        _check(lib().lsgd_easgd_step(self._h, C.byref(batch.c), _ptr(center), eta, lam))

    def sync_shadow(self):
        _check(lib().lsgd_sync_shadow(self._h))

    def get_leaders(self):
        lead = (C.c_int32 * self.G)()
        gl = C.c_int32()
        _check(lib().lsgd_get_leaders(self._h, lead, C.byref(gl)))
        return list(lead), int(gl.value)

    def set_leaders(self, local_leaders, global_leader):
        arr = (C.c_int32 * self.G)(*[int(v) for v in local_leaders])
        _check(lib().lsgd_set_leaders(self._h, arr, int(global_leader)))

    def get_losses(self):
        out = (C.c_float * self.W)()
        _check(lib().lsgd_get_losses(self._h, out))
        return list(out)
