"""Batched Leader-SGD step on one MI355X: thin Python binding over liblsgd.so.

The library (HIP kernels + C boundary declared in include/lsgd.h) does all the
work; this package only marshals arguments.  PyTorch supplies device memory
and the stream.  There is no CPU fallback: importing `binding` without the
built library raises.
"""
from .binding import (  # noqa: F401
    COMM_GLOBAL, COMM_LOCAL, FUSED_MLP_UPDATE, LEADER_EXEMPT, MOMENTUM_GRAD_ONLY, NESTEROV, PULL_UNSCALED_BY_ETA, WRITE_BF16_SHADOW,
    ExternalBatch, LsgdError, MCBatch, MLPBatch, Population, lib, lib_path, mc_pack_entries, select_pull_static, stream_probe, workspace_bytes,
    PROBE_COPY, PROBE_READ, PROBE_UPDATE,
)
