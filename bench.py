#!/usr/bin/env python3
"""Throughput of the batched LSGD step on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c2|c3|c4|c5]

Prints ONE JSON line.  Without --workload the primary record is the pull-update
bandwidth stress (W=32 x P=11.7M fp32, the largest configuration and the one
the metric's "% of peak" is quoted on) and `sub_records` holds the matrix-
completion step and the two MLP steps; with --workload X only X runs (used
for profiling).  Every record has `value` = worker-steps/s (W workers x steps
/ seconds) of the whole step with every input already resident in HBM, timed
as the median of 5 repeats of `steps` steps; `roofline` for its dominant
kernel, timed live with events on the stream the library launches on; and
`cpu_baseline`, the CPU oracle timed on a bounded sample of the same workload
on this host.  `hbm_ceilings` are streams of known size measured in the same
run (read-only, copy, and the 3-read/2-write momentum update without leader
rows, in memory order and in the update kernel's own column-chunked order).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

import numpy as np
import torch

import workloads as wl

# Bytes between the L2 caches and memory per launch, from rocprofv3 FETCH_SIZE / WRITE_SIZE runs scaled by
# reference kernels of known size (profiles/*_hbm_traffic.md).  Valid only for the kernel source they were
# taken on: reported as null once that file's code (comments and white space aside) differs.
PULL_TRAFFIC = {"file": "pull_update.hip", "code_sha256_16": "ce89fd10d8336956", "bytes_per_launch": 7.666e9,
                "key": (32, 11_689_512)}
MC_TRAFFIC = {"file": "mc_grad.hip", "code_sha256_16": "39a5db2ab05460a9", "bytes_per_launch": 3.936e8,
              "key": (16, 65536, 20000, 20000, 32)}


def _code_fingerprint(path):
    """sha256 of a source file with comments and white space removed (a reworded comment keeps the counters valid)"""
    import hashlib
    import re
    text = open(path, "r").read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    text = re.sub(r"//[^\n]*", "", text)
    text = re.sub(r"\s+", "", text)
    return hashlib.sha256(text.encode()).hexdigest()[:16]


def _traffic(rec, key):
    src = os.path.join(ROOT, "paper_1905_10395_amd", "csrc", rec["file"])
    try:
        cur = _code_fingerprint(src)
    except OSError:
        return None
    if cur != rec["code_sha256_16"] or tuple(key) != tuple(rec["key"]):
        return None
    return rec["bytes_per_launch"]


def _pull_traffic(W, P):
    return _traffic(PULL_TRAFFIC, (W, P))


METRIC = "worker-steps/sec and pull-update HBM GB/s (% of peak) at W workers, 1 MI355X"
HBM_PEAK_GBS = 8000.0
DEV = "cuda:0"


def _events_ms(fn, reps):
    """Average milliseconds per call of fn over `reps` back-to-back calls (events on the current stream)."""
    a = torch.cuda.Event(enable_timing=True)
    b = torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    a.record()
    for i in range(reps):
        fn(i)
    b.record()
    torch.cuda.synchronize()
    return a.elapsed_time(b) / reps


REPEATS = 5


def _timed_steps(step_fn, steps, warmup, repeats=REPEATS):
    """Median seconds for `steps` steps over `repeats` repeats (each bracketed by a device synchronisation),
    after `warmup` untimed steps."""
    for t in range(warmup):
        step_fn(t)
    secs = []
    t_next = warmup
    for _ in range(repeats):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for t in range(steps):
            step_fn(t_next + t)
        torch.cuda.synchronize()
        secs.append(time.perf_counter() - t0)
        t_next += steps
    return float(np.median(secs))


def _events_ms_med(fn, reps, repeats=REPEATS):
    """Median over `repeats` of the average milliseconds per call over `reps` back-to-back calls."""
    return float(np.median([_events_ms(fn, reps) for _ in range(repeats)]))


def hbm_ceilings(W=32, P=11_689_512):
    """Streams of known size on buffers of the stress shape, in memory order (lsgd_stream_probe): read-only, a
    plain copy, and the momentum update without leader rows (3 reads, 2 writes per element); and the library's
    own update kernel with both pull coefficients zero, which moves the same bytes as the last probe but in the
    column-chunked order the leader tiles need."""
    import paper_1905_10395_amd as L
    ld = wl.padded_ld(P)
    a = torch.empty((W, ld), device=DEV).normal_(std=0.05)
    b = torch.empty((W, ld), device=DEV).normal_(std=0.01)
    c = torch.zeros((W, ld), device=DEV)
    n = float(W) * ld
    ms_read = _events_ms_med(lambda i: L.stream_probe(L.PROBE_READ, a, b), 10)
    ms_copy = _events_ms_med(lambda i: L.stream_probe(L.PROBE_COPY, a, c), 10)
    c.zero_()
    ms_upd = _events_ms_med(lambda i: L.stream_probe(L.PROBE_UPDATE, a, b, c), 10)
    pop = L.Population(a, b, 1, m=c, P=P, momentum=0.9)
    ms_flat = _events_ms_med(lambda i: pop.pull_update(1e-3, 0.0, 0.0), 10)
    out = {"read_GBs": 4.0 * n / (ms_read * 1e-3) / 1e9, "copy_GBs": 8.0 * n / (ms_copy * 1e-3) / 1e9,
           "stream_3r2w_memory_order_GBs": 20.0 * n / (ms_upd * 1e-3) / 1e9,
           "stream_3r2w_chunked_order_GBs": 20.0 * W * P / (ms_flat * 1e-3) / 1e9,
           "note": "measured in this run on [32, 11689536] fp32 buffers: lsgd_stream_probe (read / copy / update, memory order) and "
                   "lsgd_pull_update(eta, 0, 0) with momentum (the update kernel's own column-chunked order)"}
    del pop, a, b, c
    torch.cuda.empty_cache()
    return out


def mfma_ceiling(n=8192, reps=10):
    """What the vendor library's plain bf16 GEMM reaches on this machine at n^3 (context for the MLP kernels' matrix-core
    figures: the datasheet's 2.5 PFLOP/s is not what a real GEMM sustains)."""
    a = torch.randn((n, n), device=DEV, dtype=torch.bfloat16)
    b = torch.randn((n, n), device=DEV, dtype=torch.bfloat16)
    c = torch.empty((n, n), device=DEV, dtype=torch.bfloat16)
    for _ in range(3):
        torch.matmul(a, b, out=c)
    ms = _events_ms_med(lambda i: torch.matmul(a, b, out=c), reps)
    return {"vendor_gemm_bf16_TFLOPs": 2.0 * n ** 3 / (ms * 1e-3) / 1e12, "shape": f"{n}x{n}x{n}",
            "note": "torch.matmul (vendor library) bf16 with fp32 accumulation, measured in this run; peak used for fractions stays 2500"}


# ------------------------------------------------------------------------------------------
# C4: pull-update bandwidth stress (leader selection + fused pull/momentum update only)
# ------------------------------------------------------------------------------------------
def run_stress(L, steps, warmup, W=32, G=4, P=11_689_512, copy_ref=False):
    ld = wl.padded_ld(P)
    gen = torch.Generator(device=DEV); gen.manual_seed(wl.MASTER_SEED)
    x = torch.randn((W, ld), device=DEV, generator=gen) * 0.05
    g = torch.randn((W, ld), device=DEV, generator=gen) * 1e-2
    m = torch.zeros((W, ld), device=DEV)
    losses = torch.rand((16, W), device=DEV, generator=gen)
    batches = [L.ExternalBatch(losses[i]) for i in range(16)]
    pop = L.Population(x, g, G, m=m, P=P, momentum=0.9)
    eta, lamL, lamG = 0.01, 0.1, 0.05
    if copy_ref:
        # a plain copy of known size (lsgd_stream_probe: reads W*ld*4 bytes, writes W*ld*4 bytes), the
        # reference that scales the FETCH_SIZE / WRITE_SIZE counters of a profiled run
        for _ in range(3):
            L.stream_probe(L.PROBE_COPY, g, m)
        m.zero_()

    def step(t):
        pop.step(batches[t % 16], eta, lamL, lamG)

    secs = _timed_steps(step, steps, warmup)
    # the update kernel alone (select once, then updates from the same leaders need kept copies;
    # a full refresh per call keeps it the same launch the step makes)
    def upd(i):
        pop.select_leaders(losses[i % 16]); pop.pull_update(eta, lamL, lamG)
    def sel(i):
        pop.select_leaders(losses[i % 16])
    ms_both = _events_ms_med(upd, max(steps, 10))
    ms_sel = _events_ms_med(sel, 200)
    ms_pull = ms_both - ms_sel
    bytes_per_launch = 20.0 * W * P
    ach = bytes_per_launch / (ms_pull * 1e-3) / 1e9
    out = {
        "workload": f"pull-update stress: W={W} x P={P} fp32 in {G} groups, momentum 0.9, select+pull only",
        "value": W * steps / secs, "unit": "worker-steps/s", "ms_per_step": secs / steps * 1e3,
        "roofline": {"kernel": "pull_rows_kernel<2,1> + pull_leaders_kernel<4,1>", "bound": "hbm", "achieved": ach, "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": ach / HBM_PEAK_GBS, "traffic": _pull_traffic(W, P),
                     "bytes_per_launch": bytes_per_launch, "ms_per_launch": ms_pull},
        "ms_select": ms_sel,
    }
    del pop, x, g, m
    torch.cuda.empty_cache()
    return out


def cpu_stress(W=32, G=4, P=11_689_512, frac=8):
    """Oracle select + update on the first P/frac columns of the same population shape."""
    import oracle
    Ps = P // frac
    x0, g0, _ = wl.stress_state(W, Ps, Ps)
    pop = oracle.Population(x0, wl.equal_group_offsets(W, G), momentum=0.9)
    pop.g[:] = g0
    reps, t0 = 0, time.perf_counter()
    while reps < 3 or time.perf_counter() - t0 < 8.0:
        pop.losses[:] = wl.stress_losses(W, reps)
        pop.select(); pop.update(0.01, 0.1, 0.05)
        reps += 1
    dt = (time.perf_counter() - t0) / reps
    return {"value": W / (dt * frac), "unit": "worker-steps/s", "cores": os.cpu_count() if _omp_threads() is None else _omp_threads(),
            "kind": "oracle", "sample": f"all {W} workers, first 1/{frac} of the columns ({Ps}), {reps} steps; "
            f"time scaled by {frac} (the update is independent per column)"}


def _omp_threads():
    v = os.environ.get("OMP_NUM_THREADS")
    return int(v) if v and v.isdigit() else None


# ------------------------------------------------------------------------------------------
# C2: matrix-completion LSGD (whole step: gradients+losses -> leaders -> pull update)
# ------------------------------------------------------------------------------------------
def make_c2():
    prob = wl.mc_problem(20000, 20000, 32, 0.01, 32 ** -0.5, noise_std=0.01)
    W, G, B, K = 16, 4, 65536, 16
    ld = wl.padded_ld(prob.P)
    x0 = wl.mc_init(W, prob, 32 ** -0.5, ld=ld)
    idx = wl.mc_batches(W, B, prob.n_obs, K)
    return prob, W, G, B, K, ld, x0, idx


def run_c2(L, steps, warmup, data):
    prob, W, G, B, K, ld, x0, idx = data
    d = lambda a: torch.from_numpy(a).to(DEV)
    x = d(x0); g = torch.zeros_like(x)
    Z = torch.zeros((G + 1, ld), device=DEV)
    rows, cols, vals, idx_d = d(prob.rows), d(prob.cols), d(prob.vals), d(idx)
    c = 0.5 * prob.n_obs / B
    packed = L.mc_pack_entries(rows, cols, vals)      # once: the observed set is fixed across steps
    batches = [L.MCBatch(prob.m, prob.n, prob.r, rows, cols, vals, idx_d[k], c, entries=packed) for k in range(K)]
    pop = L.Population(x, g, G, z_snapshot=Z, P=prob.P, largest_batch=batches[0])
    eta, lamL, lamG, tau = 0.005, 0.1, 0.05, 4

    def step(t):
        rl, rg = wl.refresh_masks(t, tau, G)
        pop.step(batches[t % K], eta, lamL, lamG, rl, rg)

    secs = _timed_steps(step, steps, warmup)
    reps = max(20, min(steps, 200))
    ms_grad = _events_ms_med(lambda i: pop.grad_loss(batches[i % K]), reps)
    ms_sel = _events_ms_med(lambda i: pop.select_leaders(), reps)

    def upd(i):
        pop.select_leaders(); pop.pull_update(eta, lamL, lamG)
    ms_pull = _events_ms_med(upd, reps) - ms_sel
    # algorithmic bytes of the gradient stage per launch: read x and write g once (2*4P per worker)
    # plus 16 B of index + entry per batch element
    grad_bytes = W * (2 * 4.0 * prob.P + 16.0 * B)
    ach = grad_bytes / (ms_grad * 1e-3) / 1e9
    lossv = pop.get_losses()

    # the same workload on Algorithm 1's schedule (small pulls to the kept copies every iteration,
    # selection + communication pull every tau iterations), and the center variable
    gamL, gamG = 0.1 / tau, 0.05 / tau

    def step_alg1(t):
        pop.step_alg1(batches[t % K], eta, gamL, gamG, lamL, lamG, (L.COMM_LOCAL | L.COMM_GLOBAL) if t % tau == 0 else 0)
    secs_alg1 = _timed_steps(step_alg1, steps, warmup)

    # Algorithm 1 in its printed order: the best workers are determined after the local step, from the
    # objective on the next sample at the new parameters (one more evaluation pass at each communication)
    def step_alg1_printed(t):
        pop.step_alg1(batches[t % K], eta, gamL, gamG, lamL, lamG, 0)
        if t % tau == 0:
            pop.loss(batches[(t + 1) % K]); pop.select_leaders(); pop.leader_pull(lamL, lamG)
    secs_alg1p = _timed_steps(step_alg1_printed, steps, warmup)
    ms_loss = _events_ms_med(lambda i: pop.loss(batches[i % K]), reps)
    center = torch.empty(ld, device=DEV)
    ms_center = _events_ms_med(lambda i: pop.center(center), reps)
    out = {
        "workload": f"matrix completion LSGD: 20000x20000 rank 32, 1% observed ({prob.n_obs}), W={W} in {G} groups, "
                    f"B={B}/worker/step, eta={eta}, lam_L={lamL}, lam_G={lamG}, leaders every {tau} steps",
        "value": W * steps / secs, "unit": "worker-steps/s", "ms_per_step": secs / steps * 1e3,
        "roofline": {"kernel": "lsgd_grad_loss stage: mc_prep + mc_side + mc_loss_finish kernels", "bound": "hbm", "achieved": ach,
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": ach / HBM_PEAK_GBS,
                     "traffic": _traffic(MC_TRAFFIC, (W, B, prob.m, prob.n, prob.r)),
                     "bytes_per_launch": grad_bytes, "ms_per_launch": ms_grad},
        "stage_ms": {"grad_loss": ms_grad, "select_leaders": ms_sel, "pull_update": ms_pull},
        "pull_update_GBs_cache_assisted": W * 12.0 * prob.P / (ms_pull * 1e-3) / 1e9,
        "cache_note": "x and g of this workload (164 MB) fit the 256 MB memory-side cache: the stage rates here are not HBM bandwidth",
        "final_mean_loss": float(np.mean(lossv)),
        "alg1_schedule": {"value": W * steps / secs_alg1, "unit": "worker-steps/s", "ms_per_step": secs_alg1 / steps * 1e3,
                          "comm_every": tau,
                          "printed_order": {"value": W * steps / secs_alg1p, "unit": "worker-steps/s",
                                            "ms_per_step": secs_alg1p / steps * 1e3, "loss_evaluation_ms": ms_loss,
                                            "note": "leaders re-selected after the local step from lsgd_loss on the next batch"}},
        "center": {"ms": ms_center, "GBs_cache_assisted": 4.0 * (W + 1) * prob.P / (ms_center * 1e-3) / 1e9},
    }
    del pop
    return out


def cpu_c2(data):
    import oracle
    prob, W, G, B, K, ld, x0, idx = data
    pop = oracle.Population(x0, wl.equal_group_offsets(W, G), P=prob.P)
    c = 0.5 * prob.n_obs / B
    reps, t0 = 0, time.perf_counter()
    while reps < 3 or time.perf_counter() - t0 < 8.0:
        rl, rg = wl.refresh_masks(reps, 4, G)
        pop.grad_loss_mc(prob.m, prob.n, prob.r, prob.rows, prob.cols, prob.vals, idx[reps % K], c)
        pop.select(rl, rg); pop.update(0.005, 0.1, 0.05, rl, rg)
        reps += 1
    dt = (time.perf_counter() - t0) / reps
    return {"value": W / dt, "unit": "worker-steps/s", "cores": _omp_threads() or os.cpu_count(), "kind": "oracle",
            "sample": f"the full workload (all {W} workers, B={B}), {reps} whole steps"}


# ------------------------------------------------------------------------------------------
# C3 / C5: MLP classifier on Gaussian-mixture batches (whole step, bf16 operands, fp32 master)
# ------------------------------------------------------------------------------------------
MLP_CFG = {
    "c3": dict(dims=[3072, 1024, 10], W=16, G=4, B=128, tau=1, staggered=False, lamL=0.1, lamG=0.05, K=4,
               name="2-layer MLP 3072-1024-10"),
    "c5": dict(dims=[3072, 4096, 4096, 4096, 10], W=8, G=2, B=256, tau=64, staggered=True, lamL=0.1, lamG=0.02, K=2,
               name="4-layer MLP 3072-4096-4096-4096-10"),
}


def mlp_flops(dims, B):
    """forward + d-weight for every layer, + d-input for every layer but the first (2 flops per MAC)"""
    f = 0
    for k in range(len(dims) - 1):
        f += 2 * 2 * B * dims[k] * dims[k + 1]
        if k > 0:
            f += 2 * B * dims[k] * dims[k + 1]
    return f


def make_mlp(cfg):
    dims, W, B, K = cfg["dims"], cfg["W"], cfg["B"], cfg["K"]
    P = wl.mlp_param_count(dims)
    ld = wl.padded_ld(P)
    x0 = wl.mlp_init(W, dims, ld=ld)
    means = wl.gmm_means(dims[0], dims[-1])
    batches = [wl.gmm_batch(W, B, means, t) for t in range(K)]
    return P, ld, x0, batches


def run_mlp(L, steps, warmup, cfg, data, fused=True, measured_bw_gbs=None):
    dims, W, G, B, K, tau = cfg["dims"], cfg["W"], cfg["G"], cfg["B"], cfg["K"], cfg["tau"]
    P, ld, x0, host_batches = data
    x = torch.from_numpy(x0).to(DEV)
    g = torch.zeros_like(x); m = torch.zeros_like(x)
    xb = torch.zeros((W, ld), dtype=torch.bfloat16, device=DEV)
    Z = torch.zeros((G + 1, ld), device=DEV) if (tau > 1 or fused) else None
    batches = []
    for Xb, y in host_batches:
        Xd = torch.from_numpy(Xb.view(np.int16)).to(DEV).view(torch.bfloat16)
        batches.append(L.MLPBatch(dims, Xd, torch.from_numpy(y).to(DEV)))
    pop = L.Population(x, g, G, m=m, z_snapshot=Z, x_bf16=xb, P=P, momentum=0.9,
                       flags=L.WRITE_BF16_SHADOW | (L.FUSED_MLP_UPDATE if fused else 0), largest_batch=batches[0])
    eta, lamL, lamG = 0.01, cfg["lamL"], cfg["lamG"]

    def step(t):
        rl, rg = wl.refresh_masks(t, tau, G, staggered=cfg["staggered"])
        pop.step(batches[t % K], eta, lamL, lamG, rl, rg)

    secs = _timed_steps(step, steps, warmup)
    reps = max(10, min(steps, 100))
    ms_grad = _events_ms_med(lambda i: pop.grad_loss(batches[i % K]), reps)
    ms_sel = _events_ms_med(lambda i: pop.select_leaders(), reps)
    ms_loss = _events_ms_med(lambda i: pop.loss(batches[i % K]), reps)

    def upd(i):
        pop.select_leaders(); pop.pull_update(eta, lamL, lamG)
    ms_pull = _events_ms_med(upd, reps) - ms_sel
    flops = float(W) * mlp_flops(dims, B)
    tf = flops / (ms_grad * 1e-3) / 1e12
    # traffic the gradient stage cannot avoid: read the bf16 weights once per product that uses them
    # (forward, d-input) and write the fp32 gradient once
    wbytes = sum(dims[k] * dims[k + 1] for k in range(len(dims) - 1))
    min_bytes = float(W) * (2.0 * wbytes * 2 + 4.0 * P)
    ms_step = secs / steps * 1e3
    if fused:
        # whole step with the update applied in the backward kernels: bf16 weights read by the forward and the
        # d-input products (the first layer has no d-input), x and m read and written, bf16 copy written
        step_bytes = float(W) * (2.0 * wbytes + 2.0 * (wbytes - dims[0] * dims[1]) + 18.0 * P)
        gbs = step_bytes / (ms_step * 1e-3) / 1e9
        roof = {"kernel": "lsgd_step, update applied in the backward kernels (gemm_bf16_kernel<..., EPI_DWU> dominant): all kernels of the step",
                "bound": "hbm", "achieved": gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": gbs / HBM_PEAK_GBS, "traffic": None,
                "bytes_per_launch": step_bytes, "ms_per_launch": ms_step,
                "mfma_TFLOPs_of_step": flops / (ms_step * 1e-3) / 1e12}
    else:
        roof = {"kernel": "lsgd_grad_loss (MLP): gemm_bf16_kernel launches", "bound": "mfma", "achieved": tf,
                "peak": 2500.0, "unit": "TFLOP/s", "frac": tf / 2500.0, "traffic": None,
                "flops_per_launch": flops, "ms_per_launch": ms_grad,
                "hbm_floor_ms": min_bytes / (HBM_PEAK_GBS * 1e9) * 1e3}
    # the gradient stage as a contraction: fraction of the bf16 matrix-core peak, and of what its arithmetic
    # intensity allows (flops per byte of unavoidable traffic x memory bandwidth, datasheet and measured)
    intensity = flops / min_bytes
    grad_stage = {"kernel": "lsgd_grad_loss (MLP): gemm_bf16_kernel launches + narrow-layer kernels", "bound": "mfma", "achieved": tf,
                  "peak": 2500.0, "unit": "TFLOP/s", "frac": tf / 2500.0, "flops_per_launch": flops, "ms_per_launch": ms_grad,
                  "min_bytes_per_launch": min_bytes, "intensity_flop_per_byte": intensity,
                  "intensity_roofline_TFLOPs": min(2500.0, intensity * HBM_PEAK_GBS / 1e3),
                  "frac_of_intensity_roofline": tf / min(2500.0, intensity * HBM_PEAK_GBS / 1e3),
                  "hbm_floor_ms": min_bytes / (HBM_PEAK_GBS * 1e9) * 1e3}
    if measured_bw_gbs:
        lim = min(2500.0, intensity * measured_bw_gbs / 1e3)
        grad_stage["intensity_roofline_measured_bw_TFLOPs"] = lim
        grad_stage["frac_of_intensity_roofline_measured_bw"] = tf / lim
        if fused:
            roof["frac_of_measured_copy_bw"] = roof["achieved"] / measured_bw_gbs
    out = {
        "workload": f"{cfg['name']}, synthetic 10-class Gaussian mixture, W={W} in {G} groups, batch {B}/worker, bf16 operands / "
                    f"fp32 master, momentum 0.9, eta={eta}, lam_L={lamL}, lam_G={lamG}, leaders every {tau} steps"
                    + (" (staggered per group)" if cfg["staggered"] else "")
                    + (", update applied inside the backward kernels" if fused else ""),
        "value": W * steps / secs, "unit": "worker-steps/s", "ms_per_step": ms_step,
        "roofline": roof,
        "stage_ms": {"grad_loss": ms_grad, "loss_only": ms_loss, "select_leaders": ms_sel, "pull_update": ms_pull,
                     "note": "separate calls (gradient through memory); the timed step " + ("fuses them" if fused else "is their sum")},
        "grad_stage_roofline": grad_stage,
        "pull_update_GBs": W * 22.0 * P / (ms_pull * 1e-3) / 1e9,
        "final_mean_loss": float(np.mean(pop.get_losses())),
    }
    del pop
    return out


def cpu_mlp(cfg, data, workers, batch_frac=1.0):
    """Oracle steps on `workers` of the W workers; with batch_frac < 1 on that share of each batch (the cost of a
    step is proportional to the batch), scaled back to whole steps."""
    import oracle
    dims, W, G, B = cfg["dims"], cfg["W"], cfg["G"], cfg["B"]
    P, ld, x0, host_batches = data
    Ws = min(workers, W)
    Bs = max(1, int(round(B * batch_frac)))
    pop = oracle.Population(x0[:Ws], np.array([0, Ws], dtype=np.int32), momentum=0.9, P=P)
    reps, t0 = 0, time.perf_counter()
    while reps < 1 or time.perf_counter() - t0 < 8.0:
        Xb, y = host_batches[reps % len(host_batches)]
        pop.grad_loss_mlp(dims, np.ascontiguousarray(Xb[:Ws, :Bs]), np.ascontiguousarray(y[:Ws, :Bs]))
        pop.select(); pop.update(0.01, cfg["lamL"], cfg["lamG"])
        reps += 1
    dt = (time.perf_counter() - t0) / reps
    what = f"full batch {B}" if Bs == B else f"{Bs} of the {B} samples of each batch (rate scaled by {Bs}/{B})"
    return {"value": Ws / dt * (Bs / B), "unit": "worker-steps/s", "cores": _omp_threads() or os.cpu_count(), "kind": "oracle",
            "sample": f"{Ws} of the {W} workers (one group), {what}, full model, {reps} whole steps"}


def _record(primary, cpu):
    rec = {"value": primary["value"], "unit": primary["unit"], "ms_per_step": primary["ms_per_step"],
           "config": {"workload": primary["workload"]}, "roofline": primary["roofline"], "cpu_baseline": cpu}
    for k in ("stage_ms", "pull_update_GBs", "pull_update_GBs_cache_assisted", "cache_note", "final_mean_loss", "ms_select",
              "alg1_schedule", "center", "grad_stage_roofline"):
        if k in primary:
            rec[k] = primary[k]
    return rec


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="all", choices=["all", "c2", "c3", "c4", "c5"],
                    help="all: the stress as primary record plus c2, c3, c5 as sub-records; else that workload alone")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle baseline legs")
    ap.add_argument("--no-fuse", action="store_true", help="MLP workloads: three-call step instead of the fused update")
    ap.add_argument("--copy-ref", action="store_true", help="also run a plain device copy of one [W,ld] buffer (counter calibration)")
    ap.add_argument("--no-ceilings", action="store_true", help="skip the stream-ceiling measurements (profiling runs of the update alone)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU; every population lives on a single device "
              "(no collectives, no sharding). Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)
    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    import paper_1905_10395_amd as L
    L.lib()

    line = {"metric": METRIC, "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "repeats": REPEATS,
            "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic"}
    which = ["c4", "c2", "c3", "c5"] if args.workload == "all" else [args.workload]
    ceil = hbm_ceilings() if args.workload in ("all", "c4") and not args.no_ceilings else None
    records = {}
    for w in which:
        if w == "c4":
            prim = run_stress(L, args.steps, args.warmup, copy_ref=args.copy_ref)
            if ceil:
                prim["roofline"]["frac_of_measured_3r2w_stream_memory_order"] = prim["roofline"]["achieved"] / ceil["stream_3r2w_memory_order_GBs"]
                prim["roofline"]["frac_of_measured_3r2w_stream_chunked_order"] = prim["roofline"]["achieved"] / ceil["stream_3r2w_chunked_order_GBs"]
            cpu = None if args.no_cpu else cpu_stress()
        elif w == "c2":
            data = make_c2()
            prim = run_c2(L, args.steps, args.warmup, data)
            cpu = None if args.no_cpu else cpu_c2(data)
            del data
        else:
            cfg = MLP_CFG[w]
            data = make_mlp(cfg)
            prim = run_mlp(L, args.steps, args.warmup, cfg, data, fused=not args.no_fuse,
                           measured_bw_gbs=ceil["copy_GBs"] if ceil else None)
            cpu = None if args.no_cpu else (cpu_mlp(cfg, data, cfg["W"]) if w == "c3" else cpu_mlp(cfg, data, 2, 0.25))
            del data
        records[w] = _record(prim, cpu)
        records[w]["dtype"] = "f32" if w in ("c2", "c4") else "bf16"
        torch.cuda.empty_cache()
    first = which[0]
    line.update(records[first])
    if ceil:
        line["hbm_ceilings"] = ceil
    if any(w in MLP_CFG for w in which):
        line["mfma_ceiling"] = mfma_ceiling()
    if len(which) > 1:
        line["sub_records"] = {w: records[w] for w in which[1:]}
    print(json.dumps(line))


if __name__ == "__main__":
    main()
