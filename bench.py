#!/usr/bin/env python3
"""Throughput of the batched LSGD step on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c2|c3|c4|c5]

Prints ONE JSON line.  `value` is worker-steps/s (W workers x steps / seconds)
of the whole step with every input already resident in HBM.  `roofline`
describes the dominant kernel of the workload, timed live with events on the
stream the library launches on; `cpu_baseline` is the CPU oracle timed on a
bounded sample of the same workload on this host.  The line also carries the
pull-update bandwidth stress (`pull_update_stress`) whichever workload is the
primary one, because the metric names both quantities.
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
PULL_TRAFFIC = {"file": "pull_update.hip", "code_sha256_16": "c1af6e928c94a4f6", "bytes_per_launch": 7.668e9,
                "key": (32, 11_689_512)}
MC_TRAFFIC = {"file": "mc_grad.hip", "code_sha256_16": "b7100f28d40b05f7", "bytes_per_launch": 3.935e8,
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


def _timed_steps(step_fn, steps, warmup):
    for t in range(warmup):
        step_fn(t)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for t in range(steps):
        step_fn(warmup + t)
    torch.cuda.synchronize()
    return (time.perf_counter() - t0)


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
        # a plain copy of known size (reads and writes W*ld*4 bytes each), the reference that scales
        # the FETCH_SIZE / WRITE_SIZE counters of a profiled run
        for _ in range(3):
            m.copy_(g)
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
    ms_both = _events_ms(upd, max(steps, 10))
    ms_sel = _events_ms(sel, 200)
    ms_pull = ms_both - ms_sel
    bytes_per_launch = 20.0 * W * P
    ach = bytes_per_launch / (ms_pull * 1e-3) / 1e9
    out = {
        "workload": f"pull-update stress: W={W} x P={P} fp32 in {G} groups, momentum 0.9, select+pull only",
        "value": W * steps / secs, "unit": "worker-steps/s", "ms_per_step": secs / steps * 1e3,
        "roofline": {"kernel": "pull_rows_kernel<4,1> + pull_leaders_kernel<4,1>", "bound": "hbm", "achieved": ach, "peak": HBM_PEAK_GBS,
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
    ms_grad = _events_ms(lambda i: pop.grad_loss(batches[i % K]), reps)
    ms_sel = _events_ms(lambda i: pop.select_leaders(), reps)

    def upd(i):
        pop.select_leaders(); pop.pull_update(eta, lamL, lamG)
    ms_pull = _events_ms(upd, reps) - ms_sel
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
    center = torch.empty(ld, device=DEV)
    ms_center = _events_ms(lambda i: pop.center(center), reps)
    out = {
        "workload": f"matrix completion LSGD: 20000x20000 rank 32, 1% observed ({prob.n_obs}), W={W} in {G} groups, "
                    f"B={B}/worker/step, eta={eta}, lam_L={lamL}, lam_G={lamG}, leaders every {tau} steps",
        "value": W * steps / secs, "unit": "worker-steps/s", "ms_per_step": secs / steps * 1e3,
        "roofline": {"kernel": "lsgd_grad_loss stage: mc_prep + mc_side + mc_loss_finish kernels", "bound": "hbm", "achieved": ach,
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": ach / HBM_PEAK_GBS,
                     "traffic": _traffic(MC_TRAFFIC, (W, B, prob.m, prob.n, prob.r)),
                     "bytes_per_launch": grad_bytes, "ms_per_launch": ms_grad},
        "stage_ms": {"grad_loss": ms_grad, "select_leaders": ms_sel, "pull_update": ms_pull},
        "pull_update_GBs": W * 12.0 * prob.P / (ms_pull * 1e-3) / 1e9,
        "final_mean_loss": float(np.mean(lossv)),
        "alg1_schedule": {"value": W * steps / secs_alg1, "unit": "worker-steps/s", "ms_per_step": secs_alg1 / steps * 1e3,
                          "comm_every": tau},
        "center": {"ms": ms_center, "GBs": 4.0 * (W + 1) * prob.P / (ms_center * 1e-3) / 1e9},
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


def run_mlp(L, steps, warmup, cfg, data, fused=True):
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
    ms_grad = _events_ms(lambda i: pop.grad_loss(batches[i % K]), reps)
    ms_sel = _events_ms(lambda i: pop.select_leaders(), reps)

    def upd(i):
        pop.select_leaders(); pop.pull_update(eta, lamL, lamG)
    ms_pull = _events_ms(upd, reps) - ms_sel
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
    out = {
        "workload": f"{cfg['name']}, synthetic 10-class Gaussian mixture, W={W} in {G} groups, batch {B}/worker, bf16 operands / "
                    f"fp32 master, momentum 0.9, eta={eta}, lam_L={lamL}, lam_G={lamG}, leaders every {tau} steps"
                    + (" (staggered per group)" if cfg["staggered"] else "")
                    + (", update applied inside the backward kernels" if fused else ""),
        "value": W * steps / secs, "unit": "worker-steps/s", "ms_per_step": ms_step,
        "roofline": roof,
        "stage_ms": {"grad_loss": ms_grad, "select_leaders": ms_sel, "pull_update": ms_pull,
                     "note": "separate calls (gradient through memory); the timed step " + ("fuses them" if fused else "is their sum")},
        "grad_loss_TFLOPs": tf,
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
    return {"value": Ws / dt * (Bs / B), "unit": "worker-steps/s", "cores": min(Ws, _omp_threads() or os.cpu_count()), "kind": "oracle",
            "sample": f"{Ws} of the {W} workers (one group), {what}, full model, {reps} whole steps"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="c2", choices=["c2", "c3", "c4", "c5"])
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle baseline leg")
    ap.add_argument("--no-stress", action="store_true", help="skip the extra pull-update stress measurement")
    ap.add_argument("--no-fuse", action="store_true", help="MLP workloads: three-call step instead of the fused update")
    ap.add_argument("--copy-ref", action="store_true", help="also run a plain device copy of one [W,ld] buffer (counter calibration)")
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

    stress = None
    if args.workload == "c4" or not args.no_stress:
        stress = run_stress(L, min(args.steps, 100), min(args.warmup, 10), copy_ref=args.copy_ref)
    line = {"metric": METRIC, "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "higher_is_better": True,
            "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic"}
    if args.workload == "c4":
        primary = stress
        cpu = None if args.no_cpu else cpu_stress()
    elif args.workload in MLP_CFG:
        cfg = MLP_CFG[args.workload]
        data = make_mlp(cfg)
        line["dtype"] = "bf16"
        primary = run_mlp(L, args.steps, args.warmup, cfg, data, fused=not args.no_fuse)
        cpu = None if args.no_cpu else (cpu_mlp(cfg, data, cfg["W"]) if args.workload == "c3" else cpu_mlp(cfg, data, 4, 0.25))
    else:
        data = make_c2()
        primary = run_c2(L, args.steps, args.warmup, data)
        cpu = None if args.no_cpu else cpu_c2(data)
    line.update({"value": primary["value"], "unit": primary["unit"], "ms_per_step": primary["ms_per_step"],
                 "config": {"workload": primary["workload"]}, "roofline": primary["roofline"],
                 "cpu_baseline": cpu})
    for k in ("stage_ms", "pull_update_GBs", "final_mean_loss", "ms_select", "alg1_schedule", "center", "grad_loss_TFLOPs"):
        if k in primary:
            line[k] = primary[k]
    if stress is not None:
        line["pull_update_stress"] = {k: stress[k] for k in ("workload", "value", "unit", "ms_per_step", "roofline")}
    if args.workload == "c4":
        line["steps"] = min(args.steps, 100); line["warmup"] = min(args.warmup, 10)
    print(json.dumps(line))


if __name__ == "__main__":
    main()
