#!/usr/bin/env python3
"""Benchmark of the rollout + Trajectory-Balance gradient step on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c2]

A step is one pass of the whole hot path over one batch of synthetic input: gfnx_rollout (fresh
Philox iteration counter each step) followed by gfnx_tb_loss_grad, inputs and outputs resident in
HBM.  Prints one JSON line: environment transitions per second (valid transitions only), the roofline
of the dominant kernel measured with HIP events in the same run, and the CPU reference timed on a
bounded sample of the same workload.
"""
import argparse
import ctypes as C
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_FP32_MFMA_TFLOPS = 157.3  # MI355X dense fp32 matrix peak

DESCRIPTIONS = {
    "c1": "2-D grid H=8, MLP 16-64-64-3, batch 16",
    "c2": "4-D grid H=20, MLP 80-256-256-5 (seeded Xavier), batch 4096, max 77 steps",
    "c2_long": "4-D grid H=20, MLP 80-256-256-5 with stop bias -8 (long walks), batch 4096",
    "c3": "bit sequences n=120 k=8, 60 modes, MLP 3855-512-512-256, batch 4096, 15 steps",
    "c4": "Ising 10x10 periodic J=0.44, MLP 300-256-256-200, batch 4096, 100 steps",
    "c5": "10-D grid H=20, MLP 200-256-256-11 (seeded Xavier), batch 16384, max 191 steps",
    "c5_long": "10-D grid H=20, MLP 200-256-256-11 with stop bias -8 (long walks), batch 16384",
}


def cpu_baseline(wl, w, seconds_target=15.0):
    """The CPU reference as it stands (untuned), on a bounded sample of the same workload."""
    from oracle import Oracle
    o32 = Oracle("f32")
    cores = min(os.cpu_count() or 1, 16)
    batch = min(wl.batch, 64)
    used = 0.0
    done_tr = 0
    sample_batches = []
    while True:
        t0 = time.perf_counter()
        out = o32.rollout(wl.env, w, wl.seed, len(sample_batches), batch=batch, nthreads=cores)
        o32.tb_loss_grad(wl.env, w, out["actions"], out["length"], wl.log_z, nthreads=cores)
        dt = time.perf_counter() - t0
        used += dt
        done_tr += int(out["length"].sum())
        sample_batches.append(batch)
        if used >= seconds_target or len(sample_batches) >= 64:
            break
        if dt < seconds_target / 8 and batch < wl.batch:
            batch = min(wl.batch, batch * 4)
    return {"value": done_tr / used, "unit": "transitions/s", "cores": cores, "kind": "oracle",
            "sample": "%d passes (rollout + TB gradient, fp32 build) over batches %s of the same workload, "
                      "%d transitions in %.1f s" % (len(sample_batches), sample_batches, done_tr, used)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="c2", choices=sorted(DESCRIPTIONS))
    ap.add_argument("--no-cpu-baseline", action="store_true")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)")

    import torch
    from paper_2511_16592_amd import gfnx
    from paper_2511_16592_amd.workloads import workloads

    if not torch.cuda.is_available():
        sys.exit("bench.py needs a GPU")
    wl = workloads()[args.workload]
    w = wl.mlp()
    sess = gfnx.Session(wl.env, w, wl.batch)
    timing = gfnx.KernelTimer()

    for i in range(args.warmup):
        sess.rollout(wl.seed, i)
        sess.tb_loss_grad(wl.log_z)
    torch.cuda.synchronize()

    timing.enable(True)
    t0 = time.perf_counter()
    for i in range(args.steps):
        sess.rollout(wl.seed, args.warmup + i)
        sess.tb_loss_grad(wl.log_z)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    kernels = timing.collect()  # {name: (launches, total ms)} from HIP events recorded on the launch stream
    timing.enable(False)

    # count the valid transitions of the timed steps (the rollout is a pure function of seed and iteration)
    transitions = 0
    for i in range(args.steps):
        sess.rollout(wl.seed, args.warmup + i)
        transitions += int(sess.length.sum().item())
    per_step = transitions / args.steps

    h1, h2, a = wl.h1, wl.h2, wl.env.dims()[2]
    flops_fwd = 2.0 * (h1 * h2 + h2 * a)  # per transition, layers 2 and 3 (layer 1 is a gather)
    flops_all = 6.0 * (h1 * h2 + h2 * a)  # forward + backward
    dom = max(kernels, key=lambda k: kernels[k][1])
    launches, total_ms = kernels[dom]
    avg_ms = total_ms / launches
    launches_per_step = launches / args.steps
    # algorithmic flops of the dominant kernel per launch
    share = {"rollout": flops_fwd, "gemm_tn_w2": 2.0 * h1 * h2, "gemm_nt_g1": 2.0 * h1 * h2,
             "gemm_tn_w3": 2.0 * h2 * a, "gemm_nt_g2": 2.0 * h2 * a}.get(dom, 0.0)
    achieved = share * per_step / launches_per_step / (avg_ms * 1e-3) / 1e12
    out = {
        "metric": "env transitions/s for rollout+TB-grad step",
        "value": transitions / elapsed,
        "unit": "transitions/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": elapsed / args.steps * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": "%s: %s" % (args.workload, DESCRIPTIONS[args.workload]),
                   "transitions_per_step": per_step},
        "roofline": {"bound": "mfma", "kernel": dom, "achieved": achieved, "peak": PEAK_FP32_MFMA_TFLOPS,
                     "unit": "TFLOP/s", "frac": achieved / PEAK_FP32_MFMA_TFLOPS, "traffic": None,
                     "avg_kernel_ms": avg_ms,
                     "whole_step_frac": flops_all * per_step / (elapsed / args.steps) / 1e12 / PEAK_FP32_MFMA_TFLOPS},
        "kernels_ms_per_step": {k: v[1] / args.steps for k, v in sorted(kernels.items(), key=lambda kv: -kv[1][1])},
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl, w)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
