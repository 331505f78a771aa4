#!/usr/bin/env python3
"""Benchmark of the rollout + Trajectory-Balance gradient step on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c2] [--no-extra] [--no-cpu-baseline]
    python bench.py --traffic --workload c2 [--steps 3]

(--no-extra skips the short runs of the other workloads, of whole training iterations and of the estimate of
P_theta(x).  --traffic is the run that the hardware-counter profiles are taken over: a few steps of the workload,
each followed by one elementwise pass over a buffer of known size that calibrates the counters, then the optimiser
update alone; it times nothing.)

A step is one pass of the whole hot path over one batch of synthetic input: gfnx_rollout (fresh
Philox iteration counter each step) followed by gfnx_tb_loss_grad, inputs and outputs resident in
HBM.  Prints one JSON line: environment transitions per second (valid transitions only), the roofline
of the dominant kernel measured with HIP events on its launch stream inside the timed region, and the
CPU reference timed on a bounded sample of the same workload.  The warm-up steps run with events
around every kernel to find the dominant one; in the timed region only that kernel carries events.
"""
import argparse
import hashlib
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
    "c3_na": "bit sequences n=64 k=4 in the non-autoregressive scheme (256 actions), MLP 1040-512-512-256, batch 4096",
    "c3_na120": "bit sequences n=120 k=8 in the non-autoregressive scheme (3840 actions), MLP 3855-512-512-3840, "
                "batch 4096",
}
KERNEL_SOURCES = ("rollout_kernel.h", "grad_kernels.h", "grad_kernels2.h", "grad_kernels3.h", "grad_kernels4.h",
                  "subtb_kernels.h", "backward_kernel.h", "gfnx_device.h", "gfnx.hip")
COPY_BYTES = 256 << 20  # the calibration pass of --traffic reads and writes this much


def kernel_source_hash():
    h = hashlib.sha256()
    for name in KERNEL_SOURCES:
        with open(os.path.join(ROOT, "paper_2511_16592_amd", "csrc", name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]


def measured_traffic(workload, kernel):
    """HBM bytes per launch of `kernel` from the committed rocprofv3 counter summary, or None when there is
    none for this workload / kernel or the kernel sources changed since the counters were taken."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    if not os.path.exists(path):
        return None
    try:
        rec = json.load(open(path))
    except ValueError:
        return None
    entry = rec.get(workload, {}).get(kernel)
    if not entry or rec.get("kernel_source_hash") != kernel_source_hash():
        return None
    return entry["bytes_per_launch"]


def flop_shares(h1, h2, a):
    """Algorithmic matrix-core flops per transition of each kernel (layer 1 is a gather / scatter)."""
    return {"rollout": 2.0 * (h1 * h2 + h2 * a), "gemm_tn_w2": 2.0 * h1 * h2, "gemm_nt_g1": 2.0 * h1 * h2,
            "gemm_tn_w3": 2.0 * h2 * a, "gemm_nt_g2": 2.0 * h2 * a}


def cpu_baseline(wl, w, seconds_target=12.0):
    """The CPU reference as it stands (untuned), on a bounded sample of the same workload."""
    from oracle import Oracle
    o32 = Oracle("f32")
    cores = min(os.cpu_count() or 1, 16)
    batch = min(wl.batch, 64)
    used, done_tr, batches = 0.0, 0, []
    while True:
        t0 = time.perf_counter()
        out = o32.rollout(wl.env, w, wl.seed, len(batches), batch=batch, nthreads=cores)
        o32.tb_loss_grad(wl.env, w, out["actions"], out["length"], wl.log_z, nthreads=cores)
        dt = time.perf_counter() - t0
        used += dt
        done_tr += int(out["length"].sum())
        batches.append(batch)
        if used >= seconds_target or len(batches) >= 160:
            break
        if dt < seconds_target / 8 and batch < wl.batch:
            batch = min(wl.batch, batch * 4)
    # the same reference on one thread, on a small batch (per-transition cost does not depend on the batch)
    t0 = time.perf_counter()
    one = o32.rollout(wl.env, w, wl.seed, 0, batch=min(wl.batch, 256), nthreads=1)
    o32.tb_loss_grad(wl.env, w, one["actions"], one["length"], wl.log_z, nthreads=1)
    single = int(one["length"].sum()) / (time.perf_counter() - t0)
    sizes = sorted(set(batches))
    mix = ", ".join("%d x %d" % (batches.count(b), b) for b in sizes)
    return {"value": done_tr / used, "unit": "transitions/s", "cores": cores, "kind": "oracle",
            "single_thread_value": single,
            "sample": "%d passes (rollout + TB gradient, binary32 build, %d threads) over batches of the same "
                      "workload (passes x trajectories: %s): %d transitions in %.1f s"
                      % (len(batches), cores, mix, done_tr, used)}


def run_workload(name, steps, warmup, events=True, epsilon=None):
    import torch
    from paper_2511_16592_amd import gfnx
    from paper_2511_16592_amd.workloads import workloads

    wl = workloads()[name]
    w = wl.mlp()
    sess = gfnx.Session(wl.env, w, wl.batch)
    timer = gfnx.KernelTimer()

    # the very first step pays one-time costs (code-object load, first-touch of the workspace): keep it out of
    # the per-kernel breakdown when there is more than one warm-up step
    cold = 1 if warmup >= 2 else 0
    for i in range(cold):
        sess.rollout(wl.seed, i, epsilon)
        sess.tb_loss_grad(wl.log_z)
    torch.cuda.synchronize()
    timer.enable(events)
    for i in range(cold, warmup):
        sess.rollout(wl.seed, i, epsilon)
        sess.tb_loss_grad(wl.log_z)
    torch.cuda.synchronize()
    breakdown = timer.collect() if events else {}
    dominant = max(breakdown, key=lambda k: breakdown[k][1]) if breakdown else None

    timer.enable(events and dominant is not None, only=dominant)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        sess.rollout(wl.seed, warmup + i, epsilon)
        sess.tb_loss_grad(wl.log_z)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    dom = timer.collect().get(dominant) if dominant else None
    timer.enable(False)

    # valid transitions of the timed steps (the rollout is a pure function of seed and iteration)
    transitions = 0
    for i in range(steps):
        sess.rollout(wl.seed, warmup + i, epsilon)
        transitions += int(sess.length.sum().item())
    torch.cuda.synchronize()
    return dict(wl=wl, weights=w, elapsed=elapsed, transitions=transitions, dominant=dominant, dom=dom,
                breakdown={k: v[1] / max(1, warmup - cold) for k, v in breakdown.items()})


def run_training(name, steps, warmup, batch=None):
    """Whole training iterations (rollout, TB loss and gradient, Adam update of the weights and of log Z on the
    device, no host round trip) from the workload's initial weights.  The policy changes from one iteration to the
    next, so the transitions are counted inside the loop: one 4-byte-per-trajectory device copy per iteration."""
    import torch
    from paper_2511_16592_amd import gfnx
    from paper_2511_16592_amd.workloads import workloads

    wl = workloads()[name]
    if batch is not None:
        wl = wl.with_batch(batch)
    sess = gfnx.Session(wl.env, wl.mlp(), wl.batch)
    sess.init_optimizer(log_z=wl.log_z, lr=1e-3, lr_log_z=1e-1)
    lengths = torch.zeros((steps, wl.batch), dtype=torch.int32, device=sess.device)
    timer = gfnx.KernelTimer()
    for i in range(warmup):
        sess.train_step(wl.seed, i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        sess.train_step(wl.seed, warmup + i)
        lengths[i].copy_(sess.length)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    timer.enable(True, only="adam")
    for i in range(5):
        sess.train_step(wl.seed, warmup + steps + i)
    torch.cuda.synchronize()
    launches, adam_ms = timer.collect().get("adam", (1, float("nan")))
    timer.enable(False)
    n_par = sum(int(v.numel()) for v in sess.w.values()) + 1
    transitions = int(lengths.sum().item())
    return {"batch": wl.batch, "iterations": steps, "ms_per_iteration": elapsed / steps * 1e3,
            "iterations_per_s": steps / elapsed, "transitions_per_s": transitions / elapsed,
            "transitions_per_iteration": transitions / steps,
            "adam_kernel": {"avg_ms": adam_ms / launches, "parameters": n_par,
                            "achieved_GBps": 28.0 * n_par / (adam_ms / launches * 1e-3) / 1e9, "peak_GBps": 8000.0}}


def run_traffic(name, steps):
    """The run that counter profiles are taken over (rocprofv3 --pmc ... -- python3 bench.py --traffic ...)."""
    import torch
    from paper_2511_16592_amd import gfnx
    from paper_2511_16592_amd.workloads import workloads

    wl = workloads()[name]
    sess = gfnx.Session(wl.env, wl.mlp(), wl.batch)
    src = torch.arange(COPY_BYTES // 4, dtype=torch.float32, device="cuda:0")
    dst = torch.empty_like(src)
    for i in range(steps):
        sess.rollout(wl.seed, i)
        sess.tb_loss_grad(wl.log_z)
        torch.add(src, 1.0, out=dst)  # a plain elementwise kernel: reads COPY_BYTES, writes COPY_BYTES
    sess.init_optimizer()
    for i in range(steps):
        sess.adam_step()  # the optimiser update alone, on the gradients of the last step
    torch.cuda.synchronize()
    return {"traffic_run": name, "steps": steps, "copy_bytes": COPY_BYTES,
            "transitions_per_step": int(sess.length.sum().item())}


def run_subtb(name, steps, lam):
    """The same step with the Subtrajectory Balance objective (lambda = 0: Detailed Balance): the network gets one
    more output, the state flow; rollout + gfnx_subtb_loss_grad."""
    import numpy as np
    import torch
    from paper_2511_16592_amd import gfnx
    from paper_2511_16592_amd.workloads import workloads, xavier_mlp

    wl = workloads()[name]
    _, obs_dim, n_actions, _ = wl.env.dims()
    w = xavier_mlp(obs_dim, wl.h1, wl.h2, n_actions + 1, wl.weight_seed)
    if wl.stop_bias:
        w["b3"][n_actions - 1] += np.float32(wl.stop_bias)
    sess = gfnx.Session(wl.env, w, wl.batch)
    for i in range(3):
        sess.rollout(wl.seed, i)
        sess.subtb_loss_grad(lam)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        sess.rollout(wl.seed, 3 + i)
        sess.subtb_loss_grad(lam)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    transitions = 0
    for i in range(steps):
        sess.rollout(wl.seed, 3 + i)
        transitions += int(sess.length.sum().item())
    return {"lambda": lam, "ms_per_step": elapsed / steps * 1e3, "transitions_per_s": transitions / elapsed,
            "transitions_per_step": transitions / steps}


def run_estimate(name, steps, n_samples=10):
    """Monte-Carlo estimate of log P_theta(x) for batch / n_samples seeded random terminal states: backward rollouts,
    teacher-forced forward evaluation along them, log-mean of P_F / P_B (the paper's evaluation uses 10 samples)."""
    import numpy as np
    import torch
    from paper_2511_16592_amd import gfnx
    from paper_2511_16592_amd.workloads import workloads

    wl = workloads()[name]
    n_states = wl.batch // n_samples
    wl = wl.with_batch(n_states * n_samples)
    sd = wl.env.dims()[0]
    rng = np.random.default_rng(wl.seed)
    if wl.env.kind == 0:
        states = rng.integers(0, wl.env.grid_side, size=(n_states, sd))
    elif wl.env.kind == 1:
        states = rng.integers(0, 1 << wl.env.k_bits, size=(n_states, sd)).astype(np.uint8).view(np.int8)
    else:
        states = 2 * rng.integers(0, 2, size=(n_states, sd)) - 1
    sess = gfnx.Session(wl.env, wl.mlp(), wl.batch)
    ts = torch.as_tensor(states, dtype=torch.int8).t().repeat_interleave(n_samples, dim=1).contiguous().to(sess.device)
    timer = gfnx.KernelTimer()

    def one(i):
        sess.terminal_state.copy_(ts)
        sess.backward_rollout(wl.seed, i)
        sess.replay_device()
        return sess.log_prob_estimate(n_states, n_samples)

    for i in range(3):
        one(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        one(3 + i)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    timer.enable(True)
    for i in range(5):
        one(3 + steps + i)
    torch.cuda.synchronize()
    bd = {k: v[1] / 5 for k, v in timer.collect().items()}
    timer.enable(False)
    transitions = int(sess.length.sum().item())
    return {"states": n_states, "samples_per_state": n_samples, "ms_per_evaluation": elapsed / steps * 1e3,
            "states_per_s": n_states * steps / elapsed, "transitions_per_s": transitions * steps / elapsed,
            "kernels_ms": {k: round(v, 5) for k, v in sorted(bd.items(), key=lambda kv: -kv[1])}}


def summary(name, r, steps):
    wl = r["wl"]
    a = wl.env.dims()[2]
    per_step = r["transitions"] / steps
    flops_all = 6.0 * (wl.h1 * wl.h2 + wl.h2 * a)
    return {"workload": "%s: %s" % (name, DESCRIPTIONS[name]), "value": r["transitions"] / r["elapsed"],
            "unit": "transitions/s", "ms_per_step": r["elapsed"] / steps * 1e3, "transitions_per_step": per_step,
            "whole_step_mfma_frac": flops_all * per_step / (r["elapsed"] / steps) / 1e12 / PEAK_FP32_MFMA_TFLOPS}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="c2", choices=sorted(DESCRIPTIONS))
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extra", action="store_true", help="skip the short runs of the other workloads")
    ap.add_argument("--traffic", action="store_true", help="the untimed run that counter profiles are taken over")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py measures one GPU: this library has no multi-GPU path (run with --gpus 1)")

    import torch
    if not torch.cuda.is_available():
        sys.exit("bench.py needs a GPU")
    if args.traffic:
        print(json.dumps(run_traffic(args.workload, min(args.steps, 3))))
        return

    r = run_workload(args.workload, args.steps, max(1, args.warmup))
    wl = r["wl"]
    a = wl.env.dims()[2]
    head = summary(args.workload, r, args.steps)
    per_step = head["transitions_per_step"]

    roofline = None
    if r["dom"]:
        launches, total_ms = r["dom"]
        avg_ms = total_ms / launches
        share = flop_shares(wl.h1, wl.h2, a).get(r["dominant"], 0.0)
        achieved = share * per_step * (args.steps / launches) / (avg_ms * 1e-3) / 1e12
        roofline = {"bound": "mfma", "kernel": r["dominant"], "achieved": achieved, "peak": PEAK_FP32_MFMA_TFLOPS,
                    "unit": "TFLOP/s", "frac": achieved / PEAK_FP32_MFMA_TFLOPS,
                    "traffic": measured_traffic(args.workload, r["dominant"]),
                    "avg_kernel_ms": avg_ms, "launches": launches,
                    "algorithmic_flops_per_launch": share * per_step * (args.steps / launches),
                    "whole_step_frac": head["whole_step_mfma_frac"],
                    "note": "the rollout's duration is bounded below by (longest trajectory of the batch) x (per-step "
                            "latency of a workgroup): short walks (c2, c5) are latency-bound, long walks and Ising "
                            "(see extra) are matrix-core-bound"}

    out = {
        "metric": "env transitions/s for rollout+TB-grad step",
        "value": head["value"], "unit": "transitions/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": head["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": head["workload"], "transitions_per_step": per_step},
        "roofline": roofline,
        "kernels_ms_per_step": {k: round(v, 5) for k, v in sorted(r["breakdown"].items(), key=lambda kv: -kv[1])},
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl, r["weights"])
    if not args.no_extra:
        # other workloads of the same path, short runs without per-kernel events (context for the headline line:
        # the 4-D grid at Xavier initialisation has ~5-step trajectories, i.e. little work per launch)
        extra = {}
        for name in ("c2_long", "c4", "c5", "c5_long", "c3", "c3_na", "c3_na120"):
            if name == args.workload:
                continue
            steps = 5 if name in ("c5_long", "c3_na120") else 20
            extra[name] = summary(name, run_workload(name, steps, 3, events=False), steps)
        out["extra"] = extra
        # the same step with epsilon-uniform exploration at the paper's rate
        out["explore_eps_1e-3"] = {name: summary(name, run_workload(name, 20, 3, events=False, epsilon=1e-3), 20)
                                   for name in ("c2", "c4", "c3")}
        # the next stage of the same path: whole training iterations (optimiser step included)
        out["train"] = {args.workload: run_training(args.workload, 50, 5), "c3": run_training("c3", 20, 3)}
        # the other two objectives of the paper's hypergrid benchmark, on the same kernels
        out["subtb"] = {"c2_db": run_subtb("c2", 20, 0.0), "c2_subtb0.9": run_subtb("c2", 20, 0.9),
                        "c2_long_subtb0.9": run_subtb("c2_long", 10, 0.9), "c5_long_subtb0.9": run_subtb("c5_long", 5, 0.9)}
        # evaluation side of the same kernels: backward rollouts + forward evaluation + estimate of P_theta(x)
        out["estimate"] = {name: run_estimate(name, 20) for name in ("c2", "c4")}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
