"""Runs a few steps of one workload plus an elementwise pass over a buffer of known size, for HBM counter runs:

    rocprofv3 --pmc FETCH_SIZE  -d <dir> -o fetch -- python3 -m paper_2511_16592_amd.traffic_probe c2
    rocprofv3 --pmc WRITE_SIZE  -d <dir> -o write -- python3 -m paper_2511_16592_amd.traffic_probe c2

The elementwise kernel (256 MiB read + 256 MiB written) calibrates what the counters report per byte.
"""
import sys

import torch

from . import gfnx
from .workloads import workloads

COPY_BYTES = 256 << 20


def main():
    name = sys.argv[1] if len(sys.argv) > 1 else "c2"
    steps = int(sys.argv[2]) if len(sys.argv) > 2 else 3
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
    print("traffic_probe", name, steps, "steps; copy bytes", COPY_BYTES, "transitions/step", int(sess.length.sum().item()))


if __name__ == "__main__":
    main()
