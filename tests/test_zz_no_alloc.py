"""gfnx_train_step_static (the entry point that allocates nothing) against gfnx_train_step.

Two calls in a row on the library's one fixed scratch array, the second with a smaller input: trajectories, loss,
gradients, updated weights, log Z and optimiser moments must be those of gfnx_train_step with a caller-provided
workspace -- bit for bit, since both run the same kernels in the same launch configuration (actions, lengths and
terminal states are integer results; the floating-point results are compared bit-exactly too, which is stricter than
the 1e-4 bar of the parity tests)."""
import ctypes as C

import numpy as np
import pytest

from paper_2511_16592_amd.workloads import grid_env, ising_env, random_mlp

pytestmark = pytest.mark.gpu
PARAM_KEYS = ("W1", "b1", "W2", "b2", "W3", "b3")


def _pair(gfnx, env, shape, batch, seed):
    w = random_mlp(*shape, seed=seed, scale=1.5)
    a, b = gfnx.Session(env, w, batch), gfnx.Session(env, w, batch)
    a.init_optimizer(log_z=0.2)
    b.init_optimizer(log_z=0.2)
    return a, b


def _same(a, b, what):
    ta, tb = a.trajectories(), b.trajectories()
    for k in ta:
        assert np.array_equal(ta[k], tb[k]), (what, k)
    ga, gb = a.gradients(), b.gradients()
    for k in ga:
        assert np.array_equal(ga[k], gb[k]), (what, k)
    wa, wb = a.weights(), b.weights()
    for k in PARAM_KEYS:
        assert np.array_equal(wa[k], wb[k]), (what, k)
        assert np.array_equal(a.adam_m[k].cpu().numpy(), b.adam_m[k].cpu().numpy()), (what, "m", k)
        assert np.array_equal(a.adam_v[k].cpu().numpy(), b.adam_v[k].cpu().numpy()), (what, "v", k)
    assert float(a.log_z.item()) == float(b.log_z.item()), what
    assert int(ta["length"].sum()) > 0


def test_static_scratch_training_iteration_matches_the_workspace_one():
    import torch
    assert torch.cuda.is_available()
    from paper_2511_16592_amd import gfnx
    gfnx.load_library()
    # first call: Ising 5 x 5, 256 wide, 60 trajectories (1500 rows: most of the scratch array is written)
    a, b = _pair(gfnx, ising_env(5), (75, 256, 256, 50), 60, seed=81)
    need = a.workspace_bytes
    assert need <= 64 << 20
    print(f"[no-alloc] call 1: ising 5x5, batch 60, workspace {need} bytes", flush=True)
    for it in range(2):
        a.train_step(31, it)
        b.train_step_static(31, it)
        _same(a, b, f"ising5 iteration {it}")
    # second call, smaller input, same array with the first call's contents still in it
    c, d = _pair(gfnx, grid_env(3, 7), (21, 256, 256, 4), 21, seed=82)
    assert c.workspace_bytes < need
    print(f"[no-alloc] call 2: grid 3x7, batch 21, workspace {c.workspace_bytes} bytes", flush=True)
    for it in range(2):
        c.train_step(32, it)
        d.train_step_static(32, it)
        _same(c, d, f"grid3x7 iteration {it}")
    # and the first shape again after the smaller one
    a.train_step(31, 2)
    b.train_step_static(31, 2)
    _same(a, b, "ising5 iteration 2")
    # too large for the array: rejected on the host, nothing launched
    big = gfnx.Session(ising_env(10), random_mlp(300, 256, 256, 200, seed=83), 4096)
    big.init_optimizer()
    assert big.workspace_bytes > 64 << 20
    with pytest.raises(gfnx.GfnxError) as err:
        big.train_step_static(1, 0)
    assert err.value.status == -4
