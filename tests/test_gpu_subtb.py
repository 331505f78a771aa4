"""GPU parity of the Subtrajectory / Detailed Balance loss and gradient (network with a flow output, hypergrid).

Bars: loss relative 1e-4 (floor 1e-6); each gradient tensor max |diff| <= 1e-4 * max |ref| + 1e-7 against the binary64
reference along the GPU's own action sequences; sampling must not see the flow output at all (bit-identical
trajectories with and without it).
"""
import math
import os

import numpy as np
import pytest

from paper_2511_16592_amd.workloads import grid_env, random_mlp, xavier_mlp
from tests.helpers import (PARAM_KEYS, enumerate_grid_trajectories, grid_dp_flows, grid_terminal_distribution,
                           grid_tv_to_reward, pack_trajectories)
from tests.test_gpu_parity import gfnx, padded_optimal_mlp, say  # noqa: F401
from tests.test_oracle_subtb import policy_part

pytestmark = pytest.mark.gpu
KEYS = ("dW1", "db1", "dW2", "db2", "dW3", "db3")
NTHREADS = min(16, os.cpu_count() or 1)


def check_subtb(oracle64, env, w, traj, grads, lam):
    g = oracle64.subtb_loss_grad(env, {k: v.astype(np.float64) for k, v in w.items()}, traj["actions"], traj["length"], lam)
    assert abs(grads["loss"] - g["loss"]) <= 1e-4 * abs(g["loss"]) + 1e-6, (grads["loss"], g["loss"])
    for k in KEYS:
        scale = np.abs(g[k]).max()
        err = np.abs(grads[k].astype(np.float64) - g[k]).max()
        assert err <= 1e-4 * scale + 1e-7, (k, float(err), float(scale))
    return g


CASES = [
    ("grid3x5_64", grid_env(3, 5), (64, 64), 200),
    ("grid2x8_b1", grid_env(2, 8), (64, 64), 1),
    ("grid3x7_256", grid_env(3, 7), (256, 256), 100),
    ("grid3x7_256_big", grid_env(3, 7), (256, 256), 5000),
    ("grid16x3_256", grid_env(16, 3), (256, 256), 90),       # 17 actions + flow: two logit tiles
    ("grid15x3_256", grid_env(15, 3), (256, 256), 50),       # 16 actions + flow = 17 outputs
    ("grid4x6_128_256", grid_env(4, 6), (128, 256), 70),
    ("grid4x20_256_long", grid_env(4, 20), (256, 256), 64),  # the c2 shape with long walks
]


@pytest.mark.parametrize("lam", [0.0, 0.9])
@pytest.mark.parametrize("case", CASES, ids=lambda c: c[0])
def test_subtb_against_reference(gfnx, oracle32, oracle64, case, lam):
    name, env, (h1, h2), batch = case
    sd, od, na, ms = env.dims()
    w = random_mlp(od, h1, h2, na + 1, seed=91, scale=1.5)
    if name.endswith("_long"):
        w["b3"][na - 1] -= 4.0
    say(f"[subtb {name}] batch={batch} lambda={lam}")
    sess = gfnx.Session(env, w, batch)
    sess.rollout(29, 1)
    sess.subtb_loss_grad(lam)
    traj, grads = sess.trajectories(), sess.gradients()
    rep = oracle32.replay(env, policy_part(w), 29, 1, traj["actions"], traj["length"], tie_tol=1e-5, nthreads=NTHREADS)
    assert (rep["violations"] == 0).all()
    check_subtb(oracle64, env, w, traj, grads, lam)
    if name.endswith("_long"):
        assert traj["length"].max() > 30


def test_flow_output_is_invisible_to_sampling(gfnx):
    env = grid_env(3, 7)
    w = random_mlp(21, 256, 256, 5, seed=92, scale=1.5)
    a = gfnx.Session(env, w, 300)
    b = gfnx.Session(env, policy_part(w), 300)
    a.rollout(7, 2)
    b.rollout(7, 2)
    ta, tb = a.trajectories(), b.trajectories()
    for k in ta:
        assert (ta[k] == tb[k]).all(), k


@pytest.mark.parametrize("lam", [0.0, 0.5, 1.0])
def test_zero_loss_under_the_proper_policy_with_true_flows(gfnx, lam):
    """Every complete trajectory of the side-4 grid, teacher-forced: detailed balance holds edge by edge."""
    side = 4
    env = grid_env(2, side)
    w, log_z = padded_optimal_mlp(side)
    F = grid_dp_flows(2, side)
    flow = np.zeros(64, np.float32)
    for i in range(side):
        for j in range(side):
            flow[i * side + j] = math.log(F[(i, j)])
    w = dict(w)
    w["W3"] = np.concatenate([w["W3"], flow[:, None]], axis=1).astype(np.float32)
    w["b3"] = np.concatenate([w["b3"], [0.0]]).astype(np.float32)
    trajs = enumerate_grid_trajectories(2, side)
    actions, length = pack_trajectories(trajs, 2 * (side - 1) + 1)
    sess = gfnx.Session(env, w, len(trajs))
    sess.replay(actions, length)
    sess.subtb_loss_grad(lam)
    g = sess.gradients()
    assert g["loss"] < 1e-10
    for k in KEYS:
        assert np.abs(g[k]).max() < 2e-6, k


def test_subtb_with_exploration_and_replay(gfnx, oracle64):
    env = grid_env(3, 5)
    w = random_mlp(15, 64, 128, 5, seed=93, scale=1.5)
    sess = gfnx.Session(env, w, 120)
    sess.rollout(31, 0, epsilon=0.4)
    sess.subtb_loss_grad(0.9)
    traj, g1 = sess.trajectories(), sess.gradients()
    check_subtb(oracle64, env, w, traj, g1, 0.9)
    sess.replay(traj["actions"], traj["length"])     # the same trajectories teacher-forced: the same gradient
    sess.subtb_loss_grad(0.9)
    g2 = sess.gradients()
    assert abs(g1["loss"] - g2["loss"]) <= 1e-6 * abs(g1["loss"])
    for k in KEYS:
        np.testing.assert_allclose(g2[k], g1[k], rtol=1e-5, atol=1e-7 * np.abs(g1[k]).max())


def test_wrong_objective_for_the_network_is_rejected(gfnx):
    env = grid_env(2, 8)
    plain = gfnx.Session(env, random_mlp(16, 64, 64, 3, seed=94), 16)
    plain.rollout(0, 0)
    with pytest.raises(gfnx.GfnxError) as err:
        plain.subtb_loss_grad(0.9)
    assert err.value.status == -3
    flow = gfnx.Session(env, random_mlp(16, 64, 64, 4, seed=94), 16)
    flow.rollout(0, 0)
    with pytest.raises(gfnx.GfnxError) as err:
        flow.tb_loss_grad(0.0)
    assert err.value.status == -3
    with pytest.raises(gfnx.GfnxError) as err:
        flow.subtb_loss_grad(1.5)
    assert err.value.status == -3
    flow.subtb_loss_grad(0.9)


@pytest.mark.parametrize("lam", [0.0, 0.9])
def test_training_with_db_and_subtb_converges(gfnx, oracle64, lam):
    """The paper's hypergrid benchmark also trains with DB and SubTB(0.9): rollout, objective, Adam (no log Z: the
    flow output at s_0 plays its part).  Criterion as for TB: total variation of the exact terminal distribution
    of the trained policy from R/Z."""
    import ctypes as C
    side = 8
    env = grid_env(2, side)
    w0 = xavier_mlp(2 * side, 64, 64, 4, seed=22)
    sess = gfnx.Session(env, w0, 16)
    sess.init_optimizer(lr=1e-3)
    state = gfnx.AdamState(sess.adam_state.m, sess.adam_state.v, None)

    def exact_tv(w):
        w64 = {k: v.astype(np.float64) for k, v in policy_part(w).items()}
        term = grid_terminal_distribution(lambda x: oracle64.policy(env, w64, list(x))[1:], 2, side)
        return grid_tv_to_reward(term, side)

    tv0 = exact_tv(w0)
    iters = 6000
    late = []  # the exact total variation at four checkpoints over the last quarter of the run
    for it in range(iters):
        sess.rollout(6, it)
        sess.subtb_loss_grad(lam)
        rc = sess.lib.gfnx_adam_step(C.byref(sess.mlp), None, C.byref(sess.cgrads), None, C.byref(state),
                                     C.byref(sess.adam_cfg), it + 1, sess._stream())
        assert rc == 0
        if it + 1 >= iters - 1500 and (it + 1) % 500 == 0:
            late.append(exact_tv(sess.weights()))
    w1 = sess.weights()
    tv1 = float(np.median(late))
    phi0 = float(w1["b3"][3] + np.maximum(np.maximum(w1["W1"][0] + w1["W1"][side] + w1["b1"], 0) @ w1["W2"] + w1["b2"], 0) @ w1["W3"][:, 3])
    say(f"[converge lambda={lam}] total variation {tv0:.3f} -> " + " ".join(f"{v:.4f}" for v in late) +
        f"; log F(s0) {phi0:.3f} (log Z {math.log(16.064):.3f})")
    # A batch of 16 makes the iterates wander: a single checkpoint can sit on a transient excursion (0.004 to 0.04
    # at iteration 6000 over rollout seeds, whatever the arithmetic of the gradient kernels), so the criterion is
    # the median of the four late checkpoints, with a loose bound on each.
    assert tv0 > 0.5 and tv1 < 0.03 and max(late) < 0.1
    assert abs(phi0 - math.log(16.064)) < 0.06


@pytest.mark.parametrize("lam", [0.0, 0.9])
def test_train_step_with_options_equals_its_three_calls(gfnx, lam):
    """gfnx_train_step_opts with exploration and a SubTB objective against rollout_explore + subtb_loss_grad + adam."""
    import ctypes as C
    env = grid_env(3, 7)
    w = xavier_mlp(21, 256, 256, 5, seed=95)
    a = gfnx.Session(env, w, 150)
    b = gfnx.Session(env, w, 150)
    a.init_optimizer()
    b.init_optimizer()
    state = gfnx.AdamState(b.adam_state.m, b.adam_state.v, None)
    for it in range(4):
        a.train_step(8, it, epsilon=0.05, subtb_lambda=lam)
        b.rollout(8, it, epsilon=0.05)
        b.subtb_loss_grad(lam)
        assert b.lib.gfnx_adam_step(C.byref(b.mlp), None, C.byref(b.cgrads), None, C.byref(state),
                                    C.byref(b.adam_cfg), it + 1, b._stream()) == 0
        ta, tb = a.trajectories(), b.trajectories()
        for k in ta:
            assert (ta[k] == tb[k]).all(), (it, k)
        wa, wb = a.weights(), b.weights()
        for k in wa:
            assert np.array_equal(wa[k], wb[k]), (it, k)
        assert float(a.loss.item()) == float(b.loss.item())
    assert float(a.log_z.item()) == 0.0   # untouched by this objective


def test_train_step_with_exploration_equals_its_three_calls(gfnx):
    env = grid_env(3, 7)
    w = xavier_mlp(21, 256, 256, 4, seed=96)
    a = gfnx.Session(env, w, 150)
    b = gfnx.Session(env, w, 150)
    a.init_optimizer(log_z=0.2)
    b.init_optimizer(log_z=0.2)
    for it in range(3):
        a.train_step(8, it, epsilon=0.1)
        b.rollout(8, it, epsilon=0.1)
        b.tb_loss_grad(float(b.log_z.item()))
        b.adam_step()
        wa, wb = a.weights(), b.weights()
        for k in wa:
            assert np.array_equal(wa[k], wb[k]), (it, k)
        assert float(a.log_z.item()) == float(b.log_z.item())
