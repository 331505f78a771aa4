"""GPU parity of epsilon-uniform exploration in the rollout against the CPU reference.

Bars as for the plain rollout: actions, lengths and terminal states bit-exact except on steps where the policy's own
draw decides and its top-2 perturbed logits are closer than 1e-5; explored steps are integer decisions and must match
exactly; scalars and gradients to 1e-4 along the GPU's own actions.
"""
import os

import numpy as np
import pytest

from paper_2511_16592_amd.workloads import bitseq_env, bitseq_na_env, grid_env, ising_env, random_mlp
from tests.test_gpu_parity import check_gradients, gfnx, relu_decisions, say  # noqa: F401  (gfnx is the module fixture)

pytestmark = pytest.mark.gpu
NTHREADS = min(16, os.cpu_count() or 1)

CASES = [
    ("grid3x5", grid_env(3, 5), (64, 64), 200, 0.5),
    ("grid3x7_256_paper_eps", grid_env(3, 7), (256, 256), 3000, 1e-3),
    ("grid3x7_256_always", grid_env(3, 7), (256, 256), 100, 1.0),
    ("grid16x3_256", grid_env(16, 3), (256, 256), 90, 0.3),
    ("ising3", ising_env(3), (64, 64), 33, 0.3),
    ("ising4_256", ising_env(4), (256, 256), 70, 0.5),
    ("ising10_256", ising_env(10), (256, 256), 24, 0.2),
    ("bitseq24", bitseq_env(24, 4, 7, mode_seed=2), (64, 64), 45, 0.5),
    ("bitseq120", bitseq_env(120, 8, 60, mode_seed=3), (64, 128), 40, 0.2),
    ("bitseq120_256", bitseq_env(120, 8, 60, mode_seed=3), (256, 256), 40, 0.2),
    ("bitseq_na24", bitseq_na_env(24, 4, 7, mode_seed=2), (64, 64), 45, 0.4),
    ("bitseq_na64_256", bitseq_na_env(64, 4, 20, mode_seed=3), (256, 256), 40, 0.2),
    ("bitseq_na16k8_paged", bitseq_na_env(16, 8, 5, mode_seed=2), (64, 64), 60, 0.4),          # 512 actions
    ("bitseq_na40k8_paged_512", bitseq_na_env(40, 8, 20, mode_seed=3), (512, 512), 40, 0.2),   # 1280 actions
    ("bitseq_na96k6_paged_paper_eps", bitseq_na_env(96, 6, 9, mode_seed=5, uniform_bits=True), (128, 128), 900, 1e-3),
]


@pytest.mark.parametrize("case", CASES, ids=lambda c: c[0])
def test_exploring_rollout_against_reference(gfnx, oracle32, oracle64, case):
    name, env, (h1, h2), batch, eps = case
    sd, od, na, ms = env.dims()
    w = random_mlp(od, h1, h2, na, seed=71, scale=1.5)
    say(f"[explore {name}] batch={batch} eps={eps}")
    sess = gfnx.Session(env, w, batch)
    sess.rollout(19, 3, epsilon=eps)
    traj = sess.trajectories()
    relu = relu_decisions(sess, traj)
    sess.tb_loss_grad(0.2)
    grads = sess.gradients()
    rep = oracle32.replay(env, w, 19, 3, traj["actions"], traj["length"], tie_tol=1e-5, nthreads=NTHREADS, epsilon=eps)
    assert (rep["violations"] == 0).all()
    clean = rep["near_ties"] == 0
    assert int(rep["near_ties"].sum()) <= 10 * 2e-5 * int(traj["length"].sum()) + 3
    assert (rep["terminal_state"] == traj["terminal_state"]).all()
    free = oracle32.rollout(env, w, 19, 3, batch=batch, nthreads=NTHREADS, epsilon=eps)
    assert (free["length"][clean] == traj["length"][clean]).all()
    assert (free["actions"][:, clean] == traj["actions"][:, clean]).all()
    ref = oracle64.replay(env, w, 19, 3, traj["actions"], traj["length"], tie_tol=1e30, nthreads=NTHREADS, epsilon=eps)
    for k in ("log_pf", "log_pb", "log_reward"):
        err = np.abs(traj[k].astype(np.float64) - ref[k]) - (1e-4 * np.abs(ref[k]) + 1e-5)
        assert (err <= 0).all(), (k, float(err.max()))
    check_gradients(oracle64, env, w, traj, grads, 0.2, relu)
    # exploration really happened (or, at the paper's rate, at about that rate)
    plain = oracle32.rollout(env, w, 19, 3, batch=batch, nthreads=NTHREADS)
    differs = (plain["actions"] != traj["actions"]).any(0).mean()
    if eps >= 0.2:
        assert differs > 0.3
    else:
        assert 0.0 < differs < 0.05


def test_epsilon_zero_is_the_plain_rollout_bit_for_bit(gfnx):
    env = grid_env(3, 7)
    w = random_mlp(21, 256, 256, 4, seed=72)
    a = gfnx.Session(env, w, 150)
    a.rollout(5, 1)
    ta = a.trajectories()
    a.rollout(5, 1, epsilon=0.0)
    tb = a.trajectories()
    for k in ta:
        assert (ta[k] == tb[k]).all()


def test_epsilon_out_of_range_is_rejected(gfnx):
    env = grid_env(2, 8)
    sess = gfnx.Session(env, random_mlp(16, 64, 64, 3, seed=73), 16)
    for bad in (-0.1, 1.5, float("nan")):
        with pytest.raises(gfnx.GfnxError) as err:
            sess.rollout(0, 0, epsilon=bad)
        assert err.value.status == -3
