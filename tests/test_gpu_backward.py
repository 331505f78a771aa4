"""GPU parity of the backward rollout and of the estimate of P_theta(x) against the CPU reference.

Bars: action bytes, lengths and recovered terminal states bit-exact (integer work: the parent drawn at each backward
move is an integer function of the Philox word); log P_B and log P_F relative 1e-4 (floor 1e-5) against the binary64
reference; the estimate within 1e-4 relative (floor 2e-5) of the reference's estimate from the same trajectories.
"""
import math
import os

import numpy as np
import pytest

from paper_2511_16592_amd.workloads import bitseq_env, bitseq_na_env, grid_env, ising_env, random_mlp, workloads
from tests.helpers import grid_reward, grid_terminal_distribution
from tests.test_oracle_backward import _random_terminal_states

pytestmark = pytest.mark.gpu
NTHREADS = min(16, os.cpu_count() or 1)


@pytest.fixture(scope="module")
def gfnx():
    import torch
    assert torch.cuda.is_available()
    from paper_2511_16592_amd import gfnx as g
    g.load_library()
    return g


def say(msg):
    print(msg, flush=True)


def _close(got, want, rel=1e-4, floor=1e-5):
    err = np.abs(got.astype(np.float64) - want) - (rel * np.abs(want) + floor)
    assert (err <= 0).all(), float(err.max())


CASES = [
    ("grid3x5", grid_env(3, 5), (64, 64), 200),
    ("grid2x8_b1", grid_env(2, 8), (64, 64), 1),
    ("grid16x3", grid_env(16, 3), (64, 64), 77),
    ("grid4x20", grid_env(4, 20), (256, 256), 4097),
    ("grid10x20", grid_env(10, 20), (256, 256), 300),
    ("bitseq24", bitseq_env(24, 4, 7, mode_seed=2), (64, 64), 45),
    ("bitseq120", bitseq_env(120, 8, 60, mode_seed=3), (64, 128), 130),
    ("ising3", ising_env(3), (64, 64), 33),
    ("ising10", ising_env(10), (256, 256), 260),
    ("bitseq_na24", bitseq_na_env(24, 4, 7, mode_seed=2), (64, 64), 45),
    ("bitseq_na64_256", bitseq_na_env(64, 4, 20, mode_seed=3), (256, 256), 130),
    ("bitseq_na40k8_paged", bitseq_na_env(40, 8, 20, mode_seed=3), (128, 64), 150),   # 1280 actions: 16-bit plane
]


@pytest.mark.parametrize("case", CASES, ids=lambda c: c[0])
def test_backward_rollout_and_forward_evaluation(gfnx, oracle64, case):
    name, env, (h1, h2), batch = case
    sd, od, na, ms = env.dims()
    say(f"[backward {name}] batch={batch}")
    rng = np.random.default_rng(50)
    ts = _random_terminal_states(env, batch, rng)
    w = random_mlp(od, h1, h2, na, seed=51)
    sess = gfnx.Session(env, w, batch)
    sess.backward_rollout(23, 4, ts)
    got = sess.trajectories()
    ref = oracle64.backward_rollout(env, 23, 4, ts)
    assert (got["length"] == ref["length"]).all()
    assert (got["actions"] == ref["actions"]).all()
    _close(got["log_pb"], ref["log_pb"])
    # forward evaluation along the drawn trajectories
    sess.replay_device()
    got = sess.trajectories()
    assert (got["terminal_state"] == ts).all()
    rep = oracle64.replay(env, w, 0, 0, ref["actions"], ref["length"], tie_tol=1e30, nthreads=NTHREADS)
    _close(got["log_pf"], rep["log_pf"])
    _close(got["log_pb"], ref["log_pb"])
    # a different iteration counter draws different parents (where there is a choice)
    sess.backward_rollout(23, 5, ts)
    other = sess.trajectories()
    if env.kind == 1:
        assert (other["actions"] == ref["actions"]).all()
    elif batch > 1:
        assert (other["actions"] != ref["actions"]).any()
    assert (other["length"] == ref["length"]).all()


def test_backward_rollout_clamps_out_of_range_states(gfnx, oracle64):
    env = grid_env(2, 8)
    w = random_mlp(16, 64, 64, 3, seed=52)
    ts = np.array([[-3, 7, 100, 0], [5, -128, 127, 0]], dtype=np.int8)
    sess = gfnx.Session(env, w, 4)
    sess.backward_rollout(1, 0, ts)
    got = sess.trajectories()
    clamped = np.clip(ts.astype(int), 0, 7)
    assert (got["length"] == clamped.sum(0) + 1).all()
    ref = oracle64.backward_rollout(env, 1, 0, clamped.astype(np.int8))
    assert (got["actions"] == ref["actions"]).all()


@pytest.mark.parametrize("n_samples", [1, 7, 64, 100])
def test_estimate_matches_reference(gfnx, oracle64, n_samples):
    env = grid_env(3, 7)
    n_states = 23
    rng = np.random.default_rng(53)
    states = rng.integers(0, 7, size=(n_states, 3)).astype(np.int8)
    w = random_mlp(21, 256, 256, 4, seed=54, scale=2.0)
    sess = gfnx.Session(env, w, n_states * n_samples)
    est = sess.estimate_log_prob(states, n_samples, seed=3, iteration=1).cpu().numpy()
    tr = sess.trajectories()
    want = oracle64.log_prob_estimate(tr["log_pf"].astype(np.float64), tr["log_pb"].astype(np.float64), n_states, n_samples)
    _close(est, want, floor=2e-5)
    # and against the reference's own chain from the same states
    ts = np.repeat(states.T, n_samples, axis=1)
    back = oracle64.backward_rollout(env, 3, 1, ts)
    rep = oracle64.replay(env, w, 0, 0, back["actions"], back["length"], tie_tol=1e30, nthreads=NTHREADS)
    chain = oracle64.log_prob_estimate(rep["log_pf"], back["log_pb"], n_states, n_samples)
    _close(est, chain, floor=2e-5)


def test_estimate_handles_tiny_probabilities(gfnx):
    import torch
    env = grid_env(2, 8)
    sess = gfnx.Session(env, random_mlp(16, 64, 64, 3, seed=55), 6)
    sess.log_pf.copy_(torch.tensor([-1000.0, -1001.0, -1002.0, -50.0, -50.0, -50.0]))
    sess.log_pb.copy_(torch.tensor([-3.0, -3.0, -3.0, 0.0, 0.0, 0.0]))
    est = sess.log_prob_estimate(2, 3).cpu().numpy()
    want = np.array([-997.0 + math.log((1 + math.exp(-1) + math.exp(-2)) / 3), -50.0])
    np.testing.assert_allclose(est, want, rtol=1e-6)


def test_estimate_is_exact_under_the_proper_policy(gfnx):
    """P_F(tau)/P_B(tau|x) = R(x)/Z on every trajectory of the policy that satisfies trajectory balance."""
    from tests.test_gpu_parity import padded_optimal_mlp
    side = 8
    env = grid_env(2, side)
    w, log_z = padded_optimal_mlp(side)
    states = np.array([(i, j) for i in range(side) for j in range(side)], dtype=np.int8)
    sess = gfnx.Session(env, w, 64 * 5)
    est = sess.estimate_log_prob(states, 5, seed=9, iteration=0).cpu().numpy()
    want = np.array([math.log(grid_reward(tuple(x), side)) - log_z for x in states])
    np.testing.assert_allclose(est, want, rtol=0, atol=2e-5)


def test_estimate_converges_to_the_exact_terminal_probability(gfnx, oracle64):
    side = 5
    env = grid_env(2, side)
    w = random_mlp(2 * side, 64, 64, 3, seed=9, scale=2.0)
    w64 = {k: v.astype(np.float64) for k, v in w.items()}
    exact = grid_terminal_distribution(lambda x: oracle64.policy(env, w64, list(x))[1:], 2, side)
    states = np.array([(4, 4), (2, 3), (0, 0), (1, 4), (3, 1)], dtype=np.int8)
    n_samples = 4000
    sess = gfnx.Session(env, w, len(states) * n_samples)
    est = np.exp(sess.estimate_log_prob(states, n_samples, seed=10, iteration=0).cpu().numpy().astype(np.float64))
    tr = sess.trajectories()
    ratio = np.exp(tr["log_pf"].astype(np.float64) - tr["log_pb"]).reshape(len(states), n_samples)
    for i, x in enumerate(states):
        sigma = ratio[i].std() / math.sqrt(n_samples)
        assert abs(est[i] - exact[tuple(x)]) <= 4.5 * sigma + 1e-4 * exact[tuple(x)], (x, est[i], exact[tuple(x)])


def test_estimate_at_benchmark_shapes(gfnx, oracle64):
    """c2 and c4 at full batch (409 states x 10 samples, the paper's N): sampled trajectories against the reference."""
    for name in ("c2", "c4"):
        wl = workloads()[name]
        n_samples, n_states = 10, wl.batch // 10
        env = wl.env
        rng = np.random.default_rng(56)
        states = _random_terminal_states(env, n_states, rng).T.copy()
        say(f"[estimate {name}] {n_states} states x {n_samples}")
        sess = gfnx.Session(env, wl.mlp(), n_states * n_samples)
        est = sess.estimate_log_prob(states, n_samples, seed=wl.seed, iteration=0).cpu().numpy()
        tr = sess.trajectories()
        pick = rng.choice(n_states, size=12, replace=False)
        cols = (pick[:, None] * n_samples + np.arange(n_samples)[None, :]).reshape(-1)
        ts = np.repeat(states[pick].T, n_samples, axis=1)
        back = oracle64.backward_rollout(env, wl.seed, 0, np.ascontiguousarray(np.repeat(states.T, n_samples, axis=1)))
        assert (back["actions"] == tr["actions"]).all() and (back["length"] == tr["length"]).all()
        rep = oracle64.replay(env, wl.mlp(), 0, 0, np.ascontiguousarray(back["actions"][:, cols]),
                              np.ascontiguousarray(back["length"][cols]), tie_tol=1e30, nthreads=NTHREADS)
        assert (rep["terminal_state"] == ts).all()
        want = oracle64.log_prob_estimate(rep["log_pf"], back["log_pb"][cols], len(pick), n_samples)
        _close(est[pick], want, floor=2e-5)
