"""Pins for epsilon-uniform exploration in the CPU reference's rollout."""
import numpy as np
import pytest

from paper_2511_16592_amd.workloads import bitseq_env, grid_env, ising_env, random_mlp
from tests.helpers import chi2_sf


def _softmax(logit, valid):
    z = np.where(valid, logit - logit[valid].max(), -np.inf)
    p = np.exp(z)
    return p / p.sum()


def test_epsilon_zero_is_the_plain_rollout(oracle32):
    env = grid_env(3, 5)
    w = random_mlp(15, 64, 64, 4, seed=61)
    a = oracle32.rollout(env, w, 7, 1, batch=50)
    b = oracle32.rollout(env, w, 7, 1, batch=50, epsilon=0.0)
    for k in a:
        assert (a[k] == b[k]).all()


@pytest.mark.parametrize("env", [grid_env(3, 5), ising_env(3), bitseq_env(24, 4, 7, mode_seed=2)],
                         ids=["grid", "ising", "bitseq"])
def test_epsilon_one_is_uniform_over_valid_actions(oracle32, oracle64, env):
    """Every action uniform over the valid ones whatever the policy says (a strongly peaked policy here)."""
    sd, od, na, ms = env.dims()
    w = random_mlp(od, 64, 64, na, seed=62, scale=6.0)
    n = 40000
    out = oracle32.rollout(env, w, 8, 0, batch=n, epsilon=1.0, nthreads=8)
    first = out["actions"][0].astype(int)
    valid0 = oracle64.policy(env, {k: v.astype(np.float64) for k, v in w.items()}, [0] * sd if env.kind != 1 else [1 << env.k_bits] * sd)[2]
    counts = np.bincount(first, minlength=na)
    assert (counts[~valid0] == 0).all()
    exp = n / valid0.sum()
    assert chi2_sf(float(((counts[valid0] - exp) ** 2 / exp).sum()), int(valid0.sum()) - 1) > 1e-4
    if env.kind == 0:
        # second step after incrementing coordinate 0 four times is impossible at step 1; use masks instead: walks that
        # reach the wall on coordinate 0 never try to cross it
        acts, length = out["actions"].astype(int), out["length"]
        for b in range(0, n, 400):
            x = np.zeros(3, int)
            for t in range(length[b] - 1):
                assert x[acts[t, b]] < env.grid_side - 1
                x[acts[t, b]] += 1
            assert acts[length[b] - 1, b] == 3
    if env.kind == 2:
        second = out["actions"][1].astype(int)
        assert ((second // 2) != (first // 2)).all()   # an assigned site is never offered again
    # log P_F stays the policy's own log-probability of the actions taken
    rep = oracle32.replay(env, w, 8, 0, out["actions"], out["length"], tie_tol=1e30)
    np.testing.assert_array_equal(rep["log_pf"], out["log_pf"])


def test_mixture_frequencies(oracle32, oracle64):
    """First action ~ (1 - eps) softmax + eps uniform (chi-square); the replay accepts the rollout's own actions
    and flags a changed explored action."""
    env = grid_env(4, 6)
    w = random_mlp(24, 64, 64, 5, seed=63, scale=3.0)
    eps, n = 0.3, 100000
    out = oracle32.rollout(env, w, 9, 2, batch=n, epsilon=eps, nthreads=8)
    logit, _lp, valid = oracle64.policy(env, {k: v.astype(np.float64) for k, v in w.items()}, [0, 0, 0, 0])
    p = (1 - eps) * _softmax(logit, valid) + eps * valid / valid.sum()
    counts = np.bincount(out["actions"][0].astype(int), minlength=5)
    assert chi2_sf(float(((counts - n * p) ** 2 / (n * p)).sum()), 4) > 1e-4
    plain = oracle32.rollout(env, w, 9, 2, batch=n, nthreads=8)
    changed = (plain["actions"][0] != out["actions"][0]).mean()
    assert 0.5 * eps * 0.6 < changed < eps                     # explored draws that differ from the policy's
    sub = slice(0, 3000)
    acts, length = np.ascontiguousarray(out["actions"][:, sub]), np.ascontiguousarray(out["length"][sub])
    rep = oracle32.replay(env, w, 9, 2, acts, length, epsilon=eps, nthreads=8)
    assert (rep["violations"] == 0).all() and (rep["near_ties"] == 0).all()
    rep0 = oracle32.replay(env, w, 9, 2, acts, length, epsilon=0.0, nthreads=8)
    assert (rep0["violations"] > 0).mean() > 0.2                # without the exploration draws many are not the argmax
    # the exploration decision does not depend on the batch split
    part = oracle32.rollout(env, w, 9, 2, batch=100, b_offset=500, epsilon=eps)
    assert (part["actions"] == out["actions"][:, 500:600]).all()


def test_small_epsilon_rate(oracle32):
    """eps = 1e-3 as in the paper's experiments: about one step in a thousand is explored."""
    env = ising_env(4)
    w = random_mlp(48, 64, 64, 32, seed=64)
    n = 4000
    a = oracle32.rollout(env, w, 10, 0, batch=n, nthreads=8)
    b = oracle32.rollout(env, w, 10, 0, batch=n, epsilon=1e-3, nthreads=8)
    first_diff = (a["actions"] != b["actions"]).any(0).mean()    # trajectories that diverged at some step
    assert 0.004 < first_diff < 0.03                              # 16 steps x 1e-3, most explored draws differ
