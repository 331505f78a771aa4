"""Pins for the non-autoregressive bit-sequence environment of the CPU reference (Appendix "Sequential
environments", non-autoregressive scheme; Appendix "Bit sequences": an action picks an empty position and a k-bit
word, the backward policy removes the word of a filled position)."""
import itertools
import math

import numpy as np

from paper_2511_16592_amd.workloads import bitseq_env, bitseq_na_env, random_mlp
from tests.helpers import chi2_sf


def _all_trajectories(length, k):
    """Every complete action sequence: an order of the positions and a word for each."""
    out = []
    for order in itertools.permutations(range(length)):
        for words in itertools.product(range(1 << k), repeat=length):
            out.append([(pos << k) + words[pos] for pos in order])
    return out


def _pack(trajs, length):
    actions = np.array(trajs, dtype=np.uint8).T.copy()  # [steps, batch]
    return actions, np.full(len(trajs), length, dtype=np.int32)


def test_dims_and_structure(oracle32):
    env = bitseq_na_env(24, 4, 5, mode_seed=2)
    assert oracle32.env_dims(env) == (6, 6 * 17, 6 * 16, 6) == env.dims()
    w = random_mlp(6 * 17, 32, 32, 96, seed=5, scale=2.0)
    out = oracle32.rollout(env, w, seed=3, iteration=0, batch=200, nthreads=4)
    assert (out["length"] == 6).all()
    acts = out["actions"].astype(int)
    pos, word = acts >> 4, acts & 15
    assert (np.sort(pos, axis=0) == np.arange(6)[:, None]).all()  # every position filled exactly once
    for b in range(200):  # the terminal string holds the word written at each position
        assert (out["terminal_state"][pos[:, b], b] == word[:, b]).all()
    assert np.allclose(out["log_pb"], -math.lgamma(7), rtol=1e-6)  # uniform over filled positions: -log 6!
    # positions are visited in many different orders (not left to right)
    assert len({tuple(pos[:, b]) for b in range(200)}) > 100


def test_exhaustive_enumeration_small(oracle64):
    """n = 6 bits, k = 2: 3 positions x 4 words = 12 actions, 3! * 4^3 = 384 complete trajectories, 64 strings.
    For any network: sum_tau P_F(tau) = 1; every string is reached by 3! orders with P_B(tau | x) = 1/3! each, so
    sum over its trajectories of P_B = 1; the reward does not depend on the order and equals the reward the
    left-to-right environment (pinned on its own) gives the same string."""
    length, k = 3, 2
    env = bitseq_na_env(6, 2, 4, mode_seed=7, uniform_bits=True)
    ar = bitseq_env(6, 2, 4, mode_seed=7, uniform_bits=True)
    w = random_mlp(3 * 5, 16, 16, 12, seed=9, scale=2.5, dtype=np.float64)
    trajs = _all_trajectories(length, k)
    assert len(trajs) == 384
    actions, lengths = _pack(trajs, length)
    r = oracle64.replay(env, w, 0, 0, actions, lengths, tie_tol=1e30, nthreads=4)
    assert (r["violations"] == 0).all()
    assert abs(np.exp(r["log_pf"]).sum() - 1.0) < 1e-12
    assert np.allclose(r["log_pb"], -math.log(6.0), atol=1e-12)
    by_string = {}
    for b, t in enumerate(trajs):
        x = tuple(int(v) for v in r["terminal_state"][:, b])
        by_string.setdefault(x, []).append(b)
    assert len(by_string) == 64 and all(len(v) == 6 for v in by_string.values())
    for x, cols in by_string.items():
        assert abs(np.exp(r["log_pb"][cols]).sum() - 1.0) < 1e-12
        assert np.ptp(r["log_reward"][cols]) == 0.0
        assert r["log_reward"][cols[0]] == oracle64.log_reward(ar, list(x)) == oracle64.log_reward(env, list(x))
    # a filled position is masked: writing to it again is a violation of the replay
    bad = actions.copy()
    bad[1, 0] = bad[0, 0] ^ 1  # same position as step 0, another word
    assert oracle64.replay(env, w, 0, 0, bad, lengths, tie_tol=1e30)["violations"][0] >= 1


def test_masked_policy_and_sampler(oracle32, oracle64):
    """At a state with positions 0 and 2 filled only the four words of position 1 are valid and carry all the
    probability; sampled first actions follow the softmax over all 12 actions (chi-square)."""
    env = bitseq_na_env(6, 2, 4, mode_seed=7, uniform_bits=True)
    w = random_mlp(15, 16, 16, 12, seed=9, scale=2.5)
    logit, logp, valid = oracle64.policy(env, {k: v.astype(np.float64) for k, v in w.items()}, [3, 4, 0])
    assert list(np.flatnonzero(valid)) == [4, 5, 6, 7]
    assert abs(np.exp(logp[valid]).sum() - 1.0) < 1e-12
    lg = logit[4:8]
    assert np.allclose(logp[4:8], lg - np.log(np.exp(lg - lg.max()).sum()) - lg.max(), atol=1e-12)
    n = 40000
    out = oracle32.rollout(env, w, seed=11, iteration=2, batch=n, nthreads=8)
    _, logp0, valid0 = oracle64.policy(env, {k: v.astype(np.float64) for k, v in w.items()}, [4, 4, 4])
    assert valid0.all()
    counts = np.bincount(out["actions"][0].astype(int), minlength=12)
    expected = np.exp(logp0) * n
    assert chi2_sf(float(((counts - expected) ** 2 / expected).sum()), 11) > 1e-4


def test_gradient_finite_differences(oracle64):
    env = bitseq_na_env(8, 2, 3, mode_seed=5, uniform_bits=True)
    w = random_mlp(4 * 5, 24, 24, 16, seed=12, scale=2.0, dtype=np.float64)
    out = oracle64.rollout(env, w, seed=4, iteration=1, batch=5)
    actions, length = out["actions"], out["length"]
    g = oracle64.tb_loss_grad(env, w, actions, length, log_z=0.3)
    delta = 0.3 + out["log_pf"] - out["log_reward"] - out["log_pb"]
    assert np.allclose(g["delta"], delta, rtol=1e-12, atol=1e-12)
    rng = np.random.default_rng(3)
    eps = 1e-6
    for k in ("W1", "b1", "W2", "b2", "W3", "b3"):
        grad = g["d" + k]
        flat = np.flatnonzero(np.abs(grad.ravel()) > 0)
        for i in rng.choice(flat, size=min(5, flat.size), replace=False):
            wp = {q: v.copy() for q, v in w.items()}
            wm = {q: v.copy() for q, v in w.items()}
            wp[k].ravel()[i] += eps
            wm[k].ravel()[i] -= eps
            fd = (oracle64.tb_loss_grad(env, wp, actions, length, log_z=0.3)["loss"] -
                  oracle64.tb_loss_grad(env, wm, actions, length, log_z=0.3)["loss"]) / (2 * eps)
            assert abs(fd - grad.ravel()[i]) <= 2e-5 * max(1.0, abs(fd)), (k, i)


def test_backward_rollout_reverses_forward(oracle64):
    """A backward rollout from a terminal string removes one filled position at a time (uniformly); replayed
    forwards its actions rebuild the string, with log P_B = -log L! whatever the order."""
    env = bitseq_na_env(10, 2, 3, mode_seed=5, uniform_bits=True)
    rng = np.random.default_rng(1)
    states = rng.integers(0, 4, size=(5, 300)).astype(np.int8)
    back = oracle64.backward_rollout(env, seed=8, iteration=0, terminal_state=states)
    assert (back["length"] == 5).all() and np.allclose(back["log_pb"], -math.lgamma(6))
    w = random_mlp(5 * 5, 16, 16, 20, seed=2, dtype=np.float64)
    fwd = oracle64.replay(env, w, 0, 0, back["actions"], back["length"], tie_tol=1e30)
    assert (fwd["violations"] == 0).all() and (fwd["terminal_state"] == states).all()
    first_removed = back["actions"][-1].astype(int) >> 2  # the last forward action is the first backward move
    counts = np.bincount(first_removed, minlength=5)
    assert chi2_sf(float(((counts - 60.0) ** 2 / 60.0).sum()), 4) > 1e-4


def test_more_than_256_actions(oracle32, oracle64):
    """n = 16, k = 8: two positions x 256 words = 512 actions, which no longer fit one byte: the action plane is
    16 bits wide there.  Structure of sampled trajectories, both steps of the policy against a dense numpy forward
    pass with the mask written out, first and second actions by chi-square (marginals over position and over the top
    bits of the word), the reward against the left-to-right environment, replay of the rollout's own actions, and
    backward rollouts."""
    env = bitseq_na_env(16, 8, 3, mode_seed=9)
    ar = bitseq_env(16, 8, 3, mode_seed=9)
    assert oracle32.env_dims(env) == (2, 2 * 257, 512, 2) == env.dims()
    w = random_mlp(514, 16, 16, 512, seed=21, scale=3.0)
    w64 = {k: v.astype(np.float64) for k, v in w.items()}
    n = 30000
    out = oracle32.rollout(env, w, seed=5, iteration=1, batch=n, nthreads=8)
    acts = out["actions"]
    assert acts.dtype == np.uint16 and acts.max() > 255 and acts.max() < 512
    pos, word = acts.astype(int) >> 8, acts.astype(int) & 255
    assert (pos[0] != pos[1]).all() and (out["length"] == 2).all()
    ts = out["terminal_state"].view(np.uint8).astype(int)
    assert (ts[pos[0], np.arange(n)] == word[0]).all() and (ts[pos[1], np.arange(n)] == word[1]).all()
    assert np.allclose(out["log_pb"], -math.log(2.0), rtol=1e-6)
    for b in range(0, n, 1500):
        x = [int(v) for v in ts[:, b]]
        assert abs(out["log_reward"][b] - oracle64.log_reward(ar, x)) < 1e-5
    # the policy at s_0 and after the first action, from a dense forward pass
    def dense_logp(state):  # state: word per position or None
        x = np.zeros(514)
        for p, v in enumerate(state):
            x[257 * p + (256 if v is None else v)] = 1.0
        h1 = np.maximum(x @ w64["W1"] + w64["b1"], 0)
        h2 = np.maximum(h1 @ w64["W2"] + w64["b2"], 0)
        lg = h2 @ w64["W3"] + w64["b3"]
        valid = np.array([state[a >> 8] is None for a in range(512)])
        lg = np.where(valid, lg, -np.inf)
        return lg - (np.log(np.exp(lg - lg.max()).sum()) + lg.max()), valid
    lp0, v0 = dense_logp([None, None])
    assert v0.all()
    _, logp, valid = oracle64.policy(env, w64, [256, 256])
    assert valid.all() and np.allclose(logp, lp0, atol=1e-12)
    lp1, v1 = dense_logp([None, 77])
    _, logp, valid = oracle64.policy(env, w64, [256, 77])
    assert (valid == v1).all() and valid[:256].all() and not valid[256:].any()
    assert np.allclose(logp[:256], lp1[:256], atol=1e-12)
    # first actions: chi-square over 32 bins (position x top 4 bits of the word)
    bins0 = np.bincount((acts[0].astype(int) >> 4), minlength=32)
    want0 = np.exp(lp0).reshape(32, 16).sum(1) * n
    assert chi2_sf(float(((bins0 - want0) ** 2 / want0).sum()), 31) > 1e-4
    # log P_F of the sampled trajectories against the dense pass (a sample of them)
    for b in range(0, n, 3000):
        st = [None, None]
        lp = dense_logp(st)[0][acts[0, b]]
        st[pos[0, b]] = word[0, b]
        lp += dense_logp(st)[0][acts[1, b]]
        assert abs(lp - out["log_pf"][b]) < 2e-4 * max(1.0, abs(lp))
    # replay of the rollout's own actions: no violation, same scalars; a second write to the same position is one
    sub = np.ascontiguousarray(acts[:, :200])
    rep = oracle32.replay(env, w, 5, 1, sub, out["length"][:200], tie_tol=1e-5, nthreads=4)
    assert (rep["violations"] == 0).all() and (rep["near_ties"] == 0).all()
    assert np.array_equal(rep["log_pf"], out["log_pf"][:200])
    bad = sub.copy()
    bad[1, 0] = bad[0, 0] ^ 1
    assert oracle32.replay(env, w, 5, 1, bad, out["length"][:200], tie_tol=1e-5)["violations"][0] >= 1
    # gradient along these actions: finite differences on a few entries of every tensor
    g = oracle64.tb_loss_grad(env, w64, sub[:, :6], out["length"][:6], log_z=0.1)
    rng = np.random.default_rng(8)
    for k in ("W1", "b1", "W2", "b2", "W3", "b3"):
        grad = g["d" + k]
        flat = np.flatnonzero(np.abs(grad.ravel()) > 0)
        for i in rng.choice(flat, size=min(3, flat.size), replace=False):
            wp = {q: v.copy() for q, v in w64.items()}
            wm = {q: v.copy() for q, v in w64.items()}
            wp[k].ravel()[i] += 1e-6
            wm[k].ravel()[i] -= 1e-6
            fd = (oracle64.tb_loss_grad(env, wp, sub[:, :6], out["length"][:6], log_z=0.1)["loss"] -
                  oracle64.tb_loss_grad(env, wm, sub[:, :6], out["length"][:6], log_z=0.1)["loss"]) / 2e-6
            assert abs(fd - grad.ravel()[i]) <= 2e-5 * max(1.0, abs(fd)), (k, i)
    # backward rollouts: 16-bit actions, reversible
    states = np.random.default_rng(2).integers(0, 256, size=(2, 400)).astype(np.uint8).view(np.int8)
    back = oracle64.backward_rollout(env, seed=3, iteration=0, terminal_state=states)
    assert back["actions"].dtype == np.uint16 and np.allclose(back["log_pb"], -math.log(2.0))
    fwd = oracle64.replay(env, w64, 0, 0, back["actions"], back["length"], tie_tol=1e30)
    assert (fwd["violations"] == 0).all() and (fwd["terminal_state"] == states).all()
    assert 140 < int((back["actions"][1].astype(int) >> 8).sum()) < 260   # either position is removed first


def test_uniform_exploration_beyond_256_actions(oracle32):
    """epsilon = 1 on the 512-action instance: every step is uniform over the valid actions whatever the policy -- the
    first action over all 512, the second over the 256 words of the other position -- and the explored action is the
    j-th valid one in increasing order, j = floor(w n / 2^32) (the integer rule both sides implement)."""
    env = bitseq_na_env(16, 8, 3, mode_seed=9)
    w = random_mlp(514, 16, 16, 512, seed=22, scale=4.0)
    n = 40000
    out = oracle32.rollout(env, w, seed=6, iteration=0, batch=n, nthreads=8, epsilon=1.0)
    a0, a1 = out["actions"][0].astype(int), out["actions"][1].astype(int)
    c0 = np.bincount(a0 >> 4, minlength=32)                      # 32 bins of 16 actions
    assert chi2_sf(float(((c0 - n / 32) ** 2 / (n / 32)).sum()), 31) > 1e-4
    assert ((a1 >> 8) != (a0 >> 8)).all()                        # the filled position is masked
    c1 = np.bincount(a1 & 255, minlength=256)
    assert chi2_sf(float(((c1 - n / 256) ** 2 / (n / 256)).sum()), 255) > 1e-4
    # the plain policy is far from uniform with these weights, so the above is the exploration's doing
    plain = oracle32.rollout(env, w, seed=6, iteration=0, batch=n, nthreads=8)
    cp = np.bincount(plain["actions"][0].astype(int) >> 4, minlength=32)
    assert chi2_sf(float(((cp - n / 32) ** 2 / (n / 32)).sum()), 31) < 1e-6
