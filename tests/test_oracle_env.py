"""Pins for the environments, rewards, backward-policy terms and trajectory bookkeeping of the CPU reference."""
import itertools
import math

import numpy as np
import pytest

from paper_2511_16592_amd.workloads import (ENV_BITSEQ, EnvSpec, bitseq_env, bitseq_modes, grid_env, ising_env,
                                            pack_bits, random_mlp, workloads, xavier_mlp)
from tests.helpers import enumerate_grid_trajectories, grid_reward, pack_trajectories


def test_env_dims_match_the_configurations(oracle64):
    expect = {"c1": (2, 16, 3, 15), "c2": (4, 80, 5, 77), "c3": (15, 3855, 256, 15),
              "c4": (100, 300, 200, 100), "c5": (10, 200, 11, 191)}
    for name, dims in expect.items():
        env = workloads()[name].env
        assert oracle64.env_dims(env) == dims
        assert env.dims() == dims


# ---------------------------------------------------------------- hypergrid
@pytest.mark.parametrize("dim,side,z", [(2, 4, 2.016), (2, 8, 16.064)])
def test_grid_partition_function_closed_form(oracle64, dim, side, z):
    """Z = R0*H^d + R1*n1^d + R2*n2^d (band sizes n1, n2), against brute force over all states."""
    total = 0.0
    for x in itertools.product(range(side), repeat=dim):
        lr = oracle64.log_reward(grid_env(dim, side), x)
        assert abs(lr - math.log(grid_reward(x, side))) < 1e-12
        total += math.exp(lr)
    assert abs(total - z) < 1e-9


def test_grid_reward_bands_side20(oracle32, oracle64):
    """Side 20: middle band {0..4,15..19}, inner band {2,3,16,17}; Z(4-D) = 5672, Z(10-D) = 15242097152."""
    env1 = grid_env(1, 20)
    vals = {x: oracle64.log_reward(env1, [x]) for x in range(20)}
    for x in range(20):
        want = 1e-3 + 0.5 * (x <= 4 or x >= 15) + 2.0 * (x in (2, 3, 16, 17))
        assert abs(vals[x] - math.log(want)) < 1e-12
        assert abs(oracle32.log_reward(env1, [x]) - math.log(want)) < 1e-6
    n1, n2 = 10, 4
    assert abs(1e-3 * 20 ** 4 + 0.5 * n1 ** 4 + 2.0 * n2 ** 4 - 5672) < 1e-9
    assert abs(1e-3 * 20 ** 10 + 0.5 * n1 ** 10 + 2.0 * n2 ** 10 - 15242097152) < 1e-3
    # a product over coordinates: one coordinate outside the band removes the term
    env4 = grid_env(4, 20)
    assert abs(oracle64.log_reward(env4, [2, 3, 16, 17]) - math.log(2.501)) < 1e-12
    assert abs(oracle64.log_reward(env4, [2, 3, 16, 4]) - math.log(0.501)) < 1e-12
    assert abs(oracle64.log_reward(env4, [2, 3, 16, 10]) - math.log(1e-3)) < 1e-12


def test_grid_threshold_is_strict_side5(oracle32, oracle64):
    """Side 5: x=1 and x=3 sit exactly on |x/4 - 0.5| = 0.25; the inequality is strict, so they earn R0 only."""
    env = grid_env(3, 5)
    for o in (oracle32, oracle64):
        assert abs(o.log_reward(env, [1, 0, 0]) - math.log(1e-3)) < 1e-6
        assert abs(o.log_reward(env, [3, 4, 0]) - math.log(1e-3)) < 1e-6
        assert abs(o.log_reward(env, [0, 4, 0]) - math.log(0.501)) < 1e-6


def test_grid_reward_is_exact_on_every_threshold(oracle32, oracle64):
    """Whenever H-1 is a multiple of 4, 5 or 10 some coordinate sits exactly on 1/4, 3/10 or 2/5 of the reward
    equation's strict inequalities (side 11: x = 2, 8 on 0.3 and x = 1, 9 on 0.4), where rounding of x/(H-1) - 0.5
    would decide the indicator.  Both builds must give the value of the equation evaluated in exact rationals, for
    every coordinate of every side from 2 to 127 and for products over two coordinates on the sides with thresholds."""
    for side in range(2, 128):
        env1 = grid_env(1, side)
        for x in range(side):
            want = math.log(grid_reward((x,), side))
            assert abs(oracle64.log_reward(env1, [x]) - want) < 1e-12, (side, x)
            assert abs(oracle32.log_reward(env1, [x]) - want) < 1e-6, (side, x)
    for side in (5, 6, 11, 21):
        env2 = grid_env(2, side)
        for x in range(side):
            for y in range(side):
                want = math.log(grid_reward((x, y), side))
                assert abs(oracle64.log_reward(env2, [x, y]) - want) < 1e-12, (side, x, y)
                assert abs(oracle32.log_reward(env2, [x, y]) - want) < 1e-6, (side, x, y)
    # the edge cells of the side-11 grid named above: on the threshold means outside the band
    assert abs(oracle64.log_reward(grid_env(2, 11), [9, 9]) - math.log(0.501)) < 1e-12
    assert abs(oracle64.log_reward(grid_env(2, 11), [8, 8]) - math.log(0.501)) < 1e-12
    assert abs(oracle32.log_reward(grid_env(2, 11), [9, 9]) - math.log(0.501)) < 1e-6
    assert abs(oracle32.log_reward(grid_env(2, 11), [8, 8]) - math.log(0.501)) < 1e-6


def test_worked_example_of_the_paper(oracle64):
    """Usage listing in "Library Details": dim 3, side 5; action 0 is not terminal and earns log-reward 0,
    the stop action is the LAST index and yields the log-reward of the state reached, here (1,0,0)."""
    env = grid_env(3, 5)
    w = random_mlp(15, 64, 64, 4, seed=1)
    actions = np.full((13, 1), 0xFF, dtype=np.uint8)
    actions[0, 0], actions[1, 0] = 0, 3
    r = oracle64.replay(env, w, 0, 0, actions, np.array([2]), tie_tol=1e30)
    assert r["violations"][0] == 0
    assert list(r["terminal_state"][:, 0]) == [1, 0, 0]
    assert abs(r["log_reward"][0] - oracle64.log_reward(env, [1, 0, 0])) == 0
    # a one-step sequence [0] does not reach a terminal state: flagged
    r1 = oracle64.replay(env, w, 0, 0, actions, np.array([1]), tie_tol=1e30)
    assert r1["violations"][0] == 1 and r1["log_reward"][0] == 0.0
    # stopping immediately is allowed and terminal
    actions[0, 0] = 3
    r2 = oracle64.replay(env, w, 0, 0, actions, np.array([1]), tie_tol=1e30)
    assert r2["violations"][0] == 0 and list(r2["terminal_state"][:, 0]) == [0, 0, 0]


def test_grid_enumeration_side4(oracle64):
    """2-D side-4 grid: exactly C(8,4)-1 = 69 complete trajectories; for ANY weights the forward
    trajectory distribution sums to 1 and so does the induced terminal distribution."""
    env = grid_env(2, 4)
    trajs = enumerate_grid_trajectories(2, 4)
    assert len(trajs) == 69 == math.comb(8, 4) - 1
    assert len({x for _a, x in trajs}) == 16
    actions, length = pack_trajectories(trajs, 7)
    for seed in (1, 2):
        w = random_mlp(8, 64, 64, 3, seed=seed, scale=4.0, dtype=np.float64)
        r = oracle64.replay(env, w, 0, 0, actions, length, tie_tol=1e30)
        assert (r["violations"] == 0).all()
        p = np.exp(r["log_pf"])
        assert abs(p.sum() - 1.0) < 1e-12
        term = {}
        for b, (_a, x) in enumerate(trajs):
            assert tuple(r["terminal_state"][:, b]) == x
            assert length[b] == sum(x) + 1
            term[x] = term.get(x, 0.0) + p[b]
        assert abs(sum(term.values()) - 1.0) < 1e-12
        # backward trajectory distribution: sum over trajectories ending in x of prod P_B equals 1
        pb = {}
        for b, (_a, x) in enumerate(trajs):
            pb[x] = pb.get(x, 0.0) + math.exp(r["log_pb"][b])
        for x, v in pb.items():
            assert abs(v - 1.0) < 1e-12


def test_grid_mask_blocks_leaving_the_grid(oracle64):
    env = grid_env(2, 4)
    w = random_mlp(8, 64, 64, 3, seed=3, dtype=np.float64)
    _, logp, valid = oracle64.policy(env, w, [3, 1])
    assert list(valid) == [False, True, True]
    assert abs(np.exp(logp[valid]).sum() - 1.0) < 1e-12
    actions = np.full((7, 1), 0xFF, dtype=np.uint8)
    actions[:5, 0] = [0, 0, 0, 0, 2]  # fourth increment of coordinate 0 would leave the grid
    r = oracle64.replay(env, w, 0, 0, actions, np.array([5]), tie_tol=1e30)
    assert r["violations"][0] == 1


def test_policy_matches_dense_one_hot_matmul(oracle64):
    """The policy network on the one-hot observation equals a dense numpy evaluation with the
    stated index layouts (grid H*i+x, bitseq 257*pos+tok, Ising 3*site+x+1)."""
    cases = [
        (grid_env(3, 5), [2, 0, 4], lambda s: [5 * i + s[i] for i in range(3)]),
        (bitseq_env(24, 8, 4, mode_seed=1), [17, 255, 256], lambda s: [257 * i + s[i] for i in range(3)]),
        (ising_env(3), [0, 1, -1, 0, 0, 1, 0, 0, -1], lambda s: [3 * i + s[i] + 1 for i in range(9)]),
    ]
    for env, state, rows in cases:
        _, od, na, _ = env.dims()
        w = random_mlp(od, 64, 64, na, seed=9, scale=2.0, dtype=np.float64)
        x = np.zeros(od)
        x[rows(state)] = 1.0
        h1 = np.maximum(x @ w["W1"] + w["b1"], 0)
        h2 = np.maximum(h1 @ w["W2"] + w["b2"], 0)
        logits = h2 @ w["W3"] + w["b3"]
        got, logp, valid = oracle64.policy(env, w, state)
        assert np.allclose(got, logits, rtol=1e-12, atol=1e-12)
        lse = np.log(np.exp(logits[valid]).sum())
        assert np.allclose(logp[valid], logits[valid] - lse, rtol=1e-12, atol=1e-12)


# ---------------------------------------------------------------- bit sequences
def test_bitseq_reward_closed_forms(oracle32, oracle64):
    bits = bitseq_modes(120, 60, seed=3)
    assert bits.shape == (60, 120)
    # every mode is a concatenation of the five 8-bit blocks
    blocks = {"00000000", "11111111", "11110000", "00001111", "00111100"}
    for m in range(60):
        for p in range(15):
            assert "".join(str(int(v)) for v in bits[m, 8 * p:8 * p + 8]) in blocks
    env = bitseq_env(120, 8, 60, mode_seed=3)

    def tokens(row):  # MSB-first tokens of a 0/1 string
        return [int("".join(str(int(v)) for v in row[8 * p:8 * p + 8]), 2) for p in range(15)]

    dist = (bits[:, None, :] != bits[None, :, :]).sum(-1)
    np.fill_diagonal(dist, 999)
    for m in (0, 7, 59):
        assert oracle64.log_reward(env, tokens(bits[m])) == 0.0
        far = int(dist[m].min())
        for j in (1, 2, 3):
            if 2 * j >= far:
                continue
            x = bits[m].copy()
            x[[5, 50, 119][:j]] ^= 1
            assert abs(oracle64.log_reward(env, tokens(x)) - (-j / 40.0)) < 1e-12
            assert abs(oracle32.log_reward(env, tokens(x)) - (-j / 40.0)) < 1e-6


def test_bitseq_reward_brute_force_small(oracle64):
    """n=8, k=4, two modes: all 256 strings against a direct Hamming-distance evaluation."""
    modes = np.array([[1, 0, 1, 1, 0, 0, 1, 0], [0, 0, 0, 1, 1, 1, 1, 0]], dtype=np.uint8)
    env = EnvSpec(kind=ENV_BITSEQ, n_bits=8, k_bits=4, modes=pack_bits(modes), beta=3.0)
    for v in range(256):
        s = [(v >> (7 - i)) & 1 for i in range(8)]
        toks = [int("".join(map(str, s[0:4])), 2), int("".join(map(str, s[4:8])), 2)]
        dmin = min(int((np.array(s) != modes[m]).sum()) for m in range(2))
        assert abs(oracle64.log_reward(env, toks) - (-3.0 * dmin / 8)) < 1e-12


def test_bitseq_rollout_structure(oracle32):
    env = bitseq_env(120, 8, 60, mode_seed=3)
    w = xavier_mlp(3855, 64, 64, 256, seed=3)
    out = oracle32.rollout(env, w, seed=3, iteration=0, batch=6)
    assert (out["length"] == 15).all()
    assert (out["log_pb"] == 0).all()
    # left-to-right: terminal token at position t is the t-th action
    assert (out["terminal_state"].view(np.uint8) == out["actions"]).all()
    for b in range(6):
        toks = [int(v) for v in out["terminal_state"].view(np.uint8)[:, b]]
        assert abs(out["log_reward"][b] - oracle32.log_reward(env, toks)) == 0


# ---------------------------------------------------------------- Ising
def test_ising_reward_closed_forms(oracle32, oracle64):
    env = ising_env(10)
    up = [1] * 100
    assert abs(oracle64.log_reward(env, up) - 88.0) < 1e-9
    assert abs(oracle64.log_reward(env, [-1] * 100) - 88.0) < 1e-9
    checker = [1 if (r + c) % 2 == 0 else -1 for r in range(10) for c in range(10)]
    assert abs(oracle64.log_reward(env, checker) + 88.0) < 1e-9
    flipped = list(up)
    flipped[37] = -1
    assert abs(oracle64.log_reward(env, flipped) - 0.44 * 192) < 1e-9
    assert abs(oracle32.log_reward(env, flipped) - 0.44 * 192) < 1e-4
    # against x^T J x with J = (coupling/2) * adjacency of the torus (every bond counted twice there)
    rng = np.random.default_rng(0)
    adj = np.zeros((100, 100))
    for r in range(10):
        for c in range(10):
            i = r * 10 + c
            for j in (r * 10 + (c + 1) % 10, ((r + 1) % 10) * 10 + c):
                adj[i, j] = adj[j, i] = 1
    assert (adj.sum(1) == 4).all()
    for _ in range(5):
        x = rng.choice([-1, 1], size=100)
        assert abs(oracle64.log_reward(env, x) - x @ (0.22 * adj) @ x) < 1e-9


def test_ising_rollout_structure(oracle32):
    env = ising_env(10)
    w = xavier_mlp(300, 64, 64, 200, seed=4)
    out = oracle32.rollout(env, w, seed=4, iteration=0, batch=5)
    assert (out["length"] == 100).all()
    assert np.allclose(out["log_pb"], -math.lgamma(101), rtol=2e-6)  # -log 100!
    assert abs(-math.lgamma(101) + 363.7393756) < 1e-6
    for b in range(5):
        sites = out["actions"][:, b] // 2
        assert sorted(sites) == list(range(100))  # every site assigned exactly once (mask works)
        spins = 2 * (out["actions"][:, b] % 2).astype(int) - 1
        x = np.zeros(100, dtype=int)
        x[sites] = spins
        assert (out["terminal_state"][:, b] == x).all()
        assert abs(out["log_reward"][b] - oracle32.log_reward(env, x)) == 0


# ---------------------------------------------------------------- bookkeeping
def test_rollout_padding_and_independence_of_batch_split(oracle32):
    """Trajectory b depends only on (seed, iteration, b): sampling columns 3..7 alone reproduces them;
    bytes after the end of a trajectory are 0xFF; a different iteration gives different trajectories."""
    env = grid_env(2, 8)
    w = xavier_mlp(16, 64, 64, 3, seed=1)
    full = oracle32.rollout(env, w, seed=0, iteration=0, batch=16)
    part = oracle32.rollout(env, w, seed=0, iteration=0, batch=5, b_offset=3)
    assert (full["actions"][:, 3:8] == part["actions"]).all()
    assert (full["log_pf"][3:8] == part["log_pf"]).all()
    for b in range(16):
        n = full["length"][b]
        assert full["actions"][n - 1, b] == 2 and (full["actions"][n:, b] == 0xFF).all()
        assert (full["actions"][:n - 1, b] < 2).all()
        assert n == full["terminal_state"][:, b].sum() + 1
    other = oracle32.rollout(env, w, seed=0, iteration=1, batch=16)
    assert (other["actions"] != full["actions"]).any()
    threaded = oracle32.rollout(env, w, seed=0, iteration=0, batch=16, nthreads=4)
    for k in ("actions", "length", "log_pf", "log_pb", "log_reward"):
        assert (threaded[k] == full[k]).all()


def test_replay_reproduces_free_run_and_flags_wrong_actions(oracle32):
    env = grid_env(4, 20)
    w = xavier_mlp(80, 64, 64, 5, seed=2)
    out = oracle32.rollout(env, w, seed=2, iteration=3, batch=64)
    r = oracle32.replay(env, w, 2, 3, out["actions"], out["length"])
    assert (r["violations"] == 0).all() and (r["near_ties"] == 0).all()
    for k in ("log_pf", "log_pb", "log_reward", "terminal_state"):
        assert (r[k] == out[k]).all()
    # planted mistake: change one sampled action to another valid one -> reported as a violation
    bad = out["actions"].copy()
    b = int(np.argmax(out["length"] >= 2))
    bad[0, b] = (bad[0, b] + 1) % 4
    r2 = oracle32.replay(env, w, 2, 3, bad, out["length"])
    assert r2["violations"][b] >= 1
    assert (np.delete(r2["violations"], b) == 0).all()


def test_replay_near_tie_margin_is_absolute_on_the_perturbed_logits(oracle32):
    """The near-tie rule of the replay: an action other than the argmax is a near tie iff its perturbed logit is
    within tie_tol (absolute) of the best one, otherwise a violation.  One-step bit sequences (a single 4-bit token,
    16 actions, no mask): the perturbed logits are rebuilt here from the policy's logits, an independent big-integer
    Philox and numpy's binary32 logarithm; the runner-up is handed to the replay with tie_tol just above and just
    below the gap.  A comparison on the raw logits, a relative one, or one against another operand fails this."""
    from tests.test_oracle_rng import philox_bigint
    env = bitseq_env(4, 4, 3, mode_seed=5, uniform_bits=True)
    w = random_mlp(17, 32, 32, 16, seed=51, scale=3.0)
    seed, iteration, batch = 77, 6, 24
    out = oracle32.rollout(env, w, seed=seed, iteration=iteration, batch=batch)
    assert (out["length"] == 1).all()
    logits, _, valid = oracle32.policy(env, w, [16])  # the empty string: the state of step 0
    assert valid.all()
    checked = 0
    for b in range(batch):
        pert = np.zeros(16, dtype=np.float32)
        for a in range(16):
            word = philox_bigint([b, 0, a // 4, iteration], [seed, 0])[a % 4]
            u = np.float32((word >> 9) + 0.5) * np.float32(2.0 ** -23)
            pert[a] = np.float32(logits[a]) + (-np.log(-np.log(u, dtype=np.float32), dtype=np.float32))
        order = np.argsort(-pert, kind="stable")
        best, second = int(order[0]), int(order[1])
        gap = float(pert[best] - pert[second])
        assert out["actions"][0, b] == best
        assert abs(out["min_margin"][b] - gap) <= 2e-6
        if gap < 1e-4 or abs(abs(float(pert[best])) - 1.0) < 0.2:
            continue  # keep clear of rounding in the gap itself, and of |best| ~ 1 where relative = absolute
        raw_gap = float(logits[best] - logits[second])
        given = out["actions"].copy()
        given[0, b] = second
        above = oracle32.replay(env, w, seed, iteration, given, out["length"], tie_tol=gap * 1.01)
        below = oracle32.replay(env, w, seed, iteration, given, out["length"], tie_tol=gap * 0.99)
        assert above["near_ties"][b] == 1 and above["violations"][b] == 0, (b, gap, raw_gap)
        assert below["near_ties"][b] == 0 and below["violations"][b] == 1, (b, gap, raw_gap)
        others = np.arange(batch) != b
        assert (above["near_ties"][others] == 0).all() and (above["violations"][others] == 0).all()
        # the third-best action is further away than the runner-up: a violation under the same tolerance
        given[0, b] = int(order[2])
        if float(pert[best] - pert[order[2]]) > gap * 1.02:
            third = oracle32.replay(env, w, seed, iteration, given, out["length"], tie_tol=gap * 1.01)
            assert third["near_ties"][b] == 0 and third["violations"][b] == 1
        checked += 1
    assert checked >= 12
