"""Pins for the counter-based RNG, the uniform/Gumbel mapping and the Gumbel-max sampler of the CPU reference."""
import math
import os

import numpy as np

from tests.helpers import chi2_sf

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "philox4x32_10_kat.txt")
M0, M1, W0, W1 = 0xD2511F53, 0xCD9E8D57, 0x9E3779B9, 0xBB67AE85


def philox_bigint(ctr, key, rounds=10):
    """Philox4x32 written with Python integers from the published round function (independent of oracle/)."""
    c = list(ctr)
    k = list(key)
    for _ in range(rounds):
        p0 = M0 * c[0]
        p1 = M1 * c[2]
        c = [((p1 >> 32) ^ c[1] ^ k[0]) & 0xFFFFFFFF, p1 & 0xFFFFFFFF,
             ((p0 >> 32) ^ c[3] ^ k[1]) & 0xFFFFFFFF, p0 & 0xFFFFFFFF]
        k = [(k[0] + W0) & 0xFFFFFFFF, (k[1] + W1) & 0xFFFFFFFF]
    return c


def read_kat():
    rows = []
    for line in open(GOLDEN):
        if line.startswith("#") or not line.strip():
            continue
        v = [int(x, 16) for x in line.split()]
        rows.append((v[0:4], v[4:6], v[6:10]))
    return rows


def test_philox_known_answers(oracle64):
    rows = read_kat()
    assert len(rows) == 3
    for ctr, key, out in rows:
        assert list(oracle64.philox(ctr, key)) == out
        assert philox_bigint(ctr, key) == out


def test_philox_matches_independent_implementation(oracle32):
    rng = np.random.default_rng(7)
    for _ in range(3000):
        ctr = [int(x) for x in rng.integers(0, 2 ** 32, size=4)]
        key = [int(x) for x in rng.integers(0, 2 ** 32, size=2)]
        assert list(oracle32.philox(ctr, key)) == philox_bigint(ctr, key)
    for b in range(64):  # the structured counters the rollout actually uses
        for t in range(8):
            ctr = [b, t, t % 3, 5]
            assert list(oracle32.philox(ctr, [11, 0])) == philox_bigint(ctr, [11, 0])


def test_philox_words_are_uniform(oracle64):
    words = np.concatenate([oracle64.philox([i, 1, 2, 3], [42, 0]) for i in range(20000)])
    counts = np.bincount((words >> 28).astype(np.int64), minlength=16)
    expected = len(words) / 16
    stat = float(((counts - expected) ** 2 / expected).sum())
    assert chi2_sf(stat, 15) > 1e-4
    for bit in (0, 9, 31):  # single bits balanced
        ones = int(((words >> bit) & 1).sum())
        assert abs(ones - len(words) / 2) < 5 * math.sqrt(len(words) / 4)


def test_uniform_mapping_is_exact_and_open(oracle32, oracle64):
    for w in (0, 1, 511, 512, 0x7FFFFFFF, 0x80000000, 0xFFFFFFFF, 0x12345678):
        exact = ((w >> 9) + 0.5) / 2 ** 23
        assert oracle32.uniform(w) == exact  # representable in binary32: 2k+1 < 2^24
        assert oracle64.uniform(w) == exact
        assert 0.0 < exact < 1.0
    assert oracle32.uniform(0) == 2.0 ** -24
    assert oracle32.uniform(0xFFFFFFFF) == 1.0 - 2.0 ** -24


def test_gumbel_closed_form(oracle32, oracle64):
    for w in (0, 0xFFFFFFFF, 0x80000000, 0x9E3779B9, 12345):
        u = ((w >> 9) + 0.5) / 2 ** 23
        g = -math.log(-math.log(u))
        assert abs(oracle64.gumbel(w) - g) <= 1e-12 * max(1.0, abs(g))
        assert abs(oracle32.gumbel(w) - g) <= 4e-6 * max(1.0, abs(g))
    # median of the standard Gumbel law is -ln ln 2, reached at u = 1/2
    assert abs(oracle64.gumbel(0x80000000) - (-math.log(math.log(2.0)))) < 1e-6


def test_gumbel_max_sampler_follows_softmax(oracle32):
    """Sampled first actions of the rollout follow the masked softmax of the policy (chi-square),
    on a state where one action is masked."""
    from paper_2511_16592_amd.workloads import grid_env, random_mlp
    env = grid_env(3, 2)  # side 2: from the origin all 3 increments + stop are valid
    w = random_mlp(6, 64, 64, 4, seed=5, scale=3.0)
    n = 40000
    out = oracle32.rollout(env, w, seed=123, iteration=9, batch=n, nthreads=8)
    _, logp, valid = oracle32.policy(env, w, [0, 0, 0])
    assert valid.all()
    counts = np.bincount(out["actions"][0], minlength=4)[:4]
    expected = np.exp(logp.astype(np.float64)) * n
    stat = float(((counts - expected) ** 2 / expected).sum())
    assert chi2_sf(stat, 3) > 1e-4
    # second step after action 0: coordinate 0 is at side-1 = 1, so action 0 must never be sampled
    first0 = out["actions"][0] == 0
    assert first0.sum() > 100
    second = out["actions"][1][first0]
    assert (second != 0).all()
    _, logp1, valid1 = oracle32.policy(env, w, [1, 0, 0])
    assert not valid1[0] and valid1[1:].all()
    counts1 = np.bincount(second, minlength=4)[1:4]
    expected1 = np.exp(logp1[1:].astype(np.float64)) * first0.sum()
    stat1 = float(((counts1 - expected1) ** 2 / expected1).sum())
    assert chi2_sf(stat1, 2) > 1e-4
