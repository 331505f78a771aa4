"""GPU parity of the optimiser step and of whole training iterations against the CPU reference.

Bars (written out here):
  * Adam on the SAME gradient sequence on both sides, binary64 reference: every parameter within
    1e-4 * (number of updates) * lr of the reference plus 4 ulp of its own binary32 value; the moments within
    1e-4 of their tensor's scale (max |g|, max g^2);
  * the fused iteration: bit-identical to the three calls it is made of;
  * a training iteration against the reference chain (replay of the GPU's actions, binary64 loss / gradient /
    Adam): the gradient bar of the parity tests gives the GPU's gradient an interval of half-width
    tau = 1e-4 * max |g| + 1e-7 around the reference's, and the updated parameter must lie in the image of that
    interval under the update (the update divides by sqrt(v), so near g = 0 it is as steep as lr / tau: a
    float-decided value like the near-tie argmax);
  * convergence: after training on the 2-D grid, the exact terminal distribution of the trained policy (visit
    probabilities pushed through the grid by the reference) is within 0.03 total variation of R/Z and log Z within
    0.03 of log of the closed-form normalising constant; fresh samples from the trained policy match that exact
    distribution (chi-square).
"""
import math
import os

import numpy as np
import pytest

from paper_2511_16592_amd.workloads import grid_env, ising_env, random_mlp, xavier_mlp
from tests.helpers import (PARAM_KEYS, OracleTrainer, chi2_sf, grid_terminal_distribution, grid_tv_to_reward)

pytestmark = pytest.mark.gpu
NTHREADS = min(16, os.cpu_count() or 1)


@pytest.fixture(scope="module")
def gfnx():
    import torch
    assert torch.cuda.is_available()
    from paper_2511_16592_amd import gfnx as g
    g.load_library()  # raises if the HIP library is missing: no fallback
    return g


def say(msg):
    print(msg, flush=True)


def _ulp32(x):
    return np.spacing(np.abs(x).astype(np.float32)).astype(np.float64)


@pytest.mark.parametrize("shape", [(16, 64, 64, 3), (80, 256, 256, 5), (27, 192, 64, 18)], ids=str)
def test_adam_step_matches_reference(gfnx, oracle64, shape):
    import torch
    n_in, h1, h2, n_act = shape
    env = {3: grid_env(2, 8), 5: grid_env(4, 20), 18: ising_env(3)}[n_act]
    w = random_mlp(n_in, h1, h2, n_act, seed=41)
    say(f"[adam {shape}]")
    sess = gfnx.Session(env, w, 16)
    lr, lr_z = 1e-3, 1e-1
    sess.init_optimizer(log_z=0.25, lr=lr, lr_log_z=lr_z)
    tr = OracleTrainer(oracle64, env, w, log_z=0.25, lr=lr, lr_log_z=lr_z)
    rng = np.random.default_rng(42)
    steps = 6
    gmax = {k: 0.0 for k in PARAM_KEYS}
    for t in range(steps):
        g = {}
        for k in PARAM_KEYS:
            a = rng.normal(size=w[k].shape) * 10.0 ** rng.integers(-5, 2, size=w[k].shape)
            a[rng.random(w[k].shape) < 0.15] = 0.0   # dead units / unused one-hot rows have exactly zero gradient
            g["d" + k] = a.astype(np.float32)
            gmax[k] = max(gmax[k], float(np.abs(g["d" + k]).max()))
            sess.grads["d" + k].copy_(torch.from_numpy(g["d" + k]))
        g["dlogz"] = float(np.float32(rng.normal()))
        sess.dlogz.fill_(g["dlogz"])
        sess.adam_step()
        tr.apply({k: (v.astype(np.float64) if isinstance(v, np.ndarray) else v) for k, v in g.items()})
        got = sess.weights()
        for k in PARAM_KEYS:
            bar = 1e-4 * (t + 1) * lr + 4 * _ulp32(tr.w[k])
            err = np.abs(got[k].astype(np.float64) - tr.w[k])
            assert (err <= bar).all(), (k, t, float((err - bar).max()))
            m = sess.adam_m[k].cpu().numpy().astype(np.float64)
            v = sess.adam_v[k].cpu().numpy().astype(np.float64)
            assert np.abs(m - tr.m[k]).max() <= 1e-4 * gmax[k]
            assert np.abs(v - tr.v[k]).max() <= 1e-4 * gmax[k] ** 2
        lz = float(sess.log_z.item())
        assert abs(lz - float(tr.log_z[0])) <= 1e-4 * (t + 1) * lr_z + 1e-6
        mv = sess.log_z_mv.cpu().numpy()
        assert abs(mv[0] - tr.mz[0]) <= 1e-4 and abs(mv[1] - tr.vz[0]) <= 1e-4
    moved = max(float(np.abs(sess.weights()[k] - w[k]).max()) for k in PARAM_KEYS)
    assert 0.5 * lr < moved <= 3.2 * steps * lr   # one update moves a parameter by at most (1-beta1)/sqrt(1-beta2) * lr


def test_adam_without_log_z(gfnx):
    """NULL log Z pointers leave log Z out; the weights still move."""
    import ctypes as C
    env = grid_env(2, 8)
    w = random_mlp(16, 64, 64, 3, seed=43)
    sess = gfnx.Session(env, w, 16)
    sess.init_optimizer(log_z=1.0)
    for k in sess.grads:
        sess.grads[k].fill_(1.0)
    st = gfnx.AdamState(sess.adam_state.m, sess.adam_state.v, None)
    rc = sess.lib.gfnx_adam_step(C.byref(sess.mlp), None, C.byref(sess.cgrads), None, C.byref(st),
                                 C.byref(sess.adam_cfg), 1, sess._stream())
    assert rc == 0
    got = sess.weights()
    for k in PARAM_KEYS:
        np.testing.assert_allclose(got[k], w[k] - 1e-3, rtol=0, atol=2e-7)
    assert float(sess.log_z.item()) == 1.0


@pytest.mark.parametrize("case", [("grid2x8", grid_env(2, 8), (16, 64, 64, 3), 16),
                                  ("grid4x6_256", grid_env(4, 6), (24, 256, 256, 5), 300),
                                  ("ising3", ising_env(3), (27, 64, 64, 18), 40)], ids=lambda c: c[0])
def test_train_step_equals_its_three_calls(gfnx, case):
    name, env, shape, batch = case
    w = xavier_mlp(*shape, seed=44)
    say(f"[train-vs-calls {name}]")
    a = gfnx.Session(env, w, batch)
    b = gfnx.Session(env, w, batch)
    a.init_optimizer(log_z=0.5)
    b.init_optimizer(log_z=0.5)
    for it in range(4):
        a.train_step(7, it)
        b.rollout(7, it)
        b.tb_loss_grad(float(b.log_z.item()))
        b.adam_step()
        ta, tb = a.trajectories(), b.trajectories()
        for k in ta:
            assert (ta[k] == tb[k]).all(), (it, k)
        ga, gb = a.gradients(), b.gradients()
        for k in ga:
            assert np.array_equal(np.asarray(ga[k]), np.asarray(gb[k])), (it, k)
        wa, wb = a.weights(), b.weights()
        for k in wa:
            assert np.array_equal(wa[k], wb[k]), (it, k)
        assert float(a.log_z.item()) == float(b.log_z.item())
    assert any(not np.array_equal(a.weights()[k], w[k]) for k in PARAM_KEYS)


def _adam_image(theta, g_lo, g_hi, m, v, t, lr, oracle64, points=5):
    """Smallest and largest updated parameter over gradients sampled across [g_lo, g_hi] (binary64 reference)."""
    lo = np.full(theta.shape, np.inf)
    hi = np.full(theta.shape, -np.inf)
    for s in np.linspace(0.0, 1.0, points):
        th, mm, vv = theta.copy(), m.copy(), v.copy()
        oracle64.adam_step(th, g_lo + s * (g_hi - g_lo), mm, vv, t, lr)
        lo, hi = np.minimum(lo, th), np.maximum(hi, th)
    return lo, hi


@pytest.mark.parametrize("case", [("grid2x8", grid_env(2, 8), (16, 64, 64, 3), 16),
                                  ("grid3x7_256", grid_env(3, 7), (21, 256, 256, 4), 200)], ids=lambda c: c[0])
def test_training_iterations_against_reference_chain(gfnx, oracle32, oracle64, case):
    name, env, shape, batch = case
    w = random_mlp(*shape, seed=45)
    lr, lr_z = 1e-3, 1e-1
    sess = gfnx.Session(env, w, batch)
    sess.init_optimizer(log_z=0.3, lr=lr, lr_log_z=lr_z)
    for it in range(3):
        say(f"[train-vs-reference {name}] iteration {it}")
        # the reference starts every iteration from the GPU's own state, so each update is judged on its own
        w_before = sess.weights()
        w64 = {k: v.astype(np.float64) for k, v in w_before.items()}
        m = {k: sess.adam_m[k].cpu().numpy().astype(np.float64) for k in PARAM_KEYS}
        v = {k: sess.adam_v[k].cpu().numpy().astype(np.float64) for k in PARAM_KEYS}
        lz = float(sess.log_z.item())
        mz, vz = [np.array([float(x)]) for x in sess.log_z_mv.cpu().numpy()]
        sess.train_step(13, it)
        traj, grads, w_after = sess.trajectories(), sess.gradients(), sess.weights()
        rep = oracle32.replay(env, w_before, 13, it, traj["actions"], traj["length"], tie_tol=1e-5, nthreads=NTHREADS)
        assert (rep["violations"] == 0).all()
        g = oracle64.tb_loss_grad(env, w64, traj["actions"], traj["length"], lz, nthreads=NTHREADS)
        assert abs(grads["loss"] - g["loss"]) <= 1e-4 * abs(g["loss"]) + 1e-6
        for k in PARAM_KEYS:
            tau = 1e-4 * np.abs(g["d" + k]).max() + 1e-7
            assert np.abs(grads["d" + k] - g["d" + k]).max() <= tau
            lo, hi = _adam_image(w64[k], g["d" + k] - tau, g["d" + k] + tau, m[k], v[k], it + 1, lr, oracle64)
            slack = 1e-4 * lr + 4 * _ulp32(w64[k])
            got = w_after[k].astype(np.float64)
            assert ((got >= lo - slack) & (got <= hi + slack)).all(), k
            # where the gradient is well away from zero the update is pinned tightly
            th = w64[k].copy()
            oracle64.adam_step(th, g["d" + k], m[k].copy(), v[k].copy(), it + 1, lr)
            firm = np.abs(g["d" + k]) > 100 * tau
            if it == 0 and firm.any():
                assert np.abs(got[firm] - th[firm]).max() <= 1e-3 * lr + 4 * _ulp32(th[firm]).max()
        tau = 1e-4 * abs(g["dlogz"]) + 1e-6
        assert abs(grads["dlogz"] - g["dlogz"]) <= tau
        lo, hi = _adam_image(np.array([lz]), np.array([g["dlogz"] - tau]), np.array([g["dlogz"] + tau]), mz, vz,
                             it + 1, lr_z, oracle64)
        assert lo[0] - 1e-4 * lr_z - 1e-6 <= float(sess.log_z.item()) <= hi[0] + 1e-4 * lr_z + 1e-6


def test_training_converges_to_the_reward_distribution(gfnx, oracle64):
    """Appendix "Hypergrid": the criterion is the total variation distance between the sampler's terminal
    distribution and R/Z (here on the 2-D grid of side 8 with the paper's batch of 16 and learning rates)."""
    import torch
    side = 8
    env = grid_env(2, side)
    w0 = xavier_mlp(2 * side, 64, 64, 3, seed=21)
    sess = gfnx.Session(env, w0, 16)
    sess.init_optimizer(log_z=0.0, lr=1e-3, lr_log_z=1e-1)

    def exact_terminal(w):
        w64 = {k: v.astype(np.float64) for k, v in w.items()}
        return grid_terminal_distribution(lambda x: oracle64.policy(env, w64, list(x))[1:], 2, side)

    tv0 = grid_tv_to_reward(exact_terminal(w0), side)
    losses = []
    iters = 4000
    for it in range(iters):
        sess.train_step(5, it)
        if it < 20 or it >= iters - 200:
            losses.append(sess.loss.clone())
        if (it + 1) % 1000 == 0:
            torch.cuda.synchronize()
            say(f"[converge] iteration {it + 1}: loss {float(sess.loss.item()):.3g}, log Z {float(sess.log_z.item()):.4f}")
    losses = [float(x.item()) for x in losses]
    w1 = sess.weights()
    term = exact_terminal(w1)
    tv1 = grid_tv_to_reward(term, side)
    log_z = float(sess.log_z.item())
    say(f"[converge] total variation {tv0:.3f} -> {tv1:.4f}; log Z {log_z:.4f} (exact {math.log(16.064):.4f})")
    assert tv0 > 0.5
    assert tv1 < 0.03
    assert abs(log_z - math.log(16.064)) < 0.03
    assert np.mean(losses[20:]) < 0.02 * np.mean(losses[:20])
    # fresh samples from the trained policy follow its exact terminal distribution
    n = 65536
    big = gfnx.Session(env, w1, n)
    big.rollout(99, 0)
    ts = big.trajectories()["terminal_state"].astype(int)
    counts = np.bincount(ts[0] * side + ts[1], minlength=side * side)
    expected = np.array([term[(i, j)] for i in range(side) for j in range(side)]) * n
    keep = expected > 5
    stat = float(((counts[keep] - expected[keep]) ** 2 / expected[keep]).sum())
    assert counts[~keep].sum() <= 10 * max(1.0, expected[~keep].sum())
    assert chi2_sf(stat, int(keep.sum()) - 1) > 1e-4
    # and the empirical distance to R/Z is small too (its floor is the sampling noise of n draws)
    probs = counts / n
    from tests.helpers import grid_reward
    target = np.array([grid_reward((i, j), side) for i in range(side) for j in range(side)]) / 16.064
    assert 0.5 * np.abs(probs - target).sum() < 0.05


def test_training_iterations_beyond_256_actions(gfnx):
    """Whole training iterations (rollout with exploration, TB gradient, Adam) on a non-autoregressive bit-sequence
    instance with 512 actions -- the paged rollout and the 16-bit action plane inside gfnx_train_step_opts: the TB loss
    falls by an order of magnitude and log Z moves towards log of the sum of the rewards."""
    from paper_2511_16592_amd.workloads import bitseq_na_env
    env = bitseq_na_env(16, 8, 4, mode_seed=6)
    w0 = xavier_mlp(2 * 257, 128, 128, 512, seed=31)
    sess = gfnx.Session(env, w0, 64)
    sess.init_optimizer(log_z=0.0, lr=1e-3, lr_log_z=1e-1)
    losses = []
    for it in range(1500):
        sess.train_step(9, it, epsilon=1e-3)
        if it < 20 or it >= 1480:
            losses.append(sess.loss.clone())
    losses = [float(x.item()) for x in losses]
    traj = sess.trajectories()
    assert traj["actions"].dtype == np.uint16 and (traj["length"] == 2).all()
    say(f"[train 512 actions] loss {np.mean(losses[:20]):.3g} -> {np.mean(losses[20:]):.3g}, log Z {float(sess.log_z.item()):.3f}")
    assert np.mean(losses[20:]) < 0.1 * np.mean(losses[:20])
    assert np.isfinite(list(sess.weights()["W3"].ravel())).all()
