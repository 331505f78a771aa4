"""Pins for the optimiser step of the CPU reference and for a whole training iteration built from it."""
import math

import numpy as np
import pytest
import torch

from paper_2511_16592_amd.workloads import grid_env, xavier_mlp
from tests.helpers import OracleTrainer, grid_terminal_distribution, grid_tv_to_reward


def test_adam_matches_library_adam(oracle64):
    """Same gradient sequence through torch.optim.Adam (binary64, CPU): parameters and both moments agree."""
    rng = np.random.default_rng(11)
    theta = rng.normal(size=(7, 5))
    p = torch.nn.Parameter(torch.tensor(theta.copy(), dtype=torch.float64))
    opt = torch.optim.Adam([p], lr=3e-3, betas=(0.9, 0.999), eps=1e-8, weight_decay=0.0)
    m, v = np.zeros_like(theta), np.zeros_like(theta)
    for t in range(1, 14):
        g = rng.normal(size=theta.shape) * 10.0 ** rng.integers(-6, 3)
        g[rng.random(theta.shape) < 0.2] = 0.0
        p.grad = torch.tensor(g.copy(), dtype=torch.float64)
        opt.step()
        oracle64.adam_step(theta, g, m, v, t, 3e-3)
        st = opt.state[p]
        np.testing.assert_allclose(theta, p.detach().numpy(), rtol=1e-12, atol=1e-15)
        np.testing.assert_allclose(m, st["exp_avg"].numpy(), rtol=1e-12, atol=1e-300)
        np.testing.assert_allclose(v, st["exp_avg_sq"].numpy(), rtol=1e-12, atol=1e-300)


def test_adam_other_betas_match_library_adam(oracle64):
    rng = np.random.default_rng(12)
    theta = rng.normal(size=33)
    p = torch.nn.Parameter(torch.tensor(theta.copy(), dtype=torch.float64))
    opt = torch.optim.Adam([p], lr=0.1, betas=(0.5, 0.9), eps=1e-3)
    m, v = np.zeros_like(theta), np.zeros_like(theta)
    for t in range(1, 6):
        g = rng.normal(size=theta.shape)
        p.grad = torch.tensor(g.copy(), dtype=torch.float64)
        opt.step()
        oracle64.adam_step(theta, g, m, v, t, 0.1, beta1=0.5, beta2=0.9, eps=1e-3)
    np.testing.assert_allclose(theta, p.detach().numpy(), rtol=1e-12)


def test_adam_constant_gradient_closed_form(oracle64):
    """With the same gradient g at every update the bias-corrected moments are exactly g and g^2, so every update
    moves the parameter by lr * g / (|g| + eps); a zero gradient never moves it."""
    g = np.array([3.0, -0.25, 1e-4, 0.0, -7e3])
    theta0 = np.array([1.0, 2.0, -3.0, 4.0, 0.5])
    theta, m, v = theta0.copy(), np.zeros(5), np.zeros(5)
    lr, eps = 1e-2, 1e-8
    for t in range(1, 40):
        oracle64.adam_step(theta, g, m, v, t, lr, eps=eps)
        np.testing.assert_allclose(theta, theta0 - t * lr * g / (np.abs(g) + eps), rtol=1e-12, atol=1e-14)
    assert theta[3] == theta0[3]
    np.testing.assert_allclose(m, (1 - 0.9 ** 39) * g, rtol=1e-12)
    np.testing.assert_allclose(v, (1 - 0.999 ** 39) * g * g, rtol=1e-10)


def test_adam_binary32_build_follows_binary64(oracle32, oracle64):
    rng = np.random.default_rng(13)
    th64 = rng.normal(size=1000)
    th32 = th64.astype(np.float32)
    th64 = th32.astype(np.float64)
    m64, v64 = np.zeros(1000), np.zeros(1000)
    m32, v32 = np.zeros(1000, np.float32), np.zeros(1000, np.float32)
    for t in range(1, 8):
        g = rng.normal(size=1000).astype(np.float32)
        oracle64.adam_step(th64, g.astype(np.float64), m64, v64, t, 1e-3)
        oracle32.adam_step(th32, g, m32, v32, t, 1e-3)
    np.testing.assert_allclose(th32, th64, rtol=1e-6, atol=1e-7)
    np.testing.assert_allclose(m32, m64, rtol=1e-5, atol=1e-6)  # sums of +-O(1) terms: absolute scale
    np.testing.assert_allclose(v32, v64, rtol=1e-4, atol=1e-9)  # 1 - float32(0.999) is 1.3e-5 off 1e-3


def test_training_iterations_approach_the_reward_distribution(oracle32, oracle64):
    """Minimising the TB objective makes the terminal distribution of P_F equal R/Z and log Z equal log of the
    true normalising constant (Background: a policy satisfying the trajectory balance constraint samples from
    R/Z; Appendix "Hypergrid": the convergence criterion is the total variation distance to R/Z).  The exact
    terminal distribution of the trained policy is computed by propagating visit probabilities through the grid."""
    side = 4
    env = grid_env(2, side)
    w0 = xavier_mlp(2 * side, 64, 64, 3, seed=21)
    tr = OracleTrainer(oracle32, env, w0, lr=1e-3, lr_log_z=1e-1)

    def tv():
        w64 = {k: v.astype(np.float64) for k, v in tr.w.items()}
        term = grid_terminal_distribution(lambda x: oracle64.policy(env, w64, list(x))[1:], 2, side)
        assert abs(sum(term.values()) - 1.0) < 1e-9
        return grid_tv_to_reward(term, side)

    tv0 = tv()
    losses = []
    for it in range(1000):
        _out, g = tr.step(seed=5, iteration=it, batch=16)
        losses.append(g["loss"])
    tv1 = tv()
    assert tv0 > 0.3
    assert tv1 < 0.02
    assert abs(float(tr.log_z[0]) - math.log(2.016)) < 0.03
    assert np.mean(losses[-100:]) < 0.05 * np.mean(losses[:20])
