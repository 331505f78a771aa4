"""Brute-force helpers written for the tests only (fp64 Python, independent of oracle/ and of the GPU code)."""
import itertools
import math

import numpy as np


def grid_reward(x, side, r0=1e-3, r1=0.5, r2=2.0):
    """Hypergrid reward, Appendix "Hypergrid" (reward equation), evaluated with exact rationals."""
    from fractions import Fraction
    in1 = in2 = True
    for xi in x:
        v = abs(Fraction(xi, side - 1) - Fraction(1, 2))
        in1 = in1 and (Fraction(1, 4) < v)
        in2 = in2 and (Fraction(3, 10) < v < Fraction(2, 5))
    return r0 + r1 * in1 + r2 * in2


def enumerate_grid_trajectories(dim, side):
    """All complete action sequences of the hypergrid DAG (increment a<dim, stop = dim)."""
    out = []

    def rec(x, prefix):
        out.append((prefix + [dim], tuple(x)))
        for i in range(dim):
            if x[i] < side - 1:
                x[i] += 1
                rec(x, prefix + [i])
                x[i] -= 1

    rec([0] * dim, [])
    return out


def pack_trajectories(trajs, max_steps):
    batch = len(trajs)
    actions = np.full((max_steps, batch), 0xFF, dtype=np.uint8)
    length = np.zeros(batch, dtype=np.int32)
    for b, (acts, _x) in enumerate(trajs):
        length[b] = len(acts)
        actions[:len(acts), b] = acts
    return actions, length


def grid_dp_flows(dim, side, r0=1e-3, r1=0.5, r2=2.0):
    """State flows F(x) of the unique proper forward policy under the uniform backward policy.

    F(x) = R(x) + sum_{i: x_i < side-1} F(x+e_i) / n(x+e_i), n(y) = #{j: y_j > 0}.
    """
    F = {}
    for x in sorted(itertools.product(range(side), repeat=dim), key=lambda s: -sum(s)):
        f = grid_reward(x, side, r0, r1, r2)
        for i in range(dim):
            if x[i] < side - 1:
                y = list(x)
                y[i] += 1
                y = tuple(y)
                f += F[y] / sum(1 for c in y if c > 0)
        F[x] = f
    return F


def grid_optimal_policy(dim, side, **kw):
    """log P_F*(a | x) for all states, invalid actions get None; also returns log Z = log F(0)."""
    F = grid_dp_flows(dim, side, **kw)
    pol = {}
    for x, f in F.items():
        lp = [None] * (dim + 1)
        lp[dim] = math.log(grid_reward(x, side, **kw) / f)
        for i in range(dim):
            if x[i] < side - 1:
                y = list(x)
                y[i] += 1
                y = tuple(y)
                lp[i] = math.log(F[y] / (sum(1 for c in y if c > 0) * f))
        pol[x] = lp
    return pol, math.log(F[tuple([0] * dim)])


def optimal_policy_mlp_2d(side, dtype=np.float64, **kw):
    """An MLP of the 2*side -> side^2 -> side^2 -> 3 shape that computes log P_F* exactly:
    hidden unit (i,j) = ReLU(onehot_0[i] + onehot_1[j] - 1) is the indicator of state (i,j),
    layer 2 is the identity, W3[(i,j), a] = log P_F*(a | (i,j))."""
    pol, log_z = grid_optimal_policy(2, side, **kw)
    n = side * side
    W1 = np.zeros((2 * side, n), dtype=dtype)
    for i in range(side):
        for j in range(side):
            W1[i, i * side + j] = 1.0
            W1[side + j, i * side + j] = 1.0
    b1 = -np.ones(n, dtype=dtype)
    W2 = np.eye(n, dtype=dtype)
    b2 = np.zeros(n, dtype=dtype)
    W3 = np.zeros((n, 3), dtype=dtype)
    for (i, j), lp in pol.items():
        for a in range(3):
            W3[i * side + j, a] = lp[a] if lp[a] is not None else 0.0
    b3 = np.zeros(3, dtype=dtype)
    return dict(W1=W1, b1=b1, W2=W2, b2=b2, W3=W3, b3=b3), log_z


def chi2_sf(stat, dof):
    from scipy.stats import chi2
    return float(chi2.sf(stat, dof))
