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


def grid_terminal_distribution(policy, dim, side):
    """Exact distribution over terminal states induced by a forward policy on the hypergrid DAG:
    visit(s0) = 1, visit(x + e_i) += visit(x) P_F(+e_i | x), P_T(x) = visit(x) P_F(stop | x).
    `policy(x)` returns (log_probs[dim+1], valid[dim+1]); stop is the last action."""
    visit = {tuple([0] * dim): 1.0}
    term = {}
    for x in sorted(itertools.product(range(side), repeat=dim), key=lambda s: sum(s)):
        v = visit.get(x, 0.0)
        logp, valid = policy(x)
        term[x] = v * math.exp(float(logp[dim]))
        for i in range(dim):
            if x[i] < side - 1:
                assert valid[i]
                y = list(x)
                y[i] += 1
                y = tuple(y)
                visit[y] = visit.get(y, 0.0) + v * math.exp(float(logp[i]))
            else:
                assert not valid[i]
    return term


def grid_tv_to_reward(term, side, **kw):
    """Total variation distance between a terminal distribution and R / Z."""
    z = sum(grid_reward(x, side, **kw) for x in term)
    return 0.5 * sum(abs(p - grid_reward(x, side, **kw) / z) for x, p in term.items())


PARAM_KEYS = ("W1", "b1", "W2", "b2", "W3", "b3")


class OracleTrainer:
    """A whole training iteration composed from the CPU reference: on-policy rollout, TB loss and gradient along
    the sampled actions, one Adam update of every weight tensor and of log Z (Appendix "Hypergrid",
    hyperparameter table: learning rate 1e-3, 1e-1 for log Z)."""

    def __init__(self, oracle, env, weights, log_z=0.0, lr=1e-3, lr_log_z=1e-1, beta1=0.9, beta2=0.999, eps=1e-8):
        self.o, self.env = oracle, env
        self.w = {k: np.array(weights[k], dtype=oracle.real) for k in PARAM_KEYS}
        self.log_z = np.array([log_z], dtype=oracle.real)
        self.m = {k: np.zeros_like(v) for k, v in self.w.items()}
        self.v = {k: np.zeros_like(v) for k, v in self.w.items()}
        self.mz, self.vz = np.zeros(1, dtype=oracle.real), np.zeros(1, dtype=oracle.real)
        self.hp = dict(beta1=beta1, beta2=beta2, eps=eps)
        self.lr, self.lr_log_z = lr, lr_log_z
        self.t = 0

    def step(self, seed, iteration, batch, nthreads=1):
        out = self.o.rollout(self.env, self.w, seed, iteration, batch, nthreads=nthreads)
        g = self.o.tb_loss_grad(self.env, self.w, out["actions"], out["length"], log_z=float(self.log_z[0]),
                                nthreads=nthreads)
        self.apply(g)
        return out, g

    def apply(self, g):
        self.t += 1
        for k in PARAM_KEYS:
            self.o.adam_step(self.w[k], g["d" + k], self.m[k], self.v[k], self.t, self.lr, **self.hp)
        self.o.adam_step(self.log_z, np.array([g["dlogz"]], dtype=self.o.real), self.mz, self.vz, self.t,
                         self.lr_log_z, **self.hp)
