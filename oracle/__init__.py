"""ctypes wrapper around the CPU reference in gfn_oracle.c.

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the CPU-baseline
leg of the benchmark.  The product package never imports this module.

`Oracle("f32")` does all arithmetic in binary32 (used where a float comparison decides the
sampled action), `Oracle("f64")` in binary64 (ground truth along a given action sequence).
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import Dict, Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "gfn_oracle.c")


def lib_path(precision: str) -> str:
    return os.path.join(_HERE, f"liboracle_{precision}.so")


def build(force: bool = False) -> None:
    """Compile the reference in both precisions with gcc (plain -O2, no contraction)."""
    for precision, ctype in (("f32", "float"), ("f64", "double")):
        out = lib_path(precision)
        if not force and os.path.exists(out) and os.path.getmtime(out) >= os.path.getmtime(_SRC):
            continue
        cmd = ["gcc", "-O2", "-ffp-contract=off", "-fPIC", "-shared", "-Wall", "-Wextra",
               f"-DORACLE_REAL={ctype}", _SRC, "-o", out, "-lm", "-lpthread"]
        subprocess.run(cmd, check=True)


class _Env(C.Structure):
    _fields_ = [("kind", C.c_int32), ("grid_dim", C.c_int32), ("grid_side", C.c_int32),
                ("r0", C.c_double), ("r1", C.c_double), ("r2", C.c_double),
                ("n_bits", C.c_int32), ("k_bits", C.c_int32), ("n_modes", C.c_int32),
                ("modes", C.c_void_p), ("beta", C.c_double),
                ("lattice_n", C.c_int32), ("coupling", C.c_double)]


class _Mlp(C.Structure):
    _fields_ = [("in_dim", C.c_int32), ("h1", C.c_int32), ("h2", C.c_int32), ("n_actions", C.c_int32),
                ("W1", C.c_void_p), ("b1", C.c_void_p), ("W2", C.c_void_p), ("b2", C.c_void_p),
                ("W3", C.c_void_p), ("b3", C.c_void_p)]


class _Grad(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("dW1", "db1", "dW2", "db2", "dW3", "db3")]


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _action_plane(actions16: np.ndarray, env) -> np.ndarray:
    """The C side keeps actions in 16 bits (padding 0xFFFF).  Environments with at most 256 actions hand them out as
    bytes (padding 0xFF), the form the rest of the tests use; wider ones keep the 16-bit plane."""
    return actions16.astype(np.uint8) if env.dims()[2] <= 256 else actions16


class Oracle:
    def __init__(self, precision: str = "f64"):
        assert precision in ("f32", "f64")
        build()
        self.precision = precision
        self.real = np.float32 if precision == "f32" else np.float64
        self.creal = C.c_float if precision == "f32" else C.c_double
        self.lib = C.CDLL(lib_path(precision))
        assert self.lib.oracle_real_bytes() == np.dtype(self.real).itemsize
        self.lib.oracle_uniform.restype = self.creal
        self.lib.oracle_gumbel.restype = self.creal
        self._keep = []

    # ---- marshalling -------------------------------------------------------
    def _env(self, env):
        modes = None
        if env.modes is not None:
            modes = np.ascontiguousarray(env.modes, dtype=np.uint32)
        e = _Env(env.kind, env.grid_dim, env.grid_side, env.r0, env.r1, env.r2, env.n_bits, env.k_bits,
                 0 if modes is None else modes.shape[0], _ptr(modes), env.beta, env.lattice_n, env.coupling)
        return e, modes

    def _mlp(self, w: Dict[str, np.ndarray]):
        arrs = {k: np.ascontiguousarray(w[k], dtype=self.real) for k in ("W1", "b1", "W2", "b2", "W3", "b3")}
        m = _Mlp(arrs["W1"].shape[0], arrs["W1"].shape[1], arrs["W2"].shape[1], arrs["W3"].shape[1],
                 *[_ptr(arrs[k]) for k in ("W1", "b1", "W2", "b2", "W3", "b3")])
        assert arrs["W2"].shape[0] == m.h1 and arrs["W3"].shape[0] == m.h2
        return m, arrs

    # ---- RNG ---------------------------------------------------------------
    def philox(self, ctr, key) -> np.ndarray:
        c = (C.c_uint32 * 4)(*[int(x) & 0xFFFFFFFF for x in ctr])
        k = (C.c_uint32 * 2)(*[int(x) & 0xFFFFFFFF for x in key])
        o = (C.c_uint32 * 4)()
        self.lib.oracle_philox4x32_10(c, k, o)
        return np.array(list(o), dtype=np.uint32)

    def uniform(self, w: int) -> float:
        return float(self.lib.oracle_uniform(C.c_uint32(int(w))))

    def gumbel(self, w: int) -> float:
        return float(self.lib.oracle_gumbel(C.c_uint32(int(w))))

    # ---- environment -------------------------------------------------------
    def env_dims(self, env):
        e, _keep = self._env(env)
        out = [C.c_int32() for _ in range(4)]
        rc = self.lib.oracle_env_dims(C.byref(e), *[C.byref(o) for o in out])
        assert rc == 0
        return tuple(o.value for o in out)

    def log_reward(self, env, state) -> float:
        e, _keep = self._env(env)
        s = np.ascontiguousarray(state, dtype=np.int32)
        out = self.creal()
        rc = self.lib.oracle_log_reward(C.byref(e), _ptr(s), C.byref(out))
        assert rc == 0
        return float(out.value)

    def policy(self, env, w, state):
        """(logits, log_probs, valid) of the forward policy at a non-terminal state."""
        e, _k1 = self._env(env)
        m, _k2 = self._mlp(w)
        s = np.ascontiguousarray(state, dtype=np.int32)
        logit = np.zeros(m.n_actions, dtype=self.real)
        logp = np.zeros(m.n_actions, dtype=self.real)
        valid = np.zeros(m.n_actions, dtype=np.int32)
        rc = self.lib.oracle_policy_logits(C.byref(e), C.byref(m), _ptr(s), _ptr(logit), _ptr(logp), _ptr(valid))
        assert rc == 0, rc
        return logit, logp, valid.astype(bool)

    # ---- rollout / replay ----------------------------------------------------
    def rollout(self, env, w, seed: int, iteration: int, batch: int, b_offset: int = 0,
                max_steps: Optional[int] = None, nthreads: int = 1, epsilon: float = 0.0) -> Dict[str, np.ndarray]:
        e, _k1 = self._env(env)
        m, _k2 = self._mlp(w)
        sd, _, _, ms = env.dims()
        T = ms if max_steps is None else max_steps
        out = dict(actions=np.zeros((T, batch), dtype=np.uint16), length=np.zeros(batch, dtype=np.int32),
                   terminal_state=np.zeros((sd, batch), dtype=np.int8),
                   log_pf=np.zeros(batch, dtype=self.real), log_pb=np.zeros(batch, dtype=self.real),
                   log_reward=np.zeros(batch, dtype=self.real), min_margin=np.zeros(batch, dtype=self.real))
        rc = self.lib.oracle_rollout(C.byref(e), C.byref(m), C.c_uint64(seed), C.c_uint64(iteration),
                                     C.c_int32(b_offset), C.c_int32(batch), C.c_int32(T),
                                     _ptr(out["actions"]), _ptr(out["length"]), _ptr(out["terminal_state"]),
                                     _ptr(out["log_pf"]), _ptr(out["log_pb"]), _ptr(out["log_reward"]),
                                     _ptr(out["min_margin"]), self.creal(epsilon), C.c_int(nthreads))
        assert rc == 0, rc
        out["actions"] = _action_plane(out["actions"], env)
        return out

    def replay(self, env, w, seed: int, iteration: int, actions: np.ndarray, length: np.ndarray,
               b_offset: int = 0, tie_tol: float = 1e-5, nthreads: int = 1, epsilon: float = 0.0) -> Dict[str, np.ndarray]:
        e, _k1 = self._env(env)
        m, _k2 = self._mlp(w)
        sd = env.dims()[0]
        actions = np.ascontiguousarray(actions, dtype=np.uint16)
        length = np.ascontiguousarray(length, dtype=np.int32)
        T, batch = actions.shape
        out = dict(terminal_state=np.zeros((sd, batch), dtype=np.int8),
                   log_pf=np.zeros(batch, dtype=self.real), log_pb=np.zeros(batch, dtype=self.real),
                   log_reward=np.zeros(batch, dtype=self.real), near_ties=np.zeros(batch, dtype=np.int32),
                   violations=np.zeros(batch, dtype=np.int32), min_margin=np.zeros(batch, dtype=self.real))
        rc = self.lib.oracle_replay(C.byref(e), C.byref(m), C.c_uint64(seed), C.c_uint64(iteration),
                                    C.c_int32(b_offset), C.c_int32(batch), C.c_int32(T), _ptr(actions), _ptr(length),
                                    _ptr(out["terminal_state"]), _ptr(out["log_pf"]), _ptr(out["log_pb"]),
                                    _ptr(out["log_reward"]), self.creal(tie_tol), _ptr(out["near_ties"]),
                                    _ptr(out["violations"]), _ptr(out["min_margin"]), self.creal(epsilon),
                                    C.c_int(nthreads))
        assert rc == 0, rc
        return out

    # ---- loss + gradient -------------------------------------------------------
    def tb_loss_grad(self, env, w, actions: np.ndarray, length: np.ndarray, log_z: float = 0.0,
                     nthreads: int = 1, kink_tol: float = 0.0) -> Dict[str, np.ndarray]:
        e, _k1 = self._env(env)
        m, arrs = self._mlp(w)
        actions = np.ascontiguousarray(actions, dtype=np.uint16)
        length = np.ascontiguousarray(length, dtype=np.int32)
        T, batch = actions.shape
        g = {("d" + k): np.zeros_like(arrs[k]) for k in ("W1", "b1", "W2", "b2", "W3", "b3")}
        gs = _Grad(*[_ptr(g[k]) for k in ("dW1", "db1", "dW2", "db2", "dW3", "db3")])
        loss, dlogz = self.creal(), self.creal()
        delta = np.zeros(batch, dtype=self.real)
        slack = np.zeros(6, dtype=self.real)
        n_kink = C.c_int64(0)
        rc = self.lib.oracle_tb_loss_grad(C.byref(e), C.byref(m), C.c_int32(batch), C.c_int32(T), _ptr(actions),
                                          _ptr(length), self.creal(log_z), C.byref(loss), C.byref(dlogz),
                                          C.byref(gs), _ptr(delta), self.creal(kink_tol), _ptr(slack),
                                          C.byref(n_kink), C.c_int(nthreads))
        assert rc == 0, rc
        g.update(loss=float(loss.value), dlogz=float(dlogz.value), delta=delta, n_kink=int(n_kink.value),
                 slack=dict(zip(("dW1", "db1", "dW2", "db2", "dW3", "db3"), slack.astype(np.float64))))
        return g

    def tb_loss_grad_follow(self, env, w, actions: np.ndarray, length: np.ndarray, relu1: np.ndarray,
                            relu2: np.ndarray, log_z: float = 0.0, kink_tol: float = 2e-6,
                            nthreads: int = 1) -> Dict[str, np.ndarray]:
        """TB loss and gradient with ReLU' taken from the given decisions where binary32 cannot decide it.

        relu1 [n, h1], relu2 [n, h2]: 0 / 1 per hidden unit, the n = sum(length) transitions ordered by column, then
        step.  Returns the gradients plus `followed`, `flipped`, `mismatched` (see oracle_tb_loss_grad_follow)."""
        e, _k1 = self._env(env)
        m, arrs = self._mlp(w)
        actions = np.ascontiguousarray(actions, dtype=np.uint16)
        length = np.ascontiguousarray(length, dtype=np.int32)
        T, batch = actions.shape
        relu1 = np.ascontiguousarray(relu1, dtype=np.uint8)
        relu2 = np.ascontiguousarray(relu2, dtype=np.uint8)
        n = int(length.sum())
        assert relu1.shape == (n, m.h1) and relu2.shape == (n, m.h2), (relu1.shape, relu2.shape, n)
        first = np.zeros(batch, dtype=np.int64)
        first[1:] = np.cumsum(length.astype(np.int64))[:-1]
        g = {("d" + k): np.zeros_like(arrs[k]) for k in ("W1", "b1", "W2", "b2", "W3", "b3")}
        gs = _Grad(*[_ptr(g[k]) for k in ("dW1", "db1", "dW2", "db2", "dW3", "db3")])
        loss, dlogz = self.creal(), self.creal()
        counts = np.zeros(3, dtype=np.int64)
        rc = self.lib.oracle_tb_loss_grad_follow(C.byref(e), C.byref(m), C.c_int32(batch), C.c_int32(T), _ptr(actions),
                                                 _ptr(length), self.creal(log_z), C.byref(loss), C.byref(dlogz),
                                                 C.byref(gs), self.creal(kink_tol), _ptr(relu1), _ptr(relu2),
                                                 _ptr(first), _ptr(counts), C.c_int(nthreads))
        assert rc == 0, rc
        g.update(loss=float(loss.value), dlogz=float(dlogz.value), followed=int(counts[0]), flipped=int(counts[1]),
                 mismatched=int(counts[2]))
        return g

    def subtb_loss_grad(self, env, w, actions: np.ndarray, length: np.ndarray, lam: float) -> Dict[str, np.ndarray]:
        """SubTB(lambda) loss (lambda = 0: DB) and gradient for a network whose last output is log F(s)."""
        e, _k1 = self._env(env)
        m, arrs = self._mlp(w)
        actions = np.ascontiguousarray(actions, dtype=np.uint16)
        length = np.ascontiguousarray(length, dtype=np.int32)
        T, batch = actions.shape
        g = {("d" + k): np.zeros_like(arrs[k]) for k in ("W1", "b1", "W2", "b2", "W3", "b3")}
        gs = _Grad(*[_ptr(g[k]) for k in ("dW1", "db1", "dW2", "db2", "dW3", "db3")])
        loss = self.creal()
        u = np.zeros((T + 1, batch), dtype=self.real)
        rc = self.lib.oracle_subtb_loss_grad(C.byref(e), C.byref(m), C.c_int32(batch), C.c_int32(T), _ptr(actions),
                                             _ptr(length), self.creal(lam), C.byref(loss), C.byref(gs), _ptr(u))
        assert rc == 0, rc
        g.update(loss=float(loss.value), u=u)
        return g

    # ---- backward rollouts ------------------------------------------------------
    def backward_rollout(self, env, seed: int, iteration: int, terminal_state: np.ndarray, b_offset: int = 0,
                         max_steps: Optional[int] = None) -> Dict[str, np.ndarray]:
        """Trajectories tau ~ P_B(. | x) for the terminal states terminal_state[state_dim, batch], in forward order."""
        e, _k1 = self._env(env)
        ts = np.ascontiguousarray(terminal_state, dtype=np.int8)
        sd, batch = ts.shape
        assert sd == env.dims()[0]
        T = env.dims()[3] if max_steps is None else max_steps
        out = dict(actions=np.zeros((T, batch), dtype=np.uint16), length=np.zeros(batch, dtype=np.int32),
                   log_pb=np.zeros(batch, dtype=self.real))
        rc = self.lib.oracle_backward_rollout(C.byref(e), C.c_uint64(seed), C.c_uint64(iteration), C.c_int32(b_offset),
                                              C.c_int32(batch), C.c_int32(T), _ptr(ts), _ptr(out["actions"]),
                                              _ptr(out["length"]), _ptr(out["log_pb"]))
        assert rc == 0, rc
        out["actions"] = _action_plane(out["actions"], env)
        return out

    def log_prob_estimate(self, log_pf: np.ndarray, log_pb: np.ndarray, n_states: int, n_samples: int) -> np.ndarray:
        """log of the mean over the n_samples trajectories of each state of P_F / P_B (samples of a state adjacent)."""
        f = np.ascontiguousarray(log_pf, dtype=self.real)
        bk = np.ascontiguousarray(log_pb, dtype=self.real)
        assert f.shape == bk.shape == (n_states * n_samples,)
        out = np.zeros(n_states, dtype=self.real)
        rc = self.lib.oracle_log_prob_estimate(_ptr(f), _ptr(bk), C.c_int32(n_states), C.c_int32(n_samples), _ptr(out))
        assert rc == 0, rc
        return out

    # ---- optimiser -------------------------------------------------------------
    def adam_step(self, theta: np.ndarray, grad: np.ndarray, m: np.ndarray, v: np.ndarray, t: int, lr: float,
                  beta1: float = 0.9, beta2: float = 0.999, eps: float = 1e-8) -> None:
        """One Adam update of `theta`, `m`, `v` in place (arrays of this oracle's precision); t counts from 1."""
        for a in (theta, m, v):
            assert a.dtype == self.real and a.flags.c_contiguous and a.shape == theta.shape
        g = np.ascontiguousarray(grad, dtype=self.real)
        assert g.shape == theta.shape
        rc = self.lib.oracle_adam_step(_ptr(theta), _ptr(g), _ptr(m), _ptr(v), C.c_int64(theta.size), C.c_int64(t),
                                       self.creal(lr), self.creal(beta1), self.creal(beta2), self.creal(eps))
        assert rc == 0, rc
