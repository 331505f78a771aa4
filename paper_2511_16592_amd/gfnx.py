"""Thin ctypes binding over libgfnx_hip.so (declared in include/gfnx.h).

Argument marshalling only: every step of the rollout and of the Trajectory-Balance gradient runs in
the HIP kernels of the library.  PyTorch is used for device memory and the stream, nothing else.  The
library is loaded on first use and a missing library is an error: there is no CPU fallback.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, Optional

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libgfnx_hip.so")

GFNX_OK = 0
EXPORTS = ("gfnx_env_dims", "gfnx_workspace_bytes", "gfnx_workspace_region", "gfnx_rollout", "gfnx_rollout_explore", "gfnx_replay",
           "gfnx_tb_loss_grad", "gfnx_subtb_loss_grad",
           "gfnx_adam_step", "gfnx_train_step", "gfnx_train_step_opts", "gfnx_train_step_static", "gfnx_backward_rollout", "gfnx_log_prob_estimate",
           "gfnx_status_string", "gfnx_timing_enable", "gfnx_timing_only", "gfnx_timing_labels", "gfnx_timing_get")


class EnvDesc(C.Structure):
    _fields_ = [("kind", C.c_int32), ("grid_dim", C.c_int32), ("grid_side", C.c_int32),
                ("r0", C.c_float), ("r1", C.c_float), ("r2", C.c_float),
                ("n_bits", C.c_int32), ("k_bits", C.c_int32), ("n_modes", C.c_int32),
                ("modes_dev", C.c_void_p), ("beta", C.c_float),
                ("lattice_n", C.c_int32), ("coupling", C.c_float)]


class Mlp(C.Structure):
    _fields_ = [("in_dim", C.c_int32), ("h1", C.c_int32), ("h2", C.c_int32), ("n_actions", C.c_int32),
                ("W1", C.c_void_p), ("b1", C.c_void_p), ("W2", C.c_void_p), ("b2", C.c_void_p),
                ("W3", C.c_void_p), ("b3", C.c_void_p)]


class MlpGrad(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("dW1", "db1", "dW2", "db2", "dW3", "db3")]


class AdamCfg(C.Structure):
    _fields_ = [("lr", C.c_float), ("lr_log_z", C.c_float), ("beta1", C.c_float), ("beta2", C.c_float),
                ("eps", C.c_float)]


class TrainOpts(C.Structure):
    _fields_ = [("epsilon", C.c_float), ("subtb_lambda", C.c_float)]


class AdamState(C.Structure):
    _fields_ = [("m", MlpGrad), ("v", MlpGrad), ("log_z_mv", C.c_void_p)]


class Traj(C.Structure):
    _fields_ = [("batch", C.c_int32), ("max_steps", C.c_int32), ("actions", C.c_void_p), ("length", C.c_void_p),
                ("terminal_state", C.c_void_p), ("log_pf", C.c_void_p), ("log_pb", C.c_void_p),
                ("log_reward", C.c_void_p), ("actions16", C.c_void_p)]


class GfnxError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"{message} (status {status})")
        self.status = status


_lib = None


def load_library() -> C.CDLL:
    """Loads libgfnx_hip.so; raises if it has not been built (run __graft_entry__.build())."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(f"{LIB_PATH} is missing: build it with `python -c 'import __graft_entry__ as g; "
                                    f"g.build()'`; there is no fallback path")
        lib = C.CDLL(LIB_PATH)
        lib.gfnx_env_dims.restype = C.c_int
        lib.gfnx_env_dims.argtypes = [C.POINTER(EnvDesc)] + [C.POINTER(C.c_int32)] * 4
        lib.gfnx_workspace_bytes.restype = C.c_size_t
        lib.gfnx_workspace_bytes.argtypes = [C.POINTER(EnvDesc), C.POINTER(Mlp), C.c_int32]
        lib.gfnx_workspace_region.restype = C.c_int
        lib.gfnx_workspace_region.argtypes = [C.POINTER(EnvDesc), C.POINTER(Mlp), C.c_int32, C.c_int32,
                                              C.POINTER(C.c_size_t), C.POINTER(C.c_size_t)]
        lib.gfnx_rollout.restype = C.c_int
        lib.gfnx_rollout.argtypes = [C.POINTER(EnvDesc), C.POINTER(Mlp), C.c_uint64, C.c_uint64, C.POINTER(Traj),
                                     C.c_void_p, C.c_size_t, C.c_void_p]
        lib.gfnx_rollout_explore.restype = C.c_int
        lib.gfnx_rollout_explore.argtypes = [C.POINTER(EnvDesc), C.POINTER(Mlp), C.c_uint64, C.c_uint64, C.c_float,
                                             C.POINTER(Traj), C.c_void_p, C.c_size_t, C.c_void_p]
        lib.gfnx_replay.restype = C.c_int
        lib.gfnx_replay.argtypes = [C.POINTER(EnvDesc), C.POINTER(Mlp), C.POINTER(Traj), C.c_void_p, C.c_size_t,
                                    C.c_void_p]
        lib.gfnx_tb_loss_grad.restype = C.c_int
        lib.gfnx_tb_loss_grad.argtypes = [C.POINTER(EnvDesc), C.POINTER(Mlp), C.POINTER(Traj), C.c_float, C.c_void_p,
                                          C.c_void_p, C.POINTER(MlpGrad), C.c_void_p, C.c_size_t, C.c_void_p]
        lib.gfnx_subtb_loss_grad.restype = C.c_int
        lib.gfnx_subtb_loss_grad.argtypes = [C.POINTER(EnvDesc), C.POINTER(Mlp), C.POINTER(Traj), C.c_float, C.c_void_p,
                                             C.POINTER(MlpGrad), C.c_void_p, C.c_size_t, C.c_void_p]
        lib.gfnx_backward_rollout.restype = C.c_int
        lib.gfnx_backward_rollout.argtypes = [C.POINTER(EnvDesc), C.c_uint64, C.c_uint64, C.POINTER(Traj), C.c_void_p]
        lib.gfnx_log_prob_estimate.restype = C.c_int
        lib.gfnx_log_prob_estimate.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p]
        lib.gfnx_adam_step.restype = C.c_int
        lib.gfnx_adam_step.argtypes = [C.POINTER(Mlp), C.c_void_p, C.POINTER(MlpGrad), C.c_void_p,
                                       C.POINTER(AdamState), C.POINTER(AdamCfg), C.c_int64, C.c_void_p]
        lib.gfnx_train_step.restype = C.c_int
        lib.gfnx_train_step.argtypes = [C.POINTER(EnvDesc), C.POINTER(Mlp), C.c_void_p, C.c_uint64, C.c_uint64,
                                        C.POINTER(Traj), C.c_void_p, C.c_void_p, C.POINTER(MlpGrad),
                                        C.POINTER(AdamState), C.POINTER(AdamCfg), C.c_int64, C.c_void_p, C.c_size_t,
                                        C.c_void_p]
        lib.gfnx_train_step_static.restype = C.c_int
        lib.gfnx_train_step_static.argtypes = [C.POINTER(EnvDesc), C.POINTER(Mlp), C.c_void_p, C.c_uint64, C.c_uint64,
                                               C.POINTER(Traj), C.c_void_p, C.c_void_p, C.POINTER(MlpGrad),
                                               C.POINTER(AdamState), C.POINTER(AdamCfg), C.c_int64, C.c_void_p]
        lib.gfnx_train_step_opts.restype = C.c_int
        lib.gfnx_train_step_opts.argtypes = [C.POINTER(EnvDesc), C.POINTER(Mlp), C.c_void_p, C.c_uint64, C.c_uint64,
                                             C.POINTER(Traj), C.c_void_p, C.c_void_p, C.POINTER(MlpGrad),
                                             C.POINTER(AdamState), C.POINTER(AdamCfg), C.POINTER(TrainOpts),
                                             C.c_int64, C.c_void_p, C.c_size_t, C.c_void_p]
        lib.gfnx_timing_enable.restype = C.c_int
        lib.gfnx_timing_enable.argtypes = [C.c_int]
        lib.gfnx_timing_only.restype = C.c_int
        lib.gfnx_timing_only.argtypes = [C.c_char_p]
        lib.gfnx_timing_labels.restype = C.c_int
        lib.gfnx_timing_get.restype = C.c_int
        lib.gfnx_timing_get.argtypes = [C.c_int, C.POINTER(C.c_char_p), C.POINTER(C.c_int32), C.POINTER(C.c_float)]
        lib.gfnx_status_string.restype = C.c_char_p
        lib.gfnx_status_string.argtypes = [C.c_int]
        _lib = lib
    return _lib


def status_string(status: int) -> str:
    return load_library().gfnx_status_string(int(status)).decode()


def _check(status: int) -> None:
    if status != GFNX_OK:
        raise GfnxError(status, status_string(status))


def env_desc(env, modes_dev_ptr: Optional[int] = None) -> EnvDesc:
    """C descriptor from a workloads.EnvSpec; modes_dev_ptr is the device address of the packed modes."""
    return EnvDesc(env.kind, env.grid_dim, env.grid_side, env.r0, env.r1, env.r2, env.n_bits, env.k_bits,
                   env.n_modes, modes_dev_ptr, env.beta, env.lattice_n, env.coupling)


def env_dims(env):
    out = [C.c_int32() for _ in range(4)]
    d = env if isinstance(env, EnvDesc) else env_desc(env)
    _check(load_library().gfnx_env_dims(C.byref(d), *[C.byref(o) for o in out]))
    return tuple(o.value for o in out)


class KernelTimer:
    """Per-kernel durations from the library's own HIP events (gfnx_timing_*)."""

    def __init__(self):
        self.lib = load_library()

    def enable(self, on: bool, only: Optional[str] = None) -> None:
        _check(self.lib.gfnx_timing_only(only.encode() if only else None))
        _check(self.lib.gfnx_timing_enable(1 if on else 0))

    def collect(self) -> Dict[str, tuple]:
        out = {}
        for i in range(self.lib.gfnx_timing_labels()):
            name, n, ms = C.c_char_p(), C.c_int32(), C.c_float()
            _check(self.lib.gfnx_timing_get(i, C.byref(name), C.byref(n), C.byref(ms)))
            if n.value:
                out[name.value.decode()] = (n.value, float(ms.value))
        return out


def _ptr(t) -> int:
    return int(t.data_ptr())


class Session:
    """Device buffers for one (environment, network, batch) and the calls of the C ABI on them."""

    def __init__(self, env, weights: Dict, batch: int, device: str = "cuda:0"):
        import torch
        self.torch = torch
        self.lib = load_library()
        self.env, self.batch, self.device = env, int(batch), torch.device(device)
        self.state_dim, self.obs_dim, self.n_actions, self.max_steps = env_dims(env)  # gfnx_env_dims
        dev = self.device
        self.modes = None
        if env.modes is not None:
            import numpy as np
            self.modes = torch.from_numpy(np.ascontiguousarray(env.modes, dtype=np.uint32).view(np.int32)).to(dev)
        self.desc = env_desc(env, None if self.modes is None else _ptr(self.modes))
        self.w = {k: torch.as_tensor(v, dtype=torch.float32).contiguous().to(dev) for k, v in weights.items()}
        self.mlp = Mlp(self.w["W1"].shape[0], self.w["W1"].shape[1], self.w["W2"].shape[1], self.w["W3"].shape[1],
                       *[_ptr(self.w[k]) for k in ("W1", "b1", "W2", "b2", "W3", "b3")])
        T, B = self.max_steps, self.batch
        # one byte per transition, or 16 bits for environments with more than 256 actions (gfnx_traj.actions16)
        self.wide_actions = self.n_actions > 256
        self.actions = torch.empty((T, B), dtype=torch.int16 if self.wide_actions else torch.uint8, device=dev)
        self.length = torch.empty(B, dtype=torch.int32, device=dev)
        self.terminal_state = torch.empty((self.state_dim, B), dtype=torch.int8, device=dev)
        self.log_pf = torch.empty(B, dtype=torch.float32, device=dev)
        self.log_pb = torch.empty(B, dtype=torch.float32, device=dev)
        self.log_reward = torch.empty(B, dtype=torch.float32, device=dev)
        self.traj = Traj(B, T, None if self.wide_actions else _ptr(self.actions), _ptr(self.length),
                         _ptr(self.terminal_state), _ptr(self.log_pf), _ptr(self.log_pb), _ptr(self.log_reward),
                         _ptr(self.actions) if self.wide_actions else None)
        self.grads = {"d" + k: torch.empty_like(v) for k, v in self.w.items()}
        self.cgrads = MlpGrad(*[_ptr(self.grads[k]) for k in ("dW1", "db1", "dW2", "db2", "dW3", "db3")])
        self.loss = torch.zeros(1, dtype=torch.float32, device=dev)
        self.dlogz = torch.zeros(1, dtype=torch.float32, device=dev)
        self.workspace_bytes = int(self.lib.gfnx_workspace_bytes(C.byref(self.desc), C.byref(self.mlp), B))
        if self.workspace_bytes == 0:
            raise GfnxError(-3, "gfnx_workspace_bytes rejected the configuration")
        self.workspace = torch.empty(self.workspace_bytes, dtype=torch.uint8, device=dev)
        assert _ptr(self.workspace) % 256 == 0

    def _stream(self) -> int:
        return int(self.torch.cuda.current_stream(self.device).cuda_stream)

    def set_weights(self, weights: Dict) -> None:
        for k, v in weights.items():
            self.w[k].copy_(self.torch.as_tensor(v, dtype=self.torch.float32))

    def rollout(self, seed: int, iteration: int, epsilon: float = None) -> None:
        """Samples the batch; with `epsilon`, through gfnx_rollout_explore (epsilon-uniform exploration)."""
        if epsilon is None:
            _check(self.lib.gfnx_rollout(C.byref(self.desc), C.byref(self.mlp), seed, iteration, C.byref(self.traj),
                                         _ptr(self.workspace), self.workspace_bytes, self._stream()))
        else:
            _check(self.lib.gfnx_rollout_explore(C.byref(self.desc), C.byref(self.mlp), seed, iteration,
                                                 float(epsilon), C.byref(self.traj), _ptr(self.workspace),
                                                 self.workspace_bytes, self._stream()))

    def _actions_tensor(self, actions):
        """Host action array [T, B] as a tensor of the plane's element type (torch has no uint16: the 16-bit plane is
        held as int16 with the same bits)."""
        import numpy as np
        if self.wide_actions:
            return self.torch.from_numpy(np.ascontiguousarray(actions, dtype=np.uint16).view(np.int16))
        return self.torch.as_tensor(actions, dtype=self.torch.uint8)

    def replay(self, actions, length) -> None:
        """Teacher-forced pass along the given host arrays actions [T, B] (uint8, or uint16 for environments with
        more than 256 actions) and length [B]."""
        torch = self.torch
        self.actions.copy_(self._actions_tensor(actions))
        self.length.copy_(torch.as_tensor(length, dtype=torch.int32))
        _check(self.lib.gfnx_replay(C.byref(self.desc), C.byref(self.mlp), C.byref(self.traj), _ptr(self.workspace),
                                    self.workspace_bytes, self._stream()))

    def workspace_rows(self, region: int, rows):
        """Device tensor [len(rows), row_bytes] (uint8) of the given rows (index t * batch + b, a device int64
        tensor) of a workspace region (gfnx_workspace_region); None where the region is not recorded."""
        off, rb = C.c_size_t(), C.c_size_t()
        rc = self.lib.gfnx_workspace_region(C.byref(self.desc), C.byref(self.mlp), self.batch, region,
                                            C.byref(off), C.byref(rb))
        if rc == -5:
            return None
        _check(rc)
        n_rows = self.max_steps * self.batch
        view = self.workspace[off.value:off.value + n_rows * rb.value].view(n_rows, rb.value)
        return view.index_select(0, rows)

    def tb_loss_grad(self, log_z: float = 0.0) -> None:
        _check(self.lib.gfnx_tb_loss_grad(C.byref(self.desc), C.byref(self.mlp), C.byref(self.traj), float(log_z),
                                          _ptr(self.loss), _ptr(self.dlogz), C.byref(self.cgrads),
                                          _ptr(self.workspace), self.workspace_bytes, self._stream()))

    # ---- backward rollouts and the estimate of P_theta(x) --------------------------
    def backward_rollout(self, seed: int, iteration: int, terminal_state=None) -> None:
        """Trajectories tau_b ~ P_B(. | x_b) for the terminal states in self.terminal_state (or the given host
        array [state_dim, batch]); fills actions (forward order), length, log_pb."""
        if terminal_state is not None:
            self.terminal_state.copy_(self.torch.as_tensor(terminal_state, dtype=self.torch.int8))
        _check(self.lib.gfnx_backward_rollout(C.byref(self.desc), seed, iteration, C.byref(self.traj), self._stream()))

    def replay_device(self) -> None:
        """Teacher-forced pass along the action bytes and lengths already on the device."""
        _check(self.lib.gfnx_replay(C.byref(self.desc), C.byref(self.mlp), C.byref(self.traj), _ptr(self.workspace),
                                    self.workspace_bytes, self._stream()))

    def log_prob_estimate(self, n_states: int, n_samples: int):
        """Device tensor [n_states] of log P_theta(x) estimated from this batch's log_pf and log_pb (the samples of
        state x at trajectory indices x * n_samples + i; n_states * n_samples = batch)."""
        assert n_states * n_samples == self.batch
        out = self.torch.empty(n_states, dtype=self.torch.float32, device=self.device)
        _check(self.lib.gfnx_log_prob_estimate(_ptr(self.log_pf), _ptr(self.log_pb), n_states, n_samples, _ptr(out),
                                               self._stream()))
        return out

    def estimate_log_prob(self, states, n_samples: int, seed: int, iteration: int):
        """log P_theta(x) for the host array states [n_states, state_dim]: backward rollouts, forward evaluation, mean."""
        torch = self.torch
        st = torch.as_tensor(states, dtype=torch.int8)
        n_states = int(st.shape[0])
        self.backward_rollout(seed, iteration, st.t().repeat_interleave(n_samples, dim=1).contiguous())
        self.replay_device()
        return self.log_prob_estimate(n_states, n_samples)

    # ---- training iterations -------------------------------------------------------
    def init_optimizer(self, log_z: float = 0.0, lr: float = 1e-3, lr_log_z: float = 1e-1, beta1: float = 0.9,
                       beta2: float = 0.999, eps: float = 1e-8) -> None:
        """Device-resident log Z and zeroed Adam moments; the update count restarts at zero."""
        torch = self.torch
        self.log_z = torch.full((1,), float(log_z), dtype=torch.float32, device=self.device)
        self.adam_m = {k: torch.zeros_like(v) for k, v in self.w.items()}
        self.adam_v = {k: torch.zeros_like(v) for k, v in self.w.items()}
        self.log_z_mv = torch.zeros(2, dtype=torch.float32, device=self.device)
        keys = ("W1", "b1", "W2", "b2", "W3", "b3")
        self.adam_state = AdamState(MlpGrad(*[_ptr(self.adam_m[k]) for k in keys]),
                                    MlpGrad(*[_ptr(self.adam_v[k]) for k in keys]), _ptr(self.log_z_mv))
        self.adam_cfg = AdamCfg(lr, lr_log_z, beta1, beta2, eps)
        self.updates = 0

    def adam_step(self) -> None:
        """One Adam update of the weights and log Z from the gradients of the last tb_loss_grad."""
        self.updates += 1
        _check(self.lib.gfnx_adam_step(C.byref(self.mlp), _ptr(self.log_z), C.byref(self.cgrads), _ptr(self.dlogz),
                                       C.byref(self.adam_state), C.byref(self.adam_cfg), self.updates,
                                       self._stream()))

    def train_step(self, seed: int, iteration: int, epsilon: float = 0.0, subtb_lambda: float = None) -> None:
        """Rollout, loss and gradient, Adam update: one call, no host round trip.  Default: on-policy Trajectory
        Balance (log Z read on the device); epsilon > 0 explores; subtb_lambda in [0, 1] trains a flow network with
        SubTB (0 = DB) instead."""
        self.updates += 1
        if epsilon == 0.0 and subtb_lambda is None:
            _check(self.lib.gfnx_train_step(C.byref(self.desc), C.byref(self.mlp), _ptr(self.log_z), seed, iteration,
                                            C.byref(self.traj), _ptr(self.loss), _ptr(self.dlogz),
                                            C.byref(self.cgrads), C.byref(self.adam_state), C.byref(self.adam_cfg),
                                            self.updates, _ptr(self.workspace), self.workspace_bytes, self._stream()))
            return
        opts = TrainOpts(float(epsilon), -1.0 if subtb_lambda is None else float(subtb_lambda))
        _check(self.lib.gfnx_train_step_opts(C.byref(self.desc), C.byref(self.mlp), _ptr(self.log_z), seed, iteration,
                                             C.byref(self.traj), _ptr(self.loss), _ptr(self.dlogz),
                                             C.byref(self.cgrads), C.byref(self.adam_state), C.byref(self.adam_cfg),
                                             C.byref(opts), self.updates, _ptr(self.workspace), self.workspace_bytes,
                                             self._stream()))

    def train_step_static(self, seed: int, iteration: int) -> None:
        """train_step on the library's own fixed scratch array (gfnx_train_step_static): no workspace is passed."""
        self.updates += 1
        _check(self.lib.gfnx_train_step_static(C.byref(self.desc), C.byref(self.mlp), _ptr(self.log_z), seed,
                                               iteration, C.byref(self.traj), _ptr(self.loss), _ptr(self.dlogz),
                                               C.byref(self.cgrads), C.byref(self.adam_state), C.byref(self.adam_cfg),
                                               self.updates, self._stream()))

    def weights(self) -> Dict:
        """Host copies (numpy) of the six weight tensors."""
        self.torch.cuda.synchronize(self.device)
        return {k: v.cpu().numpy() for k, v in self.w.items()}

    def subtb_loss_grad(self, lam: float) -> None:
        """SubTB(lambda) (lambda = 0: DB) loss and gradient; the network must have the flow output."""
        _check(self.lib.gfnx_subtb_loss_grad(C.byref(self.desc), C.byref(self.mlp), C.byref(self.traj), float(lam),
                                             _ptr(self.loss), C.byref(self.cgrads), _ptr(self.workspace),
                                             self.workspace_bytes, self._stream()))

    def trajectories(self) -> Dict:
        """Host copies (numpy) of the trajectory arrays."""
        self.torch.cuda.synchronize(self.device)
        import numpy as np
        acts = self.actions.cpu().numpy()
        return dict(actions=acts.view(np.uint16) if self.wide_actions else acts, length=self.length.cpu().numpy(),
                    terminal_state=self.terminal_state.cpu().numpy(), log_pf=self.log_pf.cpu().numpy(),
                    log_pb=self.log_pb.cpu().numpy(), log_reward=self.log_reward.cpu().numpy())

    def gradients(self) -> Dict:
        self.torch.cuda.synchronize(self.device)
        out = {k: v.cpu().numpy() for k, v in self.grads.items()}
        out["loss"] = float(self.loss.item())
        out["dlogz"] = float(self.dlogz.item())
        return out
