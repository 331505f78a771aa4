"""Seeded synthetic inputs: environment descriptors, policy weights, mode sets.

This module holds no arithmetic of the method itself (no policy evaluation, no
sampling, no reward, no loss): it only describes the five benchmark workloads and
draws their inputs from numpy's seeded generators.  Both the GPU binding and the
CPU reference used by the tests consume what it returns; neither is imported here.

The environments are the paper's synthetic ones (Appendix "Hypergrid", "Bit
sequences", "Ising model"), so these inputs are the workload itself, not a stand-in
for a dataset.
"""
from __future__ import annotations

from dataclasses import dataclass, field, replace
from typing import Dict, Optional

import numpy as np

ENV_GRID, ENV_BITSEQ, ENV_ISING, ENV_BITSEQ_NA = 0, 1, 2, 3


@dataclass(frozen=True)
class EnvSpec:
    """Plain description of an environment and its reward (host data only)."""

    kind: int
    grid_dim: int = 0
    grid_side: int = 0
    r0: float = 1e-3
    r1: float = 0.5
    r2: float = 2.0
    n_bits: int = 0
    k_bits: int = 0
    modes: Optional[np.ndarray] = None  # uint32 [n_modes, ceil(n_bits/32)]
    beta: float = 3.0
    lattice_n: int = 0
    coupling: float = 0.44

    @property
    def n_modes(self) -> int:
        return 0 if self.modes is None else int(self.modes.shape[0])

    def dims(self):
        """(state_dim, obs_dim, n_actions, max_steps)."""
        if self.kind == ENV_GRID:
            d, h = self.grid_dim, self.grid_side
            return d, d * h, d + 1, d * (h - 1) + 1
        if self.kind == ENV_BITSEQ:
            length = self.n_bits // self.k_bits
            return length, length * ((1 << self.k_bits) + 1), 1 << self.k_bits, length
        if self.kind == ENV_ISING:
            d = self.lattice_n ** 2
            return d, 3 * d, 2 * d, d
        if self.kind == ENV_BITSEQ_NA:
            length = self.n_bits // self.k_bits
            return length, length * ((1 << self.k_bits) + 1), length << self.k_bits, length
        raise ValueError("unknown environment kind")


def grid_env(dim: int, side: int, r0=1e-3, r1=0.5, r2=2.0) -> EnvSpec:
    return EnvSpec(kind=ENV_GRID, grid_dim=dim, grid_side=side, r0=r0, r1=r1, r2=r2)


def ising_env(n: int, coupling: float = 0.44) -> EnvSpec:
    return EnvSpec(kind=ENV_ISING, lattice_n=n, coupling=coupling)


# The five 8-bit building blocks of the mode set (Appendix "Bit sequences").
MODE_BLOCKS = ("00000000", "11111111", "11110000", "00001111", "00111100")


def pack_bits(bits: np.ndarray) -> np.ndarray:
    """[m, n] array of 0/1 -> uint32 [m, ceil(n/32)], string bit i in bit i%32 of word i//32."""
    m, n = bits.shape
    words = (n + 31) // 32
    out = np.zeros((m, words), dtype=np.uint32)
    for i in range(n):
        out[:, i // 32] |= (bits[:, i].astype(np.uint32) << np.uint32(i % 32))
    return out


def bitseq_modes(n_bits: int, n_modes: int, seed: int, uniform_bits: bool = False) -> np.ndarray:
    """Mode strings as a 0/1 array [n_modes, n_bits].

    Default: each mode is n_bits/8 blocks drawn with replacement from MODE_BLOCKS and
    concatenated (Appendix "Bit sequences").  uniform_bits=True draws every bit uniformly.
    """
    rng = np.random.default_rng([seed, 0x4D4F4445])
    if uniform_bits:
        return rng.integers(0, 2, size=(n_modes, n_bits), dtype=np.int64).astype(np.uint8)
    assert n_bits % 8 == 0
    blocks = np.array([[int(c) for c in s] for s in MODE_BLOCKS], dtype=np.uint8)
    pick = rng.integers(0, len(MODE_BLOCKS), size=(n_modes, n_bits // 8))
    return blocks[pick].reshape(n_modes, n_bits)


def bitseq_env(n_bits: int, k_bits: int, n_modes: int, mode_seed: int, beta: float = 3.0,
               uniform_bits: bool = False) -> EnvSpec:
    bits = bitseq_modes(n_bits, n_modes, mode_seed, uniform_bits)
    return EnvSpec(kind=ENV_BITSEQ, n_bits=n_bits, k_bits=k_bits, modes=pack_bits(bits), beta=beta)


def bitseq_na_env(n_bits: int, k_bits: int, n_modes: int, mode_seed: int, beta: float = 3.0,
                  uniform_bits: bool = False) -> EnvSpec:
    """Bit sequences in the non-autoregressive scheme (Appendix "Sequential environments"): same strings, modes
    and reward as bitseq_env; an action picks an empty position and the k-bit word written there."""
    bits = bitseq_modes(n_bits, n_modes, mode_seed, uniform_bits)
    return EnvSpec(kind=ENV_BITSEQ_NA, n_bits=n_bits, k_bits=k_bits, modes=pack_bits(bits), beta=beta)


def xavier_mlp(in_dim: int, h1: int, h2: int, n_actions: int, seed: int,
               dtype=np.float32) -> Dict[str, np.ndarray]:
    """Xavier-uniform weights (row-major [in][out]) and zero biases, drawn W1, W2, W3 in order."""
    rng = np.random.default_rng([seed, 0x57454947])
    out = {}
    for name, (fi, fo) in (("1", (in_dim, h1)), ("2", (h1, h2)), ("3", (h2, n_actions))):
        a = np.sqrt(6.0 / (fi + fo))
        out["W" + name] = rng.uniform(-a, a, size=(fi, fo)).astype(dtype)
        out["b" + name] = np.zeros(fo, dtype=dtype)
    return out


def random_mlp(in_dim: int, h1: int, h2: int, n_actions: int, seed: int, scale: float = 1.0,
               dtype=np.float32) -> Dict[str, np.ndarray]:
    """Like xavier_mlp but with non-zero biases and a gain, so every term of the forward and
    backward passes is exercised."""
    rng = np.random.default_rng([seed, 0x52414E44])
    out = {}
    for name, (fi, fo) in (("1", (in_dim, h1)), ("2", (h1, h2)), ("3", (h2, n_actions))):
        a = scale * np.sqrt(6.0 / (fi + fo))
        out["W" + name] = rng.uniform(-a, a, size=(fi, fo)).astype(dtype)
        out["b" + name] = rng.uniform(-0.1, 0.1, size=fo).astype(dtype)
    return out


@dataclass(frozen=True)
class Workload:
    name: str
    env: EnvSpec
    h1: int
    h2: int
    batch: int
    seed: int
    weight_seed: int
    log_z: float = 0.0
    stop_bias: float = 0.0  # added to b3[stop] on grids ("long-walk" variant); 0 = as initialised
    extra: dict = field(default_factory=dict)

    def mlp(self, dtype=np.float32) -> Dict[str, np.ndarray]:
        _, obs_dim, n_actions, _ = self.env.dims()
        w = xavier_mlp(obs_dim, self.h1, self.h2, n_actions, self.weight_seed, dtype)
        if self.stop_bias != 0.0:
            assert self.env.kind == ENV_GRID
            w["b3"][n_actions - 1] += dtype(self.stop_bias)
        return w

    def with_batch(self, batch: int) -> "Workload":
        return replace(self, batch=batch)


def workloads() -> Dict[str, Workload]:
    """The five configurations, the long-walk variants of the two large grids and a non-autoregressive bit-sequence
    instance."""
    w = {
        "c1": Workload("c1", grid_env(2, 8), 64, 64, batch=16, seed=0, weight_seed=1),
        "c2": Workload("c2", grid_env(4, 20), 256, 256, batch=4096, seed=2, weight_seed=2),
        "c3": Workload("c3", bitseq_env(120, 8, 60, mode_seed=3), 512, 512, batch=4096, seed=3, weight_seed=3),
        "c4": Workload("c4", ising_env(10), 256, 256, batch=4096, seed=4, weight_seed=4),
        "c5": Workload("c5", grid_env(10, 20), 256, 256, batch=16384, seed=5, weight_seed=5),
    }
    w["c2_long"] = replace(w["c2"], name="c2_long", stop_bias=-8.0)
    w["c5_long"] = replace(w["c5"], name="c5_long", stop_bias=-8.0)
    # the non-autoregressive scheme at the largest action space the kernels take: 16 positions x 16 words
    w["c3_na"] = Workload("c3_na", bitseq_na_env(64, 4, 60, mode_seed=3), 512, 512, batch=4096, seed=3, weight_seed=3)
    # ... and at the size of the paper's bit-sequence experiments: 15 positions x 256 words = 3840 actions
    w["c3_na120"] = Workload("c3_na120", bitseq_na_env(120, 8, 60, mode_seed=3), 512, 512, batch=4096, seed=3,
                             weight_seed=3)
    return w
