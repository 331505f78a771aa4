"""GPU parity: the HIP path (through the C ABI) against the CPU reference on the same seeded inputs.

Bars (written out here):
  * sampled actions, lengths and terminal states: bit-exact, except on steps where the reference's top-2
    Gumbel-perturbed logits are closer than 1e-5 (either action is then accepted; the reference follows the
    GPU's actions and counts such steps);
  * log P_F, log P_B, log R: relative 1e-4 (absolute floor 1e-5) against the binary64 reference along the
    GPU's own action sequence;
  * loss and dloss/dlogZ: relative 1e-4 (floor 1e-6); each gradient tensor: max |diff| <= 1e-4 * max |ref| + 1e-7,
    with no further allowance.  The derivative of the ReLU of a hidden unit whose pre-activation is zero to within
    binary32 rounding (|z| < 2e-6 * (|bias| + sum |terms|)) is a float-decided bit, like the near-tie argmax: there,
    and only there, the reference takes the bit the GPU recorded (read from the workspace between the rollout and
    the gradient call); every other recorded bit must equal the reference's own z > 0 -- checked for every hidden
    unit of every transition of the batch.
"""
import math
import os

import numpy as np
import pytest

from paper_2511_16592_amd.workloads import (bitseq_env, bitseq_na_env, grid_env, ising_env, random_mlp, workloads,
                                            xavier_mlp)
from tests.helpers import (chi2_sf, enumerate_grid_trajectories, grid_reward, optimal_policy_mlp_2d,
                           pack_trajectories)

pytestmark = pytest.mark.gpu
KEYS = ("dW1", "db1", "dW2", "db2", "dW3", "db3")
NTHREADS = min(16, os.cpu_count() or 1)
KINK_REL = 2e-6  # |z| below this fraction of sum|terms| (32 ulp of binary32): sign is not decidable in fp32


@pytest.fixture(scope="module")
def gfnx():
    import torch
    assert torch.cuda.is_available()
    from paper_2511_16592_amd import gfnx as g
    g.load_library()  # raises if the HIP library is missing: no fallback
    return g


def padded_optimal_mlp(side):
    """The proper policy of the 2-D grid as an MLP, its side^2 hidden units padded to the 64 the kernels need
    (the extra units are dead: bias -1, zero weights)."""
    w64, log_z = optimal_policy_mlp_2d(side)
    n = side * side
    w = dict(W1=np.zeros((2 * side, 64), np.float32), b1=-np.ones(64, np.float32),
             W2=np.zeros((64, 64), np.float32), b2=np.zeros(64, np.float32),
             W3=np.zeros((64, 3), np.float32), b3=np.zeros(3, np.float32))
    w["W1"][:, :n] = w64["W1"]
    w["W2"][:n, :n] = w64["W2"]
    w["W3"][:n] = w64["W3"]
    return w, log_z


def say(msg):
    print(msg, flush=True)


REGION_H1_SIGNS, REGION_H2_SIGNS, REGION_H2_ROWS = 0, 1, 2


def unpack_signs(packed, width):
    """[n, row_bytes] bytes of a sign-mask region -> [n, width] of 0 / 1: unit u is bit (u % 256) / 4 of the 64-bit
    little-endian word 4 * (u / 256) + u % 4 of its row (include/gfnx.h, gfnx_workspace_region)."""
    n = packed.shape[0]
    bits = np.unpackbits(np.ascontiguousarray(packed), axis=1, bitorder="little")  # [n, words * 64], word-major
    blocks = bits.reshape(n, -1, 4, 64).transpose(0, 1, 3, 2)                      # [n, block, bit l, word k]
    return np.ascontiguousarray(blocks.reshape(n, -1)[:, :width])


def relu_decisions(sess, traj):
    """The ReLU' bits the rollout recorded for every live transition, ordered column by column, step by step.  Call
    between the rollout and the gradient pass (the gradient pass consumes the workspace)."""
    import torch
    length = traj["length"].astype(np.int64)
    batch = length.shape[0]
    cols = np.repeat(np.arange(batch, dtype=np.int64), length)
    first = np.cumsum(length) - length
    steps = np.arange(int(length.sum()), dtype=np.int64) - np.repeat(first, length)
    rows = torch.as_tensor(steps * batch + cols, device=sess.device)
    h1, h2 = sess.w["W1"].shape[1], sess.w["W2"].shape[1]
    relu1 = unpack_signs(sess.workspace_rows(REGION_H1_SIGNS, rows).cpu().numpy(), h1)
    packed2 = sess.workspace_rows(REGION_H2_SIGNS, rows)
    if packed2 is None:  # narrow networks keep no h2 bits: the sign of the stored activation
        relu2 = (sess.workspace_rows(REGION_H2_ROWS, rows).view(torch.float32) > 0).to(torch.uint8).cpu().numpy()
    else:
        relu2 = unpack_signs(packed2.cpu().numpy(), h2)
    return relu1, relu2


def check_trajectories(o32, o64, env, w, seed, iteration, traj, b0=0, b1=None, free_run=True):
    """Compares columns [b0, b1) of the GPU trajectories with the reference; returns number of near-tie steps."""
    b1 = traj["length"].shape[0] if b1 is None else b1
    acts = np.ascontiguousarray(traj["actions"][:, b0:b1])
    length = np.ascontiguousarray(traj["length"][b0:b1])
    sd, _, na, ms = env.dims()
    assert (length >= 1).all() and (length <= ms).all()
    rep = o32.replay(env, w, seed, iteration, acts, length, b_offset=b0, tie_tol=1e-5, nthreads=NTHREADS)
    assert (rep["violations"] == 0).all(), "GPU action differs from the reference argmax beyond the 1e-5 margin"
    clean = rep["near_ties"] == 0
    # a step is a near tie when the reference's top-2 gap is under 1e-5 AND the GPU's rounding flips it: at most
    # a few times the ~1e-5 per step that the gap alone allows
    assert int(rep["near_ties"].sum()) <= 10 * 2e-5 * int(length.sum()) + 3, int(rep["near_ties"].sum())
    assert (rep["terminal_state"] == traj["terminal_state"][:, b0:b1]).all()
    for t in range(acts.shape[0]):  # padding after the end of each trajectory
        pad = t >= length
        if na <= 255:
            assert (acts[t][pad] == 0xFF).all()
        elif na > 256:
            assert (acts[t][pad] == 0xFFFF).all()
    if free_run:
        free = o32.rollout(env, w, seed, iteration, batch=b1 - b0, b_offset=b0, max_steps=acts.shape[0],
                           nthreads=NTHREADS)
        assert (free["length"][clean] == length[clean]).all()
        assert (free["actions"][:, clean] == acts[:, clean]).all()
        assert (free["terminal_state"][:, clean] == traj["terminal_state"][:, b0:b1][:, clean]).all()
    ref = o64.replay(env, w, seed, iteration, acts, length, b_offset=b0, tie_tol=1e30, nthreads=NTHREADS)
    for k in ("log_pf", "log_pb", "log_reward"):
        got, want = traj[k][b0:b1].astype(np.float64), ref[k]
        err = np.abs(got - want) - (1e-4 * np.abs(want) + 1e-5)
        assert (err <= 0).all(), (k, float(err.max()))
    return int(rep["near_ties"].sum())


def check_gradients(o64, env, w, traj, grads, log_z, relu=None):
    """Loss, dloss/dlogZ and the six gradient tensors against the binary64 reference along the GPU's actions, at the
    bars of the module docstring.  relu = (relu1, relu2) from relu_decisions()."""
    assert relu is not None, "the ReLU decisions of the rollout are part of every gradient check"
    g = o64.tb_loss_grad_follow(env, w, traj["actions"], traj["length"], relu[0], relu[1], log_z,
                                kink_tol=KINK_REL, nthreads=NTHREADS)
    assert g["mismatched"] == 0, "a recorded ReLU' bit differs from the reference outside the rounding margin"
    n_units = int(traj["length"].sum()) * (w["W1"].shape[1] + w["W2"].shape[1])
    assert g["followed"] <= 2e-5 * n_units + 2, g["followed"]  # the margin may only ever cover a sliver of the units
    assert abs(grads["loss"] - g["loss"]) <= 1e-4 * abs(g["loss"]) + 1e-6, (grads["loss"], g["loss"])
    assert abs(grads["dlogz"] - g["dlogz"]) <= 1e-4 * abs(g["dlogz"]) + 1e-6, (grads["dlogz"], g["dlogz"])
    worst = {}
    for k in KEYS:
        scale = np.abs(g[k]).max()
        err = np.abs(grads[k].astype(np.float64) - g[k]).max()
        worst[k] = err / (1e-4 * scale + 1e-7)
        assert err <= 1e-4 * scale + 1e-7, (k, float(err), float(scale), g["followed"], g["flipped"])
    say(f"    gradients: err/bar " + " ".join(f"{k}:{worst[k]:.2g}" for k in KEYS) +
        f"; {n_units} ReLU' bits equal to the reference's, {g['followed']} inside the rounding margin taken from "
        f"the GPU ({g['flipped']} of them the other way)")
    return g


def run_case(gfnx, o32, o64, env, w, batch, seed, iteration, log_z, name, free_run=True):
    say(f"[case {name}] batch={batch} seed={seed} iteration={iteration}")
    sess = gfnx.Session(env, w, batch)
    sess.rollout(seed, iteration)
    traj = sess.trajectories()
    relu = relu_decisions(sess, traj)
    sess.tb_loss_grad(log_z)
    grads = sess.gradients()
    ties = check_trajectories(o32, o64, env, w, seed, iteration, traj, free_run=free_run)
    check_gradients(o64, env, w, traj, grads, log_z, relu)
    say(f"[case {name}] ok: {int(traj['length'].sum())} transitions, {ties} near-tie steps, loss {grads['loss']:.6g}")
    return sess, traj, grads


# ------------------------------------------------------------------ small cases: several tiles, ragged tails
def test_c1_grid_2d_side8(gfnx, oracle32, oracle64):
    wl = workloads()["c1"]
    run_case(gfnx, oracle32, oracle64, wl.env, wl.mlp(), wl.batch, wl.seed, 0, wl.log_z, "c1")


@pytest.mark.parametrize("batch", [1, 37, 200])
def test_grid_ragged_batches(gfnx, oracle32, oracle64, batch):
    env = grid_env(3, 5)
    w = random_mlp(15, 64, 128, 4, seed=31, scale=2.0)
    run_case(gfnx, oracle32, oracle64, env, w, batch, seed=9, iteration=4, log_z=0.7, name=f"grid3x5_b{batch}")


def test_grid_long_walks(gfnx, oracle32, oracle64):
    """Stop bias -8: trajectories run to the far corner (maximum length d*(H-1)+1 occurs)."""
    env = grid_env(2, 8)
    w = xavier_mlp(16, 64, 64, 3, seed=1)
    w["b3"][2] = -8.0
    _, traj, _ = run_case(gfnx, oracle32, oracle64, env, w, 50, seed=1, iteration=0, log_z=0.0, name="grid_long")
    assert traj["length"].max() >= 14


def test_bitseq_small(gfnx, oracle32, oracle64):
    env = bitseq_env(24, 4, 7, mode_seed=2)
    w = random_mlp(6 * 17, 64, 64, 16, seed=32, scale=2.0)
    run_case(gfnx, oracle32, oracle64, env, w, 45, seed=5, iteration=1, log_z=-0.3, name="bitseq24")


def test_bitseq_odd_token_width(gfnx, oracle32, oracle64):
    """k=3: token chunks straddle the 32-bit words of the packed modes."""
    env = bitseq_env(72, 3, 5, mode_seed=4, uniform_bits=True)
    w = random_mlp(24 * 9, 64, 64, 8, seed=33, scale=2.0)
    run_case(gfnx, oracle32, oracle64, env, w, 20, seed=6, iteration=0, log_z=0.0, name="bitseq72k3")


@pytest.mark.parametrize("n", [3, 5])
def test_ising_small(gfnx, oracle32, oracle64, n):
    env = ising_env(n)
    w = random_mlp(3 * n * n, 64, 64, 2 * n * n, seed=34, scale=2.0)
    run_case(gfnx, oracle32, oracle64, env, w, 33, seed=7, iteration=2, log_z=1.5, name=f"ising{n}")


def test_different_hidden_widths(gfnx, oracle32, oracle64):
    env = grid_env(4, 6)
    w = random_mlp(24, 192, 320, 5, seed=35, scale=1.5)
    run_case(gfnx, oracle32, oracle64, env, w, 70, seed=8, iteration=3, log_z=0.2, name="grid_h192_320")


def _wide_cases():
    """256-wide networks on small environments: the on-chip-W2 rollout, the bf16 one-hot contraction with a ragged
    number of one-hot columns, the one-sweep logit backward (<= 16 logits) and the GEMM pair (17..32 logits),
    slot refill (batch > 4096), and unequal hidden widths on the fast gradient kernels."""
    return [
        ("grid3x7_256", grid_env(3, 7), (21, 256, 256, 4), 100),
        ("grid3x7_256_refill", grid_env(3, 7), (21, 256, 256, 4), 5000),
        ("grid16x3_256", grid_env(16, 3), (48, 256, 256, 17), 90),
        ("ising3_256", ising_env(3), (27, 256, 256, 18), 40),
        ("bitseq24k4_256", bitseq_env(24, 4, 7, mode_seed=2), (6 * 17, 256, 256, 16), 45),
        ("grid4x6_128_256", grid_env(4, 6), (24, 128, 256, 5), 70),
        ("grid4x6_256_64", grid_env(4, 6), (24, 256, 64, 5), 70),
        # 512-wide: four layer-2 tiles per wave in the rollout, the split-contraction input-gradient kernel
        ("bitseq24k4_512", bitseq_env(24, 4, 7, mode_seed=2), (6 * 17, 512, 512, 16), 150),
        ("grid4x6_512_384", grid_env(4, 6), (24, 512, 384, 5), 70),
        # Ising one-hot layer-1 gradient at 256 wide, 50 one-hot columns in use
        ("ising5_256", ising_env(5), (75, 256, 256, 50), 40),
        ("grid11x2_320_192", grid_env(2, 11), (22, 320, 192, 3), 300),
    ]


@pytest.mark.parametrize("case", _wide_cases(), ids=lambda c: c[0])
def test_wide_networks_small_envs(gfnx, oracle32, oracle64, case):
    name, env, (n_in, h1, h2, n_act), batch = case
    w = random_mlp(n_in, h1, h2, n_act, seed=36, scale=1.5)
    run_case(gfnx, oracle32, oracle64, env, w, batch, seed=11, iteration=5, log_z=0.4, name=name)


def _na_cases():
    """Bit sequences in the non-autoregressive scheme (position, word): one and two logit chunks per lane, resident
    and streamed layer 2, one-bit words (two positions per chunk of four actions), words that straddle the 32-bit
    words of the packed modes, the largest action space the kernels take (256), a batch with slot refill."""
    return [
        ("na12k2", bitseq_na_env(12, 2, 5, mode_seed=2, uniform_bits=True), (64, 64), 60),
        ("na24k4", bitseq_na_env(24, 4, 7, mode_seed=2), (64, 128), 45),
        ("na8k1", bitseq_na_env(8, 1, 4, mode_seed=4, uniform_bits=True), (64, 64), 70),
        ("na21k3", bitseq_na_env(21, 3, 5, mode_seed=4, uniform_bits=True), (128, 64), 33),
        ("na24k4_256", bitseq_na_env(24, 4, 7, mode_seed=2), (256, 256), 90),
        ("na64k4_256", bitseq_na_env(64, 4, 20, mode_seed=3), (256, 256), 300),
        ("na64k4_512_refill", bitseq_na_env(64, 4, 20, mode_seed=3), (512, 512), 4200),
        ("na40k5", bitseq_na_env(40, 5, 9, mode_seed=6, uniform_bits=True), (192, 64), 50),
    ]


@pytest.mark.parametrize("case", _na_cases(), ids=lambda c: c[0])
def test_non_autoregressive_bit_sequences(gfnx, oracle32, oracle64, case):
    name, env, (h1, h2), batch = case
    sd, od, na, ms = env.dims()
    w = random_mlp(od, h1, h2, na, seed=39, scale=1.5)
    _, traj, _ = run_case(gfnx, oracle32, oracle64, env, w, batch, seed=17, iteration=3, log_z=0.3, name=name)
    assert (traj["length"] == ms).all()
    pos = traj["actions"].astype(int) >> env.k_bits
    assert (np.sort(pos, axis=0) == np.arange(ms)[:, None]).all()       # every position filled exactly once
    assert np.allclose(traj["log_pb"], -math.lgamma(ms + 1), rtol=1e-5)  # uniform over the filled positions
    if batch >= 60:
        assert len({tuple(pos[:, b]) for b in range(batch)}) > batch // 3  # in many different orders


def _na_wide_cases():
    """More than 256 actions (16-bit action plane, logits in pages of 256): two to five pages, words of 5, 6 and 8
    bits, hidden widths from 64 to 512, a batch with several groups of 16 trajectories per workgroup."""
    return [
        ("na16k8", bitseq_na_env(16, 8, 5, mode_seed=2), (64, 64), 50),
        ("na16k8_b1", bitseq_na_env(16, 8, 5, mode_seed=2), (64, 64), 1),
        ("na24k8_128_192", bitseq_na_env(24, 8, 7, mode_seed=3), (128, 192), 37),
        ("na80k5", bitseq_na_env(80, 5, 6, mode_seed=4, uniform_bits=True), (64, 128), 33),
        ("na96k6_256", bitseq_na_env(96, 6, 9, mode_seed=5, uniform_bits=True), (256, 256), 70),
        ("na40k8_512", bitseq_na_env(40, 8, 20, mode_seed=3), (512, 512), 300),
        ("na16k8_groups", bitseq_na_env(16, 8, 5, mode_seed=2), (64, 64), 4200),
    ]


@pytest.mark.parametrize("case", _na_wide_cases(), ids=lambda c: c[0])
def test_non_autoregressive_bit_sequences_beyond_256_actions(gfnx, oracle32, oracle64, case):
    name, env, (h1, h2), batch = case
    sd, od, na, ms = env.dims()
    assert na > 256 and na % 256 == 0
    w = random_mlp(od, h1, h2, na, seed=41, scale=1.5)
    _, traj, _ = run_case(gfnx, oracle32, oracle64, env, w, batch, seed=19, iteration=2, log_z=0.2, name=name)
    assert traj["actions"].dtype == np.uint16 and (traj["length"] == ms).all()
    pos = traj["actions"].astype(int) >> env.k_bits
    assert (np.sort(pos, axis=0) == np.arange(ms)[:, None]).all()       # every position filled exactly once
    assert np.allclose(traj["log_pb"], -math.lgamma(ms + 1), rtol=1e-5)  # uniform over the filled positions
    if batch >= 60:
        assert traj["actions"].max() > 255


def test_teacher_forced_pass_beyond_256_actions(gfnx, oracle64):
    """gfnx_replay along given 16-bit actions: the rollout's own actions give its scalars and gradient back; an
    action on a filled position cuts that trajectory without touching the others."""
    env = bitseq_na_env(24, 8, 7, mode_seed=3)
    sd, od, na, ms = env.dims()
    w = random_mlp(od, 64, 128, na, seed=43, scale=1.5)
    sess = gfnx.Session(env, w, 90)
    sess.rollout(23, 1)
    sess.tb_loss_grad(0.1)
    traj, g1 = sess.trajectories(), sess.gradients()
    sess.replay(traj["actions"], traj["length"])
    sess.tb_loss_grad(0.1)
    again, g2 = sess.trajectories(), sess.gradients()
    for k in ("log_pf", "log_pb", "log_reward"):
        np.testing.assert_allclose(again[k], traj[k], rtol=1e-6, atol=1e-6)
    assert (again["terminal_state"] == traj["terminal_state"]).all()
    for k in KEYS:
        # (dW1 is summed with atomics: the order of the additions differs from launch to launch)
        np.testing.assert_allclose(g2[k], g1[k], rtol=1e-4, atol=1e-6 * np.abs(g1[k]).max())
    bad = traj["actions"].copy()
    bad[1, 5] = bad[0, 5] ^ 1   # the position filled at step 0 again
    sess.replay(bad, traj["length"])
    cut = sess.trajectories()
    ref = oracle64.replay(env, {k: v.astype(np.float64) for k, v in w.items()}, 0, 0, np.ascontiguousarray(bad[:1, 5:6]),
                          np.array([1], np.int32), tie_tol=1e30)
    assert abs(cut["log_pf"][5] - ref["log_pf"][0]) < 1e-4 * abs(ref["log_pf"][0]) + 1e-5   # the first step only
    keep = np.arange(90) != 5
    np.testing.assert_allclose(cut["log_pf"][keep], traj["log_pf"][keep], rtol=1e-6, atol=1e-6)
    # sequences that stop early (given lengths 1 and 2 of 3): the scalars of the steps taken, nothing more
    short = traj["length"].copy()
    short[7], short[20] = 1, 2
    sess.replay(traj["actions"], short)
    part = sess.trajectories()
    w64 = {k: v.astype(np.float64) for k, v in w.items()}
    for b, n in ((7, 1), (20, 2)):
        ref = oracle64.replay(env, w64, 0, 0, np.ascontiguousarray(traj["actions"][:n, b:b + 1]), np.array([n], np.int32),
                              tie_tol=1e30)
        assert abs(part["log_pf"][b] - ref["log_pf"][0]) < 1e-4 * abs(ref["log_pf"][0]) + 1e-5
        assert abs(part["log_pb"][b] - ref["log_pb"][0]) < 1e-5
    keep = (np.arange(90) != 7) & (np.arange(90) != 20)
    np.testing.assert_allclose(part["log_pf"][keep], traj["log_pf"][keep], rtol=1e-6, atol=1e-6)


def test_full_paper_size_non_autoregressive_bit_sequences(gfnx, oracle32, oracle64):
    """The paper's own bit-sequence setting: n = 120, k = 8 (15 positions x 256 words = 3840 actions), 60 modes,
    batch 4096, MLP 3855 - 512 - 512 - 3840: every action, scalar and gradient tensor against the reference."""
    env = bitseq_na_env(120, 8, 60, mode_seed=3)
    sd, od, na, ms = env.dims()
    assert (od, na, ms) == (3855, 3840, 15)
    w = xavier_mlp(od, 512, 512, na, seed=3)
    _, traj, _ = run_case(gfnx, oracle32, oracle64, env, w, 4096, seed=3, iteration=0, log_z=0.0, name="na120k8_4096")
    pos = traj["actions"].astype(int) >> 8
    assert (np.sort(pos, axis=0) == np.arange(15)[:, None]).all()


def test_action_space_limits_of_the_non_autoregressive_kind(gfnx):
    """More than 256 actions must come in whole pages of 256 (n = 60, k = 5: 384 actions is refused)."""
    env = bitseq_na_env(60, 5, 4, mode_seed=3, uniform_bits=True)
    with pytest.raises(gfnx.GfnxError) as err:
        gfnx.Session(env, random_mlp(12 * 33, 64, 64, 384, seed=1), 16)
    assert err.value.status in (-3, -5)


def test_rollout_is_deterministic_and_batch_split_invariant(gfnx):
    wl = workloads()["c1"]
    w = wl.mlp()
    a = gfnx.Session(wl.env, w, 64)
    a.rollout(3, 5)
    ta = a.trajectories()
    a.rollout(3, 5)
    tb = a.trajectories()
    for k in ta:
        assert (ta[k] == tb[k]).all()
    small = gfnx.Session(wl.env, w, 20)  # trajectory b depends on (seed, iteration, b) only
    small.rollout(3, 5)
    ts = small.trajectories()
    assert (ts["actions"] == ta["actions"][:, :20]).all()
    assert (ts["log_pf"] == ta["log_pf"][:20]).all()
    a.rollout(3, 6)
    assert (a.trajectories()["actions"] != ta["actions"]).any()


@pytest.mark.parametrize("batch", [3, 4, 5, 21, 260])
def test_wide_grid_few_running_trajectories(gfnx, oracle32, oracle64, batch):
    """256-wide grid policies switch to the four-slot matrix path whenever a workgroup has at most four running
    trajectories: batches of 3 and 4 never leave it, 5 enters it as soon as one walk ends, 21 and 260 mix full and
    nearly empty workgroups; long walks (stop bias -3) keep the tail long."""
    env = grid_env(3, 9)
    w = random_mlp(27, 256, 256, 4, seed=37, scale=1.5)
    w["b3"][3] -= 3.0
    _, traj, _ = run_case(gfnx, oracle32, oracle64, env, w, batch, seed=14, iteration=2, log_z=0.1,
                          name=f"grid3x9_256_b{batch}")
    assert traj["length"].max() >= 10


def test_wide_grid_batch_split_changes_rounding_only(gfnx):
    """The path a step takes depends on how many trajectories of the workgroup still run, so the same trajectory in
    a different batch sees sums rounded in a different order: same actions (no near-tie here), floats to 1e-6."""
    env = grid_env(3, 9)
    w = random_mlp(27, 256, 256, 4, seed=37, scale=1.5)
    a = gfnx.Session(env, w, 64)
    a.rollout(3, 5)
    ta = a.trajectories()
    small = gfnx.Session(env, w, 3)
    small.rollout(3, 5)
    ts = small.trajectories()
    assert (ts["actions"] == ta["actions"][:, :3]).all() and (ts["length"] == ta["length"][:3]).all()
    np.testing.assert_allclose(ts["log_pf"], ta["log_pf"][:3], rtol=1e-6, atol=1e-6)
    a.rollout(3, 5)
    tb = a.trajectories()
    for k in ta:
        assert (ta[k] == tb[k]).all()   # the same launch twice is bit-identical


def test_trajectory_buffer_longer_than_the_environment_needs(gfnx, oracle32, oracle64):
    """traj->max_steps may exceed the environment's: the extra steps stay 0xFF padding and nothing else moves."""
    import torch
    env = grid_env(3, 5)
    w = random_mlp(15, 64, 128, 4, seed=38, scale=1.5)
    sess = gfnx.Session(env, w, 90)
    extra = 6
    T = sess.max_steps + extra
    sess.actions = torch.zeros((T, 90), dtype=torch.uint8, device=sess.device)
    sess.traj = gfnx.Traj(90, T, int(sess.actions.data_ptr()), int(sess.length.data_ptr()),
                          int(sess.terminal_state.data_ptr()), int(sess.log_pf.data_ptr()),
                          int(sess.log_pb.data_ptr()), int(sess.log_reward.data_ptr()))
    sess.rollout(15, 2)
    traj = sess.trajectories()
    relu = relu_decisions(sess, traj)
    sess.tb_loss_grad(0.3)
    grads = sess.gradients()
    assert (traj["actions"][sess.max_steps:] == 0xFF).all()
    ref = gfnx.Session(env, w, 90)
    ref.rollout(15, 2)
    ref.tb_loss_grad(0.3)
    t2, g2 = ref.trajectories(), ref.gradients()
    assert (traj["actions"][:sess.max_steps] == t2["actions"]).all()
    for k in ("length", "terminal_state", "log_pf", "log_pb", "log_reward"):
        assert (traj[k] == t2[k]).all()
    for k in KEYS:
        assert np.array_equal(grads[k], g2[k])
    check_trajectories(oracle32, oracle64, env, w, 15, 2, traj)
    check_gradients(oracle64, env, w, traj, grads, 0.3, relu)


def test_longest_supported_walks(gfnx, oracle32, oracle64):
    """15-D grid of side 18: 256 steps at most (the supported maximum), 270 one-hot inputs (more than the 256 the
    one-hot contraction takes: the per-trajectory segment-sum path of the layer-1 gradient), stop bias -8."""
    env = grid_env(15, 18)
    assert env.dims()[3] == 256
    w = xavier_mlp(270, 64, 64, 16, seed=41)
    w["b3"][15] = -8.0
    _, traj, _ = run_case(gfnx, oracle32, oracle64, env, w, 24, seed=12, iteration=1, log_z=0.0, name="grid15x18")
    assert traj["length"].max() >= 200


def test_kernel_timing_interface(gfnx):
    """gfnx_timing_*: per-label launch counts and times; the label filter keeps only the chosen kernel."""
    import torch
    wl = workloads()["c1"]
    sess = gfnx.Session(wl.env, wl.mlp(), wl.batch)
    timer = gfnx.KernelTimer()
    timer.enable(True)
    for i in range(3):
        sess.rollout(wl.seed, i)
        sess.tb_loss_grad(0.0)
    torch.cuda.synchronize()
    rec = timer.collect()
    assert rec["rollout"][0] == 3 and rec["rollout"][1] > 0.0
    assert {"prepare", "rows", "reduce"} <= set(rec)
    timer.enable(True, only="rollout")
    sess.rollout(wl.seed, 9)
    sess.tb_loss_grad(0.0)
    torch.cuda.synchronize()
    rec = timer.collect()
    assert set(rec) == {"rollout"} and rec["rollout"][0] == 1
    timer.enable(False)
    sess.rollout(wl.seed, 10)
    torch.cuda.synchronize()
    assert timer.collect() == {}


def test_replay_cuts_a_trajectory_at_an_impossible_action(gfnx, oracle64):
    """A given action that is impossible in its state ends that trajectory there (no fault, no effect on the
    others); the other trajectories match the reference as usual."""
    env = grid_env(2, 4)
    trajs = enumerate_grid_trajectories(2, 4)[:32]
    actions, length = pack_trajectories(trajs, 7)
    w = random_mlp(8, 64, 64, 3, seed=37, scale=2.0)
    sess = gfnx.Session(env, w, len(trajs))
    sess.replay(actions, length)
    good = sess.trajectories()
    bad_actions = actions.copy()
    victim = int(np.argmax(length))
    bad_actions[1, victim] = 200  # not an action of this environment
    sess.replay(bad_actions, length)
    got = sess.trajectories()
    others = np.arange(len(trajs)) != victim
    for k in ("log_pf", "log_pb", "log_reward"):
        assert (got[k][others] == good[k][others]).all(), k
    assert (got["terminal_state"][:, others] == good["terminal_state"][:, others]).all()
    assert np.isfinite(got["log_pf"][victim]) and np.isfinite(got["log_reward"][victim])
    sess.tb_loss_grad(0.1)
    g = sess.gradients()
    assert all(np.isfinite(g[k]).all() for k in KEYS) and np.isfinite(g["loss"])


# ------------------------------------------------------------------ teacher-forced pass and the DP-optimal policy
def test_replay_of_all_trajectories_and_optimal_policy(gfnx, oracle64):
    """All 69 complete trajectories of the 2-D side-4 grid, teacher-forced: with the proper forward policy
    (embedded in an MLP) every TB residual is zero, so loss and all gradients vanish; sum_tau P_F(tau) = 1."""
    side = 4
    env = grid_env(2, side)
    trajs = enumerate_grid_trajectories(2, side)
    actions, length = pack_trajectories(trajs, 7)
    w, log_z = padded_optimal_mlp(side)
    sess = gfnx.Session(env, w, len(trajs))
    sess.replay(actions, length)
    sess.tb_loss_grad(log_z)
    traj, grads = sess.trajectories(), sess.gradients()
    assert abs(np.exp(traj["log_pf"].astype(np.float64)).sum() - 1.0) < 1e-5
    delta = log_z + traj["log_pf"] - traj["log_reward"] - traj["log_pb"]
    assert np.abs(delta).max() < 5e-6
    assert grads["loss"] < 1e-10 and abs(grads["dlogz"]) < 1e-5
    for k in KEYS:
        assert np.abs(grads[k]).max() < 1e-5, k
    for b, (_a, x) in enumerate(trajs):
        assert tuple(traj["terminal_state"][:, b]) == x
    # a random network on the same trajectories: full parity of scalars and gradients
    wr = random_mlp(8, 64, 64, 3, seed=36, scale=3.0)
    sess.set_weights(wr)
    sess.replay(actions, length)
    traj = sess.trajectories()
    relu = relu_decisions(sess, traj)
    sess.tb_loss_grad(0.4)
    grads = sess.gradients()
    ref = oracle64.replay(env, wr, 0, 0, actions, length, tie_tol=1e30)
    for k in ("log_pf", "log_pb", "log_reward"):
        assert np.allclose(traj[k], ref[k], rtol=1e-4, atol=1e-5)
    check_gradients(oracle64, env, wr, dict(actions=actions, length=length), grads, 0.4, relu)


def test_sampler_reaches_reward_distribution_on_gpu(gfnx):
    """Sampling on the GPU with the proper policy gives terminal states ~ R/Z (chi-square, 16 states)."""
    side = 4
    env = grid_env(2, side)
    w, _ = padded_optimal_mlp(side)
    n = 65536
    sess = gfnx.Session(env, w, n)
    sess.rollout(4242, 0)
    traj = sess.trajectories()
    idx = traj["terminal_state"][0].astype(int) * side + traj["terminal_state"][1].astype(int)
    counts = np.bincount(idx, minlength=16)
    probs = np.array([grid_reward((i, j), side) for i in range(side) for j in range(side)]) / 2.016
    stat = float(((counts - probs * n) ** 2 / (probs * n)).sum())
    assert chi2_sf(stat, 15) > 1e-4
    assert (traj["length"] == traj["terminal_state"].sum(0) + 1).all()


# ------------------------------------------------------------------ full-size configurations (as benchmarked)
def _full_size(gfnx, o32, o64, name, sample, full_grad, iteration=0):
    wl = workloads()[name]
    w = wl.mlp()
    say(f"[full {name}] batch={wl.batch} seed={wl.seed} iteration={iteration}")
    sess = gfnx.Session(wl.env, w, wl.batch)
    sess.rollout(wl.seed, iteration)
    traj = sess.trajectories()
    relu = relu_decisions(sess, traj) if full_grad else None
    sess.tb_loss_grad(wl.log_z)
    grads = sess.gradients()
    sd, _, na, ms = wl.env.dims()
    assert (traj["length"] >= 1).all() and (traj["length"] <= ms).all()
    ties = 0
    if sample is None:  # every trajectory of the batch against the reference
        ties = check_trajectories(o32, o64, wl.env, w, wl.seed, iteration, traj)
    else:
        for b0, b1 in sample:  # contiguous column blocks
            ties += check_trajectories(o32, o64, wl.env, w, wl.seed, iteration, traj, b0, min(b1, wl.batch))
    # properties that hold at any size
    delta = wl.log_z + traj["log_pf"].astype(np.float64) - traj["log_reward"] - traj["log_pb"]
    assert abs(grads["loss"] - np.mean(delta ** 2)) <= 1e-4 * np.mean(delta ** 2) + 1e-6
    assert abs(grads["dlogz"] - 2 * np.mean(delta)) <= 1e-4 * abs(2 * np.mean(delta)) + 1e-6
    assert abs(grads["db3"].sum()) <= 1e-4 * np.abs(grads["db3"]).max() * na + 1e-7
    if wl.env.kind == 2:
        assert np.allclose(traj["log_pb"], -math.lgamma(sd + 1), rtol=1e-5)
    if wl.env.kind == 1:
        assert (traj["log_pb"] == 0).all() and (traj["length"] == ms).all()
    if wl.env.kind == 0:
        assert (traj["length"] == traj["terminal_state"].astype(int).sum(0) + 1).all()
    if full_grad:
        check_gradients(o64, wl.env, w, traj, grads, wl.log_z, relu)
    say(f"[full {name}] ok: {int(traj['length'].sum())} transitions, {ties} near-tie steps")


def test_full_c2(gfnx, oracle32, oracle64):
    _full_size(gfnx, oracle32, oracle64, "c2", sample=None, full_grad=True)


def test_full_c2_long_walk(gfnx, oracle32, oracle64):
    _full_size(gfnx, oracle32, oracle64, "c2_long", sample=None, full_grad=True)


def test_full_c3(gfnx, oracle32, oracle64):
    _full_size(gfnx, oracle32, oracle64, "c3", sample=None, full_grad=True)


def test_full_c4(gfnx, oracle32, oracle64):
    _full_size(gfnx, oracle32, oracle64, "c4", sample=None, full_grad=True)


def test_full_c5(gfnx, oracle32, oracle64):
    _full_size(gfnx, oracle32, oracle64, "c5", sample=None, full_grad=True)


def test_full_c5_long_walk(gfnx, oracle32, oracle64):
    """3.1 M transitions: trajectories are checked on a sample; the gradient through the identities above
    (the full reference gradient at this size takes minutes on the host) and through the reduced batch below."""
    _full_size(gfnx, oracle32, oracle64, "c5_long", sample=[(0, 256), (4096, 4608), (16128, 16384)], full_grad=False)
    wl = workloads()["c5_long"]
    run_case(gfnx, oracle32, oracle64, wl.env, wl.mlp(), 256, wl.seed, 1, wl.log_z, "c5_long_b256", free_run=False)


def test_grid_reward_on_the_thresholds_side11(gfnx, oracle32, oracle64):
    """Side 11: x = 2, 8 sit exactly on |x/10 - 0.5| = 0.3 and x = 1, 9 on 0.4 (strict inequalities of the reward
    equation: on the threshold means outside the band).  The batch must reach such cells, and every log-reward must
    be the equation's value in exact rationals."""
    env = grid_env(2, 11)
    w = random_mlp(22, 64, 64, 3, seed=43, scale=1.0)
    w["b3"][2] -= 2.0
    _, traj, _ = run_case(gfnx, oracle32, oracle64, env, w, 3000, seed=21, iteration=0, log_z=0.0, name="grid2x11")
    ts = traj["terminal_state"].astype(int)
    on_edge = np.isin(ts, (1, 2, 8, 9)).all(axis=0)
    assert on_edge.sum() >= 20, int(on_edge.sum())
    want = np.array([math.log(grid_reward((int(x), int(y)), 11)) for x, y in ts.T])
    assert np.abs(traj["log_reward"] - want).max() < 1e-6
    assert {round(float(v), 4) for v in traj["log_reward"][on_edge]} <= {round(math.log(1e-3), 4), round(math.log(0.501), 4)}
