"""Host-side checks of the C ABI that need no GPU: the library loads, exports every declared symbol,
and validates its arguments before launching anything."""
import ctypes as C
import os
import re

import pytest

from paper_2511_16592_amd import gfnx
from paper_2511_16592_amd.workloads import bitseq_env, bitseq_na_env, grid_env, ising_env, workloads

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(gfnx.LIB_PATH):
        import __graft_entry__
        __graft_entry__.build()
    return gfnx.load_library()


def test_every_declared_symbol_is_exported(lib):
    header = open(os.path.join(ROOT, "include", "gfnx.h")).read()
    declared = set(re.findall(r"\b(gfnx_[a-z_]+)\s*\(", header))
    assert declared == set(gfnx.EXPORTS)
    for name in declared:
        assert getattr(lib, name) is not None


def test_env_dims_of_the_five_configurations(lib):
    expect = {"c1": (2, 16, 3, 15), "c2": (4, 80, 5, 77), "c3": (15, 3855, 256, 15),
              "c4": (100, 300, 200, 100), "c5": (10, 200, 11, 191)}
    for name, dims in expect.items():
        assert gfnx.env_dims(workloads()[name].env) == dims


def test_status_strings(lib):
    assert gfnx.status_string(0) == "GFNX_OK"
    for code in range(-6, 0):
        assert gfnx.status_string(code).startswith("GFNX_E_")


def _mlp(in_dim, h1, h2, a, ptr=0x1000):
    return gfnx.Mlp(in_dim, h1, h2, a, ptr, ptr, ptr, ptr, ptr, ptr)


def _traj(batch, steps, ptr=0x1000):
    return gfnx.Traj(batch, steps, ptr, ptr, ptr, ptr, ptr, ptr)


def test_bad_environment_descriptors(lib):
    bad = [grid_env(0, 8), grid_env(17, 8), grid_env(2, 1), grid_env(2, 200), ising_env(2), ising_env(11),
           bitseq_env(120, 7, 4, 1), bitseq_env(120, 8, 4, 1)]
    for i, env in enumerate(bad):
        d = gfnx.env_desc(env, 0x1000)
        if i == len(bad) - 1:
            d.kind = 7
        out = C.c_int32()
        assert lib.gfnx_env_dims(C.byref(d), C.byref(out), None, None, None) == -2
    assert lib.gfnx_env_dims(None, None, None, None, None) == -1


def test_workspace_size_and_argument_validation(lib):
    env = grid_env(2, 8)
    d = gfnx.env_desc(env)
    m = _mlp(16, 64, 64, 3)
    need = lib.gfnx_workspace_bytes(C.byref(d), C.byref(m), 16)
    assert need > 0 and need % 256 == 0
    assert lib.gfnx_workspace_bytes(C.byref(d), C.byref(m), 32) > need
    assert lib.gfnx_workspace_bytes(C.byref(d), C.byref(_mlp(16, 64, 64, 5)), 16) == 0   # neither env's n_actions nor +1
    assert lib.gfnx_workspace_bytes(C.byref(d), C.byref(_mlp(15, 64, 64, 3)), 16) == 0   # in_dim != obs_dim
    assert lib.gfnx_workspace_bytes(C.byref(d), C.byref(_mlp(16, 48, 64, 3)), 16) == 0   # h1 not a multiple of 64
    assert lib.gfnx_workspace_bytes(C.byref(d), C.byref(m), 0) == 0
    t = _traj(16, 15)
    ws = 0x10000
    call = lambda dd, mm, tt, w, n: lib.gfnx_rollout(dd, mm, 0, 0, tt, w, n, None)
    assert call(None, C.byref(m), C.byref(t), ws, need) == -1
    assert call(C.byref(d), None, C.byref(t), ws, need) == -1
    assert call(C.byref(d), C.byref(m), None, ws, need) == -1
    assert call(C.byref(d), C.byref(gfnx.Mlp(16, 64, 64, 3, 0, 0, 0, 0, 0, 0)), C.byref(t), ws, need) == -1
    assert call(C.byref(d), C.byref(_mlp(16, 64, 64, 5)), C.byref(t), ws, need) == -3
    assert call(C.byref(d), C.byref(_mlp(16, 64, 640, 3)), C.byref(t), ws, need) == -5
    assert call(C.byref(d), C.byref(m), C.byref(_traj(16, 14)), ws, need) == -3          # max_steps too small
    assert call(C.byref(d), C.byref(m), C.byref(_traj(0, 15)), ws, need) == -3
    assert call(C.byref(d), C.byref(m), C.byref(gfnx.Traj(16, 15, 0, 0, 0, 0, 0, 0)), ws, need) == -1
    assert call(C.byref(d), C.byref(m), C.byref(t), None, need) == -4
    assert call(C.byref(d), C.byref(m), C.byref(t), ws + 4, need) == -4                  # misaligned
    assert call(C.byref(d), C.byref(m), C.byref(t), ws, need - 1) == -4
    bs = gfnx.env_desc(bitseq_env(120, 8, 60, 3), None)                                   # modes pointer missing
    assert call(C.byref(bs), C.byref(_mlp(3855, 512, 512, 256)), C.byref(_traj(4, 15)), ws, 1 << 40) == -1
    g = gfnx.MlpGrad(0x1000, 0x1000, 0x1000, 0x1000, 0x1000, 0)
    assert lib.gfnx_tb_loss_grad(C.byref(d), C.byref(m), C.byref(t), 0.0, 0x1000, 0x1000, C.byref(g), ws, need, None) == -1
    assert lib.gfnx_tb_loss_grad(C.byref(d), C.byref(m), C.byref(t), 0.0, None, 0x1000, C.byref(g), ws, need, None) == -1
    assert lib.gfnx_replay(C.byref(d), C.byref(m), C.byref(t), ws, need - 1, None) == -4
    explore = lambda eps, n: lib.gfnx_rollout_explore(C.byref(d), C.byref(m), 0, 0, eps, C.byref(t), ws, n, None)
    assert explore(-0.01, need) == -3 and explore(1.01, need) == -3 and explore(float("nan"), need) == -3
    assert explore(0.5, need - 1) == -4


def test_workspace_sizes_of_the_benchmark_configurations(lib):
    gib = 1 << 30
    for name, limit in (("c2", 2 * gib), ("c3", 1 * gib), ("c4", 4 * gib), ("c5", 20 * gib)):
        wl = workloads()[name]
        _, od, na, _ = wl.env.dims()
        d = gfnx.env_desc(wl.env, 0x1000)
        need = lib.gfnx_workspace_bytes(C.byref(d), C.byref(_mlp(od, wl.h1, wl.h2, na)), wl.batch)
        assert 0 < need < limit, (name, need)


def test_optimiser_argument_validation(lib):
    """gfnx_adam_step / gfnx_train_step reject bad arguments on the host, before any launch."""
    p = 0x1000
    m = _mlp(16, 64, 64, 3)
    g = gfnx.MlpGrad(p, p, p, p, p, p)
    st = gfnx.AdamState(gfnx.MlpGrad(p, p, p, p, p, p), gfnx.MlpGrad(p, p, p, p, p, p), p)
    cfg = gfnx.AdamCfg(1e-3, 1e-1, 0.9, 0.999, 1e-8)
    call = lambda mm, lz, gg, dz, ss, cc, step: lib.gfnx_adam_step(mm, lz, gg, dz, ss, cc, step, None)
    assert call(None, p, C.byref(g), p, C.byref(st), C.byref(cfg), 1) == -1
    assert call(C.byref(m), p, None, p, C.byref(st), C.byref(cfg), 1) == -1
    assert call(C.byref(m), p, C.byref(g), p, None, C.byref(cfg), 1) == -1
    assert call(C.byref(m), p, C.byref(g), p, C.byref(st), None, 1) == -1
    assert call(C.byref(m), p, C.byref(gfnx.MlpGrad(p, p, p, 0, p, p)), p, C.byref(st), C.byref(cfg), 1) == -1
    bad_state = gfnx.AdamState(gfnx.MlpGrad(p, p, p, p, p, p), gfnx.MlpGrad(p, 0, p, p, p, p), p)
    assert call(C.byref(m), p, C.byref(g), p, C.byref(bad_state), C.byref(cfg), 1) == -1
    assert call(C.byref(m), p, C.byref(g), None, C.byref(st), C.byref(cfg), 1) == -1   # log Z given only in part
    assert call(C.byref(m), p, C.byref(g), p, C.byref(st), C.byref(cfg), 0) == -3      # updates count from 1
    assert call(C.byref(_mlp(16, 0, 64, 3)), p, C.byref(g), p, C.byref(st), C.byref(cfg), 1) == -3
    for bad in (gfnx.AdamCfg(1e-3, 1e-1, 1.0, 0.999, 1e-8), gfnx.AdamCfg(1e-3, 1e-1, 0.9, -0.1, 1e-8),
                gfnx.AdamCfg(-1e-3, 1e-1, 0.9, 0.999, 1e-8), gfnx.AdamCfg(1e-3, 1e-1, 0.9, 0.999, float("nan"))):
        assert call(C.byref(m), p, C.byref(g), p, C.byref(st), C.byref(bad), 1) == -3
    # the fused iteration: its own pointers, then the same checks, then those of the rollout
    d = gfnx.env_desc(grid_env(2, 8))
    t = _traj(16, 15)
    need = lib.gfnx_workspace_bytes(C.byref(d), C.byref(m), 16)
    train = lambda lz, step, ws_bytes: lib.gfnx_train_step(C.byref(d), C.byref(m), lz, 0, 0, C.byref(t), p, p,
                                                          C.byref(g), C.byref(st), C.byref(cfg), step, 0x10000,
                                                          ws_bytes, None)
    assert train(None, 1, need) == -1
    assert train(p, 0, need) == -3
    assert train(p, 1, need - 1) == -4


def test_backward_rollout_and_estimate_argument_validation(lib):
    p = 0x1000
    d = gfnx.env_desc(grid_env(2, 8))
    t = _traj(16, 15)
    call = lambda dd, tt: lib.gfnx_backward_rollout(dd, 0, 0, tt, None)
    assert call(None, C.byref(t)) == -1
    assert call(C.byref(d), None) == -1
    assert call(C.byref(d), C.byref(gfnx.Traj(16, 15, p, p, 0, p, p, p))) == -1       # no terminal states
    assert call(C.byref(d), C.byref(gfnx.Traj(16, 15, p, p, p, p, 0, p))) == -1       # no log_pb
    assert call(C.byref(d), C.byref(_traj(16, 14))) == -3
    assert call(C.byref(d), C.byref(_traj(0, 15))) == -3
    assert call(C.byref(gfnx.env_desc(grid_env(2, 1))), C.byref(t)) == -2
    assert call(C.byref(gfnx.env_desc(grid_env(16, 100))), C.byref(_traj(16, 1600))) == -5   # walks longer than 256
    est = lambda f, b, ns, n, o: lib.gfnx_log_prob_estimate(f, b, ns, n, o, None)
    assert est(None, p, 4, 4, p) == -1 and est(p, None, 4, 4, p) == -1 and est(p, p, 4, 4, None) == -1
    assert est(p, p, 0, 4, p) == -3 and est(p, p, 4, 0, p) == -3
    assert est(p, p, 1 << 20, 1 << 20, p) == -5


def test_flow_network_shapes_are_validated_on_the_host(lib):
    """A network with one output more than the environment has actions is a flow network: grids only, and only the
    matching objective accepts it."""
    p = 0x1000
    d = gfnx.env_desc(grid_env(2, 8))
    flow, plain = _mlp(16, 64, 64, 4), _mlp(16, 64, 64, 3)
    assert lib.gfnx_workspace_bytes(C.byref(d), C.byref(flow), 16) > lib.gfnx_workspace_bytes(C.byref(d), C.byref(plain), 16)
    assert lib.gfnx_workspace_bytes(C.byref(d), C.byref(_mlp(16, 64, 64, 5)), 16) == 0
    ising = gfnx.env_desc(ising_env(3))
    assert lib.gfnx_workspace_bytes(C.byref(ising), C.byref(_mlp(27, 64, 64, 19)), 16) == 0   # no flow output there
    t = _traj(16, 15)
    g = gfnx.MlpGrad(p, p, p, p, p, p)
    need = lib.gfnx_workspace_bytes(C.byref(d), C.byref(flow), 16)
    sub = lambda mm, lam, n: lib.gfnx_subtb_loss_grad(C.byref(d), C.byref(mm), C.byref(t), lam, p, C.byref(g), 0x10000, n, None)
    assert sub(plain, 0.9, need) == -3
    assert sub(flow, -0.1, need) == -3 and sub(flow, 1.1, need) == -3 and sub(flow, float("nan"), need) == -3
    assert sub(flow, 0.9, need - 1) == -4
    assert lib.gfnx_tb_loss_grad(C.byref(d), C.byref(flow), C.byref(t), 0.0, p, p, C.byref(g), 0x10000, need, None) == -3


def test_train_step_options_are_validated_on_the_host(lib):
    p = 0x1000
    d = gfnx.env_desc(grid_env(2, 8))
    flow, plain = _mlp(16, 64, 64, 4), _mlp(16, 64, 64, 3)
    t = _traj(16, 15)
    g = gfnx.MlpGrad(p, p, p, p, p, p)
    st = gfnx.AdamState(gfnx.MlpGrad(p, p, p, p, p, p), gfnx.MlpGrad(p, p, p, p, p, p), p)
    cfg = gfnx.AdamCfg(1e-3, 1e-1, 0.9, 0.999, 1e-8)

    def call(mm, opts, lz=p, need_of=None):
        need = lib.gfnx_workspace_bytes(C.byref(d), C.byref(need_of or mm), 16)
        return lib.gfnx_train_step_opts(C.byref(d), C.byref(mm), lz, 0, 0, C.byref(t), p, lz, C.byref(g), C.byref(st),
                                        C.byref(cfg), None if opts is None else C.byref(opts), 1, 0x10000, need - 1,
                                        None)

    assert call(plain, None) == -1
    assert call(plain, gfnx.TrainOpts(-0.1, -1.0)) == -3 and call(plain, gfnx.TrainOpts(1.1, -1.0)) == -3
    assert call(plain, gfnx.TrainOpts(0.0, 1.5)) == -3 and call(plain, gfnx.TrainOpts(0.0, float("nan"))) == -3
    assert call(plain, gfnx.TrainOpts(0.0, 0.9)) == -3           # SubTB needs the flow output
    assert call(flow, gfnx.TrainOpts(0.0, -1.0)) == -3           # TB must not have it
    assert call(plain, gfnx.TrainOpts(0.1, -1.0), lz=None) == -1  # TB needs log Z
    assert call(plain, gfnx.TrainOpts(0.1, -1.0)) == -4          # everything else fine: only the workspace is short
    assert call(flow, gfnx.TrainOpts(0.1, 0.9), lz=None) == -4   # SubTB: log Z pointers may be NULL


def test_workspace_regions(lib):
    """gfnx_workspace_region: the recorded ReLU' bits lie inside the workspace, rows of 32 bytes per 256 hidden
    units; networks of at most 16 outputs with h2 = 256 record no h2 bits (GFNX_E_UNSUPPORTED) but do have h2 rows."""
    off, rb = C.c_size_t(), C.c_size_t()
    cases = [(grid_env(4, 20), _mlp(80, 256, 256, 5), 4096, 77, False),
             (ising_env(10), _mlp(300, 256, 256, 200), 512, 100, True),
             (bitseq_env(120, 8, 4, 1), _mlp(3855, 512, 512, 256), 64, 15, True),
             (grid_env(2, 8), _mlp(16, 64, 128, 3), 16, 15, True)]
    for env, m, batch, steps, has_h2_bits in cases:
        d = gfnx.env_desc(env, 0x1000)
        need = lib.gfnx_workspace_bytes(C.byref(d), C.byref(m), batch)
        rows = steps * batch
        assert lib.gfnx_workspace_region(C.byref(d), C.byref(m), batch, 0, C.byref(off), C.byref(rb)) == 0
        assert rb.value == 32 * ((m.h1 + 255) // 256) and off.value % 256 == 0
        assert off.value + rows * rb.value <= need
        rc = lib.gfnx_workspace_region(C.byref(d), C.byref(m), batch, 1, C.byref(off), C.byref(rb))
        assert rc == (0 if has_h2_bits else -5)
        if has_h2_bits:
            assert rb.value == 32 * ((m.h2 + 255) // 256) and off.value + rows * rb.value <= need
        assert lib.gfnx_workspace_region(C.byref(d), C.byref(m), batch, 2, C.byref(off), C.byref(rb)) == 0
        assert rb.value == 4 * m.h2 and off.value + rows * rb.value <= need
        assert lib.gfnx_workspace_region(C.byref(d), C.byref(m), batch, 3, C.byref(off), C.byref(rb)) == -3
        assert lib.gfnx_workspace_region(C.byref(d), C.byref(m), batch, 0, None, C.byref(rb)) == -1
        assert lib.gfnx_workspace_region(C.byref(d), C.byref(m), 0, 0, C.byref(off), C.byref(rb)) == -3
    assert lib.gfnx_workspace_region(None, C.byref(_mlp(16, 64, 64, 3)), 4, 0, C.byref(off), C.byref(rb)) == -1


def test_static_scratch_entry_point_rejects_oversize_on_the_host(lib):
    """gfnx_train_step_static: a configuration whose workspace exceeds the fixed 64 MiB array is refused with
    GFNX_E_WORKSPACE before the runtime is touched (so this runs without a GPU); NULL and shape errors come first."""
    env = ising_env(10)
    d = gfnx.env_desc(env)
    m = _mlp(300, 256, 256, 200)
    assert lib.gfnx_workspace_bytes(C.byref(d), C.byref(m), 4096) > (64 << 20)
    t = _traj(4096, 100)
    g = gfnx.MlpGrad(*[0x1000] * 6)
    st = gfnx.AdamState(g, g, 0x1000)
    cfg = gfnx.AdamCfg(1e-3, 1e-1, 0.9, 0.999, 1e-8)
    call = lambda dd, mm, tt: lib.gfnx_train_step_static(dd, mm, 0x1000, 0, 0, tt, 0x1000, 0x1000, C.byref(g),
                                                          C.byref(st), C.byref(cfg), 1, None)
    assert call(C.byref(d), C.byref(m), C.byref(t)) == -4
    assert call(None, C.byref(m), C.byref(t)) == -1
    assert call(C.byref(d), C.byref(m), None) == -1
    assert call(C.byref(d), C.byref(_mlp(299, 256, 256, 200)), C.byref(t)) == -3
    small = _traj(16, 100)
    assert lib.gfnx_workspace_bytes(C.byref(d), C.byref(m), 16) <= (64 << 20)


def test_non_autoregressive_bit_sequence_dims_and_limits(lib):
    """gfnx_env_dims of the (position, word) environment; up to 256 actions use the byte plane; more (the paper's
    n = 120, k = 8 instance: 3840 actions) must be a multiple of 256 and need the 16-bit plane of gfnx_traj."""
    assert gfnx.env_dims(bitseq_na_env(24, 4, 3, 1)) == (6, 6 * 17, 6 * 16, 6)
    assert gfnx.env_dims(bitseq_na_env(64, 4, 3, 1)) == (16, 16 * 17, 256, 16)
    assert gfnx.env_dims(bitseq_na_env(120, 8, 3, 1)) == (15, 3855, 3840, 15)
    d = gfnx.env_desc(bitseq_na_env(64, 4, 3, 1), 0x1000)
    assert lib.gfnx_workspace_bytes(C.byref(d), C.byref(_mlp(16 * 17, 256, 256, 256)), 64) > 0
    big = gfnx.env_desc(bitseq_na_env(120, 8, 3, 1), 0x1000)
    need = lib.gfnx_workspace_bytes(C.byref(big), C.byref(_mlp(3855, 256, 256, 3840)), 64)
    assert need > 64 * 15 * 3840 * 4          # the logit rows of every transition are part of it
    t = _traj(64, 15)                          # byte plane only: the 16-bit plane is missing
    assert lib.gfnx_rollout(C.byref(big), C.byref(_mlp(3855, 256, 256, 3840)), 0, 0, C.byref(t), 0x10000, need,
                            None) == -1
    t16 = gfnx.Traj(64, 15, None, 0x1000, 0x1000, 0x1000, 0x1000, 0x1000, 0x1000)
    assert lib.gfnx_rollout(C.byref(big), C.byref(_mlp(3855, 256, 256, 3840)), 0, 0, C.byref(t16), 0x10000, need - 1,
                            None) == -4        # everything else accepted: only the workspace is too small
    odd = gfnx.env_desc(bitseq_na_env(60, 5, 3, 1, uniform_bits=True), 0x1000)   # 12 x 32 = 384 actions
    assert lib.gfnx_workspace_bytes(C.byref(odd), C.byref(_mlp(12 * 33, 64, 64, 384)), 64) == 0
    bad = gfnx.env_desc(bitseq_na_env(64, 4, 3, 1), 0x1000)
    bad.k_bits = 5
    out = C.c_int32()
    assert lib.gfnx_env_dims(C.byref(bad), C.byref(out), None, None, None) == -2
