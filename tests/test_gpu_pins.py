"""The oracle's hand-computed pins, repeated on the GPU through the snapshot
calls: the same fixed facts must hold for the HIP path itself."""
import numpy as np
import pytest

from paper_2210_00882_amd import synth
from helpers import GpuRollout, assert_close

pytestmark = pytest.mark.gpu


def forced_action_params(cfg, action):
    """All-zero networks whose policy bias makes `action` certain (p > 1 - 1e-25)."""
    p = np.zeros(cfg.param_count, dtype=np.float32)
    n_pol = synth.net_param_count(cfg.obs_dim, cfg.hidden, 5)
    b3 = np.full(5, -30.0, dtype=np.float32)
    b3[action] = 30.0
    p[n_pol - 5:n_pol] = b3
    return p


def test_single_step_by_hand():
    cfg = synth.particle("p1", 1, 1, 64, 2, 1000, idx=0)
    with GpuRollout(cfg, forced_action_params(cfg, 1), 1) as gpu:
        gpu.set_state(np.array([[0.5, -0.25, 0.0, 0.0, 0.0, 0.0]], dtype=np.float32))
        tr = gpu.run(1)
        es, g = gpu.get_state()
    assert tr["actions"][0, 0] == 1
    assert_close(tr["obs"][0, 0], [0, 0, 0.5, -0.25, -0.5, 0.25], 1e-6, "obs before")
    assert_close(tr["obs"][1, 0], [0.1, 0, 0.51, -0.25, -0.51, 0.25], 1e-6, "obs after")
    assert_close(tr["rewards"][0, 0], -np.sqrt(0.3226), 1e-6, "reward")
    assert_close(es[0], [0.51, -0.25, 0.1, 0.0, 0.0, 0.0], 1e-6, "state")
    assert g[0] == 1 and tr["dones"][0, 0] == 0
    assert abs(tr["logp"][0, 0]) < 1e-6


def test_damping_and_constant_force_closed_forms():
    T = 30
    cfg = synth.particle("p1", 2, 1, 64, T, 1000, idx=0)
    v0 = np.array([0.8, -0.4])
    p0 = np.array([0.1, 0.2])
    t = np.arange(T + 1)
    with GpuRollout(cfg, forced_action_params(cfg, 0), 1) as gpu:
        st = np.array([[p0[0], p0[1], v0[0], v0[1], 0.3, 0.3]] * 2, dtype=np.float32)
        gpu.set_state(st)
        tr = gpu.run(T)
    assert (tr["actions"] == 0).all()
    assert_close(tr["obs"][:, 0, 0:2], v0[None] * 0.75 ** t[:, None], 1e-5, "v_t = v0 0.75^t")
    assert_close(tr["obs"][:, 0, 2:4], p0[None] + 0.3 * v0[None] * (1 - 0.75 ** t[:, None]), 1e-5, "p_t")
    with GpuRollout(cfg, forced_action_params(cfg, 1), 1) as gpu:
        gpu.set_state(np.array([[0, 0, 0, 0, 1, 1]] * 2, dtype=np.float32))
        tr = gpu.run(T)
    v = 0.4 * (1 - 0.75 ** t)
    assert_close(tr["obs"][:, 1, 0], v, 1e-5, "v_t = 0.4 (1 - 0.75^t)")
    assert_close(tr["obs"][:, 1, 2], 0.1 * np.cumsum(v), 1e-5, "p_t")
    assert (tr["obs"][:, :, 1] == 0).all() and (tr["obs"][:, :, 3] == 0).all()


def test_collision_thresholds():
    cfg = synth.particle("p2", 3, 2, 64, 1, 1000, idx=0)
    st = np.zeros((3, 12), dtype=np.float32)
    for e, dist in enumerate([0.299, 0.301, 0.05]):
        st[e] = [0, 0, 0, 0, dist, 0, 0, 0, 0, 0, dist, 0]   # landmarks under the agents
    with GpuRollout(cfg, forced_action_params(cfg, 0), 1) as gpu:
        gpu.set_state(st)
        tr = gpu.run(1)
    assert_close(tr["rewards"][0, ::2], [-1.0, 0.0, -1.0], 1e-6, "collision penalties")
    assert (tr["rewards"][0, ::2] == tr["rewards"][0, 1::2]).all()


def test_lingauss_norm_law():
    # no noise and (numerically) zero action: |s_t| = 0.98^t |s_0|, r_t = -0.98^(2t) |s_0|^2
    T = 40
    cfg = synth.CONFIGS[4].with_(num_envs=33, T=T, noise_std=0.0)
    dyn = synth.make_dynamics(cfg)
    p = np.zeros(cfg.param_count, dtype=np.float32)
    n_pol = synth.net_param_count(17, 256, 12)
    p[n_pol - 6:n_pol] = -30.0   # log-std bias: actions of size e^-30
    with GpuRollout(cfg, p, 5, dyn) as gpu:
        tr = gpu.run(T)
    n0 = np.linalg.norm(tr["obs"][0].astype(np.float64), axis=-1)
    t = np.arange(T + 1)
    assert_close(np.linalg.norm(tr["obs"].astype(np.float64), axis=-1), n0[None] * 0.98 ** t[:, None], 1e-4, "norm law")
    assert_close(tr["rewards"], -(n0[None] ** 2) * 0.98 ** (2 * t[:T, None]), 1e-4, "reward law")
    assert (np.abs(tr["actions"]) < 1e-10).all()
