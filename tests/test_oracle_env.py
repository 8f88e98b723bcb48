"""Pins of the oracle's environments: hand-computed steps, closed forms,
thresholds and invariants that follow from the stated dynamics alone."""
import numpy as np
import pytest

from oracle import ref
from paper_2210_00882_amd import synth


def particle_env(N, L=None, ep=25):
    L = N if L is None else L
    return ref.Env(ref.PARTICLE, N, L, 4 + 2 * L + 4 * (N - 1), 1, ep)


def test_particle_single_step_by_hand():
    # one agent at (0.5,-0.25) at rest, landmark at the origin, action 1 (+x):
    # v' = 0*0.75 + 1*0.1 = (0.1, 0); p' = p + 0.1*v' = (0.51,-0.25);
    # reward = -|p'| = -sqrt(0.51^2 + 0.25^2) = -sqrt(0.3226)
    env = particle_env(1)
    s = np.array([0.5, -0.25, 0.0, 0.0, 0.0, 0.0])
    s1, r, _ = ref.particle_move(env, s, [1])
    np.testing.assert_allclose(s1, [0.51, -0.25, 0.1, 0.0, 0.0, 0.0], atol=1e-15)
    assert r == pytest.approx(-np.sqrt(0.3226), abs=1e-14)
    assert r == pytest.approx(-0.567979, abs=1e-6)
    np.testing.assert_allclose(ref.env_obs(env, s1)[0], [0.1, 0, 0.51, -0.25, -0.51, 0.25], atol=1e-15)
    # then a no-op: v'' = 0.075, p'' = 0.51 + 0.0075
    s2, r2, _ = ref.particle_move(env, s1, [0])
    np.testing.assert_allclose(s2, [0.5175, -0.25, 0.075, 0.0, 0.0, 0.0], atol=1e-15)
    assert r2 == pytest.approx(-np.hypot(0.5175, 0.25), abs=1e-14)


@pytest.mark.parametrize("action,dv", [(0, (0, 0)), (1, (0.1, 0)), (2, (-0.1, 0)), (3, (0, 0.1)), (4, (0, -0.1))])
def test_action_force_table(action, dv):
    env = particle_env(1)
    s1, _, _ = ref.particle_move(env, np.zeros(6), [action])
    np.testing.assert_allclose(s1[2:4], dv, atol=1e-16)
    np.testing.assert_allclose(s1[0:2], 0.1 * np.array(dv), atol=1e-16)


def test_damping_closed_form():
    # zero action: v_t = v0 * 0.75^t, p_t = p0 + 0.1 * sum_{s=1..t} v_s = p0 + 0.3 v0 (1 - 0.75^t)
    env = particle_env(1)
    v0 = np.array([0.8, -0.4])
    p0 = np.array([0.1, 0.2])
    s = np.concatenate([p0, v0, [0.3, 0.3]])
    for t in range(1, 40):
        s, _, _ = ref.particle_move(env, s, [0])
        np.testing.assert_allclose(s[2:4], v0 * 0.75 ** t, rtol=1e-12)
        np.testing.assert_allclose(s[0:2], p0 + 0.3 * v0 * (1 - 0.75 ** t), rtol=1e-12)


def test_constant_force_closed_form():
    # action 1 forever from rest: v_t = 0.4 (1 - 0.75^t) (terminal 0.4 = force*dt/damping)
    env = particle_env(1)
    s = np.array([0.0, 0.0, 0.0, 0.0, 1.0, 1.0])
    psum = 0.0
    for t in range(1, 60):
        s, _, _ = ref.particle_move(env, s, [1])
        v = 0.4 * (1 - 0.75 ** t)
        psum += 0.1 * v
        assert s[2] == pytest.approx(v, rel=1e-12)
        assert s[0] == pytest.approx(psum, rel=1e-12)
        assert s[1] == 0.0 and s[3] == 0.0
    assert s[2] == pytest.approx(0.4, abs=1e-6)


def test_collision_threshold_and_count():
    env = particle_env(2)
    far = [5.0, 5.0, 6.0, 6.0]  # landmarks
    def reward(pa, pb, lms=far):
        s = np.array([pa[0], pa[1], 0, 0, pb[0], pb[1], 0, 0] + list(lms), dtype=float)
        return ref.particle_move(env, s, [0, 0])
    # distance 0.299 < 0.30 -> one colliding pair; 0.301 -> none
    _, r_in, m_in = reward((0, 0), (0.299, 0), [0, 0, 0.299, 0])
    _, r_out, m_out = reward((0, 0), (0.301, 0), [0, 0, 0.301, 0])
    assert r_in == pytest.approx(-1.0, abs=1e-12)
    assert r_out == pytest.approx(0.0, abs=1e-12)
    assert m_in == pytest.approx(0.001, abs=1e-9) and m_out == pytest.approx(0.001, abs=1e-9)
    # exactly 2*radius is not a collision (strict inequality); 0.3 = 2*0.15 exactly in double
    _, r_eq, _ = reward((0, 0), (0.3, 0), [0, 0, 0.3, 0])
    assert r_eq == pytest.approx(0.0, abs=1e-12)
    # three mutually overlapping agents: 3 pairs
    env3 = particle_env(3)
    s = np.array([0, 0, 0, 0, 0.1, 0, 0, 0, 0, 0.1, 0, 0, 0, 0, 0.1, 0, 0, 0.1], dtype=float)
    _, r3, _ = ref.particle_move(env3, s, [0, 0, 0])
    assert r3 == pytest.approx(-3.0, abs=1e-12)


def test_reward_is_sum_of_nearest_agent_distances():
    # 2 agents, 2 landmarks; landmark 0 nearest to agent 1, landmark 1 nearest to agent 1 too
    env = particle_env(2)
    s = np.array([-1, -1, 0, 0, 1, 1, 0, 0, 1, 0, 0.5, 1], dtype=float)
    _, r, _ = ref.particle_move(env, s, [0, 0])
    assert r == pytest.approx(-(1.0 + 0.5), abs=1e-14)
    # brute force on random states, asymmetric N != L
    rng = np.random.default_rng(3)
    env = particle_env(3, L=2)
    for _ in range(50):
        s = rng.uniform(-1, 1, env.S)
        s[2:12:4] = 0
        s[3:12:4] = 0
        P = s[:12].reshape(3, 4)[:, :2]
        Lm = s[12:].reshape(2, 2)
        want = -sum(min(np.linalg.norm(P[i] - Lm[k]) for i in range(3)) for k in range(2))
        want -= sum(np.linalg.norm(P[i] - P[j]) < 0.3 for i in range(3) for j in range(i + 1, 3))
        _, r, _ = ref.particle_move(env, s, [0, 0, 0])
        assert r == pytest.approx(want, abs=1e-13) and r <= 0


def test_obs_layout_three_agents():
    env = particle_env(3)
    assert env.D == 18
    s = np.array([1, 2, 0.1, 0.2, 3, 4, 0.3, 0.4, 5, 6, 0.5, 0.6, 10, 20, 30, 40, 50, 60], dtype=float)
    o = ref.env_obs(env, s)
    # agent 1: v, p, landmarks - p, then agents 0 and 2 relative, then 4 zeros
    np.testing.assert_allclose(o[1], [0.3, 0.4, 3, 4, 7, 16, 27, 36, 47, 56, -2, -2, 2, 2, 0, 0, 0, 0])
    np.testing.assert_allclose(o[0][10:14], [2, 2, 4, 4])
    np.testing.assert_allclose(o[2][10:14], [-4, -4, -2, -2])
    assert (o[:, 14:] == 0).all()


def test_reset_draws():
    env = particle_env(3)
    seed = 77
    s = ref.env_reset(env, seed, 9, 4)
    for e in range(6):
        w = ref.draw(seed, 9, e, 4, 1, 0)
        xy = [2 * ref.uniform(w[0]) - 1, 2 * ref.uniform(w[1]) - 1]
        if e < 3:
            np.testing.assert_array_equal(s[4 * e:4 * e + 2], xy)
            np.testing.assert_array_equal(s[4 * e + 2:4 * e + 4], [0, 0])
        else:
            np.testing.assert_array_equal(s[12 + 2 * (e - 3):14 + 2 * (e - 3)], xy)
    # uniform on [-1,1)^2: mean 0, variance 1/3
    pos = np.array([ref.env_reset(env, seed, i, 0) for i in range(4000)])
    xs = np.concatenate([pos[:, 0:12:4].ravel(), pos[:, 1:12:4].ravel(), pos[:, 12:].ravel()])
    assert xs.min() >= -1 and xs.max() < 1
    assert abs(xs.mean()) < 4 * np.sqrt(1 / 3 / xs.size)
    assert abs(xs.var() - 1 / 3) < 0.01


def test_done_and_reset_schedule():
    env = particle_env(2, ep=5)
    seed = 5
    s = ref.env_reset(env, seed, 3, 0)
    for g in range(12):
        s_new, r, d, _ = ref.env_step(env, seed, 3, g, s, [1, 3])
        assert d == int((g + 1) % 5 == 0)
        if d:
            np.testing.assert_array_equal(s_new, ref.env_reset(env, seed, 3, (g + 1) // 5))
        else:
            moved, r2, _ = ref.particle_move(env, s, [1, 3])
            np.testing.assert_array_equal(s_new, moved)
            assert r == r2
        s = s_new


def lingauss_env(noise=0.01):
    cfg = synth.CONFIGS[4]
    A, B = synth.make_dynamics(cfg)
    return ref.Env(ref.LINGAUSS, 1, 0, 17, 6, 1000, A=A, B=B, noise_std=noise), A.astype(float), B.astype(float)


def test_dynamics_matrix_is_scaled_orthogonal():
    _, A, B = lingauss_env()
    np.testing.assert_allclose(A.T @ A, 0.98 ** 2 * np.eye(17), atol=1e-5)
    assert abs(B.var() - 0.1) < 0.05


def test_lingauss_norm_law():
    # no noise, zero action: |s_t| = 0.98^t |s_0| and r_t = -0.98^(2t) |s_0|^2
    env, A, _ = lingauss_env(noise=0.0)
    rng = np.random.default_rng(0)
    s0 = rng.standard_normal(17)
    s = s0.copy()
    for t in range(50):
        s, r = ref.lingauss_move(env, s, np.zeros(6), np.zeros(17))
        assert r == pytest.approx(-(0.98 ** (2 * t)) * (s0 @ s0), rel=1e-5)
        assert np.linalg.norm(s) == pytest.approx(0.98 ** (t + 1) * np.linalg.norm(s0), rel=1e-5)


def test_lingauss_move_against_numpy():
    env, A, B = lingauss_env()
    rng = np.random.default_rng(1)
    for _ in range(20):
        s, a, eps = rng.standard_normal(17), rng.standard_normal(6), rng.standard_normal(17)
        s1, r = ref.lingauss_move(env, s, a, eps)
        np.testing.assert_allclose(s1, A @ s + B @ a + 0.01 * eps, rtol=1e-13, atol=1e-14)
        assert r == pytest.approx(-(s @ s + 0.01 * a @ a), rel=1e-14)


def test_lingauss_step_noise_stream_and_reset():
    env, A, B = lingauss_env()
    seed = 11
    s = ref.env_reset(env, seed, 2, 0)
    np.testing.assert_array_equal(s, ref.normals(seed, 2, 0, 0, 1, 17))
    a = np.arange(6) * 0.1
    s1, r, d, _ = ref.env_step(env, seed, 2, 41, s, a)
    want, r2 = ref.lingauss_move(env, s, a, ref.normals(seed, 2, 0, 41, 2, 17))
    np.testing.assert_array_equal(s1, want)
    assert d == 0 and r == r2
    s2, _, d, _ = ref.env_step(env, seed, 2, 999, s, a)
    assert d == 1
    np.testing.assert_array_equal(s2, ref.normals(seed, 2, 0, 1, 1, 17))
