"""Pins of the oracle's pursuit ("tag") env: CPU only.

The env is a synthetic stand-in defined in oracle/msrl_ref.c (the paper names the task of its
GPU-only experiment, section 7.3, Fig. 10, and gives no formulas).  It is pinned to things other than itself:
the particle env's move (already pinned) when bodies never touch, conservation of momentum by the
contact forces, a two-body case worked out by hand, the speed limit, rewards and observations
rebuilt with array operations, and the routing of the per-role parameter sets in the rollout loop.
"""
import numpy as np
import pytest

from oracle import ref

N, NC, L = 4, 3, 2
D = 4 + 2 * L + 4 * (N - 1)


def make_env(**kw):
    args = dict(num_chasers=NC, accel_c=3.0, accel_r=4.0, vmax_c=1.0, vmax_r=1.3, radius_c=0.075, radius_r=0.05,
                contact_force=100.0, contact_margin=1e-3, dt=0.1, damping=0.25)
    args.update(kw)
    return ref.Env(ref.TAG, N, L, D, 1, 7, **args)


def random_state(rng, spread=1.0):
    s = np.zeros(4 * N + 2 * L)
    s[:4 * N] = rng.uniform(-1, 1, 4 * N) * np.tile([spread, spread, 0.5, 0.5], N)
    s[4 * N:] = rng.uniform(-1, 1, 2 * L)
    return s


def test_without_contact_the_move_is_the_particle_env_move():
    rng = np.random.default_rng(0)
    # bodies so small that they never touch, no speed limit, one force for both roles
    env = make_env(accel_c=1.0, accel_r=1.0, vmax_c=1e9, vmax_r=1e9, radius_c=1e-9, radius_r=1e-9)
    plain = ref.Env(ref.PARTICLE, N, L, 4 + 2 * L + 4 * (N - 1), 1, 7, dt=0.1, damping=0.25, force=1.0, radius=1e-9)
    for _ in range(20):
        s = random_state(rng, spread=3.0)
        a = rng.integers(0, 5, N)
        s_tag, _, _ = ref.tag_move(env, s, a)
        s_plain, _, _ = ref.particle_move(plain, s, a)
        np.testing.assert_allclose(s_tag, s_plain, rtol=0, atol=1e-13)


def test_contact_forces_conserve_momentum():
    rng = np.random.default_rng(1)
    env = make_env(damping=0.0, vmax_c=1e9, vmax_r=1e9, radius_c=0.3, radius_r=0.25)
    hits = 0
    for _ in range(50):
        s = random_state(rng, spread=0.4)           # crowded: bodies overlap
        v0 = s[:4 * N].reshape(N, 4)[:, 2:].sum(0)
        s1, _, _ = ref.tag_move(env, s, np.zeros(N, dtype=np.int32))
        v1 = s1[:4 * N].reshape(N, 4)[:, 2:].sum(0)
        np.testing.assert_allclose(v1, v0, rtol=0, atol=1e-10)
        hits += np.abs(s1[:4 * N].reshape(N, 4)[:, 2:] - s[:4 * N].reshape(N, 4)[:, 2:]).max() > 1e-3
    assert hits > 40        # and the bodies did push each other


def test_two_bodies_by_hand():
    # chaser at the origin, runner 0.1 to the right; radii 0.075 + 0.05 -> overlap 0.025
    env = ref.Env(ref.TAG, 2, 0, 4 + 4, 1, 7, num_chasers=1, damping=0.0, dt=0.1, vmax_c=1e9, vmax_r=1e9,
                  radius_c=0.075, radius_r=0.05, contact_force=100.0, contact_margin=1e-3)
    s = np.array([0.0, 0.0, 0.0, 0.0, 0.1, 0.0, 0.0, 0.0])
    s1, r, mg = ref.tag_move(env, s, [0, 0])
    m = 1e-3
    pen = m * np.logaddexp(0.0, 0.025 / m)            # smooth max(0, overlap): 0.025 to 1e-13
    assert pen == pytest.approx(0.025, abs=1e-12)
    dv = 100.0 * pen * 0.1
    np.testing.assert_allclose(s1, [-dv * 0.1, 0, -dv, 0, 0.1 + dv * 0.1, 0, dv, 0], atol=1e-13)
    # after the move they are 0.1 + 2 * 0.025 = 0.15 apart: no contact any more
    np.testing.assert_array_equal(r, [0.0, 0.0])
    assert mg == pytest.approx(0.15 - 0.125, abs=1e-12)
    # barely apart: the smooth overlap is m * log(1 + exp(-gap / m))
    s = np.array([0.0, 0.0, 0.0, 0.0, 0.1255, 0.0, 0.0, 0.0])
    s1, _, _ = ref.tag_move(env, s, [0, 0])
    assert s1[6] == pytest.approx(100.0 * m * np.log1p(np.exp(-0.5)) * 0.1, rel=1e-12)
    # an action is a force of accel(role): the runner accelerates more
    s = np.array([0.0, 0.0, 0.0, 0.0, 1.0, 0.0, 0.0, 0.0])
    s1, _, _ = ref.tag_move(env, s, [3, 3])
    assert s1[3] == pytest.approx(3.0 * 0.1) and s1[7] == pytest.approx(4.0 * 0.1)


def test_speed_limit_keeps_the_direction():
    rng = np.random.default_rng(2)
    env = make_env(damping=0.0)
    for _ in range(30):
        s = random_state(rng, spread=3.0)
        s[:4 * N].reshape(N, 4)[:, 2:] *= 6.0          # fast
        a = np.zeros(N, dtype=np.int32)
        s1, _, _ = ref.tag_move(env, s, a)
        v0, v1 = s[:4 * N].reshape(N, 4)[:, 2:], s1[:4 * N].reshape(N, 4)[:, 2:]
        lim = np.array([1.0] * NC + [1.3] * (N - NC))
        sp0, sp1 = np.linalg.norm(v0, axis=1), np.linalg.norm(v1, axis=1)
        np.testing.assert_allclose(sp1, np.minimum(sp0, lim), rtol=1e-12)
        np.testing.assert_allclose(v1 / sp1[:, None], v0 / sp0[:, None], atol=1e-12)
        np.testing.assert_allclose(s1[:4 * N].reshape(N, 4)[:, :2], s[:4 * N].reshape(N, 4)[:, :2] + 0.1 * v1, atol=1e-13)


def test_rewards_rebuilt_with_array_operations():
    rng = np.random.default_rng(3)
    env = make_env(radius_c=0.2, radius_r=0.15)
    seen = set()
    for _ in range(200):
        s = random_state(rng, spread=rng.choice([0.3, 1.4]))
        s1, r, mg = ref.tag_move(env, s, rng.integers(0, 5, N))
        p = s1[:4 * N].reshape(N, 4)[:, :2]
        d = np.linalg.norm(p[:NC, None, :] - p[None, NC:, :], axis=2)       # chasers x runners
        touch = d < 0.35
        want = np.empty(N)
        want[:NC] = 10.0 * touch.sum()
        want[NC:] = -10.0 * touch.sum(0) - 10.0 * np.maximum(np.abs(p[NC:]) - 1.0, 0.0).sum(1)
        np.testing.assert_allclose(r, want, atol=1e-12)
        assert mg == pytest.approx(np.abs(d - 0.35).min(), abs=1e-12)
        seen.add((int(touch.sum()) > 0, bool((np.abs(p[NC:]) > 1).any())))
    assert len(seen) == 4        # with and without contact, inside and outside the arena


def test_observation_rebuilt_with_array_operations():
    rng = np.random.default_rng(4)
    env = make_env()
    s = random_state(rng)
    o = ref.env_obs(env, s)
    a = s[:4 * N].reshape(N, 4)
    lm = s[4 * N:].reshape(L, 2)
    for i in range(N):
        others = [j for j in range(N) if j != i]
        want = np.concatenate([a[i, 2:], a[i, :2], (lm - a[i, :2]).ravel(), (a[others, :2] - a[i, :2]).ravel(),
                               a[others, 2:].ravel()])
        np.testing.assert_array_equal(o[i], want)
    assert o.shape == (N, D)


def test_step_done_and_reset_as_the_particle_env():
    env = make_env()
    s = ref.env_reset(env, 9, 3, 0)
    plain = ref.Env(ref.PARTICLE, N, L, D, 1, 7)
    np.testing.assert_array_equal(s, ref.env_reset(plain, 9, 3, 0))
    s1, r, d, _ = ref.env_step(env, 9, 3, 5, s, [0, 1, 2, 3])
    assert d == 0 and r.shape == (N,)
    s2, r, d, _ = ref.env_step(env, 9, 3, 6, s1, [0, 1, 2, 3])       # step 7 of 7: done, episode 1 starts
    assert d == 1
    np.testing.assert_array_equal(s2, ref.env_reset(env, 9, 3, 1))


def test_rollout_uses_one_parameter_set_per_role():
    rng = np.random.default_rng(5)
    env = make_env()
    pol = ref.Policy(D, 16, 5)
    params = rng.normal(0, 0.5, 2 * pol.param_count)
    state, g = ref.init(env, 77, 0, 3)
    s0 = state.copy()
    tr = ref.rollout(env, pol, 77, 0, state, g, params, 5)
    n = pol.param_count
    for e in range(3):
        for i in range(N):
            m = e * N + i
            role = params[:n] if i < NC else params[n:]
            lg, v = ref.policy_value(pol, role, tr["obs"][0, m])
            np.testing.assert_array_equal(tr["logits"][0, m], lg)
            assert tr["values"][0, m] == v
            a, lp, _ = ref.sample(pol, 77, e, i, 0, lg)
            assert tr["actions"][0, m] == a and tr["logp"][0, m] == lp
        s1, r, d, _ = ref.env_step(env, 77, e, 0, s0[e], tr["actions"][0, e * N:(e + 1) * N])
        np.testing.assert_array_equal(tr["rewards"][0, e * N:(e + 1) * N], r)
        np.testing.assert_array_equal(tr["obs"][1, e * N:(e + 1) * N], ref.env_obs(env, s1))
    assert (tr["dones"].sum(0) == 0).all() and (g == 5).all()


def test_rollout_with_a_centralised_critic_per_role():
    # value_in_dim = N * D with the pursuit env: every role has its own critic on the env's joint
    # observation, and a role's parameter set is counted with the critic at that width.  A runner's value
    # must come from the second set's critic (on the joint observation), a chaser's from the first set's.
    rng = np.random.default_rng(6)
    env = make_env()
    pol = ref.Policy(D, 16, 5, value_in_dim=N * D)
    n = pol.param_count
    assert n == ref.net_param_count(D, 16, 5) + ref.net_param_count(N * D, 16, 1)
    params = rng.normal(0, 0.5, 2 * n)
    state, g = ref.init(env, 78, 0, 2)
    tr = ref.rollout(env, pol, 78, 0, state, g, params, 2)
    n_pi = pol.policy_param_count
    for t in range(3):
        for e in range(2):
            joint = tr["obs"][t, e * N:(e + 1) * N]
            v_role = [ref.central_value(pol, params[:n], joint), ref.central_value(pol, params[n:], joint)]
            # the critic of a set is the plain network of its parameters on the concatenated rows
            for k, role in enumerate((params[:n], params[n:])):
                np.testing.assert_allclose(v_role[k], ref.mlp(N * D, 16, 1, role[n_pi:], joint.ravel())[0], rtol=1e-14)
            assert abs(v_role[0] - v_role[1]) > 1e-3
            for i in range(N):
                m = e * N + i
                k = 0 if i < NC else 1
                assert tr["values"][t, m] == v_role[k]
                if t < 2:
                    role = params[:n] if k == 0 else params[n:]
                    np.testing.assert_array_equal(tr["logits"][t, m], ref.mlp(D, 16, 5, role[:n_pi], tr["obs"][t, m]))
