"""GPU parity of the pursuit ("tag") env rollout against the CPU oracle, through the C ABI.

Stage-wise like the other parity tests: every stage of a step is checked on what the GPU itself
produced for the stage before (observation rows -> networks of the agent's role -> sampler -> move,
contact forces, per-role rewards, done / reset -> next observation rows).  Tolerances as in
helpers.py; a reward may differ by one contact (10) where a chaser-runner distance lies within 1e-5
of the contact distance.
"""
import numpy as np
import pytest

from oracle import ref
from paper_2210_00882_amd import synth
from helpers import EDGE, GpuRollout, TOL_BF16, TOL_F32, assert_close, check_gae, close, _logp_of

pytestmark = pytest.mark.gpu

SEED = 0x7A6C0FFEE


def tag_env(cfg):
    return ref.Env(ref.TAG, cfg.num_agents, cfg.num_landmarks, cfg.obs_dim, 1, cfg.episode_len,
                   dt=np.float32(cfg.dt), damping=np.float32(cfg.damping), num_chasers=cfg.num_chasers,
                   accel_c=np.float32(cfg.accel_c), accel_r=np.float32(cfg.accel_r), vmax_c=np.float32(cfg.vmax_c),
                   vmax_r=np.float32(cfg.vmax_r), radius_c=np.float32(cfg.radius_c), radius_r=np.float32(cfg.radius_r),
                   contact_force=np.float32(cfg.contact_force), contact_margin=np.float32(cfg.contact_margin))


def state_from_obs(cfg, rows):
    N, L = cfg.num_agents, cfg.num_landmarks
    s = np.zeros(4 * N + 2 * L)
    for i in range(N):
        s[4 * i:4 * i + 2] = rows[i][2:4]
        s[4 * i + 2:4 * i + 4] = rows[i][0:2]
    s[4 * N:] = rows[0][4:4 + 2 * L].astype(np.float64) + np.tile(rows[0][2:4].astype(np.float64), L)
    return s


def check(cfg, tr, env, pol, params, env_ids, g0, T):
    N = cfg.num_agents
    n_role = pol.param_count
    TOL_NET = TOL_BF16 if cfg.dtype == synth.BF16 else TOL_F32
    stats = {"rows": 0, "action_edge": 0, "contact_edge": 0, "contacts": 0}
    for k, e in enumerate(env_ids):
        rows = slice(e * N, (e + 1) * N)
        for t in range(T + 1):
            g = int(g0[k]) + t
            o_gpu = tr["obs"][t, rows]
            s = state_from_obs(cfg, o_gpu)
            assert_close(o_gpu, ref.env_obs(env, s), TOL_F32, f"obs rows env {e} t {t}")
            for i in range(N):
                m = e * N + i
                prm = params[:n_role] if i < cfg.num_chasers else params[n_role:]
                lg, v = ref.policy_value(pol, prm, o_gpu[i])
                assert_close(tr["values"][t, m], v, TOL_NET, f"value env {e} agent {i} t {t}")
                if t < T:
                    assert_close(tr["logits"][t, m], lg, TOL_NET, f"logits env {e} agent {i} t {t}")
            if t == T:
                break
            acts = []
            for i in range(N):
                m = e * N + i
                a_o, lp_o, mg = ref.sample(pol, SEED, e, i, g, tr["logits"][t, m])
                a_g = int(tr["actions"][t, m])
                if a_g != a_o:
                    assert mg < EDGE, f"action env {e} agent {i} t {t}: gpu {a_g} oracle {a_o} margin {mg}"
                    stats["action_edge"] += 1
                    _, lp_o = _logp_of(tr["logits"][t, m], a_g)
                assert_close(tr["logp"][t, m], lp_o, TOL_F32, f"logp env {e} agent {i} t {t}")
                acts.append(a_g)
                stats["rows"] += 1
            s1, r, d, mg = ref.env_step(env, SEED, e, g, s, acts)
            assert (tr["dones"][t, rows] == d).all(), f"done env {e} t {t}"
            r_gpu = tr["rewards"][t, rows]
            if not np.all(close(r_gpu, r, TOL_F32)):
                assert mg < EDGE, f"rewards env {e} t {t}: gpu {r_gpu} oracle {r} (contact margin {mg})"
                stats["contact_edge"] += 1
            stats["contacts"] += int(r[0] > 0)
            assert_close(tr["obs"][t + 1, rows], ref.env_obs(env, s1), TOL_F32, f"next obs env {e} t {t}")
    return stats


@pytest.mark.parametrize("tiles,E", [(1, 70), (4, 70), (4, 300)])
@pytest.mark.parametrize("nc,nr,L", [(3, 1, 2), (2, 2, 1)])
def test_tag_rollout_every_env_and_step(nc, nr, L, tiles, E):
    # both workgroup shapes (one or four 32-env tiles, msrl_env_cfg.tag_tiles): E = 70 is
    # one ragged workgroup of four tiles with an empty tile, E = 300 three workgroups with a ragged last tile
    tag_parity(nc, nr, L, tiles, E, 20 if E < 100 else 8, 100)


@pytest.mark.parametrize("nc,nr,L,tiles", [(1, 1, 0, 0), (1, 1, 2, 4), (1, 3, 4, 4), (3, 1, 0, 1), (4, 4, 4, 0),
                                           (7, 1, 3, 0), (1, 7, 0, 0), (5, 2, 1, 0), (2, 6, 4, 0), (3, 3, 3, 0),
                                           (4, 1, 4, 0), (6, 1, 2, 0)])
def test_tag_shapes_off_the_benchmark(nc, nr, L, tiles):
    # every (chasers, runners) up to 8 agents with up to 4 landmarks is compiled: a sample of the corners
    tag_parity(nc, nr, L, tiles, 45, 8, 10)


@pytest.mark.parametrize("nc,nr,L", [(3, 1, 2), (1, 1, 0), (2, 2, 1), (4, 3, 4), (1, 6, 2), (5, 1, 0)])
def test_tag_with_fp32_networks(nc, nr, L):
    # fp32 networks (twice the LDS: compiled where the four of them still fit, i.e. all but the largest shapes),
    # to the fp32 tolerance
    tag_parity(nc, nr, L, 0, 45, 8, 10, dtype=synth.F32)


def test_tag_fp32_shapes_that_do_not_fit():
    from paper_2210_00882_amd import binding as B
    big = synth.tag("tagbig", 8, 4, 4, 4, 64, 4, 4, dtype=synth.F32)     # four fp32 networks of 41 inputs: 169 KB
    with pytest.raises(B.MsrlError) as e:
        B.msrl_rollout_init(B.make_env_cfg(big, None, None)[0], B.make_policy_cfg(big), 1)
    assert e.value.code == B.MSRL_EUNSUPPORTED
    four = synth.tag("tag4", 8, 3, 1, 2, 64, 4, 4, dtype=synth.F32)      # four tiles per workgroup: bf16 only
    with pytest.raises(B.MsrlError) as e:
        B.msrl_rollout_init(B.make_env_cfg(four, None, None, tag_tiles=4)[0], B.make_policy_cfg(four), 1)
    assert e.value.code == B.MSRL_EUNSUPPORTED


def tag_parity(nc, nr, L, tiles, E, T, min_contacts, dtype=synth.BF16):
    # big bodies, so that contact forces and contact rewards occur in most steps
    cfg = synth.tag("tag", E, nc, nr, L, 64, T, 7, dtype=dtype, idx=50 + nc).with_(radius_c=0.3, radius_r=0.25)
    env = tag_env(cfg)
    pol = ref.Policy(cfg.obs_dim, cfg.hidden, 5, bf16=dtype == synth.BF16)
    params = synth.make_params(cfg, bias_std=0.1).astype(np.float64)
    assert params.size == 2 * pol.param_count
    with GpuRollout(cfg, params.astype(np.float32), SEED, tag_tiles=tiles) as gpu:
        es0, g0 = gpu.get_state()
        np.testing.assert_array_equal(es0[3], ref.env_reset(env, SEED, 3, 0).astype(np.float32))
        shift = (np.arange(cfg.num_envs) * 3 + 1).astype(np.int64)     # a different episode phase per env
        gpu.set_state(None, shift)
        ids = list(range(cfg.num_envs))
        total = {}
        g = shift.copy()
        for call in range(2):
            tr = gpu.run(cfg.T)
            st = check(cfg, tr, env, pol, params, ids, g, cfg.T)
            check_gae(cfg, tr)
            g = g + cfg.T
            es, gg = gpu.get_state()
            np.testing.assert_array_equal(gg, g)
            for e in ids[:6]:
                assert_close(tr["obs"][cfg.T, e * cfg.num_agents:(e + 1) * cfg.num_agents],
                             ref.env_obs(env, es[e].astype(np.float64)), 1e-6, "state writeback")
            for k, v in st.items():
                total[k] = total.get(k, 0) + v
    assert total["rows"] == 2 * cfg.T * cfg.M
    assert total["contacts"] > min_contacts  # the contact path was exercised
    # chasers share their reward, runners do not see it
    r = tr["rewards"].reshape(cfg.T, cfg.num_envs, cfg.num_agents)
    assert (r[:, :, :nc] == r[:, :, :1]).all() and (r[:, :, :nc] >= 0).all() and (r[:, :, nc:] <= 0).all()


def test_tag_at_the_benchmarks_size_sampled():
    # 25,000 envs (100,000 agents): the launch bench.py times, which takes four tiles per workgroup by itself
    cfg = synth.tag("tag_100k_agents", 25000, 3, 1, 2, 64, 12, 5, idx=58)
    env = tag_env(cfg)
    pol = ref.Policy(cfg.obs_dim, cfg.hidden, 5, bf16=True)
    params = synth.make_params(cfg, bias_std=0.1).astype(np.float64)
    rng = np.random.default_rng(2)
    ids = [0, 31, 32, 127, 128, cfg.num_envs - 1] + sorted(rng.choice(cfg.num_envs, 6, replace=False).tolist())
    with GpuRollout(cfg, params.astype(np.float32), SEED) as gpu:
        tr = gpu.run(cfg.T)
        _, g = gpu.get_state()
    assert (g == cfg.T).all()
    st = check(cfg, tr, env, pol, params, ids, np.zeros(len(ids), dtype=np.int64), cfg.T)
    assert st["rows"] == len(ids) * cfg.num_agents * cfg.T
    check_gae(cfg, tr)
    r = tr["rewards"].reshape(cfg.T, cfg.num_envs, cfg.num_agents)
    assert (r[:, :, :3] == r[:, :, :1]).all() and (r[:, :, :3] >= 0).all() and (r[:, :, 3:] <= 0).all()
    assert np.isfinite(tr["values"]).all() and ((tr["actions"] >= 0) & (tr["actions"] < 5)).all()


def test_tag_default_bodies_and_errors():
    from paper_2210_00882_amd import binding as B
    cfg = synth.tag("tag", 33, 3, 1, 2, 64, 9, 4, idx=60)
    env = tag_env(cfg)
    pol = ref.Policy(cfg.obs_dim, cfg.hidden, 5, bf16=True)
    params = synth.make_params(cfg, bias_std=0.1).astype(np.float64)
    with GpuRollout(cfg, params.astype(np.float32), SEED) as gpu:
        tr = gpu.run(cfg.T)
        check(cfg, tr, env, pol, params, list(range(cfg.num_envs)), np.zeros(cfg.num_envs, dtype=np.int64), cfg.T)
        with pytest.raises(B.MsrlError) as e:   # the measurement variants have no pursuit kernel
            B.msrl_measure_phase(gpu.state, gpu.params, 2, gpu.dev, B.MSRL_PHASE_ENV)
        assert e.value.code == B.MSRL_EUNSUPPORTED
    assert B.msrl_param_count(B.make_policy_cfg(cfg)) == cfg.param_count == 2 * pol.param_count
    env_cfg, keep = B.make_env_cfg(cfg, None, None)
    one_role = B.make_policy_cfg(cfg)
    one_role.roles = 1
    with pytest.raises(B.MsrlError):
        B.msrl_rollout_init(env_cfg, one_role, 1)
    for bad in (synth.tag("tag9", 8, 5, 4, 2, 64, 4, 4),       # more than 8 agents per env
                synth.tag("tagl5", 8, 3, 3, 5, 64, 4, 4),      # more than 4 landmarks
                synth.tag("tagl3", 8, 1, 1, 3, 64, 4, 4),      # more landmarks than agents
                synth.tag("tagh", 8, 3, 1, 2, 128, 4, 4)):     # networks that do not fit the LDS four at a time
        with pytest.raises(B.MsrlError) as e:
            B.msrl_rollout_init(B.make_env_cfg(bad, None, None)[0], B.make_policy_cfg(bad), 1)
        assert e.value.code == B.MSRL_EUNSUPPORTED, bad.name
    c5 = synth.tag("tag5", 8, 4, 1, 2, 64, 4, 4)               # four tiles x five agents exceed a workgroup
    e5 = B.make_env_cfg(c5, None, None, tag_tiles=4)[0]
    with pytest.raises(B.MsrlError) as e:
        B.msrl_rollout_init(e5, B.make_policy_cfg(c5), 1)
    assert e.value.code == B.MSRL_EINVAL
    with pytest.raises(B.MsrlError):            # a learner holds one parameter set
        B.msrl_learner_init(B.make_policy_cfg(cfg), 64)


@pytest.mark.parametrize("path", ["on_chip", "device_memory"])
def test_learner_gradient_per_role_on_a_tag_trajectory(path):
    # Listing 1 runs one learner per role.  The learner holds one parameter set and is pointed at its role's
    # rows of the stored trajectory by an msrl_row_select (nothing is gathered on the device side); the oracle
    # gets the same rows gathered by the test.  Both learner paths; gradient per output unit, statistics,
    # msrl_rows_mean, and the update loop over a selection against the same loop on gathered rows.
    import torch
    from paper_2210_00882_amd import binding as B
    from test_gpu_learner import check_gradient_per_unit
    cfg = synth.tag("tag", 40, 3, 1, 2, 64, 8, 8, idx=61).with_(radius_c=0.3, radius_r=0.25)
    pol = ref.Policy(cfg.obs_dim, cfg.hidden, 5, bf16=True)
    params = synth.make_params(cfg, bias_std=0.1).astype(np.float64)
    n_role = pol.param_count
    with GpuRollout(cfg, params.astype(np.float32), SEED) as gpu:
        tr = gpu.run(cfg.T, logits=False)
    N, T = cfg.num_agents, cfg.T
    agent = np.tile(np.arange(cfg.M) % N, T)                       # agent slot of every flattened row
    flat = {k: tr[k][:T].reshape(T * cfg.M, *tr[k].shape[2:]) for k in ("obs", "actions", "logp", "adv", "ret", "rewards")}
    one = B.make_policy_cfg(cfg)
    one.roles = 1
    lib_path = B.MSRL_LEARNER_PATH_AUTO if path == "on_chip" else B.MSRL_LEARNER_PATH_DEVICE_MEMORY
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    for role, sel, rs in ((0, agent < cfg.num_chasers, B.msrl_row_select(N, 0, cfg.num_chasers)),
                          (1, agent >= cfg.num_chasers, B.msrl_row_select(N, cfg.num_chasers, N - cfg.num_chasers))):
        rows = {k: np.ascontiguousarray(v[sel]) for k, v in flat.items()}
        R = int(sel.sum())
        prm = params[role * n_role:(role + 1) * n_role]
        hp = dict(clip=0.2, vf_coef=0.5, ent_coef=0.01)
        # old log-probabilities shifted so that both branches of the clipped objective occur
        lp_old_all = (flat["logp"] - np.random.default_rng(role).choice([-0.4, 0.0, 0.4], T * cfg.M)).astype(np.float32)
        lp_old = lp_old_all[sel]
        _, g_ref, st_ref = ref.ppo_loss(pol, ref.ppo_cfg(**hp), prm, rows["obs"], rows["actions"], lp_old,
                                        rows["adv"], rows["ret"])
        L = B.msrl_learner_init_path(one, R, lib_path)
        try:
            grad = torch.empty(n_role, dtype=torch.float32, device="cuda")
            stats = torch.zeros(5, dtype=torch.float32, device="cuda")
            full = [dev(flat["obs"]), dev(flat["actions"]), dev(lp_old_all), dev(flat["adv"]), dev(flat["ret"])]
            B.msrl_ppo_grad(L, dev(prm.astype(np.float32)), *full, B.make_ppo_cfg(**hp), grad, stats, rows=rs)
            torch.cuda.synchronize()
            g = grad.cpu().numpy().astype(np.float64)
            st = stats.cpu().numpy().astype(np.float64) / R
            # the same rows, gathered by the test and passed without a selection: the same gradient up to
            # the order of the float additions
            gathered = [dev(rows["obs"]), dev(rows["actions"]), dev(lp_old), dev(rows["adv"]), dev(rows["ret"])]
            grad2 = torch.empty_like(grad)
            B.msrl_ppo_grad(L, dev(prm.astype(np.float32)), *gathered, B.make_ppo_cfg(**hp), grad2)
            torch.cuda.synchronize()
            g2 = grad2.cpu().numpy().astype(np.float64)
            assert np.abs(g - g2).max() <= 1e-5 * np.abs(g2).max()
            # mean reward of the role's rows
            mean = torch.full((1,), -7.0, device="cuda")
            B.msrl_rows_mean(dev(flat["rewards"]), mean, rows=rs)
            torch.cuda.synchronize()
            np.testing.assert_allclose(float(mean[0]), rows["rewards"].astype(np.float64).mean(), rtol=1e-5, atol=1e-6)
            # update loop: 2 passes x 3 minibatches over the selection == over the gathered rows
            pc = B.make_ppo_cfg(lr=1e-3, **hp)
            pa, pb = dev(prm.astype(np.float32)), dev(prm.astype(np.float32))
            ma, va, mb, vb = (torch.zeros_like(pa) for _ in range(4))
            Lu = B.msrl_learner_init_path(one, -(-R // 3) + 3, lib_path)
            try:
                ka = B.msrl_ppo_update(Lu, pa, ma, va, 0, 2, 3, *full, pc, rows=rs)
                kb = B.msrl_ppo_update(Lu, pb, mb, vb, 0, 2, 3, *gathered, pc)
                torch.cuda.synchronize()
            finally:
                B.msrl_learner_destroy(Lu)
            assert ka == kb == 6
            diff = np.abs(pa.cpu().numpy() - pb.cpu().numpy())
            assert diff.max() <= 2 * 1e-3 * 6 + 1e-6 and (diff > 1e-4).mean() < 0.01    # (Adam on noise-level entries)
            # bad selections
            for bad in (B.msrl_row_select(N, 3, 2), B.msrl_row_select(0, 0, 1), B.msrl_row_select(N, -1, 1),
                        B.msrl_row_select(N, 0, 0)):
                with pytest.raises(B.MsrlError) as e:
                    B.msrl_ppo_grad(L, dev(prm.astype(np.float32)), *full, B.make_ppo_cfg(**hp), grad, stats, rows=bad)
                assert e.value.code == B.MSRL_EINVAL
        finally:
            B.msrl_learner_destroy(L)
        assert 0.05 < st_ref[3] < 0.95
        np.testing.assert_allclose(st[[0, 1, 2, 4]], st_ref[[0, 1, 2, 4]], rtol=2e-2, atol=2e-2)
        one_cfg = cfg.with_(kind=synth.PARTICLE)     # (a single role's learner: shapes only)
        check_gradient_per_unit(f"role {role} {path}", one_cfg, pol, g, g_ref, 2e-2)


def test_training_loop_with_a_learner_per_role():
    # Trainer.train of Listing 1 on the pursuit env: rollout + GAE, then one update per role on that
    # role's rows.  Checked here: it runs, stays finite and moves both parameter sets; and the
    # chasers, whose reward is the number of contacts, come to touch the runners more often.
    from paper_2210_00882_amd import train
    cfg = synth.tag("tag", 1024, 3, 1, 2, 64, 32, 32, idx=62).with_(radius_c=0.15, radius_r=0.1)
    params = synth.make_params(cfg, bias_std=0.0, seed=9)
    final, hist = train.ppo_train(cfg, params, 40, 321, lr=1e-3, gamma=0.95, lam=0.95)
    hist = np.asarray(hist)
    assert np.isfinite(final).all() and np.isfinite(hist).all()
    n = params.size // 2
    assert np.abs(final[:n] - params[:n]).max() > 1e-3 and np.abs(final[n:] - params[n:]).max() > 1e-3
    assert (hist[:, 0] >= 0).all() and (hist[:, 1] <= 0).all()
    first, last = hist[:5, 0].mean(), hist[-5:, 0].mean()
    assert last > 2.0 * first, (first, last)     # measured: 0.34 -> 2.2 contacts x 10 per step
