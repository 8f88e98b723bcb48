"""GPU parity of the rollout with a centralised critic (multi-agent PPO, section 2.1 of the paper):
the policy network acts on an agent's own observation row, the value network on the joint
observation of the env's agents, one value per env.  The oracle side of the comparison is
ref.central_value on the N observation rows the GPU itself produced.
"""
import numpy as np
import pytest

from paper_2210_00882_amd import synth
from test_gpu_parity import run_and_check

pytestmark = pytest.mark.gpu


def _values_shared_per_env(cfg, tr):
    v = tr["values"].reshape(tr["values"].shape[0], cfg.num_envs, cfg.num_agents)
    assert (v == v[:, :, :1]).all()
    assert np.isfinite(v).all() and np.abs(v).max() > 0


@pytest.mark.parametrize("E,T,ep", [(50, 20, 6), (1, 4, 3), (21, 9, 25)])
def test_p3_central_critic_every_env_and_step(E, T, ep):
    # 20 envs per workgroup: several workgroups and a ragged last one; two calls in a row
    cfg = synth.particle("p3central", E, 3, 64, T, ep, dtype=synth.BF16, idx=50).with_(central_critic=True)
    assert cfg.value_in_dim == 3 * cfg.obs_dim
    tr, stats = run_and_check(cfg, T, calls=2)
    assert stats["rows"] == 2 * T * cfg.M and stats["mlp_rows"] == 2 * (T + 1) * cfg.M
    _values_shared_per_env(cfg, tr)


@pytest.mark.parametrize("N,H", [(2, 64), (4, 64), (5, 64), (7, 64), (10, 64), (4, 128), (6, 128), (7, 128), (9, 128),
                                 (10, 128), (7, 256), (8, 256), (9, 256)])
def test_central_critic_shapes_off_the_benchmark(N, H):
    # one wave per 32-unit chunk, the envs of a workgroup as the columns of the critic's tile: compiled for
    # 64 units from 2 agents per env, 128 from 4, 256 from 7 (up to 10 each)
    cfg = synth.particle(f"central{N}_{H}", 50, N, H, 9, 4, dtype=synth.BF16, idx=70 + N).with_(central_critic=True)
    tr, stats = run_and_check(cfg, 9, calls=2)
    assert stats["mlp_rows"] == 2 * 10 * cfg.M
    _values_shared_per_env(cfg, tr)


@pytest.mark.parametrize("N,H", [(2, 64), (3, 64), (5, 64), (8, 64), (4, 128), (6, 128), (8, 128)])
def test_central_critic_with_fp32_networks(N, H):
    # fp32 networks: 64 and 128 units, up to 8 agents per env; to the fp32 tolerance
    cfg = synth.particle(f"central{N}_{H}f", 50, N, H, 9, 4, dtype=synth.F32, idx=90 + N).with_(central_critic=True)
    tr, stats = run_and_check(cfg, 9, calls=2)
    assert stats["mlp_rows"] == 2 * 10 * cfg.M
    _values_shared_per_env(cfg, tr)


def test_central_critic_shapes_that_do_not_fit():
    from paper_2210_00882_amd import binding as B
    shapes = [(3, 128, synth.BF16), (6, 256, synth.BF16), (2, 256, synth.BF16),   # more envs per workgroup than the 32 columns of the critic's tile
              (9, 64, synth.F32), (9, 128, synth.F32), (7, 256, synth.F32)]       # fp32: the LDS, the ring of tile registers
    for N, H, dt in shapes:
        cfg = synth.particle("c", 8, N, H, 4, 4, dtype=dt, idx=1).with_(central_critic=True)
        with pytest.raises(B.MsrlError) as e:
            B.msrl_rollout_init(B.make_env_cfg(cfg, None, None)[0], B.make_policy_cfg(cfg), 1)
        assert e.value.code == B.MSRL_EUNSUPPORTED


@pytest.mark.parametrize("T", [1, 2, 3])
def test_central_critic_shortest_rollouts(T):
    # the value leaves the kernel two steps behind the step it belongs to: the shortest rollouts are all tail
    cfg = synth.particle("p3central", 23, 3, 64, T, 2, dtype=synth.BF16, idx=53).with_(central_critic=True)
    tr, stats = run_and_check(cfg, T, calls=3)
    assert stats["mlp_rows"] == 3 * (T + 1) * cfg.M
    _values_shared_per_env(cfg, tr)


def test_central_value_depends_on_every_agents_row():
    # with the critic's layer 1 zero except on the rows of one agent, the value must still change when
    # that agent is the last of the env: a critic that only saw the row's own observation would not
    cfg = synth.particle("p3central", 30, 3, 64, 5, 25, dtype=synth.BF16, idx=51).with_(central_critic=True)
    params = synth.make_params(cfg, bias_std=0.1)
    n_pi = cfg.param_count - (cfg.value_in_dim * cfg.hidden + cfg.hidden + cfg.hidden * cfg.hidden + cfg.hidden +
                              cfg.hidden + 1)
    w1 = params[n_pi:n_pi + cfg.value_in_dim * cfg.hidden].reshape(cfg.value_in_dim, cfg.hidden)
    w1[:2 * cfg.obs_dim] = 0       # the critic looks at agent 2's row only
    from helpers import GpuRollout, oracle_setup
    import helpers
    env, pol, p64, _ = oracle_setup(cfg, params=params)
    with GpuRollout(cfg, p64.astype(np.float32), 7) as gpu:
        tr = gpu.run(cfg.T)
    helpers.check_trajectory(cfg, tr, env, pol, p64, 7, list(range(cfg.num_envs)), 0, cfg.T)
    _values_shared_per_env(cfg, tr)
    v = tr["values"][0].reshape(cfg.num_envs, 3)[:, 0]
    assert np.unique(np.round(v, 4)).size > cfg.num_envs // 2     # differs from env to env


def test_cfg5_central_critic_sampled():
    # the benchmark's networks and agent count (4099 envs: many workgroups and a ragged tail)
    cfg = synth.CONFIGS[5].with_(num_envs=4099, T=12, central_critic=True)
    rng = np.random.default_rng(8)
    ids = [0, 1, 2, cfg.num_envs - 1] + sorted(rng.choice(cfg.num_envs, 5, replace=False).tolist())
    tr, _ = run_and_check(cfg, cfg.T, env_ids=ids)
    _values_shared_per_env(cfg, tr)
    assert (tr["obs"][:, :, 42:] == 0).all()


def test_central_critic_error_paths():
    from paper_2210_00882_amd import binding as B
    import torch
    cfg = synth.particle("p3central", 8, 3, 64, 4, 4, dtype=synth.BF16, idx=52).with_(central_critic=True)
    pc = B.make_policy_cfg(cfg)
    assert B.msrl_param_count(pc) == cfg.param_count
    env_cfg, keep = B.make_env_cfg(cfg, None, None)
    # more than two hidden layers: refused
    for bad in (cfg.with_(hidden_layers=3),):
        with pytest.raises(B.MsrlError):
            B.msrl_rollout_init(env_cfg, B.make_policy_cfg(bad), 1)
    pc_bad = B.make_policy_cfg(cfg)
    pc_bad.value_in_dim = 2 * cfg.obs_dim
    with pytest.raises(B.MsrlError):
        B.msrl_rollout_init(env_cfg, pc_bad, 1)
    pc_odd = B.make_policy_cfg(cfg)
    pc_odd.value_in_dim = 2 * cfg.obs_dim + 1          # the learner takes whole rows per group only
    with pytest.raises(B.MsrlError):
        B.msrl_learner_init(pc_odd, 64)
    st = B.msrl_rollout_init(env_cfg, pc, 1)
    try:
        params = B.upload_params(cfg, synth.make_params(cfg))
        obs = torch.zeros((cfg.M, cfg.obs_dim), device="cuda")
        B.msrl_observe(st, obs)
        a = torch.zeros(cfg.M, dtype=torch.int32, device="cuda")
        lp = torch.zeros(cfg.M, device="cuda")
        B.msrl_act(st, params, obs, a, lp, lp.clone())        # (checked against the oracle in test_gpu_steps.py)
        out = B.alloc_traj(cfg, 2, logits=False, gae=False)
        with pytest.raises(B.MsrlError) as e:                 # no measurement variants with a centralised critic
            B.msrl_measure_phase(st, params, 2, out, B.MSRL_PHASE_MLP)
        assert e.value.code == B.MSRL_EUNSUPPORTED
        torch.cuda.synchronize()
    finally:
        B.msrl_rollout_destroy(st)


def test_learner_and_rollout_agree_on_the_critic_and_the_update_fits_it():
    # the trajectory of a rollout with a centralised critic, fed to the learner as it is stored: the learner's
    # value network (groups of N consecutive rows) must see what the rollout kernel's critic saw, so its summed
    # squared error against ret equals the one computed from the rollout's own values; a few update steps on
    # the same rows then fit the critic to the returns
    import torch
    from paper_2210_00882_amd import binding as B
    cfg = synth.particle("p3central", 64, 3, 64, 10, 5, dtype=synth.BF16, idx=54).with_(central_critic=True)
    T, N, R = cfg.T, cfg.num_agents, cfg.T * cfg.M
    env_cfg, keep = B.make_env_cfg(cfg, None, None)
    pc = B.make_policy_cfg(cfg)
    params = synth.make_params(cfg, bias_std=0.1)                    # bfloat16-representable values
    acting = B.upload_params(cfg, params)
    master = torch.from_numpy(params.astype(np.float32)).cuda()
    st = B.msrl_rollout_init(env_cfg, pc, 99)
    L = B.msrl_learner_init(pc, R)
    try:
        out = B.alloc_traj(cfg, T, logits=False, gae=True)
        B.msrl_rollout_gae(st, acting, T, cfg.gamma, cfg.lam, out)
        rows = lambda t: t.reshape(-1, *t.shape[2:])
        batch = [rows(out["obs"][:T]), rows(out["actions"]), rows(out["logp"]), rows(out["adv"]), rows(out["ret"])]
        grad, stats = torch.empty_like(master), torch.zeros(5, device="cuda")
        hp = B.make_ppo_cfg(lr=3e-3)
        B.msrl_ppo_grad(L, master, *batch, hp, grad, stats)
        torch.cuda.synchronize()
        err = (out["values"][:T] - out["ret"]).reshape(T, cfg.num_envs, N)[:, :, 0]
        want = float((err.double() ** 2).sum())
        got = float(stats[1])
        assert want > 0 and abs(got - want) <= 2e-2 * want, (got, want)
        # logp of the stored actions under the same parameters: ratio 1, nothing clipped
        assert float(stats[3]) == 0 and abs(float(stats[4])) / R < 1e-3
        m, v = torch.zeros_like(master), torch.zeros_like(master)
        B.msrl_ppo_update(L, master, m, v, 0, 10, 2, *batch, hp)
        B.msrl_ppo_grad(L, master, *batch, hp, grad, stats)
        torch.cuda.synchronize()
        assert float(stats[1]) < 0.6 * got, (float(stats[1]), got)
    finally:
        B.msrl_learner_destroy(L)
        B.msrl_rollout_destroy(st)


def test_training_loop_with_a_centralised_critic_runs():
    from paper_2210_00882_amd import train
    cfg = synth.particle("p3central", 256, 3, 64, 25, 25, dtype=synth.BF16, idx=55).with_(central_critic=True)
    params = synth.make_params(cfg, bias_std=0.0, seed=5)
    new, hist = train.ppo_train(cfg, params, 6, 321, lr=1e-3)
    assert np.isfinite(hist).all() and np.isfinite(new).all() and all(h < 0 for h in hist)
    n_pi = cfg.param_count - (cfg.value_in_dim * cfg.hidden + cfg.hidden + cfg.hidden * cfg.hidden + cfg.hidden +
                              cfg.hidden + 1)
    assert np.abs(new[:n_pi] - params[:n_pi]).max() > 0 and np.abs(new[n_pi:] - params[n_pi:]).max() > 0


def test_update_loop_cuts_its_blocks_at_group_boundaries():
    # 37 groups of 3 rows in 4 minibatches: blocks of 27, 27, 27 and 30 rows (the oracle's rule); the loop equals
    # msrl_ppo_grad + msrl_adam_step on those blocks, and lands where the oracle's loop lands
    import torch
    from oracle import ref
    from paper_2210_00882_amd import binding as B
    from test_gpu_learner import make_batch
    cfg = synth.particle("p3c", 8, 3, 64, 4, 4, synth.F32, 13).with_(central_critic=True)
    G, R, mb, iters = 3, 3 * 37, 4, 2
    params = synth.make_params(cfg, bias_std=0.1).astype(np.float64)
    pol, obs, actions, logp_old, adv, ret = make_batch(cfg, R, 17, params)
    c = B.make_ppo_cfg(lr=1e-3)
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    d = [dev(x) for x in (obs, actions, logp_old, adv, ret)]
    L = B.msrl_learner_init(B.make_policy_cfg(cfg), 30)
    try:
        pa = dev(params.astype(np.float32)); ma = torch.zeros_like(pa); va = torch.zeros_like(pa)
        k = B.msrl_ppo_update(L, pa, ma, va, 0, iters, mb, *d, c)
        assert k == iters * mb
        pb = dev(params.astype(np.float32)); mbuf = torch.zeros_like(pb); vb = torch.zeros_like(pb)
        gr, kk, blk = torch.empty_like(pb), 0, R // mb // G * G
        assert blk == 27
        for it in range(iters):
            for b in range(mb):
                sl = slice(blk * b, R if b == mb - 1 else blk * b + blk)
                B.msrl_ppo_grad(L, pb, d[0][sl], d[1][sl], d[2][sl], d[3][sl], d[4][sl], c, gr)
                kk += 1
                B.msrl_adam_step(pb, mbuf, vb, gr, kk, c)
        torch.cuda.synchronize()
        diff = np.abs(pa.cpu().numpy() - pb.cpu().numpy())
        assert diff.max() <= 2 * 1e-3 * kk + 1e-6 and (diff > 1e-4).mean() < 0.01
        po, mo, vo = params.copy(), np.zeros_like(params), np.zeros_like(params)
        ref.ppo_update(pol, ref.ppo_cfg(lr=1e-3), po, mo, vo, 0, iters, mb, obs, actions, logp_old, adv, ret)
        loss = lambda p: ref.ppo_loss(pol, ref.ppo_cfg(), p, obs, actions, logp_old, adv, ret, want_grad=False)[0]
        l0, l_ref, l_gpu = loss(params), loss(po), loss(pa.cpu().numpy().astype(np.float64))
        assert l_ref < l0 and abs(l_gpu - l_ref) <= 0.02 * abs(l0 - l_ref) + 1e-6
        with pytest.raises(B.MsrlError):     # rows that are no whole groups
            B.msrl_ppo_update(L, pa, ma, va, k, 1, 4, d[0][:R - 1], d[1][:R - 1], d[2][:R - 1], d[3][:R - 1], d[4][:R - 1], c)
    finally:
        B.msrl_learner_destroy(L)
