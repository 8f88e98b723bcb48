"""Step-granular calls (msrl_observe / msrl_act / msrl_env_step) through the C ABI.

The fused rollout is checked against the oracle in test_gpu_parity.py; here the split calls are
checked (a) to reproduce the fused call bit for bit, and (b) directly against the oracle's
environment step for actions the test chooses itself.
"""
import numpy as np
import pytest

from helpers import GpuRollout, TOL_F32, assert_close, oracle_setup
from oracle import ref
from paper_2210_00882_amd import synth

pytestmark = pytest.mark.gpu


def split_rollout(gpu, T, logits=True):
    """T x { observe / act / env_step } -> the arrays msrl_rollout_step would fill."""
    import torch
    B, cfg = gpu.B, gpu.cfg
    M, D = cfg.M, cfg.obs_dim
    tr = B.alloc_traj(cfg, T, logits=logits, gae=False)
    for v in tr.values():
        if v is not None:
            v.fill_(-77 if v.dtype != torch.uint8 else 77)
    B.msrl_observe(gpu.state, tr["obs"][0])
    for t in range(T):
        B.msrl_act(gpu.state, gpu.params, tr["obs"][t], tr["actions"][t], tr["logp"][t], tr["values"][t],
                   tr["logits"][t] if logits else None)
        B.msrl_env_step(gpu.state, tr["actions"][t], tr["rewards"][t], tr["dones"][t], tr["obs"][t + 1])
    # values[T]: one more evaluation whose sampled outputs are dropped
    scratch_a = torch.empty_like(tr["actions"][0])
    scratch_l = torch.empty(M, dtype=torch.float32, device="cuda")
    B.msrl_act(gpu.state, gpu.params, tr["obs"][T], scratch_a, scratch_l, tr["values"][T], None)
    torch.cuda.synchronize()
    return {k: (None if v is None else v.cpu().numpy()) for k, v in tr.items()}


@pytest.mark.parametrize("which", ["n3_f32_ragged", "n1_f32", "n6_f32", "n3_bf16", "n10_bf16", "lingauss"])
def test_split_calls_reproduce_the_fused_rollout(which):
    cfg = {
        "n3_f32_ragged": synth.CONFIGS[1].with_(num_envs=53, episode_len=4),
        "n1_f32": synth.particle("p1", 70, 1, 64, 6, 3, synth.F32, 11),
        "n6_f32": synth.CONFIGS[3].with_(num_envs=77, episode_len=5),
        "n3_bf16": synth.particle("p3b", 45, 3, 64, 6, 3, synth.BF16, 12),
        "n10_bf16": synth.CONFIGS[5].with_(num_envs=100, episode_len=3),
        "lingauss": synth.CONFIGS[4].with_(num_envs=150, episode_len=3),
    }[which]
    T = 7
    _, _, params, dyn = oracle_setup(cfg)
    with GpuRollout(cfg, params.astype(np.float32), 31, dyn=dyn) as gpu:
        fused = gpu.run(T, gae=False, logits=True)
        es_f, g_f = gpu.get_state()
    with GpuRollout(cfg, params.astype(np.float32), 31, dyn=dyn) as gpu:
        split = split_rollout(gpu, T)
        es_s, g_s = gpu.get_state()
    for k in ("obs", "actions", "logp", "rewards", "dones", "values", "logits"):
        np.testing.assert_array_equal(fused[k], split[k], err_msg=k)
    np.testing.assert_array_equal(es_f, es_s)
    np.testing.assert_array_equal(g_f, g_s)
    assert (g_s == T).all()


def test_env_step_against_the_oracle_for_chosen_actions():
    import torch
    cfg = synth.CONFIGS[1].with_(num_envs=41, episode_len=3)
    env, _, params, _ = oracle_setup(cfg)
    N, M, D = cfg.num_agents, cfg.M, cfg.obs_dim
    rng = np.random.default_rng(5)
    seed = 77
    with GpuRollout(cfg, params.astype(np.float32), seed) as gpu:
        B = gpu.B
        obs = torch.empty((M, D), dtype=torch.float32, device="cuda")
        rew = torch.empty(M, dtype=torch.float32, device="cuda")
        done = torch.empty(M, dtype=torch.uint8, device="cuda")
        for step in range(4):                       # crosses an episode end (reset draws)
            es, g = gpu.get_state()
            acts = rng.integers(0, 5, size=M).astype(np.int32)
            B.msrl_env_step(gpu.state, torch.from_numpy(acts).cuda(), rew, done, obs)
            torch.cuda.synchronize()
            r_gpu, d_gpu, o_gpu = rew.cpu().numpy(), done.cpu().numpy(), obs.cpu().numpy()
            es1, g1 = gpu.get_state()
            assert (g1 == g + 1).all()
            for e in range(cfg.num_envs):
                s = es[e].astype(np.float64)
                s2, r, d, margin = ref.env_step(env, seed, e, int(g[e]), s, acts[e * N:(e + 1) * N])
                if margin > 1e-5:   # no pair distance within 1e-5 of the collision threshold
                    assert_close(r_gpu[e * N:(e + 1) * N], np.full(N, r), TOL_F32, f"reward env {e} step {step}")
                assert (d_gpu[e * N:(e + 1) * N] == d).all()
                assert_close(es1[e], s2, TOL_F32, f"state env {e} step {step}")
                assert_close(o_gpu[e * N:(e + 1) * N], ref.env_obs(env, es1[e].astype(np.float64)), TOL_F32,
                             f"next obs env {e} step {step}")


def test_observe_and_act_leave_the_state_alone_and_argument_errors():
    import torch
    cfg = synth.CONFIGS[1].with_(num_envs=9)
    _, _, params, _ = oracle_setup(cfg)
    M, D = cfg.M, cfg.obs_dim
    with GpuRollout(cfg, params.astype(np.float32), 3) as gpu:
        B = gpu.B
        es0, g0 = gpu.get_state()
        obs = torch.empty((M, D), dtype=torch.float32, device="cuda")
        a = torch.empty(M, dtype=torch.int32, device="cuda")
        lp = torch.empty(M, dtype=torch.float32, device="cuda")
        v = torch.empty(M, dtype=torch.float32, device="cuda")
        B.msrl_observe(gpu.state, obs)
        B.msrl_act(gpu.state, gpu.params, obs, a, lp, v)
        B.msrl_act(gpu.state, gpu.params, obs, a, lp, v)
        torch.cuda.synchronize()
        es1, g1 = gpu.get_state()
        np.testing.assert_array_equal(es0, es1)
        np.testing.assert_array_equal(g0, g1)
        with pytest.raises(B.MsrlError) as e:
            B.msrl_act(gpu.state, gpu.params, obs, a, lp, None)
        assert e.value.code == B.MSRL_EINVAL
        with pytest.raises(B.MsrlError) as e:
            B.msrl_env_step(gpu.state, a, None, None, obs)
        assert e.value.code == B.MSRL_EINVAL
