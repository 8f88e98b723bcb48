"""msrl_rollout_gae_static (the entry point that allocates nothing: packed parameters in a static
device array, env batch in caller-owned buffers) against msrl_rollout_gae on an msrl_state.

Both run the same kernels on the same inputs, so every output is compared bit for bit: two calls in a
row on one configuration (the second continues the trajectory), then a smaller configuration of another
shape (a smaller parameter image in the same array, which still holds the larger one), then the pursuit
env (four parameter sets), and the refusals.  Runs last in the suite and also alone in a fresh process.
"""
import numpy as np
import pytest

from helpers import GpuRollout, oracle_setup
from paper_2210_00882_amd import synth

pytestmark = pytest.mark.gpu

KEYS = ("obs", "actions", "logp", "rewards", "dones", "values", "adv", "ret")


def run_both(cfg, seed, T, calls, tag_tiles=0):
    """`calls` consecutive calls of T steps through both entry points; asserts bit-equality of every
    trajectory tensor and of the env state afterwards."""
    import torch
    from paper_2210_00882_amd import binding as B
    params = synth.make_params(cfg, bias_std=0.1)
    with GpuRollout(cfg, params, seed, tag_tiles=tag_tiles) as gpu:
        es0, g0 = gpu.get_state()
        shift = (np.arange(cfg.num_envs) % 5).astype(np.int64)       # different episode phases
        gpu.set_state(None, g0 + shift)
        es_dev = torch.from_numpy(es0).cuda()
        g_dev = torch.from_numpy(g0 + shift).cuda()
        for call in range(calls):
            want = gpu.run(T, gae=True, logits=False)
            out = B.alloc_traj(cfg, T, logits=False, gae=True)
            for v in out.values():
                if v is not None:
                    v.fill_(-55 if v.dtype != torch.uint8 else 55)
            B.msrl_rollout_gae_static(gpu.env_cfg, gpu.pol_cfg, seed, es_dev, g_dev, gpu.params, T, cfg.gamma, cfg.lam, out)
            torch.cuda.synchronize()
            for k in KEYS:
                np.testing.assert_array_equal(out[k].cpu().numpy(), want[k], err_msg=f"{cfg.name} call {call}: {k}")
            es1, g1 = gpu.get_state()
            np.testing.assert_array_equal(es_dev.cpu().numpy(), es1, err_msg=f"{cfg.name} call {call}: env state")
            np.testing.assert_array_equal(g_dev.cpu().numpy(), g1, err_msg=f"{cfg.name} call {call}: counters")
            assert (g1 == g0 + shift + (call + 1) * T).all()


def test_static_entry_point_matches_the_allocating_one():
    from paper_2210_00882_amd import binding as B
    # the benchmark's shape (10 agents, 256-unit bf16 networks: a 386 KiB image), ragged workgroups
    run_both(synth.CONFIGS[5].with_(num_envs=70, episode_len=4), 41, 6, calls=2)
    # then a smaller input: 3 agents, 64-unit fp32 networks (the array still holds the larger image)
    run_both(synth.CONFIGS[1].with_(num_envs=21, episode_len=3), 42, 5, calls=2)
    # centralised critic (policy image + a critic image of another layout)
    run_both(synth.CONFIGS[5].with_(num_envs=33, episode_len=4, central_critic=True), 43, 5, calls=1)
    # pursuit env: four networks, both workgroup shapes
    run_both(synth.tag("tag", 70, 3, 1, 2, 64, 6, 4, idx=50), 44, 6, calls=2, tag_tiles=1)
    run_both(synth.tag("tag", 70, 3, 1, 2, 64, 6, 4, idx=50), 44, 6, calls=1, tag_tiles=4)
    # and the first configuration again
    run_both(synth.CONFIGS[5].with_(num_envs=70, episode_len=4), 41, 6, calls=1)


def test_static_entry_point_refusals():
    import torch
    from paper_2210_00882_amd import binding as B

    def call(cfg, dyn=None, T=3, drop=None):
        A, Bm = dyn if dyn is not None else (None, None)
        e, _keep = B.make_env_cfg(cfg, A, Bm)
        p = B.make_policy_cfg(cfg)
        es = torch.zeros((cfg.num_envs, cfg.env_state_size), dtype=torch.float32, device="cuda")
        g = torch.zeros(cfg.num_envs, dtype=torch.int64, device="cuda")
        params = B.upload_params(cfg, synth.make_params(cfg))
        out = B.alloc_traj(cfg, max(T, 1), logits=False, gae=True)
        if drop:
            out[drop] = None
        B.msrl_rollout_gae_static(e, p, 1, es, g, params, T, 0.99, 0.95, out)

    small = synth.CONFIGS[1].with_(num_envs=8)
    # an image beyond the array: seven hidden layers of 256 units
    with pytest.raises(B.MsrlError) as ei:
        call(synth.CONFIGS[5].with_(num_envs=8, hidden_layers=7))
    assert ei.value.code == B.MSRL_EUNSUPPORTED and "static scratch" in str(ei.value)
    with pytest.raises(B.MsrlError) as ei:
        call(synth.CONFIGS[4].with_(num_envs=8), dyn=synth.make_dynamics(synth.CONFIGS[4]))
    assert ei.value.code == B.MSRL_EUNSUPPORTED
    with pytest.raises(B.MsrlError) as ei:
        call(small, T=0)
    assert ei.value.code == B.MSRL_EINVAL
    with pytest.raises(B.MsrlError) as ei:
        call(small, drop="adv")
    assert ei.value.code == B.MSRL_EINVAL
    with pytest.raises(B.MsrlError) as ei:
        call(small.with_(hidden=96))
    assert ei.value.code == B.MSRL_EUNSUPPORTED
    call(small)            # and a valid call still works afterwards
    torch.cuda.synchronize()
