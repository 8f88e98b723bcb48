"""Behaviour of the C ABI on the device beyond numerics: determinism, optional
outputs, call equivalences, argument errors raised before any launch."""
import numpy as np
import pytest

from paper_2210_00882_amd import synth
from helpers import GpuRollout, oracle_setup

pytestmark = pytest.mark.gpu


def small_cfg():
    return synth.CONFIGS[1].with_(num_envs=77, episode_len=6)


def test_two_runs_are_bit_identical():
    cfg = small_cfg()
    _, _, params, _ = oracle_setup(cfg)
    runs = []
    for _ in range(2):
        with GpuRollout(cfg, params.astype(np.float32), 99) as gpu:
            runs.append(gpu.run(21))
    for k in runs[0]:
        np.testing.assert_array_equal(runs[0][k], runs[1][k])


def test_optional_logits_and_step_vs_fused_call():
    cfg = small_cfg()
    _, _, params, _ = oracle_setup(cfg)
    with GpuRollout(cfg, params.astype(np.float32), 5) as gpu:
        full = gpu.run(15, gae=True, logits=True)
    with GpuRollout(cfg, params.astype(np.float32), 5) as gpu:
        bare = gpu.run(15, gae=False, logits=False)
        # adv / ret are not touched by msrl_rollout_step; logits were not requested
        assert bare["logits"] is None and bare["adv"] is None
    for k in ("obs", "actions", "logp", "rewards", "dones", "values"):
        np.testing.assert_array_equal(full[k], bare[k])


def test_one_long_call_equals_two_short_ones():
    cfg = small_cfg()
    _, _, params, _ = oracle_setup(cfg)
    with GpuRollout(cfg, params.astype(np.float32), 5) as gpu:
        whole = gpu.run(17)
    with GpuRollout(cfg, params.astype(np.float32), 5) as gpu:
        a = gpu.run(8)
        b = gpu.run(9)
    for k in ("actions", "logp", "rewards", "dones"):
        np.testing.assert_array_equal(whole[k], np.concatenate([a[k], b[k]]))
    np.testing.assert_array_equal(whole["obs"][8:], b["obs"])
    np.testing.assert_array_equal(whole["values"][:8], a["values"][:8])


def test_state_snapshot_round_trip():
    cfg = small_cfg()
    _, _, params, _ = oracle_setup(cfg)
    with GpuRollout(cfg, params.astype(np.float32), 5) as gpu:
        gpu.run(7)
        es, g = gpu.get_state()
        ref_run = gpu.run(5)
        gpu.set_state(es, g)
        again = gpu.run(5)
    for k in ref_run:
        np.testing.assert_array_equal(ref_run[k], again[k])


def test_argument_errors():
    import torch
    cfg = small_cfg()
    _, _, params, _ = oracle_setup(cfg)
    with GpuRollout(cfg, params.astype(np.float32), 5) as gpu:
        B = gpu.B
        out = B.alloc_traj(cfg, 4, logits=False, gae=False)
        with pytest.raises(B.MsrlError) as e:
            B.msrl_rollout_step(gpu.state, gpu.params, 0, out)
        assert e.value.code == B.MSRL_EINVAL
        with pytest.raises(B.MsrlError) as e:           # adv / ret missing for the fused call
            B.msrl_rollout_gae(gpu.state, gpu.params, 4, 0.99, 0.95, out)
        assert e.value.code == B.MSRL_EINVAL
        broken = dict(out)
        broken["rewards"] = None
        with pytest.raises(B.MsrlError):
            B.msrl_rollout_step(gpu.state, gpu.params, 4, broken)
        with pytest.raises(B.MsrlError):
            B.msrl_state_set(gpu.state, None, np.full(cfg.num_envs, -1, dtype=np.int64))
        # the state is still usable after rejected calls
        B.msrl_rollout_step(gpu.state, gpu.params, 4, out)
        torch.cuda.synchronize()
        assert int(out["dones"].max()) <= 1


@pytest.mark.parametrize("which", ["f32_small", "bf16_big"])
def test_env_phase_equals_the_full_kernel_with_zero_parameters(which):
    # the measurement variant that skips the networks must be the rollout an all-zero parameter
    # buffer gives: logits 0, values 0, uniform categorical draws
    import torch
    if which == "f32_small":
        cfg = synth.CONFIGS[1].with_(num_envs=53, episode_len=7)
    else:
        cfg = synth.CONFIGS[5].with_(num_envs=100, T=12, episode_len=5)
    T = 12
    zeros = np.zeros(cfg.param_count, dtype=np.float32)
    with GpuRollout(cfg, zeros, 21) as gpu:
        full = gpu.run(T, gae=False, logits=True)
    with GpuRollout(cfg, zeros, 21) as gpu:
        B = gpu.B
        dev = B.alloc_traj(cfg, T, logits=True, gae=False)
        B.msrl_measure_phase(gpu.state, gpu.params, T, dev, B.MSRL_PHASE_ENV)
        torch.cuda.synchronize()
        _, g = gpu.get_state()
        env_only = {k: (None if v is None else v.cpu().numpy()) for k, v in dev.items()}
    assert (g == T).all()
    for k in ("obs", "actions", "logp", "rewards", "dones", "values", "logits"):
        np.testing.assert_array_equal(full[k], env_only[k])
    assert (env_only["logits"] == 0).all() and (env_only["values"] == 0).all()
    np.testing.assert_allclose(env_only["logp"], np.log(0.2), rtol=1e-6)


def test_mlp_phase_leaves_the_state_alone():
    import torch
    cfg = synth.CONFIGS[5].with_(num_envs=60, T=6)
    _, _, params, _ = oracle_setup(cfg)
    with GpuRollout(cfg, params.astype(np.float32), 3) as gpu:
        B = gpu.B
        es0, g0 = gpu.get_state()
        dev = B.alloc_traj(cfg, 6, logits=False, gae=False)
        B.msrl_measure_phase(gpu.state, gpu.params, 6, dev, B.MSRL_PHASE_MLP)
        torch.cuda.synchronize()
        es1, g1 = gpu.get_state()
        assert bool(torch.isfinite(dev["rewards"][0]).all())
    np.testing.assert_array_equal(es0, es1)
    np.testing.assert_array_equal(g0, g1)
    with GpuRollout(synth.CONFIGS[2].with_(num_envs=8), np.zeros(synth.CONFIGS[2].param_count, np.float32), 1) as gpu:
        dev = gpu.B.alloc_traj(gpu.cfg, 2, gae=False)
        with pytest.raises(gpu.B.MsrlError) as e:   # not compiled for this configuration
            gpu.B.msrl_measure_phase(gpu.state, gpu.params, 2, dev, gpu.B.MSRL_PHASE_MLP)
        assert e.value.code == gpu.B.MSRL_EUNSUPPORTED


def test_clock_variant_computes_the_same_rollout():
    # the variant that also records in-kernel clocks must write every output of the plain kernel,
    # and monotonically increasing stamps for the waves of the first workgroup
    import torch
    cfg = synth.CONFIGS[5].with_(num_envs=100, T=8, episode_len=5)
    T = 8
    _, _, params, _ = oracle_setup(cfg)
    with GpuRollout(cfg, params.astype(np.float32), 9) as gpu:
        plain = gpu.run(T, gae=False, logits=False)
    with GpuRollout(cfg, params.astype(np.float32), 9) as gpu:
        B = gpu.B
        dev = B.alloc_traj(cfg, T, logits=False, gae=False)
        with pytest.raises(B.MsrlError) as e:           # the stamps need a buffer
            B.msrl_measure_phase(gpu.state, gpu.params, T, dev, B.MSRL_PHASE_CLOCKS)
        assert e.value.code == B.MSRL_EINVAL
        stamps = torch.zeros(256, dtype=torch.float32, device="cuda")
        B.msrl_measure_phase(gpu.state, gpu.params, T, dict(dev, logits=stamps), B.MSRL_PHASE_CLOCKS)
        torch.cuda.synchronize()
        timed = {k: v.cpu().numpy() for k, v in dev.items() if v is not None}
        c = stamps.cpu().numpy().reshape(8, 32)
    for k in ("obs", "actions", "logp", "rewards", "dones", "values"):
        np.testing.assert_array_equal(plain[k], timed[k])
    order = [0, 1, 2, 3, 4, 5, 6, 8, 9, 10, 11, 12, 14, 15, 16]
    assert (np.diff(c[:, order], axis=1) > 0).all()
    assert (c[:, 16] < 5e6).all()


def test_fused_call_replays_from_a_hip_graph():
    # the call enqueues kernels only (no allocation, no memset), so it can be captured once and
    # replayed: replay k must equal the k-th eager call of a second, identical state
    import torch
    cfg = synth.CONFIGS[1].with_(num_envs=40, episode_len=4)
    T = 6
    _, _, params, _ = oracle_setup(cfg)
    with GpuRollout(cfg, params.astype(np.float32), 13) as gpu:
        eager = [gpu.run(T, gae=True, logits=False) for _ in range(4)]
    with GpuRollout(cfg, params.astype(np.float32), 13) as gpu:
        B = gpu.B
        dev = B.alloc_traj(cfg, T, logits=False, gae=True)
        stream = torch.cuda.Stream()
        stream.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(stream):
            B.msrl_rollout_gae(gpu.state, gpu.params, T, cfg.gamma, cfg.lam, dev, stream=stream)   # call 0, eager
        stream.synchronize()
        first = {k: v.cpu().numpy() for k, v in dev.items() if v is not None}
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=stream):
            B.msrl_rollout_gae(gpu.state, gpu.params, T, cfg.gamma, cfg.lam, dev, stream=torch.cuda.current_stream())
        for k in first:
            np.testing.assert_array_equal(first[k], eager[0][k], err_msg=k)
        for rep in range(1, 4):
            graph.replay()
            torch.cuda.synchronize()
            got = {k: v.cpu().numpy() for k, v in dev.items() if v is not None}
            for k in got:
                np.testing.assert_array_equal(got[k], eager[rep][k], err_msg=f"{k} replay {rep}")
            _ = torch.ones(1000, device="cuda").sum().item()   # unrelated eager work between replays
