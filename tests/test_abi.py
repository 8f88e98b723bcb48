"""Host-side checks of the C ABI that need no GPU: the library loads, exports
every symbol include/msrl.h declares, and rejects bad arguments before it
touches the device."""
import ctypes as C
import os
import re

import pytest

from paper_2210_00882_amd import binding as B, synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "msrl.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(msrl_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = B.load()
    names = declared_functions()
    assert set(names) == set(B.EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None


def test_param_count_and_state_size():
    for idx, want in [(1, 10_880 + 2 * (64 + 64) + 5 + 1), (5, 163_328 + 4 * 256 + 6)]:
        cfg = synth.CONFIGS[idx]
        assert B.msrl_param_count(B.make_policy_cfg(cfg)) == want == cfg.param_count
        e, _ = B.make_env_cfg(cfg)
        assert B.msrl_env_state_size(e) == cfg.env_state_size
    bad = B.msrl_policy_cfg(18, 0, 5, 0, 0)
    assert B.msrl_param_count(bad) == 0


@pytest.mark.parametrize("mutate,code", [
    (dict(num_envs=0), B.MSRL_EINVAL),
    (dict(episode_len=0), B.MSRL_EINVAL),
    (dict(obs_dim=17), B.MSRL_EINVAL),            # particle obs_dim must be 4 + 2L + 4(N-1)
    (dict(out_dim=4), B.MSRL_EINVAL),             # categorical particle policy has 5 outputs
    (dict(hidden=96), B.MSRL_EUNSUPPORTED),       # valid but not compiled
    # fp32 networks of 256 units: at most 7 agents per env (the layer-1 tiles of both networks stay in LDS)
    (dict(hidden=256, num_agents=8, num_landmarks=8, obs_dim=48), B.MSRL_EUNSUPPORTED),
    (dict(num_agents=11, num_landmarks=11, obs_dim=66), B.MSRL_EUNSUPPORTED),   # more than 10 agents per env
    (dict(num_agents=3, num_landmarks=2, obs_dim=16), B.MSRL_EUNSUPPORTED),     # landmarks != agents
])
def test_init_rejects_bad_configurations_before_touching_the_device(mutate, code):
    cfg = synth.CONFIGS[1].with_(**mutate)
    e, _ = B.make_env_cfg(cfg)
    p = B.make_policy_cfg(cfg)
    with pytest.raises(B.MsrlError) as ei:
        B.msrl_rollout_init(e, p, 1)
    assert ei.value.code == code and len(B.msrl_last_error()) > 10


@pytest.mark.parametrize("roles", [-1, 3, 7])
def test_init_rejects_bad_wave_roles_before_touching_the_device(roles):
    cfg = synth.CONFIGS[1]
    e, _ = B.make_env_cfg(cfg, wave_roles=roles)
    with pytest.raises(B.MsrlError) as ei:
        B.msrl_rollout_init(e, B.make_policy_cfg(cfg), 1)
    assert ei.value.code == B.MSRL_EINVAL and "wave_roles" in B.msrl_last_error()
    # the field belongs to the particle env
    lg = synth.CONFIGS[4].with_(num_envs=8)
    A, Bm = synth.make_dynamics(lg)
    e, keep = B.make_env_cfg(lg, A, Bm, wave_roles=2)
    with pytest.raises(B.MsrlError) as ei:
        B.msrl_rollout_init(e, B.make_policy_cfg(lg), 1)
    assert ei.value.code == B.MSRL_EINVAL


def test_null_and_size_checks():
    lib = B.load()
    assert lib.msrl_rollout_init(None, None, 0, None) == B.MSRL_EINVAL
    assert lib.msrl_rollout_step(None, None, 1, None, None) == B.MSRL_EINVAL
    assert lib.msrl_rollout_gae(None, None, 1, 0.99, 0.95, None, None) == B.MSRL_EINVAL
    assert lib.msrl_gae(None, None, None, -1, 4, 0.99, 0.95, None, None, None) == B.MSRL_EINVAL
    assert lib.msrl_gae(None, None, None, 4, 4, 0.99, 0.95, None, None, None) == B.MSRL_EINVAL
    assert lib.msrl_gae(None, None, None, 0, 4, 0.99, 0.95, None, None, None) == B.MSRL_OK
    assert lib.msrl_state_get(None, None, None) == B.MSRL_EINVAL
    assert lib.msrl_rollout_shape(None, None, None, None) == B.MSRL_EINVAL
    lib.msrl_rollout_destroy(None)
