"""Seeded synthetic inputs: the five benchmark configurations and their tensors.

This module holds no arithmetic of the method itself (no env step, network,
sampler or GAE): it only names shapes and draws input values, so that the HIP
path and the CPU oracle can be fed the same numbers.  numpy + torch (CPU) only.

The particle configurations stand in for the multi-agent particle tasks the
paper evaluates on (section 7.4: n agents cover n landmarks, collisions are
penalised); the linear-Gaussian one stands in for the 17-observation /
6-action continuous-control task with 1000-step episodes of section 7.2.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np

PARTICLE, LINGAUSS, TAG = 0, 1, 2
F32, BF16 = 0, 1
CATEGORICAL, DIAG_GAUSSIAN = 0, 1


@dataclass(frozen=True)
class Config:
    name: str
    kind: int
    num_envs: int
    num_agents: int
    num_landmarks: int
    obs_dim: int
    act_dim: int
    hidden: int
    out_dim: int
    dtype: int
    dist: int
    T: int
    episode_len: int
    dt: float = 0.1
    damping: float = 0.25
    force: float = 1.0
    radius: float = 0.15
    noise_std: float = 0.01
    act_cost: float = 0.01
    gamma: float = 0.99
    lam: float = 0.95
    env_seed: int = 0
    param_seed: int = 0
    hidden_layers: int = 2   # tanh layers of `hidden` units in front of the output layer
    central_critic: bool = False   # value net on the joint observation of the env's agents (one value per env)
    # pursuit ("tag") env: the first num_chasers agents chase the others; one parameter set per role
    num_chasers: int = 0
    accel_c: float = 3.0
    accel_r: float = 4.0
    vmax_c: float = 1.0
    vmax_r: float = 1.3
    radius_c: float = 0.075
    radius_r: float = 0.05
    contact_force: float = 100.0
    contact_margin: float = 1e-3
    extra: dict = field(default_factory=dict)

    @property
    def M(self) -> int:
        return self.num_envs * self.num_agents

    @property
    def roles(self) -> int:
        return 2 if self.kind == TAG else 1

    @property
    def env_state_size(self) -> int:
        if self.kind != LINGAUSS:
            return 4 * self.num_agents + 2 * self.num_landmarks
        return self.obs_dim

    @property
    def param_count(self) -> int:
        return self.roles * (net_param_count(self.obs_dim, self.hidden, self.out_dim, self.hidden_layers) +
                             net_param_count(self.value_in_dim, self.hidden, 1, self.hidden_layers))

    @property
    def value_in_dim(self) -> int:
        return self.num_agents * self.obs_dim if self.central_critic else self.obs_dim

    def with_(self, **kw) -> "Config":
        d = dict(self.__dict__)
        d.update(kw)
        return Config(**d)


def net_param_count(i: int, h: int, o: int, layers: int = 2) -> int:
    return i * h + h + (layers - 1) * (h * h + h) + h * o + o


def particle(name, E, N, H, T, ep, dtype=F32, idx=0) -> Config:
    return Config(name=name, kind=PARTICLE, num_envs=E, num_agents=N, num_landmarks=N,
                  obs_dim=6 * N, act_dim=1, hidden=H, out_dim=5, dtype=dtype, dist=CATEGORICAL,
                  T=T, episode_len=ep, env_seed=0x5EED0000 + idx, param_seed=1000 + idx)


def tag(name, E, NC, NR, L, H, T, ep, dtype=BF16, idx=0) -> Config:
    """Pursuit env: NC chasers, NR runners, L landmarks; observation 4 + 2L + 4(N-1) wide."""
    N = NC + NR
    return Config(name=name, kind=TAG, num_envs=E, num_agents=N, num_landmarks=L,
                  obs_dim=4 + 2 * L + 4 * (N - 1), act_dim=1, hidden=H, out_dim=5, dtype=dtype, dist=CATEGORICAL,
                  T=T, episode_len=ep, env_seed=0x5EED0000 + idx, param_seed=1000 + idx, num_chasers=NC)


def lingauss(name, E, S, K, H, T, ep, idx=0) -> Config:
    return Config(name=name, kind=LINGAUSS, num_envs=E, num_agents=1, num_landmarks=0,
                  obs_dim=S, act_dim=K, hidden=H, out_dim=2 * K, dtype=F32, dist=DIAG_GAUSSIAN,
                  T=T, episode_len=ep, env_seed=0x5EED0000 + idx, param_seed=1000 + idx)


CONFIGS = {
    1: particle("cfg1_particle_64x3_h64_f32", 64, 3, 64, 100, 25, F32, 1),
    2: particle("cfg2_particle_4096x3_h64_f32", 4096, 3, 64, 128, 25, F32, 2),
    3: particle("cfg3_particle_16384x6_h128_f32", 16384, 6, 128, 128, 50, F32, 3),
    4: lingauss("cfg4_lingauss_32768_s17a6_h256_f32", 32768, 17, 6, 256, 256, 1000, 4),
    5: particle("cfg5_particle_65536x10_h256_bf16", 65536, 10, 256, 200, 50, BF16, 5),
}


def make_params(cfg: Config, bias_std: float = 0.0, seed: int | None = None) -> np.ndarray:
    """Flat float32 parameter vector, policy net then value net, each
    W1 b1 W2 b2 W3 b3 (one more W b per hidden layer beyond two) with W[in, out]; weights ~ N(0, 1/fan_in), biases ~
    N(0, bias_std^2) (0 in the benchmark recipe).  For BF16 configurations every
    value is rounded to a bfloat16-representable float32."""
    rng = np.random.default_rng(cfg.param_seed if seed is None else seed)
    parts = []
    for k, out in enumerate((cfg.out_dim, 1) * cfg.roles):   # per role: policy net, value net
        dims = [cfg.value_in_dim if k % 2 else cfg.obs_dim] + [cfg.hidden] * cfg.hidden_layers + [out]
        for fan_in, fan_out in zip(dims[:-1], dims[1:]):
            parts.append((rng.standard_normal((fan_in, fan_out)) / np.sqrt(fan_in)).ravel())
            parts.append(rng.standard_normal(fan_out) * bias_std)
    p = np.concatenate(parts).astype(np.float32)
    assert p.size == cfg.param_count
    if cfg.dtype == BF16:
        p = to_bf16_representable(p)
    return p


def to_bf16_representable(x: np.ndarray) -> np.ndarray:
    import torch
    return torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(torch.bfloat16).to(torch.float32).numpy()


def make_dynamics(cfg: Config, seed: int = 2000):
    """A = 0.98 * (seeded random orthogonal matrix), B ~ N(0, 0.1) (variance),
    both float32, row-major [D, D] and [D, act_dim]."""
    rng = np.random.default_rng(seed)
    q, r = np.linalg.qr(rng.standard_normal((cfg.obs_dim, cfg.obs_dim)))
    q = q * np.sign(np.diag(r))[None, :]
    A = (0.98 * q).astype(np.float32)
    B = (rng.standard_normal((cfg.obs_dim, cfg.act_dim)) * np.sqrt(0.1)).astype(np.float32)
    return A, B


def make_gae_inputs(T: int, M: int, episode_len: int, seed: int = 7):
    """Rewards <= 0 of the particle scale, values ~ N(0,1), dones on every
    episode_len-th step (shifted per column block so columns differ)."""
    rng = np.random.default_rng(seed)
    r = (-np.abs(rng.standard_normal((T, M))) * 2.0).astype(np.float32)
    v = rng.standard_normal((T + 1, M)).astype(np.float32)
    phase = rng.integers(0, max(1, episode_len), size=M)
    t = np.arange(T)[:, None]
    d = (((t + phase[None, :] + 1) % max(1, episode_len)) == 0).astype(np.uint8)
    return r, v, d
