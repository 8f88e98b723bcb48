"""ctypes front end of the CPU oracle (oracle/msrl_ref.c, oracle/msrl_learn_ref.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
cpu_baseline leg of bench.py.  Nothing in the product package imports it, and it
imports nothing from the product package.

Every array is float64 / int32 / uint8 / int64 numpy, C-contiguous.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "msrl_ref.c")
_SRCS = [_SRC, os.path.join(_HERE, "msrl_learn_ref.c")]
_LIB = os.path.join(_HERE, "libmsrl_ref.so")

PARTICLE, LINGAUSS, TAG = 0, 1, 2
CATEGORICAL, DIAG_GAUSSIAN = 0, 1


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, no fast-math)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < max(os.path.getmtime(f) for f in _SRCS):
        subprocess.check_call(
            ["gcc", "-O2", "-std=c99", "-fPIC", "-shared", "-Wall", "-o", _LIB, *_SRCS, "-lm"]
        )
    return _LIB


class EnvCfg(C.Structure):
    _fields_ = [
        ("kind", C.c_int32), ("num_agents", C.c_int32), ("num_landmarks", C.c_int32),
        ("obs_dim", C.c_int32), ("act_dim", C.c_int32), ("episode_len", C.c_int32),
        ("dt", C.c_double), ("damping", C.c_double), ("force", C.c_double), ("radius", C.c_double),
        ("A", C.c_void_p), ("B", C.c_void_p),
        ("noise_std", C.c_double), ("act_cost", C.c_double),
        ("num_chasers", C.c_int32), ("pad_", C.c_int32),
        ("accel_c", C.c_double), ("accel_r", C.c_double), ("vmax_c", C.c_double), ("vmax_r", C.c_double),
        ("radius_c", C.c_double), ("radius_r", C.c_double),
        ("contact_force", C.c_double), ("contact_margin", C.c_double),
    ]


class PolicyCfg(C.Structure):
    _fields_ = [("in_dim", C.c_int32), ("hidden", C.c_int32), ("out_dim", C.c_int32),
                ("bf16", C.c_int32), ("dist", C.c_int32), ("hidden_layers", C.c_int32),
                ("value_in_dim", C.c_int32)]


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.ref_uniform.restype = C.c_double
        _lib.ref_uniform.argtypes = [C.c_uint32]
        _lib.ref_bf16_round.restype = C.c_double
        _lib.ref_bf16_round.argtypes = [C.c_double]
        _lib.ref_net_param_count.restype = C.c_size_t
        _lib.ref_net_param_count_l.restype = C.c_size_t
        _lib.ref_env_state_size.restype = C.c_int
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


class Env:
    """Environment configuration (keeps A and B alive)."""

    def __init__(self, kind, num_agents, num_landmarks, obs_dim, act_dim, episode_len,
                 dt=0.1, damping=0.25, force=1.0, radius=0.15, A=None, B=None,
                 noise_std=0.01, act_cost=0.01, num_chasers=0, accel_c=3.0, accel_r=4.0, vmax_c=1.0, vmax_r=1.3,
                 radius_c=0.075, radius_r=0.05, contact_force=100.0, contact_margin=1e-3):
        self.A = None if A is None else _f64(A)
        self.B = None if B is None else _f64(B)
        self.c = EnvCfg(kind, num_agents, num_landmarks, obs_dim, act_dim, episode_len,
                        float(dt), float(damping), float(force), float(radius), _p(self.A), _p(self.B),
                        float(noise_std), float(act_cost), num_chasers, 0, float(accel_c), float(accel_r),
                        float(vmax_c), float(vmax_r), float(radius_c), float(radius_r), float(contact_force),
                        float(contact_margin))
        self.num_chasers = num_chasers
        self.kind, self.N, self.L, self.D, self.K = kind, num_agents, num_landmarks, obs_dim, act_dim
        self.episode_len = episode_len
        self.S = int(lib().ref_env_state_size(C.byref(self.c)))


class Policy:
    def __init__(self, in_dim, hidden, out_dim, bf16=False, dist=CATEGORICAL, hidden_layers=2, value_in_dim=0):
        self.c = PolicyCfg(in_dim, hidden, out_dim, int(bf16), dist, hidden_layers, value_in_dim)
        self.in_dim, self.hidden, self.out_dim, self.bf16, self.dist = in_dim, hidden, out_dim, bool(bf16), dist
        self.hidden_layers = hidden_layers
        self.value_in_dim = value_in_dim or in_dim     # wider than in_dim: centralised critic on the joint observation

    @property
    def policy_param_count(self):
        return net_param_count(self.in_dim, self.hidden, self.out_dim, self.hidden_layers)

    @property
    def param_count(self):
        return self.policy_param_count + net_param_count(self.value_in_dim, self.hidden, 1, self.hidden_layers)


def net_param_count(i, h, o, layers=2):
    return int(lib().ref_net_param_count_l(C.c_int(i), C.c_int(h), C.c_int(o), C.c_int(layers)))


# ------------------------------------------------------------------ random numbers
def philox(ctr, key):
    c = (C.c_uint32 * 4)(*[int(x) & 0xFFFFFFFF for x in ctr])
    k = (C.c_uint32 * 2)(*[int(x) & 0xFFFFFFFF for x in key])
    o = (C.c_uint32 * 4)()
    lib().ref_philox4x32_10(c, k, o)
    return [int(x) for x in o]


def draw(seed, env, entity, time, stream, block):
    o = (C.c_uint32 * 4)()
    lib().ref_draw(C.c_uint64(seed), C.c_uint32(env), C.c_uint32(entity), C.c_uint32(time),
                   C.c_uint32(stream), C.c_uint32(block), o)
    return [int(x) for x in o]


def uniform(w):
    return float(lib().ref_uniform(C.c_uint32(w)))


def normal_pair(w0, w1):
    o = (C.c_double * 2)()
    lib().ref_normal_pair(C.c_uint32(w0), C.c_uint32(w1), o)
    return float(o[0]), float(o[1])


def normals(seed, env, entity, time, stream, n):
    out = np.zeros(n, dtype=np.float64)
    lib().ref_normals(C.c_uint64(seed), C.c_uint32(env), C.c_uint32(entity), C.c_uint32(time),
                      C.c_uint32(stream), C.c_int(n), _p(out))
    return out


def bf16_round(x):
    return float(lib().ref_bf16_round(C.c_double(x)))


# ------------------------------------------------------------------ networks / sampling
def mlp(i, h, o, params, x, bf16=False, layers=2):
    params, x = _f64(params), _f64(x)
    assert params.size == net_param_count(i, h, o, layers) and x.size == i
    y = np.zeros(o, dtype=np.float64)
    lib().ref_mlp_l(C.c_int(i), C.c_int(h), C.c_int(o), C.c_int(layers), _p(params), _p(x), _p(y),
                    C.c_int(int(bf16)))
    return y


def policy_value(pol: Policy, params, x):
    params, x = _f64(params), _f64(x)
    assert params.size == pol.param_count and x.size == pol.in_dim
    lg = np.zeros(pol.out_dim, dtype=np.float64)
    v = C.c_double()
    lib().ref_policy_value(C.byref(pol.c), _p(params), _p(x), _p(lg), C.byref(v))
    return lg, float(v.value)


def central_value(pol: Policy, params, joint):
    """Value of an env from the joint observation of its agents (centralised critic)."""
    params, joint = _f64(params), _f64(joint).ravel()
    assert params.size == pol.param_count and joint.size == pol.value_in_dim
    v = C.c_double()
    lib().ref_central_value(C.byref(pol.c), _p(params), _p(joint), C.byref(v))
    return float(v.value)


def categorical(logits, u):
    logits = _f64(logits)
    a, lp, mg = C.c_int32(), C.c_double(), C.c_double()
    lib().ref_categorical(_p(logits), C.c_int(logits.size), C.c_double(u), C.byref(a), C.byref(lp), C.byref(mg))
    return int(a.value), float(lp.value), float(mg.value)


def gaussian(mean, logstd, eps):
    mean, logstd, eps = _f64(mean), _f64(logstd), _f64(eps)
    a = np.zeros(mean.size, dtype=np.float64)
    lp = C.c_double()
    lib().ref_gaussian(_p(mean), _p(logstd), _p(eps), C.c_int(mean.size), _p(a), C.byref(lp))
    return a, float(lp.value)


def sample(pol: Policy, seed, env, agent, g, logits):
    """-> (action (int or float64 array), logp, margin)."""
    logits = _f64(logits)
    ai, lp, mg = C.c_int32(), C.c_double(), C.c_double()
    af = np.zeros(64, dtype=np.float64)
    lib().ref_sample(C.byref(pol.c), C.c_uint64(seed), C.c_uint32(env), C.c_uint32(agent),
                     C.c_uint32(int(g) & 0xFFFFFFFF), _p(logits), C.byref(ai), _p(af), C.byref(lp), C.byref(mg))
    if pol.dist == CATEGORICAL:
        return int(ai.value), float(lp.value), float(mg.value)
    return af[: pol.out_dim // 2].copy(), float(lp.value), float(mg.value)


# ------------------------------------------------------------------ environments
def env_obs(env: Env, s):
    s = _f64(s)
    assert s.size == env.S
    o = np.zeros((env.N, env.D), dtype=np.float64)
    lib().ref_env_obs(C.byref(env.c), _p(s), _p(o))
    return o


def env_reset(env: Env, seed, env_id, episode):
    s = np.zeros(env.S, dtype=np.float64)
    lib().ref_env_reset(C.byref(env.c), C.c_uint64(seed), C.c_uint32(env_id), C.c_uint32(episode), _p(s))
    return s


def particle_move(env: Env, s, actions):
    """-> (new state, reward, collision margin); no done/reset handling."""
    s = _f64(s).copy()
    a = np.ascontiguousarray(actions, dtype=np.int32)
    assert s.size == env.S and a.size == env.N
    r, mg = C.c_double(), C.c_double()
    lib().ref_particle_move(C.byref(env.c), _p(s), _p(a), C.byref(r), C.byref(mg))
    return s, float(r.value), float(mg.value)


def lingauss_move(env: Env, s, a, eps):
    s, a, eps = _f64(s).copy(), _f64(a), _f64(eps)
    assert s.size == env.D and a.size == env.K and eps.size == env.D
    r = C.c_double()
    lib().ref_lingauss_move(C.byref(env.c), _p(s), _p(a), _p(eps), C.byref(r))
    return s, float(r.value)


def tag_move(env: Env, s, actions):
    """-> (new state, rewards [N], contact margin); no done/reset handling."""
    s = _f64(s).copy()
    a = np.ascontiguousarray(actions, dtype=np.int32)
    assert s.size == env.S and a.size == env.N
    r, mg = np.zeros(env.N), C.c_double()
    lib().ref_tag_move(C.byref(env.c), _p(s), _p(a), _p(r), C.byref(mg))
    return s, r, float(mg.value)


def env_step(env: Env, seed, env_id, g, s, actions):
    """One env_step incl. done and reset -> (new state, reward (per agent for the pursuit env), done, margin)."""
    s = _f64(s).copy()
    assert s.size == env.S
    r, d, mg = C.c_double(), C.c_uint8(), C.c_double()
    if env.kind == TAG:
        a = np.ascontiguousarray(actions, dtype=np.int32)
        assert a.size == env.N
        rr = np.zeros(env.N)
        lib().ref_env_step_tag(C.byref(env.c), C.c_uint64(seed), C.c_uint32(env_id), C.c_int64(int(g)),
                               _p(s), _p(a), _p(rr), C.byref(d), C.byref(mg))
        return s, rr, int(d.value), float(mg.value)
    if env.kind == PARTICLE:
        a = np.ascontiguousarray(actions, dtype=np.int32)
        assert a.size == env.N
        lib().ref_env_step(C.byref(env.c), C.c_uint64(seed), C.c_uint32(env_id), C.c_int64(int(g)),
                           _p(s), _p(a), None, C.byref(r), C.byref(d), C.byref(mg))
    else:
        a = _f64(actions)
        assert a.size == env.K
        lib().ref_env_step(C.byref(env.c), C.c_uint64(seed), C.c_uint32(env_id), C.c_int64(int(g)),
                           _p(s), None, _p(a), C.byref(r), C.byref(d), C.byref(mg))
    return s, float(r.value), int(d.value), float(mg.value)


def init(env: Env, seed, env0, E):
    state = np.zeros((E, env.S), dtype=np.float64)
    g = np.zeros(E, dtype=np.int64)
    lib().ref_init(C.byref(env.c), C.c_uint64(seed), C.c_int(env0), C.c_int(E), _p(state), _p(g))
    return state, g


def rollout(env: Env, pol: Policy, seed, env0, state, g, params, T, want_logits=True):
    """Advances state and g in place; returns a dict of trajectory arrays."""
    assert state.dtype == np.float64 and state.flags.c_contiguous and g.dtype == np.int64
    E = state.shape[0]
    assert state.shape == (E, env.S) and g.shape == (E,)
    params = _f64(params)
    assert params.size == pol.param_count * (2 if env.kind == TAG else 1)   # one parameter set per role
    M = E * env.N
    out = {
        "obs": np.zeros((T + 1, M, env.D)),
        "logp": np.zeros((T, M)),
        "rewards": np.zeros((T, M)),
        "dones": np.zeros((T, M), dtype=np.uint8),
        "values": np.zeros((T + 1, M)),
        "logits": np.zeros((T, M, pol.out_dim)) if want_logits else None,
    }
    if pol.dist == CATEGORICAL:
        out["actions"] = np.zeros((T, M), dtype=np.int32)
        ai, af = out["actions"], None
    else:
        out["actions"] = np.zeros((T, M, env.K))
        ai, af = None, out["actions"]
    lib().ref_rollout(C.byref(env.c), C.byref(pol.c), C.c_uint64(seed), C.c_int(env0), C.c_int(E),
                      _p(state), _p(g), _p(params), C.c_int(T), _p(out["obs"]), _p(ai), _p(af),
                      _p(out["logp"]), _p(out["rewards"]), _p(out["dones"]), _p(out["values"]),
                      _p(out["logits"]))
    return out


def gae(rewards, values, dones, gamma, lam):
    r, V = _f64(rewards), _f64(values)
    d = np.ascontiguousarray(dones, dtype=np.uint8)
    T, M = r.shape if r.ndim == 2 else (r.shape[0], 1)
    assert V.size == (T + 1) * M and d.size == T * M
    adv = np.zeros((T, M))
    ret = np.zeros((T, M))
    lib().ref_gae(_p(r), _p(V), _p(d), C.c_int(T), C.c_int64(M), C.c_double(gamma), C.c_double(lam),
                  _p(adv), _p(ret))
    return adv.reshape(r.shape), ret.reshape(r.shape)


# ------------------------------------------------------------------ batch helpers (statistical pins)
def categorical_counts(pol: Policy, seed, g, logits, n):
    logits = _f64(logits)
    counts = np.zeros(pol.out_dim, dtype=np.int64)
    lib().ref_categorical_counts(C.byref(pol.c), C.c_uint64(seed), C.c_uint32(g), _p(logits),
                                 C.c_int64(n), _p(counts))
    return counts


def normals_many(seed, stream, n):
    out = np.zeros(n, dtype=np.float64)
    lib().ref_normals_many(C.c_uint64(seed), C.c_uint32(stream), C.c_int64(n), _p(out))
    return out


def words_many(seed, stream, n):
    out = np.zeros(n, dtype=np.uint32)
    lib().ref_words_many(C.c_uint64(seed), C.c_uint32(stream), C.c_int64(n), _p(out))
    return out


# ------------------------------------------------------------------ learner (policy update)
class PpoCfg(C.Structure):
    _fields_ = [("clip", C.c_double), ("vf_coef", C.c_double), ("ent_coef", C.c_double),
                ("lr", C.c_double), ("beta1", C.c_double), ("beta2", C.c_double), ("adam_eps", C.c_double)]


def ppo_cfg(clip=0.2, vf_coef=0.5, ent_coef=0.01, lr=3e-4, beta1=0.9, beta2=0.999, adam_eps=1e-8):
    return PpoCfg(clip, vf_coef, ent_coef, lr, beta1, beta2, adam_eps)


def _actions(pol: "Policy", actions):
    if pol.dist == CATEGORICAL:
        ai = np.ascontiguousarray(actions, dtype=np.int32)
        return ai, None, ai.ctypes.data_as(C.c_void_p), None
    af = _f64(actions)
    return None, af, None, _p(af)


def ppo_loss(pol: "Policy", cfg: PpoCfg, params, obs, actions, logp_old, adv, ret, want_grad=True):
    """-> (loss, grad or None, stats[5]) of the clipped-surrogate objective over the given rows."""
    params, obs, logp_old, adv, ret = map(_f64, (params, obs, logp_old, adv, ret))
    R = logp_old.size
    assert obs.size == R * pol.in_dim and params.size == pol.param_count
    ai, af, pi, pf = _actions(pol, actions)
    grad = np.zeros(params.size) if want_grad else None
    stats = np.zeros(5)
    f = lib().ref_ppo_loss
    f.restype = C.c_double
    loss = f(C.byref(pol.c), C.byref(cfg), _p(params), C.c_int64(R), _p(obs), pi, pf, _p(logp_old), _p(adv),
             _p(ret), _p(grad) if want_grad else None, _p(stats))
    return float(loss), grad, stats


def adam_step(cfg: PpoCfg, params, m, v, grad, k):
    """In place on params, m, v (float64 arrays); k = 1-based step counter."""
    lib().ref_adam_step(C.byref(cfg), _p(params), _p(m), _p(v), _p(_f64(grad)), C.c_size_t(params.size),
                        C.c_int64(k))


def ppo_update(pol: "Policy", cfg: PpoCfg, params, m, v, step, iters, minibatches, obs, actions, logp_old, adv, ret):
    """-> (mean minibatch loss, new step counter); params, m, v are updated in place."""
    obs, logp_old, adv, ret = map(_f64, (obs, logp_old, adv, ret))
    ai, af, pi, pf = _actions(pol, actions)
    k = C.c_int64(step)
    f = lib().ref_ppo_update
    f.restype = C.c_double
    loss = f(C.byref(pol.c), C.byref(cfg), _p(params), _p(m), _p(v), C.byref(k), C.c_int64(logp_old.size),
             C.c_int(iters), C.c_int(minibatches), _p(obs), pi, pf, _p(logp_old), _p(adv), _p(ret))
    return float(loss), int(k.value)
