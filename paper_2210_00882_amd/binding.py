"""Thin ctypes binding of libmsrl.so: the functions of include/msrl.h under the
same names.  Argument marshalling only -- every step of the path runs in the HIP
kernels.  torch is used for device memory and streams; tensors are passed as raw
device pointers.  There is no CPU fallback: a missing library raises.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmsrl.so")

MSRL_OK, MSRL_EINVAL, MSRL_ENOMEM, MSRL_EDEVICE, MSRL_EUNSUPPORTED = 0, -1, -2, -3, -4
MSRL_ENV_PARTICLE, MSRL_ENV_LINGAUSS = 0, 1
MSRL_F32, MSRL_BF16 = 0, 1
MSRL_CATEGORICAL, MSRL_DIAG_GAUSSIAN = 0, 1
MSRL_PHASE_ENV, MSRL_PHASE_MLP, MSRL_PHASE_CLOCKS = 1, 2, 3

EXPORTS = (
    "msrl_param_count", "msrl_env_state_size", "msrl_rollout_init", "msrl_rollout_step", "msrl_gae",
    "msrl_rollout_gae", "msrl_rollout_gae_static", "msrl_measure_phase", "msrl_rollout_shape", "msrl_observe", "msrl_act", "msrl_env_step",
    "msrl_learner_init", "msrl_learner_init_path", "msrl_learner_destroy", "msrl_ppo_grad", "msrl_rows_mean", "msrl_adam_step", "msrl_ppo_update", "msrl_params_cast", "msrl_state_get", "msrl_state_set", "msrl_rollout_destroy", "msrl_last_error",
)


class msrl_env_cfg(C.Structure):
    _fields_ = [
        ("kind", C.c_int32), ("num_envs", C.c_int32), ("num_agents", C.c_int32),
        ("num_landmarks", C.c_int32), ("obs_dim", C.c_int32), ("act_dim", C.c_int32),
        ("episode_len", C.c_int32),
        ("dt", C.c_float), ("damping", C.c_float), ("force", C.c_float), ("radius", C.c_float),
        ("A", C.c_void_p), ("B", C.c_void_p),
        ("noise_std", C.c_float), ("act_cost", C.c_float),
        ("num_chasers", C.c_int32), ("accel_c", C.c_float), ("accel_r", C.c_float),
        ("vmax_c", C.c_float), ("vmax_r", C.c_float), ("radius_c", C.c_float), ("radius_r", C.c_float),
        ("contact_force", C.c_float), ("contact_margin", C.c_float),
        ("tag_tiles", C.c_int32),
        ("wave_roles", C.c_int32),
    ]


class msrl_policy_cfg(C.Structure):
    _fields_ = [("in_dim", C.c_int32), ("hidden", C.c_int32), ("out_dim", C.c_int32),
                ("dtype", C.c_int32), ("dist", C.c_int32), ("hidden_layers", C.c_int32), ("roles", C.c_int32),
                ("value_in_dim", C.c_int32)]


class msrl_traj(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in
                ("obs", "actions", "logp", "rewards", "dones", "values", "logits", "adv", "ret")]


class msrl_row_select(C.Structure):
    _fields_ = [("group", C.c_int32), ("first", C.c_int32), ("count", C.c_int32)]


class msrl_ppo_cfg(C.Structure):
    _fields_ = [(n, C.c_float) for n in ("clip", "vf_coef", "ent_coef", "lr", "beta1", "beta2", "adam_eps")]


class MsrlError(RuntimeError):
    def __init__(self, code, message):
        super().__init__(f"msrl error {code}: {message}")
        self.code = code


_lib = None


def load():
    """Loads libmsrl.so (built by `python -m paper_2210_00882_amd.build`)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2210_00882_amd.build`; "
            "there is no fallback path")
    lib = C.CDLL(LIB_PATH)
    vp, i32, i64, f32, u64 = C.c_void_p, C.c_int32, C.c_int64, C.c_float, C.c_uint64
    lib.msrl_param_count.restype = C.c_size_t
    lib.msrl_param_count.argtypes = [C.POINTER(msrl_policy_cfg)]
    lib.msrl_env_state_size.restype = C.c_size_t
    lib.msrl_env_state_size.argtypes = [C.POINTER(msrl_env_cfg)]
    lib.msrl_rollout_init.restype = C.c_int
    lib.msrl_rollout_init.argtypes = [C.POINTER(msrl_env_cfg), C.POINTER(msrl_policy_cfg), u64, C.POINTER(vp)]
    lib.msrl_rollout_step.restype = C.c_int
    lib.msrl_rollout_step.argtypes = [vp, vp, i32, C.POINTER(msrl_traj), vp]
    lib.msrl_gae.restype = C.c_int
    lib.msrl_gae.argtypes = [vp, vp, vp, i32, i64, f32, f32, vp, vp, vp]
    lib.msrl_rollout_gae.restype = C.c_int
    lib.msrl_rollout_gae.argtypes = [vp, vp, i32, f32, f32, C.POINTER(msrl_traj), vp]
    lib.msrl_rollout_gae_static.restype = C.c_int
    lib.msrl_rollout_gae_static.argtypes = [C.POINTER(msrl_env_cfg), C.POINTER(msrl_policy_cfg), u64, vp, vp, vp, i32,
                                            f32, f32, C.POINTER(msrl_traj), vp]
    lib.msrl_measure_phase.restype = C.c_int
    lib.msrl_rollout_shape.restype = C.c_int
    lib.msrl_rollout_shape.argtypes = [vp, C.POINTER(i32), C.POINTER(i32), C.POINTER(i32)]
    lib.msrl_measure_phase.argtypes = [vp, vp, i32, C.POINTER(msrl_traj), i32, vp]
    lib.msrl_observe.restype = C.c_int
    lib.msrl_observe.argtypes = [vp, vp, vp]
    lib.msrl_act.restype = C.c_int
    lib.msrl_act.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp]
    lib.msrl_env_step.restype = C.c_int
    lib.msrl_env_step.argtypes = [vp, vp, vp, vp, vp, vp]
    lib.msrl_learner_init.restype = C.c_int
    lib.msrl_learner_init.argtypes = [C.POINTER(msrl_policy_cfg), i64, C.POINTER(vp)]
    lib.msrl_learner_init_path.restype = C.c_int
    lib.msrl_learner_init_path.argtypes = [C.POINTER(msrl_policy_cfg), i64, i32, C.POINTER(vp)]
    lib.msrl_learner_destroy.restype = None
    lib.msrl_learner_destroy.argtypes = [vp]
    lib.msrl_ppo_grad.restype = C.c_int
    lib.msrl_ppo_grad.argtypes = [vp, vp, i64, vp, vp, vp, vp, vp, C.POINTER(msrl_row_select),
                                  C.POINTER(msrl_ppo_cfg), vp, vp, vp]
    lib.msrl_rows_mean.restype = C.c_int
    lib.msrl_rows_mean.argtypes = [vp, i64, C.POINTER(msrl_row_select), vp, vp]
    lib.msrl_adam_step.restype = C.c_int
    lib.msrl_adam_step.argtypes = [vp, vp, vp, vp, i64, i64, C.POINTER(msrl_ppo_cfg), vp]
    lib.msrl_params_cast.restype = C.c_int
    lib.msrl_params_cast.argtypes = [vp, vp, i64, i32, vp]
    lib.msrl_ppo_update.restype = C.c_int
    lib.msrl_ppo_update.argtypes = [vp, vp, vp, vp, C.POINTER(i64), i64, i32, i32, vp, vp, vp, vp, vp,
                                    C.POINTER(msrl_row_select), C.POINTER(msrl_ppo_cfg), vp]
    lib.msrl_state_get.restype = C.c_int
    lib.msrl_state_get.argtypes = [vp, vp, vp]
    lib.msrl_state_set.restype = C.c_int
    lib.msrl_state_set.argtypes = [vp, vp, vp]
    lib.msrl_rollout_destroy.restype = None
    lib.msrl_rollout_destroy.argtypes = [vp]
    lib.msrl_last_error.restype = C.c_char_p
    lib.msrl_last_error.argtypes = []
    _lib = lib
    return lib


def msrl_last_error() -> str:
    return load().msrl_last_error().decode()


def _check(rc):
    if rc != MSRL_OK:
        raise MsrlError(rc, msrl_last_error())


def _ptr(t):
    """Device pointer of a torch tensor (or None)."""
    if t is None:
        return None
    assert t.is_cuda and t.is_contiguous(), "device tensors must be contiguous CUDA/HIP tensors"
    return C.c_void_p(t.data_ptr())


def _stream(stream):
    import torch
    s = torch.cuda.current_stream() if stream is None else stream
    return C.c_void_p(s.cuda_stream)


def make_env_cfg(cfg, A=None, B=None, tag_tiles=0, wave_roles=0):
    """msrl_env_cfg from a synth.Config; A, B float32 host arrays for lingauss.
    Returns (struct, keepalive)."""
    keep = []
    pa = pb = None
    if A is not None:
        A = np.ascontiguousarray(A, dtype=np.float32)
        B = np.ascontiguousarray(B, dtype=np.float32)
        keep = [A, B]
        pa, pb = A.ctypes.data, B.ctypes.data
    e = msrl_env_cfg(cfg.kind, cfg.num_envs, cfg.num_agents, cfg.num_landmarks, cfg.obs_dim, cfg.act_dim,
                     cfg.episode_len, cfg.dt, cfg.damping, cfg.force, cfg.radius, pa, pb,
                     cfg.noise_std, cfg.act_cost, cfg.num_chasers, cfg.accel_c, cfg.accel_r, cfg.vmax_c, cfg.vmax_r,
                     cfg.radius_c, cfg.radius_r, cfg.contact_force, cfg.contact_margin, tag_tiles, wave_roles)
    return e, keep


def make_policy_cfg(cfg):
    return msrl_policy_cfg(cfg.obs_dim, cfg.hidden, cfg.out_dim, cfg.dtype, cfg.dist, cfg.hidden_layers, cfg.roles,
                           cfg.value_in_dim if cfg.central_critic else 0)


def msrl_param_count(policy_cfg: msrl_policy_cfg) -> int:
    return int(load().msrl_param_count(C.byref(policy_cfg)))


def msrl_env_state_size(env_cfg: msrl_env_cfg) -> int:
    return int(load().msrl_env_state_size(C.byref(env_cfg)))


def msrl_rollout_init(env_cfg: msrl_env_cfg, policy_cfg: msrl_policy_cfg, seed: int) -> C.c_void_p:
    st = C.c_void_p()
    _check(load().msrl_rollout_init(C.byref(env_cfg), C.byref(policy_cfg), C.c_uint64(seed), C.byref(st)))
    return st


def msrl_rollout_destroy(state) -> None:
    load().msrl_rollout_destroy(state)


def _traj(out: dict) -> msrl_traj:
    t = msrl_traj()
    for name, _ in msrl_traj._fields_:
        v = out.get(name)
        setattr(t, name, None if v is None else v.data_ptr())
    return t


def msrl_rollout_step(state, params, T: int, out: dict, stream=None) -> None:
    """out: dict of preallocated device tensors (see alloc_traj)."""
    tr = _traj(out)
    _check(load().msrl_rollout_step(state, _ptr(params), C.c_int32(T), C.byref(tr), _stream(stream)))


def msrl_gae(rewards, values, dones, gamma: float, lam: float, adv, ret, stream=None) -> None:
    T = rewards.shape[0]
    M = rewards.numel() // T if T else 0
    _check(load().msrl_gae(_ptr(rewards), _ptr(values), _ptr(dones), C.c_int32(T), C.c_int64(M),
                           C.c_float(gamma), C.c_float(lam), _ptr(adv), _ptr(ret), _stream(stream)))


def msrl_rollout_gae(state, params, T: int, gamma: float, lam: float, out: dict, stream=None) -> None:
    tr = _traj(out)
    _check(load().msrl_rollout_gae(state, _ptr(params), C.c_int32(T), C.c_float(gamma), C.c_float(lam),
                                   C.byref(tr), _stream(stream)))


MSRL_STATIC_SCRATCH_BYTES = 1 << 20


def msrl_rollout_gae_static(env_cfg: msrl_env_cfg, policy_cfg: msrl_policy_cfg, seed: int, env_state, step_counters,
                            params, T: int, gamma: float, lam: float, out: dict, stream=None) -> None:
    """env_state float32 [E, S] and step_counters int64 [E]: device tensors, advanced in place."""
    tr = _traj(out)
    _check(load().msrl_rollout_gae_static(C.byref(env_cfg), C.byref(policy_cfg), C.c_uint64(seed), _ptr(env_state),
                                          _ptr(step_counters), _ptr(params), C.c_int32(T), C.c_float(gamma),
                                          C.c_float(lam), C.byref(tr), _stream(stream)))


def msrl_measure_phase(state, params, T: int, out: dict, phase: int, stream=None) -> None:
    tr = _traj(out)
    _check(load().msrl_measure_phase(state, _ptr(params), C.c_int32(T), C.byref(tr), C.c_int32(phase),
                                     _stream(stream)))


def msrl_rollout_shape(state) -> tuple:
    """-> (workgroups, waves per workgroup, waves that own a row block)"""
    wg, w, rw = C.c_int32(), C.c_int32(), C.c_int32()
    _check(load().msrl_rollout_shape(state, C.byref(wg), C.byref(w), C.byref(rw)))
    return wg.value, w.value, rw.value


def msrl_observe(state, obs, stream=None) -> None:
    _check(load().msrl_observe(state, _ptr(obs), _stream(stream)))


def msrl_act(state, params, obs, actions, logp, values, logits=None, stream=None) -> None:
    _check(load().msrl_act(state, _ptr(params), _ptr(obs), _ptr(actions), _ptr(logp), _ptr(values),
                           _ptr(logits), _stream(stream)))


def msrl_env_step(state, actions, rewards, dones, next_obs, stream=None) -> None:
    _check(load().msrl_env_step(state, _ptr(actions), _ptr(rewards), _ptr(dones), _ptr(next_obs),
                                _stream(stream)))


def make_ppo_cfg(clip=0.2, vf_coef=0.5, ent_coef=0.01, lr=3e-4, beta1=0.9, beta2=0.999, adam_eps=1e-8):
    return msrl_ppo_cfg(clip, vf_coef, ent_coef, lr, beta1, beta2, adam_eps)


MSRL_LEARNER_PATH_AUTO, MSRL_LEARNER_PATH_DEVICE_MEMORY = 0, 1


def msrl_learner_init(policy_cfg: msrl_policy_cfg, max_rows: int) -> C.c_void_p:
    L = C.c_void_p()
    _check(load().msrl_learner_init(C.byref(policy_cfg), C.c_int64(max_rows), C.byref(L)))
    return L


def msrl_learner_init_path(policy_cfg: msrl_policy_cfg, max_rows: int, path: int) -> C.c_void_p:
    L = C.c_void_p()
    _check(load().msrl_learner_init_path(C.byref(policy_cfg), C.c_int64(max_rows), C.c_int32(path), C.byref(L)))
    return L


def msrl_learner_destroy(learner) -> None:
    load().msrl_learner_destroy(learner)


def _selected(n_rows: int, rows):
    """(number of selected rows, pointer argument) for a row selection over arrays of n_rows rows."""
    if rows is None:
        return n_rows, None
    if rows.group < 1:      # (the library rejects it)
        return n_rows, C.byref(rows)
    return n_rows // rows.group * rows.count, C.byref(rows)


def msrl_ppo_grad(learner, params, obs, actions, logp_old, adv, ret, cfg: msrl_ppo_cfg, grad, stats=None,
                  stream=None, rows: msrl_row_select | None = None) -> None:
    """All tensors on the device; params / grad float32 [param_count].  rows: optional msrl_row_select over the
    rows of the given arrays (one role's rows of a stored trajectory); default every row."""
    R, sel = _selected(logp_old.numel(), rows)
    _check(load().msrl_ppo_grad(learner, _ptr(params), C.c_int64(R), _ptr(obs), _ptr(actions),
                                _ptr(logp_old), _ptr(adv), _ptr(ret), sel, C.byref(cfg), _ptr(grad), _ptr(stats),
                                _stream(stream)))


def msrl_rows_mean(x, out, rows: msrl_row_select | None = None, stream=None) -> None:
    """out[0] (device float32) <- mean of x (one float per row) over the selected rows."""
    R, sel = _selected(x.numel(), rows)
    _check(load().msrl_rows_mean(_ptr(x), C.c_int64(R), sel, _ptr(out), _stream(stream)))


def msrl_adam_step(params, m, v, grad, k: int, cfg: msrl_ppo_cfg, stream=None) -> None:
    _check(load().msrl_adam_step(_ptr(params), _ptr(m), _ptr(v), _ptr(grad), C.c_int64(params.numel()),
                                 C.c_int64(k), C.byref(cfg), _stream(stream)))


def msrl_params_cast(master, out, dtype: int, stream=None) -> None:
    _check(load().msrl_params_cast(_ptr(master), _ptr(out), C.c_int64(master.numel()), C.c_int32(dtype),
                                   _stream(stream)))


def msrl_ppo_update(learner, params, m, v, step: int, iters: int, minibatches: int, obs, actions, logp_old, adv,
                    ret, cfg: msrl_ppo_cfg, stream=None, rows: msrl_row_select | None = None) -> int:
    """-> the new step counter; params, m, v (float32, device) are updated in place."""
    k = C.c_int64(step)
    R, sel = _selected(logp_old.numel(), rows)
    _check(load().msrl_ppo_update(learner, _ptr(params), _ptr(m), _ptr(v), C.byref(k),
                                  C.c_int64(R), C.c_int32(iters), C.c_int32(minibatches),
                                  _ptr(obs), _ptr(actions), _ptr(logp_old), _ptr(adv), _ptr(ret), sel, C.byref(cfg),
                                  _stream(stream)))
    return int(k.value)


def msrl_state_get(state, num_envs: int, state_size: int):
    es = np.zeros((num_envs, state_size), dtype=np.float32)
    g = np.zeros(num_envs, dtype=np.int64)
    _check(load().msrl_state_get(state, es.ctypes.data_as(C.c_void_p), g.ctypes.data_as(C.c_void_p)))
    return es, g


def msrl_state_set(state, env_state=None, step_counters=None) -> None:
    es = None if env_state is None else np.ascontiguousarray(env_state, dtype=np.float32)
    g = None if step_counters is None else np.ascontiguousarray(step_counters, dtype=np.int64)
    _check(load().msrl_state_set(state,
                                 None if es is None else es.ctypes.data_as(C.c_void_p),
                                 None if g is None else g.ctypes.data_as(C.c_void_p)))


# ------------------------------------------------------------------ device-memory helpers (plumbing)
def alloc_traj(cfg, T: int, device="cuda:0", logits: bool = False, gae: bool = True) -> dict:
    """Caller-owned trajectory tensors of the shapes msrl_traj documents."""
    import torch
    M, D = cfg.M, cfg.obs_dim
    out = {
        "obs": torch.empty((T + 1, M, D), dtype=torch.float32, device=device),
        "logp": torch.empty((T, M), dtype=torch.float32, device=device),
        "rewards": torch.empty((T, M), dtype=torch.float32, device=device),
        "dones": torch.empty((T, M), dtype=torch.uint8, device=device),
        "values": torch.empty((T + 1, M), dtype=torch.float32, device=device),
        "logits": torch.empty((T, M, cfg.out_dim), dtype=torch.float32, device=device) if logits else None,
        "adv": torch.empty((T, M), dtype=torch.float32, device=device) if gae else None,
        "ret": torch.empty((T, M), dtype=torch.float32, device=device) if gae else None,
    }
    if cfg.dist == MSRL_CATEGORICAL:
        out["actions"] = torch.empty((T, M), dtype=torch.int32, device=device)
    else:
        out["actions"] = torch.empty((T, M, cfg.act_dim), dtype=torch.float32, device=device)
    return out


def upload_params(cfg, params_f32: np.ndarray, device="cuda:0"):
    """Parameter vector as a device tensor of the policy dtype."""
    import torch
    t = torch.from_numpy(np.ascontiguousarray(params_f32, dtype=np.float32))
    if cfg.dtype == MSRL_BF16:
        t = t.to(torch.bfloat16)
    return t.to(device)
