"""The training loop of Listing 1 (Trainer.train) on one GPU, the paper's "GPU only" distribution
policy: every iteration collects `T` steps from all environments (msrl_rollout_gae) and runs the
learner's update on them (msrl_ppo_update).  Calls of the C ABI only: torch holds the buffers.
"""
from __future__ import annotations

import numpy as np

from . import binding as B, synth


def ppo_train(cfg: synth.Config, params_f32: np.ndarray, iterations: int, seed: int, *, lr=1e-3, iters=4,
              minibatches=4, clip=0.2, vf_coef=0.5, ent_coef=0.01, gamma=None, lam=None, dyn=None):
    """-> (final float32 master parameters as numpy, list of the mean reward per step of every iteration)."""
    import torch
    T, M = cfg.T, cfg.M
    gamma = cfg.gamma if gamma is None else gamma
    lam = cfg.lam if lam is None else lam
    A, Bm = dyn if dyn is not None else (None, None)
    env_cfg, keep = B.make_env_cfg(cfg, A, Bm)
    pol_cfg = B.make_policy_cfg(cfg)
    state = B.msrl_rollout_init(env_cfg, pol_cfg, seed)
    learner = B.msrl_learner_init(pol_cfg, -(-T * M // minibatches) + minibatches)
    try:
        master = torch.from_numpy(np.ascontiguousarray(params_f32, dtype=np.float32)).cuda()
        m, v = torch.zeros_like(master), torch.zeros_like(master)
        acting = master if cfg.dtype == synth.F32 else torch.empty(master.numel(), dtype=torch.bfloat16, device="cuda")
        out = B.alloc_traj(cfg, T, logits=False, gae=True)
        pc = B.make_ppo_cfg(clip=clip, vf_coef=vf_coef, ent_coef=ent_coef, lr=lr)
        rows = lambda t: t.reshape(-1, *t.shape[2:])
        step, history = 0, []
        for _ in range(iterations):
            if acting is not master:
                B.msrl_params_cast(master, acting, B.MSRL_BF16)
            B.msrl_rollout_gae(state, acting, T, gamma, lam, out)
            step = B.msrl_ppo_update(learner, master, m, v, step, iters, minibatches, rows(out["obs"][:T]),
                                     rows(out["actions"]), rows(out["logp"]), rows(out["adv"]), rows(out["ret"]), pc)
            history.append(float(out["rewards"].mean()))   # syncs
        return master.cpu().numpy(), history
    finally:
        B.msrl_learner_destroy(learner)
        B.msrl_rollout_destroy(state)
