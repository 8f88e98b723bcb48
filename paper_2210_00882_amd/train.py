"""The training loop of Listing 1 (Trainer.train) on one GPU, the paper's "GPU only" distribution
policy: every iteration collects `T` steps from all environments (msrl_rollout_gae) and runs the
learner's update on them (msrl_ppo_update).  Calls of the C ABI only: torch holds the buffers.
"""
from __future__ import annotations

import numpy as np

from . import binding as B, synth


def ppo_train(cfg: synth.Config, params_f32: np.ndarray, iterations: int, seed: int, *, lr=1e-3, iters=4,
              minibatches=4, clip=0.2, vf_coef=0.5, ent_coef=0.01, gamma=None, lam=None, dyn=None):
    """-> (final float32 master parameters as numpy, list of the mean reward per step of every iteration;
    for the pursuit env, which has a parameter set per role, a (chasers, runners) pair per iteration)."""
    import torch
    T, M, N = cfg.T, cfg.M, cfg.num_agents
    gamma = cfg.gamma if gamma is None else gamma
    lam = cfg.lam if lam is None else lam
    A, Bm = dyn if dyn is not None else (None, None)
    env_cfg, keep = B.make_env_cfg(cfg, A, Bm)
    pol_cfg = B.make_policy_cfg(cfg)
    state = B.msrl_rollout_init(env_cfg, pol_cfg, seed)
    # one learner per role, each fed the rows of its agents (every row when there is one role)
    roles = cfg.roles
    one_role = B.make_policy_cfg(cfg)
    one_role.roles = 1
    n_role = B.msrl_param_count(one_role)
    agent = torch.arange(T * M, device="cuda") % N
    if roles == 1:
        row_sets = [None]
    else:
        row_sets = [torch.nonzero(agent < cfg.num_chasers).flatten(), torch.nonzero(agent >= cfg.num_chasers).flatten()]
    counts = [T * M if r is None else int(r.numel()) for r in row_sets]
    # (the last block takes the remainder; with a centralised critic the blocks hold whole groups of N rows)
    learners = [B.msrl_learner_init(one_role, -(-c // minibatches) + minibatches * N) for c in counts]
    try:
        master = torch.from_numpy(np.ascontiguousarray(params_f32, dtype=np.float32)).cuda()
        assert master.numel() == roles * n_role
        m, v = torch.zeros_like(master), torch.zeros_like(master)
        acting = master if cfg.dtype == synth.F32 else torch.empty(master.numel(), dtype=torch.bfloat16, device="cuda")
        out = B.alloc_traj(cfg, T, logits=False, gae=True)
        pc = B.make_ppo_cfg(clip=clip, vf_coef=vf_coef, ent_coef=ent_coef, lr=lr)
        rows = lambda t: t.reshape(-1, *t.shape[2:])
        steps, history = [0] * roles, []
        for _ in range(iterations):
            if acting is not master:
                B.msrl_params_cast(master, acting, B.MSRL_BF16)
            B.msrl_rollout_gae(state, acting, T, gamma, lam, out)
            batch = [rows(out["obs"][:T]), rows(out["actions"]), rows(out["logp"]), rows(out["adv"]), rows(out["ret"])]
            for r in range(roles):
                sel = batch if row_sets[r] is None else [t.index_select(0, row_sets[r]) for t in batch]
                sl = slice(r * n_role, (r + 1) * n_role)
                steps[r] = B.msrl_ppo_update(learners[r], master[sl], m[sl], v[sl], steps[r], iters, minibatches,
                                             *sel, pc)
            rew = out["rewards"]
            if roles == 1:
                history.append(float(rew.mean()))   # syncs
            else:
                per_agent = rew.reshape(T, cfg.num_envs, N).mean(dim=(0, 1)).cpu().numpy()
                history.append((float(per_agent[:cfg.num_chasers].mean()), float(per_agent[cfg.num_chasers:].mean())))
        return master.cpu().numpy(), history
    finally:
        for L in learners:
            B.msrl_learner_destroy(L)
        B.msrl_rollout_destroy(state)
