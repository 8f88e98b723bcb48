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
    # (Listing 1: one learner per role; a role's rows are named by a row selection, nothing is copied)
    if roles == 1:
        row_sets = [None]
    else:
        row_sets = [B.msrl_row_select(N, 0, cfg.num_chasers), B.msrl_row_select(N, cfg.num_chasers, N - cfg.num_chasers)]
    counts = [T * M if r is None else T * cfg.num_envs * r.count for r in row_sets]
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
        steps = [0] * roles
        mean_rew = torch.empty((iterations, roles), dtype=torch.float32, device="cuda")   # written by msrl_rows_mean
        for it in range(iterations):
            if acting is not master:
                B.msrl_params_cast(master, acting, B.MSRL_BF16)
            B.msrl_rollout_gae(state, acting, T, gamma, lam, out)
            batch = [rows(out["obs"][:T]), rows(out["actions"]), rows(out["logp"]), rows(out["adv"]), rows(out["ret"])]
            for r in range(roles):
                sl = slice(r * n_role, (r + 1) * n_role)
                steps[r] = B.msrl_ppo_update(learners[r], master[sl], m[sl], v[sl], steps[r], iters, minibatches,
                                             *batch, pc, rows=row_sets[r])
            for r in range(roles):
                B.msrl_rows_mean(out["rewards"], mean_rew[it, r:r + 1], rows=row_sets[r])
        hist = mean_rew.cpu().numpy()            # read back once, after the loop
        history = [float(h[0]) for h in hist] if roles == 1 else [(float(h[0]), float(h[1])) for h in hist]
        return master.cpu().numpy(), history
    finally:
        for L in learners:
            B.msrl_learner_destroy(L)
        B.msrl_rollout_destroy(state)
