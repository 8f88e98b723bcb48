/*
 * msrl.h -- C ABI of the fused actor+environment rollout fragment and the
 * GAE advantage/return pass, for one AMD MI355X (gfx950).
 *
 * What the calls compute follows the MAPPO listing of the paper (Listing 1,
 * section 3): Actor.act is "policy network -> action -> env_step -> reward,
 * new_state", Trainer.train runs it `duration` times and stores every step
 * (replay_buffer_insert), Learner.learn evaluates the critic on state and
 * next_state and calls gae().  Section 6 (distribution policy DP-D, "GPU
 * only") places that whole loop in one device fragment and section 5.2 fuses
 * the replicas of a fragment by batching their tensors; here the batch axis is
 * M = num_envs * num_agents rows.
 *
 * Conventions
 *   - Every function returns MSRL_OK (0) or a negative msrl_status and never
 *     throws or aborts.  msrl_last_error() returns a thread-local message for
 *     the last failing call of the calling thread.
 *   - "DEVICE" pointers are HIP device memory of the device that was current
 *     when msrl_rollout_init ran; "HOST" pointers are ordinary host memory.
 *   - The caller owns every tensor it passes in; the library owns msrl_state.
 *   - Work is enqueued on `hip_stream` (a hipStream_t passed as void*, NULL =
 *     the null stream) and the call returns without waiting; the caller
 *     synchronises.  msrl_state_get/set synchronise the device themselves.
 *   - Row index m = env * num_agents + agent.  All trajectory tensors are
 *     time-major and row-major: element (t, m, j) of a [T, M, J] tensor is at
 *     offset (t*M + m)*J + j.
 *   - Two calls that use the same msrl_state must not overlap in time.
 *
 * Random numbers: Philox4x32-10 (Salmon et al., SC'11), key = the 64-bit seed
 * (low word, high word), counter = (env, entity, time, stream<<16 | block):
 *   stream 0  action noise   entity = agent,          time = env step counter g
 *   stream 1  reset draws    entity = agent | N+landmark (particle), 0 (lingauss),
 *                            time = episode index
 *   stream 2  env noise      entity = 0,               time = env step counter g
 * A 32-bit word w gives u = (w >> 8) * 2^-24 in [0,1); normals come in pairs by
 * Box-Muller from (w0, w1): radius sqrt(-2 ln(((w0>>8)+1) * 2^-24)), angle
 * 2*pi*(w1>>8)*2^-24, first normal = r cos, second = r sin; words (0,1) and
 * (2,3) of block b give normals 4b..4b+3.
 */
#ifndef MSRL_H
#define MSRL_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct msrl_state msrl_state; /* opaque, library-owned */

typedef enum {
  MSRL_OK = 0,
  MSRL_EINVAL = -1,       /* bad argument or inconsistent configuration */
  MSRL_ENOMEM = -2,       /* device or host allocation failed */
  MSRL_EDEVICE = -3,      /* a HIP runtime call failed */
  MSRL_EUNSUPPORTED = -4  /* valid configuration with no compiled kernel */
} msrl_status;

typedef enum { MSRL_ENV_PARTICLE = 0, MSRL_ENV_LINGAUSS = 1, MSRL_ENV_TAG = 2 } msrl_env_kind;
typedef enum { MSRL_F32 = 0, MSRL_BF16 = 1 } msrl_dtype;
typedef enum { MSRL_CATEGORICAL = 0, MSRL_DIAG_GAUSSIAN = 1 } msrl_dist;

/*
 * Environment (the `env` entry of the algorithm configuration, section 3).
 *
 * MSRL_ENV_PARTICLE: num_agents point masses and num_landmarks landmarks in the
 *   plane.  Per step, per agent: v <- v*(1-damping) + F(action)*dt, then
 *   p <- p + v*dt with the new v; F = force * {(0,0),(+1,0),(-1,0),(0,+1),(0,-1)}
 *   for actions 0..4.  Reward, shared by the env's agents and evaluated after
 *   the move: -(sum over landmarks of the distance to the nearest agent)
 *   -(number of unordered agent pairs closer than 2*radius).  Observation of
 *   agent i, obs_dim = 4 + 2*num_landmarks + 4*(num_agents-1) floats:
 *   [v, p, landmark_k - p (k ascending), p_j - p (j != i ascending), zeros].
 *   The 2*(num_agents-1) trailing slots are zero by construction; the kernels
 *   store them but leave the matching rows of W1 out of the contraction, so a
 *   non-finite weight in those rows does not reach the outputs.
 *   Reset draws every agent and landmark position uniform in [-1,1)^2, v = 0.
 *   act_dim is ignored.  Kernels are compiled for num_landmarks == num_agents =
 *   1 .. 10 with 64, 128 or 256 hidden units, fp32 and bf16 networks, two to
 *   eight hidden layers (fp32 networks of 256 units: at most 7 agents, the
 *   design keeps the first layer of both networks in LDS); anything else is
 *   MSRL_EUNSUPPORTED.
 * MSRL_ENV_LINGAUSS: num_agents = 1, num_landmarks = 0, state = observation of
 *   obs_dim floats; s' = A s + B a + noise_std * N(0,I); reward
 *   -(s.s + act_cost * a.a) on the state before the step.  Reset: s ~ N(0,I).
 * MSRL_ENV_TAG: pursuit variant of the particle env (a stand-in for the task of
 *   the GPU-only experiment, section 7.3, Fig. 10): the first num_chasers agents chase
 *   the others ("runners"), with one parameter set per role (see
 *   msrl_policy_cfg.roles).  State and reset as MSRL_ENV_PARTICLE.  Observation
 *   of agent i, obs_dim = 4 + 2*num_landmarks + 4*(num_agents-1):
 *   [v, p, landmark_k - p, p_j - p (j != i ascending), v_j (j != i ascending)].
 *   Per step, with the positions before the move: F_i = accel(role) *
 *   direction(action) + sum_{j != i} contact_force * pen(d_ij) * (p_i - p_j) /
 *   d_ij, pen(d) = m * log(1 + exp((r_i + r_j - d) / m)), m = contact_margin;
 *   v <- v*(1-damping) + F*dt, |v| limited to vmax(role), p <- p + v*dt.
 *   Rewards on the new positions ("contact": d < radius_c + radius_r between a
 *   chaser and a runner): every chaser +10 per contact of any chaser; a runner
 *   -10 per chaser in contact with it, -10 * (max(0,|px|-1) + max(0,|py|-1)).
 *   Supported by msrl_rollout_step / msrl_rollout_gae, the step-granular calls
 *   (msrl_observe / msrl_act / msrl_env_step) and the snapshot calls; not by
 *   msrl_measure_phase.
 *   Kernels are compiled for every (num_chasers, runners) with at most 8
 *   agents per env, 0 .. 4 landmarks (never more than agents), networks of 64
 *   hidden units and two hidden layers, bf16 or - except for the largest
 *   shapes - fp32 (the four networks stay in LDS: 160 KiB must hold them);
 *   anything else is MSRL_EUNSUPPORTED.
 *   The kernel has two workgroup shapes with identical results (one or four
 *   tiles of 32 envs; four only with at most 4 agents per env and bf16
 *   networks); tag_tiles = 0
 *   lets msrl_rollout_init pick by num_envs, 1 or 4 fixes the shape (EINVAL
 *   for any other value, for 4 with more than 4 agents, and for a non-zero
 *   value with another env kind).
 *
 * MSRL_ENV_PARTICLE with 64-unit networks (or 128-unit bf16 networks) of two
 *   hidden layers and a per-agent critic has two kernel shapes with identical
 *   results: a wave evaluates the policy and then the value network of its 32
 *   rows, or two waves share the rows, one network each, with every weight
 *   resident on chip (a step is then half as long a chain of instructions and
 *   has no stage barriers).  wave_roles = 0 lets msrl_rollout_init pick (64
 *   units: always two waves, with two or four row blocks per workgroup by
 *   num_envs; 128 units: two waves while the workgroups of that shape run in
 *   one round), 1 or 2 fixes the shape (EINVAL for any other value or another
 *   env kind, EUNSUPPORTED for 2 where it is not compiled).
 *
 * An episode ends (done = 1, then reset) on every step whose counter g
 * satisfies (g+1) % episode_len == 0; g counts the env's steps since init.
 */
typedef struct {
  int32_t kind;           /* msrl_env_kind */
  int32_t num_envs;       /* E >= 1 */
  int32_t num_agents;     /* N >= 1 */
  int32_t num_landmarks;  /* L */
  int32_t obs_dim;        /* D */
  int32_t act_dim;        /* lingauss: action width; particle: ignored */
  int32_t episode_len;    /* >= 1 */
  float dt, damping, force, radius;  /* particle */
  const float* A;         /* lingauss: HOST [D, D] row-major, copied at init */
  const float* B;         /* lingauss: HOST [D, act_dim] row-major, copied at init */
  float noise_std;        /* lingauss */
  float act_cost;         /* lingauss */
  /* tag */
  int32_t num_chasers;    /* 1 .. num_agents-1 */
  float accel_c, accel_r;    /* force of an action: chasers, runners */
  float vmax_c, vmax_r;      /* speed limits */
  float radius_c, radius_r;  /* body radii */
  float contact_force, contact_margin;
  int32_t tag_tiles;      /* 0: chosen by the library; 1 or 4: 32-env tiles per workgroup */
  int32_t wave_roles;     /* particle env: 0 chosen by the library; 1: a wave evaluates both networks of its
                             rows; 2: two waves per row block, one per network (see above) */
} msrl_env_cfg;

/*
 * Policy network in_dim - hidden - hidden - out_dim with tanh, and a value
 * network in_dim - hidden - hidden - 1 of the same dtype, both shared by all
 * agents.  out_dim = 5 for MSRL_CATEGORICAL (particle env) and 2*act_dim for
 * MSRL_DIAG_GAUSSIAN (means, then log standard deviations).
 * MSRL_BF16: parameters are bfloat16; the layer inputs (observation, h1, h2)
 * are rounded to bfloat16 (nearest even), products are accumulated in fp32,
 * bias add and tanh are fp32; logits and values are fp32.
 *
 * Parameter buffer: policy then value, each
 *   W1[in_dim, hidden] b1[hidden] W2[hidden, hidden] b2[hidden] W3[hidden, out] b3[out]
 * with W row-major [in, out], so that y = x W + b.
 *
 * hidden_layers (0 means 2; 2..8): number of tanh layers of `hidden` units in
 * front of the output layer (the evaluation of the paper, section 7.1, uses a
 * seven-layer network).  Each layer beyond two adds one W[hidden, hidden]
 * b[hidden] pair in front of W3.  More than two layers are supported by
 * msrl_rollout_step / msrl_rollout_gae, by the step-granular calls and by the
 * learner; msrl_measure_phase returns MSRL_EUNSUPPORTED for them.
 *
 * roles (0 means 1; 2 for MSRL_ENV_TAG): number of parameter sets.  The
 * parameter buffer holds them one after the other (policy then value each);
 * role 0 are the chasers.
 *
 * value_in_dim (0 means in_dim): input width of the value network.  The only
 * other value accepted is num_agents * in_dim: a centralised critic (multi-
 * agent PPO, section 2.1 of the paper) that takes the joint observation of an
 * env, the rows of its agents one after the other, and gives one value per env;
 * values[t, m] then holds that value on every row of the env.  W1 of the value
 * network is [value_in_dim, hidden].  Supported by msrl_rollout_step /
 * msrl_rollout_gae and the step-granular calls on the particle env with
 * networks of two hidden layers (msrl_act then takes the joint observation of
 * an env from the rows the caller gives for its agents); kernels are compiled
 * for bfloat16 networks of 64 hidden units with 2 .. 10 agents per env, 128
 * with 4 .. 10 and 256 with 7 .. 10 (the envs of a workgroup must fit the 32
 * columns of the critic's tile), and for fp32 networks of 64 units with
 * 2 .. 8 and 128 with 4 .. 8 agents; anything else is MSRL_EUNSUPPORTED; and
 * by the learner (any multiple
 * G of in_dim: the value network then reads groups of G consecutive rows, see
 * msrl_ppo_grad).
 */
typedef struct {
  int32_t in_dim, hidden, out_dim;
  int32_t dtype;  /* msrl_dtype */
  int32_t dist;   /* msrl_dist */
  int32_t hidden_layers;
  int32_t roles;
  int32_t value_in_dim;
} msrl_policy_cfg;

/*
 * Trajectory of one call (the replay buffer contents of Listing 1).  All
 * DEVICE pointers, caller-owned, non-overlapping.
 */
typedef struct {
  float* obs;        /* [T+1, M, D]; obs[T] is the observation after the last step */
  void* actions;     /* categorical: int32 [T, M]; Gaussian: float [T, M, act_dim] */
  float* logp;       /* [T, M] log-probability (density) of the action taken */
  float* rewards;    /* [T, M] */
  uint8_t* dones;    /* [T, M] 0/1 */
  float* values;     /* [T+1, M]; values[T] = V(obs[T]) */
  float* logits;     /* optional (NULL allowed): [T, M, out_dim] policy-net outputs */
  float* adv;        /* [T, M]; written by msrl_rollout_gae only */
  float* ret;        /* [T, M]; written by msrl_rollout_gae only */
} msrl_traj;

/* Number of elements (not bytes) of the parameter buffer; 0 if cfg is invalid. */
size_t msrl_param_count(const msrl_policy_cfg* cfg);

/* Number of floats of env state per env in msrl_state_get/set:
 * particle 4*N + 2*L laid out [agent0 (px,py,vx,vy), agent1 ..., landmark0 (x,y), ...];
 * lingauss D.  0 if cfg is invalid. */
size_t msrl_env_state_size(const msrl_env_cfg* cfg);

/*
 * Creates the env batch on the current device: allocates the library-owned
 * state, copies A and B, sets every step counter to 0 and draws the initial
 * state of episode 0 (the reset of Trainer.train, Listing 1).  EINVAL for null
 * pointers, non-positive sizes, obs_dim != in_dim, an obs_dim or out_dim that
 * does not match the env kind; EUNSUPPORTED if no kernel was compiled for the
 * (env kind, sizes, hidden, dtype) combination.
 */
int msrl_rollout_init(const msrl_env_cfg* env, const msrl_policy_cfg* policy,
                      uint64_t seed, msrl_state** out);

/*
 * T steps of Actor.act for every env (Listing 1; the `duration` loop of
 * Trainer.train), starting from the state the previous call left: observation,
 * both networks, action sampling, env step, reward, done, reset; fills
 * out->obs, actions, logp, rewards, dones, values (and logits if non-NULL) and
 * advances the state.  params: DEVICE buffer of msrl_param_count elements of
 * the policy dtype.  out->adv and out->ret are not touched.
 */
int msrl_rollout_step(msrl_state* st, const void* params, int32_t T,
                      msrl_traj* out, void* hip_stream);

/*
 * Generalised advantage estimation over a stored trajectory (the gae() and
 * discounted_reward() calls of Learner.learn, Listing 1).  For every column m,
 * with A_T = 0:
 *   delta_t = r_t + gamma*(1-d_t)*V_{t+1} - V_t
 *   A_t     = delta_t + gamma*lambda*(1-d_t)*A_{t+1}
 *   ret_t   = A_t + V_t
 * rewards, dones, adv, ret: DEVICE [T, M]; values: DEVICE [T+1, M].
 * T == 0 or M == 0 is a no-op that returns MSRL_OK.
 */
int msrl_gae(const float* rewards, const float* values, const uint8_t* dones,
             int32_t T, int64_t M, float gamma, float lambda,
             float* adv, float* ret, void* hip_stream);

/* msrl_rollout_step followed by msrl_gae on its outputs, enqueued on the same
 * stream: the fused rollout+GAE path.  Needs out->adv and out->ret. */
int msrl_rollout_gae(msrl_state* st, const void* params, int32_t T,
                     float gamma, float lambda, msrl_traj* out, void* hip_stream);

/*
 * msrl_rollout_gae for callers that cannot allocate device memory and cannot let the library do it
 * either: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  It
 * takes no msrl_state and calls no hipMalloc / hipFree or any other allocating routine.
 *   - The env batch is the caller's: env_state DEVICE [num_envs, msrl_env_state_size] floats and
 *     step_counters DEVICE [num_envs] int64, in the layout of msrl_state_get / msrl_state_set; both
 *     are read at the start and advanced in place, so consecutive calls continue the trajectory as
 *     consecutive msrl_rollout_gae calls do.  (An initial state can come from msrl_state_get of a
 *     state made at set-up time, or from the caller's own draws.)
 *   - The re-ordered parameter image, which msrl_rollout_init would allocate, lives in a static
 *     device array of the library of MSRL_STATIC_SCRATCH_BYTES per GPU (held until the process
 *     ends).  A configuration whose image is larger (e.g. 256-unit networks with more than three
 *     hidden layers) is refused with MSRL_EUNSUPPORTED, as is MSRL_ENV_LINGAUSS (its dynamics
 *     matrices are HOST pointers and would need a device copy).
 *   - The first call on a device looks the array's address up (hipGetSymbolAddress); make that
 *     call outside a graph capture.
 *   - Every call on a GPU uses that GPU's one array: two such calls that overlap in time on one
 *     GPU (different streams or threads) race; calls on one stream are ordered and safe.
 * Same arguments, results and errors as msrl_rollout_init(env, policy, seed) followed by
 * msrl_rollout_gae otherwise (env->A and env->B are ignored).
 */
#define MSRL_STATIC_SCRATCH_BYTES (1u << 20)
int msrl_rollout_gae_static(const msrl_env_cfg* env, const msrl_policy_cfg* policy, uint64_t seed,
                            float* env_state, int64_t* step_counters, const void* params, int32_t T,
                            float gamma, float lambda, msrl_traj* out, void* hip_stream);

/*
 * Measurement only (phase rooflines of the rollout kernel; not part of the
 * method).  Same arguments as msrl_rollout_step.
 *   MSRL_PHASE_ENV: the rollout with both networks skipped.  Logits and values
 *     are 0, i.e. exactly what msrl_rollout_step computes for an all-zero
 *     parameter buffer: every output is defined, the state advances.
 *   MSRL_PHASE_MLP: T evaluations of both networks on the observation of the
 *     current state; no env step, no state change.  The contents of `out` are
 *     unspecified afterwards (only rewards[0, :] is written, with a checksum).
 *   MSRL_PHASE_CLOCKS: the full rollout (every output of msrl_rollout_step is
 *     written, the state advances), except that out->logits, which must not be
 *     NULL and needs room for 32 floats per wave of a workgroup (256 floats
 *     suffice), receives no logits but clock stamps: for each wave w of the
 *     first workgroup, float 32*w + i is the number of shader-clock cycles from
 *     the start of step T/2 to the end of phase i of that step, with i = 1
 *     observation rows built and stored, 2 policy layer 1, 3..6 policy weight
 *     stages, 8 value layer 1, 9..12 value weight stages, 14 logits and values
 *     ready, 15 sampling and move, 16 end of step (reward, done, reset).
 * EUNSUPPORTED if the variant was not compiled for the state's configuration.
 */
typedef enum { MSRL_PHASE_ENV = 1, MSRL_PHASE_MLP = 2, MSRL_PHASE_CLOCKS = 3 } msrl_phase;
int msrl_measure_phase(msrl_state* st, const void* params, int32_t T, msrl_traj* out,
                       int32_t phase, void* hip_stream);

/*
 * The launch shape msrl_rollout_init chose for the fused rollout of this state
 * (host call, no device work): workgroups per launch, waves per workgroup, and
 * how many of those waves own a block of 32 rows (all of them, or half with
 * msrl_env_cfg.wave_roles = 2).  Any of the three pointers may be NULL.  Nothing
 * in the results depends on the shape; the call is there so that tests and
 * benchmarks can tell which kernel shape they ran.  EINVAL for a NULL state.
 */
int msrl_rollout_shape(const msrl_state* st, int32_t* workgroups, int32_t* waves, int32_t* row_waves);

/*
 * Step-granular calls: the two halves of Actor.act (Listing 1) as calls of their
 * own, for deployments that keep actor and environment in different fragments
 * (distribution policies DP-A and DP-B of section 6, Table 2, run the policy
 * inference as a device fragment and the environment elsewhere; the dedicated
 * environment fragments of the evaluation do the opposite).  All pointers DEVICE.
 *
 *   msrl_observe   obs [M, D] <- observation of the current state.
 *   msrl_act       both networks and the sampling on the rows of `obs` [M, D]:
 *                  actions (int32 [M] or float [M, act_dim]), logp [M], values
 *                  [M], optional logits [M, out_dim].  The noise is the one msrl_rollout_step would
 *                  draw at the state's step counters; the state is not changed.
 *                  params may be NULL: then the parameters of the most recent call
 *                  on this state that passed some (msrl_act, msrl_rollout_step, ...)
 *                  are used again without being re-ordered once more -- for an actor
 *                  fragment that acts many times between two parameter updates
 *                  (EINVAL if there was no such call).  The caller must not have
 *                  changed that buffer's meaning in between: the library keeps its
 *                  own re-ordered copy and does not look at the buffer again.
 *                  The rows must be observations of this env kind: for the
 *                  particle env the 2*(num_agents-1) trailing slots are taken to
 *                  be zero (they are not multiplied).
 *   msrl_env_step  applies `actions` (one step of msrl_traj.actions: int32 [M],
 *                  values outside 0..4 move nothing; or float [M, act_dim]):
 *                  move, reward, done, reset, step counters + 1; rewards [M],
 *                  dones [M], next_obs [M, D] = observation of the new state.
 * T repetitions of { act on the current observation; env_step } produce exactly
 * the trajectory of one msrl_rollout_step(T) call.
 */
int msrl_observe(msrl_state* st, float* obs, void* hip_stream);
int msrl_act(msrl_state* st, const void* params, const float* obs, void* actions,
             float* logp, float* values, float* logits, void* hip_stream);
int msrl_env_step(msrl_state* st, const void* actions, float* rewards, uint8_t* dones,
                  float* next_obs, void* hip_stream);

/*
 * Learner: the policy update that Learner.learn runs after gae() (Listing 1:
 * mappo_net_train(action, state, adv, r), `iter` times).  The paper names the
 * algorithm (multi-agent PPO) and nothing else; what is computed is the clipped
 * surrogate of PPO with a squared-error value loss and an entropy bonus,
 *   rho = exp(logp_theta(a|s) - logp_old),
 *   L = mean_rows( -min(rho A, clip(rho, 1-clip, 1+clip) A)
 *                  + vf_coef (V_theta(s) - ret)^2 - ent_coef H(pi_theta(.|s)) ),
 * its gradient with respect to all parameters of both networks, and Adam with
 * bias correction.  Parameters, moments and gradients are float32 in the
 * parameter layout of msrl_policy_cfg, whatever the policy dtype; for
 * MSRL_BF16 the networks are evaluated as in the rollout (weights and layer
 * inputs rounded to bfloat16, fp32 accumulation) and the backward contractions
 * take bfloat16 operands too; roundings count as the identity in the
 * derivative.  A row is one (t, m) entry of a stored trajectory: obs [R, D],
 * actions int32 [R] or float [R, act_dim], logp_old, adv, ret [R].  All
 * pointers DEVICE except cfg and step_counter (HOST).
 *
 * Centralised critic (value_in_dim = G * in_dim, G > 1; multi-agent PPO,
 * section 2.1 of the paper): the rows come in groups of G consecutive rows, the
 * agents of one env at one step (the row order of a stored trajectory); the
 * value network reads a group's rows as one input and has one target per group,
 * ret of the group's first row, and the value term is the mean over the groups:
 *   L = mean_rows( policy term - ent_coef H ) + vf_coef mean_groups (V_theta(group) - ret)^2.
 * R must then be a multiple of G (EINVAL otherwise), and msrl_ppo_update cuts
 * its blocks at group boundaries.
 *
 * Rows of one role.  Listing 1 runs one learner per agent role, each on the rows of its own agents;
 * in a stored trajectory those rows are interleaved with the other roles' (row = (t, env, agent)).
 * msrl_row_select names them without a copy: selected row r (0 <= r < R) is row
 *   (r / count) * group + first + r % count
 * of obs, actions, logp_old, adv and ret, i.e. with group = num_agents the agents first ..
 * first + count - 1 of every env at every step.  NULL selects every row (row r is row r).  EINVAL
 * unless group >= 1, first >= 0, count >= 1, first + count <= group, and for a selection together
 * with a centralised critic (which reads whole groups of rows).
 */
typedef struct { int32_t group, first, count; } msrl_row_select;
typedef struct msrl_learner msrl_learner; /* opaque: workspaces for up to max_rows rows per call */
typedef struct {
  float clip, vf_coef, ent_coef;
  float lr, beta1, beta2, adam_eps;
} msrl_ppo_cfg;

/* Allocates the workspaces.  EINVAL unless hidden is a multiple of 32 and out_dim <= 32.
 * bfloat16 networks with two hidden layers of 64, 128 or 256 units, a categorical policy of at most
 * 16 actions and at most 62 inputs take the path that keeps the activations on chip (with a
 * centralised critic: the policy network only); everything else the path through device memory.
 * Both compute the same gradient (the same rounding points in bfloat16 mode). */
int msrl_learner_init(const msrl_policy_cfg* policy, int64_t max_rows, msrl_learner** out);
/* The same with the choice of path made by the caller (tests and measurements: it keeps the
 * device-memory kernels covered for configurations that would take the on-chip path).
 * MSRL_LEARNER_PATH_AUTO is msrl_learner_init; EINVAL for an unknown path. */
typedef enum { MSRL_LEARNER_PATH_AUTO = 0, MSRL_LEARNER_PATH_DEVICE_MEMORY = 1 } msrl_learner_path;
int msrl_learner_init_path(const msrl_policy_cfg* policy, int64_t max_rows, int32_t path, msrl_learner** out);
void msrl_learner_destroy(msrl_learner* learner);

/*
 * grad [msrl_param_count] <- dL/dparams over the R given rows (1 <= R <=
 * max_rows); stats (optional, 5 floats) <- sums over the rows of: the policy
 * term, (V - ret)^2 (with a centralised critic: the sum over the R / G groups),
 * the entropy, 1 where the clipped branch of the min is active, logp_old - logp.
 * grad is summed in a fixed order: the same inputs give the same bits on every
 * call.  The five statistics (and msrl_rows_mean's result) are added up with
 * float atomics over a few bins, so their last bits can differ between calls.
 */
int msrl_ppo_grad(msrl_learner* learner, const float* params, int64_t R, const float* obs,
                  const void* actions, const float* logp_old, const float* adv, const float* ret,
                  const msrl_row_select* rows, const msrl_ppo_cfg* cfg, float* grad, float* stats,
                  void* hip_stream);

/* One Adam step on n parameters, in place; k >= 1 is the number of this step. */
int msrl_adam_step(float* params, float* m, float* v, const float* grad, int64_t n, int64_t k,
                   const msrl_ppo_cfg* cfg, void* hip_stream);

/* out [n] (policy dtype: float or bfloat16, nearest even) <- master [n] (float): the parameter
 * buffer msrl_rollout_step takes, from the learner's float32 master copy. */
int msrl_params_cast(const float* master, void* out, int64_t n, int32_t dtype, void* hip_stream);

/*
 * The training loop of Learner.learn: `iters` passes over the R rows, each
 * split into `minibatches` consecutive blocks of rows (the last one takes the
 * remainder; no block may exceed max_rows), one msrl_ppo_grad + msrl_adam_step
 * per block.  *step_counter (HOST): Adam steps taken so far, advanced by
 * iters * minibatches.
 */
int msrl_ppo_update(msrl_learner* learner, float* params, float* m, float* v, int64_t* step_counter,
                    int64_t R, int32_t iters, int32_t minibatches, const float* obs,
                    const void* actions, const float* logp_old, const float* adv, const float* ret,
                    const msrl_row_select* rows, const msrl_ppo_cfg* cfg, void* hip_stream);

/* out[0] (DEVICE) <- mean of x over the R selected rows (x: DEVICE, one float per row; rows as above,
 * NULL = rows 0 .. R-1): e.g. the mean reward of one role's agents over a stored trajectory. */
int msrl_rows_mean(const float* x, int64_t R, const msrl_row_select* rows, float* out, void* hip_stream);

/*
 * Snapshot / restore of the env batch.  env_state: HOST
 * [num_envs, msrl_env_state_size] floats; step_counters: HOST [num_envs] int64
 * (only the low 32 bits enter the Philox counter).  Either pointer may be NULL
 * to skip that part.  Both calls wait for the device.
 */
int msrl_state_get(msrl_state* st, float* env_state, int64_t* step_counters);
int msrl_state_set(msrl_state* st, const float* env_state, const int64_t* step_counters);

/* Frees the state (NULL allowed). */
void msrl_rollout_destroy(msrl_state* st);

/* Message of the last error on this thread ("" if none). */
const char* msrl_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* MSRL_H */
