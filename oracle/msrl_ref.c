/*
 * msrl_ref.c -- CPU oracle for the fused rollout fragment and the GAE pass.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the
 * HIP library is checked against.  Only the tests, the smoke check and the
 * cpu_baseline leg of the benchmark may call it; the product path never does.
 * It shares no code, header or table with the HIP sources.
 *
 * Scalar loops in the order step -> env -> agent, double precision throughout,
 * except where a floating-point value decides an integer (the categorical
 * draw), which is taken in float like the device does.
 *
 * What is computed follows Listing 1 of the paper (section 3): Actor.act =
 * policy network, action, env_step giving reward and new_state; Trainer.train
 * repeats it and stores each step; Learner.learn evaluates the critic and calls
 * gae().  The paper fixes no arithmetic for these; the concrete environment,
 * network, sampling and GAE definitions are the ones stated with each function
 * below.
 *
 * Pins (tests/test_oracle_*.py): hand-computed particle steps, damping and
 * constant-force closed forms, collision thresholds, the 0.98^t norm law of
 * the linear-Gaussian env, GAE against a brute-force discounted sum and worked
 * values, MLP special cases against numpy, sampled-action frequencies against
 * softmax probabilities over 10^6 draws, normal moments, Philox multiply/round
 * structure against big-integer arithmetic and uniformity statistics.
 * ref_philox4x32_10 reproduces the published known-answer vectors of
 * Philox4x32-10 (tests/golden/philox4x32_10_kat.txt).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define REF_ENV_TAG 2
#define REF_ENV_PARTICLE 0
#define REF_ENV_LINGAUSS 1
#define REF_CATEGORICAL 0
#define REF_DIAG_GAUSSIAN 1

typedef struct {
  int32_t kind, num_agents, num_landmarks, obs_dim, act_dim, episode_len;
  double dt, damping, force, radius;
  const double* A; /* [D, D] row-major */
  const double* B; /* [D, act_dim] row-major */
  double noise_std, act_cost;
  /* pursuit ("tag") variant of the particle env: the first num_chasers agents chase the others */
  int32_t num_chasers, pad_;
  double accel_c, accel_r;   /* force of an action, chasers / runners */
  double vmax_c, vmax_r;     /* speed limit */
  double radius_c, radius_r; /* body radius */
  double contact_force, contact_margin;
} ref_env_cfg;

typedef struct {
  int32_t in_dim, hidden, out_dim;
  int32_t bf16; /* 0: exact arithmetic on the given values; 1: bf16 rounding points */
  int32_t dist;
  int32_t hidden_layers; /* tanh layers of `hidden` units in front of the output layer; 0 means 2 */
  int32_t value_in_dim;  /* input width of the value net; 0 means in_dim.  N * in_dim: a centralised
                            critic on the joint observation of the env's N agents */
} ref_policy_cfg;

/* ---------------------------------------------------------------- Philox */

/* One Philox4x32 round followed by the key schedule, ten times
 * (Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as easy as 1, 2, 3",
 * SC'11, Philox-4x32 with the multipliers and Weyl key increments given there). */
void ref_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]) {
  uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
  uint32_t k0 = key[0], k1 = key[1];
  for (int round = 0; round < 10; ++round) {
    uint64_t p0 = (uint64_t)0xD2511F53u * c0;
    uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
    uint32_t hi0 = (uint32_t)(p0 >> 32), lo0 = (uint32_t)p0;
    uint32_t hi1 = (uint32_t)(p1 >> 32), lo1 = (uint32_t)p1;
    uint32_t n0 = hi1 ^ c1 ^ k0;
    uint32_t n1 = lo1;
    uint32_t n2 = hi0 ^ c3 ^ k1;
    uint32_t n3 = lo0;
    c0 = n0; c1 = n1; c2 = n2; c3 = n3;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* Words of the stream block (env, entity, time, stream, block) under `seed`. */
void ref_draw(uint64_t seed, uint32_t env, uint32_t entity, uint32_t time,
              uint32_t stream, uint32_t block, uint32_t out[4]) {
  uint32_t ctr[4] = {env, entity, time, (stream << 16) | block};
  uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
  ref_philox4x32_10(ctr, key, out);
}

/* u in [0,1): the top 24 bits of the word. */
double ref_uniform(uint32_t w) { return (double)(w >> 8) * (1.0 / 16777216.0); }

/* Box-Muller pair from two words; the radius uses a uniform in (0,1]. */
void ref_normal_pair(uint32_t w0, uint32_t w1, double out[2]) {
  double u1 = (double)((w0 >> 8) + 1u) * (1.0 / 16777216.0);
  double u2 = (double)(w1 >> 8) * (1.0 / 16777216.0);
  double r = sqrt(-2.0 * log(u1));
  double th = 6.283185307179586476925286766559 * u2;
  out[0] = r * cos(th);
  out[1] = r * sin(th);
}

/* n standard normals of a stream: block b supplies normals 4b..4b+3. */
void ref_normals(uint64_t seed, uint32_t env, uint32_t entity, uint32_t time,
                 uint32_t stream, int n, double* out) {
  for (int i = 0; i < n; i += 4) {
    uint32_t w[4];
    double e[4];
    ref_draw(seed, env, entity, time, stream, (uint32_t)(i / 4), w);
    ref_normal_pair(w[0], w[1], e);
    ref_normal_pair(w[2], w[3], e + 2);
    for (int j = 0; j < 4 && i + j < n; ++j) out[i + j] = e[j];
  }
}

/* ---------------------------------------------------------------- bf16 */

/* Nearest-even rounding of a value to bfloat16 (through float), as a double. */
double ref_bf16_round(double x) {
  float f = (float)x;
  uint32_t b;
  memcpy(&b, &f, 4);
  if ((b & 0x7F800000u) == 0x7F800000u) return (double)f; /* inf / nan unchanged */
  uint32_t lsb = (b >> 16) & 1u;
  b += 0x7FFFu + lsb;
  b &= 0xFFFF0000u;
  memcpy(&f, &b, 4);
  return (double)f;
}

/* ---------------------------------------------------------------- networks */

/* One dense layer y = act(x W + b), W row-major [in, out]. */
static void dense(const double* W, const double* b, int in, int out, const double* x,
                  double* y, int do_tanh, int bf16) {
  for (int o = 0; o < out; ++o) {
    double acc = 0.0;
    for (int i = 0; i < in; ++i) {
      double w = bf16 ? ref_bf16_round(W[(size_t)i * out + o]) : W[(size_t)i * out + o];
      double xi = bf16 ? ref_bf16_round(x[i]) : x[i];
      acc += xi * w;
    }
    acc += b[o];
    y[o] = do_tanh ? tanh(acc) : acc;
  }
}

/* in - H - ... - H - out network with L >= 1 tanh hidden layers of H units (the paper's
 * evaluation uses a deeper policy than its listings: section 7.1, "seven-layer DNN"; the depth is a
 * parameter here); params = W1 b1, then W b per further hidden layer, then the output layer's
 * W b, every W stored [inputs, outputs].  bf16 = 1 rounds every layer input and every weight to
 * bfloat16; sums, bias add and tanh are not rounded. */
void ref_mlp_l(int in, int H, int out, int L, const double* params, const double* x, double* y,
               int bf16) {
  double* ha = (double*)malloc(sizeof(double) * (size_t)H);
  double* hb = (double*)malloc(sizeof(double) * (size_t)H);
  const double* P = params;
  dense(P, P + (size_t)in * H, in, H, x, ha, 1, bf16);
  P += (size_t)in * H + H;
  for (int l = 1; l < L; ++l) {
    dense(P, P + (size_t)H * H, H, H, ha, hb, 1, bf16);
    P += (size_t)H * H + H;
    double* t = ha;
    ha = hb;
    hb = t;
  }
  dense(P, P + (size_t)H * out, H, out, ha, y, 0, bf16);
  free(ha);
  free(hb);
}

/* the two-hidden-layer network of the benchmark configurations: W1 b1 W2 b2 W3 b3 */
void ref_mlp(int in, int H, int out, const double* params, const double* x, double* y,
             int bf16) {
  ref_mlp_l(in, H, out, 2, params, x, y, bf16);
}

size_t ref_net_param_count_l(int in, int H, int out, int L) {
  return (size_t)in * H + H + (size_t)(L - 1) * ((size_t)H * H + H) + (size_t)H * out + out;
}

size_t ref_net_param_count(int in, int H, int out) { return ref_net_param_count_l(in, H, out, 2); }

static int layers_of(const ref_policy_cfg* p) { return p->hidden_layers > 0 ? p->hidden_layers : 2; }

/* Policy outputs and value of one observation row; params = policy net, value net. */
void ref_policy_value(const ref_policy_cfg* p, const double* params, const double* x,
                      double* logits, double* value) {
  const int L = layers_of(p);
  ref_mlp_l(p->in_dim, p->hidden, p->out_dim, L, params, x, logits, p->bf16);
  ref_mlp_l(p->in_dim, p->hidden, 1, L,
            params + ref_net_param_count_l(p->in_dim, p->hidden, p->out_dim, L), x, value, p->bf16);
}

/* Centralised critic (multi-agent PPO, section 2.1: the critic takes joint information of all agents): the
 * value network takes the joint observation of an env, the N rows of its agents one after the
 * other, and gives one value for the env.  params as above, the value net value_in_dim wide. */
void ref_central_value(const ref_policy_cfg* p, const double* params, const double* joint,
                       double* value) {
  const int L = layers_of(p);
  ref_mlp_l(p->value_in_dim, p->hidden, 1, L,
            params + ref_net_param_count_l(p->in_dim, p->hidden, p->out_dim, L), joint, value, p->bf16);
}

/* ---------------------------------------------------------------- sampling */

/* Categorical draw by inverse CDF.  The decision is taken in float: z = logit -
 * max, p_k = exp(z_k) / sum, c_k = running sum in index order, action = first k
 * with u < c_k (last index if none).  logp = z_a - log(sum exp z) in double.
 * margin = min_k |c_k - u|: how close the draw was to a bin edge. */
void ref_categorical(const double* logits, int n, double u, int32_t* action, double* logp,
                     double* margin) {
  float z[64], e[64];
  float mx = (float)logits[0];
  for (int k = 1; k < n; ++k)
    if ((float)logits[k] > mx) mx = (float)logits[k];
  float s = 0.0f;
  for (int k = 0; k < n; ++k) {
    z[k] = (float)logits[k] - mx;
    e[k] = expf(z[k]);
    s += e[k];
  }
  float uf = (float)u, c = 0.0f;
  int a = n - 1, found = 0;
  double mg = 1.0;
  for (int k = 0; k < n; ++k) {
    c += e[k] / s;
    if (!found && uf < c) { a = k; found = 1; }
    if (k < n - 1 && fabs((double)c - (double)uf) < mg) mg = fabs((double)c - (double)uf);
  }
  double mxd = logits[0], sd = 0.0;
  for (int k = 1; k < n; ++k)
    if (logits[k] > mxd) mxd = logits[k];
  for (int k = 0; k < n; ++k) sd += exp(logits[k] - mxd);
  *action = a;
  *logp = (logits[a] - mxd) - log(sd);
  *margin = mg;
}

/* Diagonal Gaussian: a = mean + exp(logstd) * eps,
 * logp = sum(-eps^2/2 - logstd - ln(2 pi)/2). */
void ref_gaussian(const double* mean, const double* logstd, const double* eps, int n,
                  double* a, double* logp) {
  double lp = 0.0;
  for (int d = 0; d < n; ++d) {
    a[d] = mean[d] + exp(logstd[d]) * eps[d];
    lp += -0.5 * eps[d] * eps[d] - logstd[d] - 0.91893853320467274178;
  }
  *logp = lp;
}

/* Action of (env, agent) at step counter g from the policy outputs. */
void ref_sample(const ref_policy_cfg* p, uint64_t seed, uint32_t env, uint32_t agent,
                uint32_t g, const double* logits, int32_t* action_i, double* action_f,
                double* logp, double* margin) {
  if (p->dist == REF_CATEGORICAL) {
    uint32_t w[4];
    ref_draw(seed, env, agent, g, 0, 0, w);
    ref_categorical(logits, p->out_dim, ref_uniform(w[0]), action_i, logp, margin);
  } else {
    int n = p->out_dim / 2;
    double eps[64];
    ref_normals(seed, env, agent, g, 0, n, eps);
    ref_gaussian(logits, logits + n, eps, n, action_f, logp);
    *margin = 1.0;
  }
}

/* ---------------------------------------------------------------- particle env */

/* state of one env: [agent i: px,py,vx,vy] * N, then [landmark k: x,y] * L. */

void ref_particle_obs(int N, int L, int D, const double* s, double* obs /* [N, D] */) {
  const double* lm = s + 4 * N;
  for (int i = 0; i < N; ++i) {
    double* o = obs + (size_t)i * D;
    double px = s[4 * i], py = s[4 * i + 1];
    int f = 0;
    o[f++] = s[4 * i + 2];
    o[f++] = s[4 * i + 3];
    o[f++] = px;
    o[f++] = py;
    for (int k = 0; k < L; ++k) {
      o[f++] = lm[2 * k] - px;
      o[f++] = lm[2 * k + 1] - py;
    }
    for (int j = 0; j < N; ++j) {
      if (j == i) continue;
      o[f++] = s[4 * j] - px;
      o[f++] = s[4 * j + 1] - py;
    }
    while (f < D) o[f++] = 0.0; /* silent communication slots */
  }
}

void ref_particle_reset(uint64_t seed, uint32_t env, uint32_t episode, int N, int L, double* s) {
  uint32_t w[4];
  for (int i = 0; i < N; ++i) {
    ref_draw(seed, env, (uint32_t)i, episode, 1, 0, w);
    s[4 * i] = 2.0 * ref_uniform(w[0]) - 1.0;
    s[4 * i + 1] = 2.0 * ref_uniform(w[1]) - 1.0;
    s[4 * i + 2] = 0.0;
    s[4 * i + 3] = 0.0;
  }
  for (int k = 0; k < L; ++k) {
    ref_draw(seed, env, (uint32_t)(N + k), episode, 1, 0, w);
    s[4 * N + 2 * k] = 2.0 * ref_uniform(w[0]) - 1.0;
    s[4 * N + 2 * k + 1] = 2.0 * ref_uniform(w[1]) - 1.0;
  }
}

/* Point-mass move of every agent, then the shared reward on the new positions.
 * coll_margin: smallest |distance - 2 radius| over the agent pairs. */
void ref_particle_move(const ref_env_cfg* c, double* s, const int32_t* actions, double* reward,
                       double* coll_margin) {
  static const double FX[5] = {0.0, 1.0, -1.0, 0.0, 0.0};
  static const double FY[5] = {0.0, 0.0, 0.0, 1.0, -1.0};
  int N = c->num_agents, L = c->num_landmarks;
  for (int i = 0; i < N; ++i) {
    double* a = s + 4 * i;
    int act = actions[i];
    a[2] = a[2] * (1.0 - c->damping) + FX[act] * c->force * c->dt;
    a[3] = a[3] * (1.0 - c->damping) + FY[act] * c->force * c->dt;
    a[0] += a[2] * c->dt;
    a[1] += a[3] * c->dt;
  }
  double r = 0.0, mg = 1e30;
  for (int k = 0; k < L; ++k) {
    double best = 1e300;
    for (int i = 0; i < N; ++i) {
      double dx = s[4 * i] - s[4 * N + 2 * k], dy = s[4 * i + 1] - s[4 * N + 2 * k + 1];
      double d = sqrt(dx * dx + dy * dy);
      if (d < best) best = d;
    }
    r -= best;
  }
  for (int i = 0; i < N; ++i)
    for (int j = i + 1; j < N; ++j) {
      double dx = s[4 * i] - s[4 * j], dy = s[4 * i + 1] - s[4 * j + 1];
      double d = sqrt(dx * dx + dy * dy);
      if (d < 2.0 * c->radius) r -= 1.0;
      if (fabs(d - 2.0 * c->radius) < mg) mg = fabs(d - 2.0 * c->radius);
    }
  *reward = r;
  if (coll_margin) *coll_margin = mg;
}

/* ---------------------------------------------------------------- pursuit ("tag") env
 *
 * The workload of the paper's GPU-only experiment (section 7.3, Fig. 10) is a pursuit task of the
 * multi-agent particle family: heterogeneous agents (chasers and runners) with a policy per role,
 * rewards per role, and bodies that push each other apart.  The paper gives no formulas; this is a
 * synthetic stand-in defined here:
 *   state        as the particle env: agents (px, py, vx, vy), then landmarks (x, y); reset alike
 *   observation  of agent i: v_i, p_i, landmark_k - p_i (all k), p_j - p_i (all j != i, index
 *                order), v_j (all j != i): D = 4 + 2L + 4(N-1)
 *   move         F_i = accel(role_i) * direction(action_i) + sum_{j != i} contact(i, j),
 *                contact(i, j) = contact_force * pen(d_ij) * (p_i - p_j) / d_ij,
 *                pen(d) = m * softplus((r_i + r_j - d) / m), m = contact_margin (a smooth
 *                max(0, overlap)); v <- v (1 - damping) + F dt; |v| limited to vmax(role);
 *                p <- p + v dt.  All forces use the positions before the move.
 *   reward       on the new positions, "contact" = d_ij < r_i + r_j between a chaser and a runner:
 *                every chaser +10 per contact of any chaser; runner j -10 per chaser in contact
 *                with it, - 10 * sum over the two axes of max(0, |p| - 1) (leaving the arena).
 */
static int tag_is_chaser(const ref_env_cfg* c, int i) { return i < c->num_chasers; }

void ref_tag_obs(const ref_env_cfg* c, const double* s, double* obs /* [N, D] */) {
  const int N = c->num_agents, L = c->num_landmarks, D = c->obs_dim;
  const double* lm = s + 4 * N;
  for (int i = 0; i < N; ++i) {
    double* o = obs + (size_t)i * D;
    const double px = s[4 * i], py = s[4 * i + 1];
    int f = 0;
    o[f++] = s[4 * i + 2];
    o[f++] = s[4 * i + 3];
    o[f++] = px;
    o[f++] = py;
    for (int k = 0; k < L; ++k) {
      o[f++] = lm[2 * k] - px;
      o[f++] = lm[2 * k + 1] - py;
    }
    for (int j = 0; j < N; ++j) {
      if (j == i) continue;
      o[f++] = s[4 * j] - px;
      o[f++] = s[4 * j + 1] - py;
    }
    for (int j = 0; j < N; ++j) {
      if (j == i) continue;
      o[f++] = s[4 * j + 2];
      o[f++] = s[4 * j + 3];
    }
    while (f < D) o[f++] = 0.0;
  }
}

static double softplus(double x) { return (x > 0.0 ? x : 0.0) + log1p(exp(-fabs(x))); }

/* Move of every agent, then the per-agent rewards on the new positions.
 * margin: smallest |distance - (r_i + r_j)| over the chaser-runner pairs after the move. */
void ref_tag_move(const ref_env_cfg* c, double* s, const int32_t* actions, double* rewards /* [N] */,
                  double* margin) {
  static const double FX[5] = {0.0, 1.0, -1.0, 0.0, 0.0};
  static const double FY[5] = {0.0, 0.0, 0.0, 1.0, -1.0};
  const int N = c->num_agents;
  double fx[64], fy[64];
  for (int i = 0; i < N; ++i) {
    const int ci = tag_is_chaser(c, i);
    const double acc = ci ? c->accel_c : c->accel_r, ri = ci ? c->radius_c : c->radius_r;
    fx[i] = acc * FX[actions[i]];
    fy[i] = acc * FY[actions[i]];
    for (int j = 0; j < N; ++j) {
      if (j == i) continue;
      const double rj = tag_is_chaser(c, j) ? c->radius_c : c->radius_r;
      const double dx = s[4 * i] - s[4 * j], dy = s[4 * i + 1] - s[4 * j + 1];
      const double d = sqrt(dx * dx + dy * dy);
      const double pen = c->contact_margin * softplus((ri + rj - d) / c->contact_margin);
      if (d > 0.0) {
        fx[i] += c->contact_force * pen * dx / d;
        fy[i] += c->contact_force * pen * dy / d;
      }
    }
  }
  for (int i = 0; i < N; ++i) {
    double* a = s + 4 * i;
    const double vmax = tag_is_chaser(c, i) ? c->vmax_c : c->vmax_r;
    a[2] = a[2] * (1.0 - c->damping) + fx[i] * c->dt;
    a[3] = a[3] * (1.0 - c->damping) + fy[i] * c->dt;
    const double sp = sqrt(a[2] * a[2] + a[3] * a[3]);
    if (sp > vmax) {
      a[2] *= vmax / sp;
      a[3] *= vmax / sp;
    }
    a[0] += a[2] * c->dt;
    a[1] += a[3] * c->dt;
  }
  double mg = 1e30;
  int total = 0;
  int per_runner[64];
  for (int j = 0; j < N; ++j) per_runner[j] = 0;
  for (int i = 0; i < N; ++i) {
    if (!tag_is_chaser(c, i)) continue;
    for (int j = 0; j < N; ++j) {
      if (tag_is_chaser(c, j)) continue;
      const double dx = s[4 * i] - s[4 * j], dy = s[4 * i + 1] - s[4 * j + 1];
      const double d = sqrt(dx * dx + dy * dy), dmin = c->radius_c + c->radius_r;
      if (d < dmin) {
        total += 1;
        per_runner[j] += 1;
      }
      if (fabs(d - dmin) < mg) mg = fabs(d - dmin);
    }
  }
  for (int i = 0; i < N; ++i) {
    if (tag_is_chaser(c, i)) {
      rewards[i] = 10.0 * total;
    } else {
      const double ox = fabs(s[4 * i]) - 1.0, oy = fabs(s[4 * i + 1]) - 1.0;
      rewards[i] = -10.0 * per_runner[i] - 10.0 * ((ox > 0.0 ? ox : 0.0) + (oy > 0.0 ? oy : 0.0));
    }
  }
  if (margin) *margin = mg;
}

/* ---------------------------------------------------------------- linear-Gaussian env */

/* reward on (s, a) before the move; then s <- A s + B a + noise_std * eps. */
void ref_lingauss_move(const ref_env_cfg* c, double* s, const double* a, const double* eps,
                       double* reward) {
  int D = c->obs_dim, K = c->act_dim;
  double ss = 0.0, aa = 0.0;
  for (int i = 0; i < D; ++i) ss += s[i] * s[i];
  for (int j = 0; j < K; ++j) aa += a[j] * a[j];
  *reward = -(ss + c->act_cost * aa);
  double* n = (double*)malloc(sizeof(double) * (size_t)D);
  for (int i = 0; i < D; ++i) {
    double acc = 0.0;
    for (int j = 0; j < D; ++j) acc += c->A[(size_t)i * D + j] * s[j];
    for (int j = 0; j < K; ++j) acc += c->B[(size_t)i * K + j] * a[j];
    n[i] = acc + c->noise_std * eps[i];
  }
  memcpy(s, n, sizeof(double) * (size_t)D);
  free(n);
}

/* ---------------------------------------------------------------- env interface */

int ref_env_state_size(const ref_env_cfg* c) {
  return c->kind != REF_ENV_LINGAUSS ? 4 * c->num_agents + 2 * c->num_landmarks : c->obs_dim;
}

void ref_env_reset(const ref_env_cfg* c, uint64_t seed, uint32_t env, uint32_t episode,
                   double* s) {
  if (c->kind != REF_ENV_LINGAUSS)
    ref_particle_reset(seed, env, episode, c->num_agents, c->num_landmarks, s);
  else
    ref_normals(seed, env, 0, episode, 1, c->obs_dim, s);
}

void ref_env_obs(const ref_env_cfg* c, const double* s, double* obs /* [N, D] */) {
  if (c->kind == REF_ENV_PARTICLE)
    ref_particle_obs(c->num_agents, c->num_landmarks, c->obs_dim, s, obs);
  else if (c->kind == REF_ENV_TAG)
    ref_tag_obs(c, s, obs);
  else
    memcpy(obs, s, sizeof(double) * (size_t)c->obs_dim);
}

/* One env_step of env `env` whose step counter is g: move, reward, done, and the
 * reset that follows a done.  actions: int32 [N] (particle) or double [act_dim]. */
void ref_env_step(const ref_env_cfg* c, uint64_t seed, uint32_t env, int64_t g, double* s,
                  const int32_t* actions_i, const double* actions_f, double* reward,
                  uint8_t* done, double* margin) {
  if (c->kind == REF_ENV_PARTICLE) {
    ref_particle_move(c, s, actions_i, reward, margin);
  } else {
    double eps[256];
    ref_normals(seed, env, 0, (uint32_t)g, 2, c->obs_dim, eps);
    ref_lingauss_move(c, s, actions_f, eps, reward);
    if (margin) *margin = 1e30;
  }
  *done = (uint8_t)(((g + 1) % c->episode_len) == 0);
  if (*done) ref_env_reset(c, seed, env, (uint32_t)((g + 1) / c->episode_len), s);
}

/* The pursuit env's step: rewards per agent [N]; done and reset as above. */
void ref_env_step_tag(const ref_env_cfg* c, uint64_t seed, uint32_t env, int64_t g, double* s,
                      const int32_t* actions, double* rewards, uint8_t* done, double* margin) {
  ref_tag_move(c, s, actions, rewards, margin);
  *done = (uint8_t)(((g + 1) % c->episode_len) == 0);
  if (*done) ref_env_reset(c, seed, env, (uint32_t)((g + 1) / c->episode_len), s);
}

/* ---------------------------------------------------------------- rollout */

/* Initial state of envs env0 .. env0+E-1 (global ids): episode 0, counters 0. */
void ref_init(const ref_env_cfg* c, uint64_t seed, int env0, int E, double* state, int64_t* g) {
  int S = ref_env_state_size(c);
  for (int e = 0; e < E; ++e) {
    ref_env_reset(c, seed, (uint32_t)(env0 + e), 0, state + (size_t)e * S);
    g[e] = 0;
  }
}

/*
 * T steps for envs env0 .. env0+E-1.  Trajectory tensors are time-major over
 * M = E * N rows: obs [T+1, M, D], actions_i int32 [T, M] or actions_f
 * [T, M, act_dim], logp/rewards/values(+1 row)/dones [T, M], logits
 * [T, M, out_dim] (may be NULL).  state and g are advanced in place.
 */
void ref_rollout(const ref_env_cfg* c, const ref_policy_cfg* p, uint64_t seed, int env0, int E,
                 double* state, int64_t* g, const double* params, int T, double* obs,
                 int32_t* actions_i, double* actions_f, double* logp, double* rewards,
                 uint8_t* dones, double* values, double* logits) {
  int N = c->num_agents, D = c->obs_dim, S = ref_env_state_size(c), O = p->out_dim;
  int K = c->act_dim;
  size_t M = (size_t)E * N;
  double* lg = (double*)malloc(sizeof(double) * (size_t)O);
  int32_t* ai = (int32_t*)malloc(sizeof(int32_t) * (size_t)N);
  double af[64];
  for (int t = 0; t <= T; ++t) {
    for (int e = 0; e < E; ++e) {
      double* s = state + (size_t)e * S;
      double* o = obs + ((size_t)t * M + (size_t)e * N) * D;
      ref_env_obs(c, s, o);
      for (int i = 0; i < N; ++i) {
        size_t m = (size_t)e * N + i;
        double v;
        /* pursuit env: one parameter set (policy net, value net) per role, chasers first */
        const double* prm = params;
        if (c->kind == REF_ENV_TAG && i >= c->num_chasers) {
          const int Lh = p->hidden_layers > 0 ? p->hidden_layers : 2;
          prm += ref_net_param_count_l(p->in_dim, p->hidden, p->out_dim, Lh) +
                 ref_net_param_count_l(p->value_in_dim > 0 ? p->value_in_dim : p->in_dim, p->hidden, 1, Lh);
        }
        if (p->value_in_dim > 0 && p->value_in_dim != p->in_dim) {
          /* centralised critic: policy on the agent's row, value on the env's joint observation */
          const int Lh = p->hidden_layers > 0 ? p->hidden_layers : 2;
          ref_mlp_l(p->in_dim, p->hidden, p->out_dim, Lh, prm, o + (size_t)i * D, lg, p->bf16);
          ref_central_value(p, prm, o, &v);
        } else {
          ref_policy_value(p, prm, o + (size_t)i * D, lg, &v);
        }
        values[(size_t)t * M + m] = v;
        if (t == T) continue;
        double lp, mg;
        ref_sample(p, seed, (uint32_t)(env0 + e), (uint32_t)i, (uint32_t)g[e], lg, &ai[i], af,
                   &lp, &mg);
        logp[(size_t)t * M + m] = lp;
        if (logits) memcpy(logits + ((size_t)t * M + m) * O, lg, sizeof(double) * (size_t)O);
        if (p->dist == REF_CATEGORICAL)
          actions_i[(size_t)t * M + m] = ai[i];
        else
          memcpy(actions_f + ((size_t)t * M + m) * K, af, sizeof(double) * (size_t)K);
      }
      if (t == T) continue;
      double r, rr[64];
      uint8_t d;
      if (c->kind == REF_ENV_TAG)
        ref_env_step_tag(c, seed, (uint32_t)(env0 + e), g[e], s, ai, rr, &d, NULL);
      else
        ref_env_step(c, seed, (uint32_t)(env0 + e), g[e], s, ai, af, &r, &d, NULL);
      g[e] += 1;
      for (int i = 0; i < N; ++i) {
        rewards[(size_t)t * M + (size_t)e * N + i] = c->kind == REF_ENV_TAG ? rr[i] : r;
        dones[(size_t)t * M + (size_t)e * N + i] = d;
      }
    }
  }
  free(lg);
  free(ai);
}

/* ---------------------------------------------------------------- GAE */

/* Reverse recurrence per column:
 *   delta_t = r_t + gamma (1-d_t) V_{t+1} - V_t,
 *   A_t = delta_t + gamma lambda (1-d_t) A_{t+1}, A_T = 0;  ret_t = A_t + V_t. */
void ref_gae(const double* r, const double* V, const uint8_t* d, int T, int64_t M, double gamma,
             double lambda, double* adv, double* ret) {
  for (int64_t m = 0; m < M; ++m) {
    double next = 0.0;
    for (int t = T - 1; t >= 0; --t) {
      double nd = 1.0 - (double)d[(size_t)t * M + m];
      double delta = r[(size_t)t * M + m] + gamma * nd * V[(size_t)(t + 1) * M + m] -
                     V[(size_t)t * M + m];
      next = delta + gamma * lambda * nd * next;
      adv[(size_t)t * M + m] = next;
      ret[(size_t)t * M + m] = next + V[(size_t)t * M + m];
    }
  }
}

/* ---------------------------------------------------------------- batch helpers */

/* Loops used by the statistical pins: n draws of ref_sample for fixed policy
 * outputs, env = 0..n-1 (agent 0, step counter g). */
void ref_categorical_counts(const ref_policy_cfg* p, uint64_t seed, uint32_t g,
                            const double* logits, int64_t n, int64_t* counts) {
  for (int64_t e = 0; e < n; ++e) {
    int32_t a;
    double lp, mg;
    ref_sample(p, seed, (uint32_t)e, 0, g, logits, &a, NULL, &lp, &mg);
    counts[a] += 1;
  }
}

/* First n normals (4 per env) of stream `stream`, env = 0 .. */
void ref_normals_many(uint64_t seed, uint32_t stream, int64_t n, double* out) {
  for (int64_t i = 0; i < n; i += 4) {
    double e[4];
    ref_normals(seed, (uint32_t)(i / 4), 0, 0, stream, 4, e);
    for (int j = 0; j < 4 && i + j < n; ++j) out[i + j] = e[j];
  }
}

/* Word 0 of n consecutive env counters of a stream. */
void ref_words_many(uint64_t seed, uint32_t stream, int64_t n, uint32_t* out) {
  for (int64_t i = 0; i < n; ++i) {
    uint32_t w[4];
    ref_draw(seed, (uint32_t)i, 0, 0, stream, 0, w);
    out[i] = w[0];
  }
}
