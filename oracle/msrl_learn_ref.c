/*
 * msrl_learn_ref.c -- CPU oracle of the learner's policy update (the next hot-path
 * row after rollout + GAE); the HIP entry points msrl_ppo_grad / msrl_adam_step /
 * msrl_ppo_update are checked against it.
 *
 * TEST INFRASTRUCTURE ONLY, like msrl_ref.c: plain scalar loops in double
 * precision, no code shared with the HIP sources.
 *
 * What is computed follows Listing 1 of the paper (section 3): after
 * discounted_reward() and gae(), Learner.learn calls
 * mappo_net_train(action, state, adv, r) `iter` times and averages the returned
 * loss.  The paper names the algorithm (multi-agent PPO) and fixes nothing else;
 * the definition used here is the clipped-surrogate objective of PPO with a
 * squared-error value loss and an entropy bonus, one Adam step per minibatch:
 *
 *   rho_n  = exp(logp_theta(a_n | s_n) - logp_old_n)
 *   Lpi_n  = -min(rho_n A_n, clip(rho_n, 1-eps, 1+eps) A_n)
 *   Lv_n   = (V_theta(s_n) - ret_n)^2
 *   L      = mean_n(Lpi_n + c_v Lv_n - c_e H_n),   H_n = entropy of pi_theta(.|s_n)
 *
 * with the policy and value networks of msrl_ref.c (same parameter layout, same
 * bf16 rounding points in the forward pass, any number of hidden layers).
 *
 * Centralised critic (multi-agent PPO, section 2.1 of the paper; value_in_dim =
 * G * in_dim): the rows come in groups of G consecutive rows, the agents of one
 * env at one step; the value network takes the group's rows one after the other
 * as one input and has one target per group, the return of the group's first row
 * (with a shared reward and a shared value every row of the group has the same).
 * The value term is then the mean over the R / G groups:
 *
 *   L = mean_n(Lpi_n - c_e H_n) + c_v mean_g (V_theta(s_gG .. s_gG+G-1) - ret_gG)^2
 *
 * In bf16 mode the derivative treats every rounding of the forward pass as the
 * identity (straight-through): dL/dW uses the rounded layer input, dL/d(input)
 * uses the rounded weight.  The paper fixes no precision for the update; the
 * reading taken for bf16 networks is that the backward contractions take bf16
 * operands just as the forward ones do.  So, in bf16 mode only:
 *   - dL/dy is rounded to bf16 where the loss produces it;
 *   - tanh' is 1 - a^2 with a the ROUNDED activation (the value the forward pass
 *     handed to the next layer);
 *   - every dL/d(pre-activation) = (sum_o W[i,o] d_o) (1 - a_i^2) is rounded to
 *     bf16 where it is produced; the sum itself is not rounded (it is an
 *     accumulator, fp32 in a kernel, double here);
 *   - weight gradients are sums over the rows of (rounded input) x (rounded d),
 *     bias gradients sums of the rounded d; the sums are not rounded.
 * At rho exactly on a clip edge, or where both branches of the min are equal, the
 * unclipped branch gives the derivative.
 *
 * Adam (Kingma & Ba, 2015) with bias correction, step counter k >= 1:
 *   m <- b1 m + (1-b1) g;  v <- b2 v + (1-b2) g^2;
 *   theta <- theta - lr * (m / (1-b1^k)) / (sqrt(v / (1-b2^k)) + adam_eps)
 *
 * Pins (tests/test_oracle_learner.py): loss and every gradient against an
 * automatic-differentiation library on the same formulas (both distributions,
 * all clip regimes; bf16: straight-through forward roundings, the backward
 * roundings as gradient hooks of that library, and the distance to the gradient
 * without backward roundings), central finite differences of the
 * loss, closed forms for all-zero parameters, exact zero policy gradient when
 * every row is clipped, Adam against its one- and two-step closed forms.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define REF_CATEGORICAL 0
#define REF_DIAG_GAUSSIAN 1

typedef struct {
  int32_t in_dim, hidden, out_dim;
  int32_t bf16;
  int32_t dist;
  int32_t hidden_layers; /* tanh layers in front of the output layer; 0 means 2 */
  int32_t value_in_dim;  /* 0 or in_dim: value net on the row; G * in_dim: centralised critic on groups of G rows */
} ref_policy_cfg;

typedef struct {
  double clip, vf_coef, ent_coef;
  double lr, beta1, beta2, adam_eps;
} ref_ppo_cfg;

double ref_bf16_round(double x); /* msrl_ref.c */
size_t ref_net_param_count(int in, int H, int out);
size_t ref_net_param_count_l(int in, int H, int out, int L);

static double rnd(double x, int bf16) { return bf16 ? ref_bf16_round(x) : x; }

/* Forward pass of one network with L tanh hidden layers of H units on one row (parameter layout
 * and rounding points of ref_mlp_l), keeping what the backward pass needs: xin (rounded input),
 * act[l] (tanh output of hidden layer l = 0 .. L-1, unrounded), y. */
static void net_forward(int in, int H, int out, int L, const double* P, const double* x, int bf16,
                        double* xin, double* act, double* y) {
  for (int i = 0; i < in; ++i) xin[i] = rnd(x[i], bf16);
  const double* W = P;
  const double* b = W + (size_t)in * H;
  for (int o = 0; o < H; ++o) {
    double s = 0.0;
    for (int i = 0; i < in; ++i) s += xin[i] * rnd(W[(size_t)i * H + o], bf16);
    act[o] = tanh(s + b[o]);
  }
  W = b + H;
  for (int l = 1; l < L; ++l) {
    b = W + (size_t)H * H;
    const double* ain = act + (size_t)(l - 1) * H;
    double* aout = act + (size_t)l * H;
    for (int o = 0; o < H; ++o) {
      double s = 0.0;
      for (int i = 0; i < H; ++i) s += rnd(ain[i], bf16) * rnd(W[(size_t)i * H + o], bf16);
      aout[o] = tanh(s + b[o]);
    }
    W = b + H;
  }
  b = W + (size_t)H * out;
  const double* alast = act + (size_t)(L - 1) * H;
  for (int o = 0; o < out; ++o) {
    double s = 0.0;
    for (int i = 0; i < H; ++i) s += rnd(alast[i], bf16) * rnd(W[(size_t)i * out + o], bf16);
    y[o] = s + b[o];
  }
}

/* Backward pass of one row: G += dL/dP given dy_in = dL/dy (straight-through across the roundings of
 * the forward pass; in bf16 mode dy and every dL/d(pre-activation) are rounded to bf16 and tanh' uses
 * the rounded activation, see the header).
 * delta: scratch [L, H] (dL/d pre-activation of every hidden layer). */
static void net_backward(int in, int H, int out, int L, const double* P, int bf16, const double* xin,
                         const double* act, const double* dy_in, double* G, double* delta) {
  double* dy = (double*)malloc(sizeof(double) * (size_t)out);
  for (int o = 0; o < out; ++o) dy[o] = rnd(dy_in[o], bf16);
  /* offsets of the layers' W inside the flat vector */
  const size_t first = (size_t)in * H + H, mid = (size_t)H * H + H;
  const size_t oWout = first + (size_t)(L - 1) * mid;
  /* output layer */
  {
    const double* alast = act + (size_t)(L - 1) * H;
    double* dl = delta + (size_t)(L - 1) * H;
    for (int o = 0; o < out; ++o) G[oWout + (size_t)H * out + o] += dy[o];
    for (int i = 0; i < H; ++i) {
      double da = 0.0;
      const double a_in = rnd(alast[i], bf16);
      for (int o = 0; o < out; ++o) {
        G[oWout + (size_t)i * out + o] += a_in * dy[o];
        da += rnd(P[oWout + (size_t)i * out + o], bf16) * dy[o];
      }
      dl[i] = rnd(da * (1.0 - a_in * a_in), bf16);
    }
  }
  /* hidden layers L-1 .. 1 (inputs: the hidden layer before) */
  for (int l = L - 1; l >= 1; --l) {
    const size_t oW = first + (size_t)(l - 1) * mid, ob = oW + (size_t)H * H;
    const double* ain = act + (size_t)(l - 1) * H;
    const double* dl = delta + (size_t)l * H;
    double* dprev = delta + (size_t)(l - 1) * H;
    for (int o = 0; o < H; ++o) G[ob + o] += dl[o];
    for (int i = 0; i < H; ++i) {
      double da = 0.0;
      const double a_in = rnd(ain[i], bf16);
      for (int o = 0; o < H; ++o) {
        G[oW + (size_t)i * H + o] += a_in * dl[o];
        da += rnd(P[oW + (size_t)i * H + o], bf16) * dl[o];
      }
      dprev[i] = rnd(da * (1.0 - a_in * a_in), bf16);
    }
  }
  /* layer 1 */
  for (int o = 0; o < H; ++o) G[(size_t)in * H + o] += delta[o];
  for (int i = 0; i < in; ++i)
    for (int o = 0; o < H; ++o) G[(size_t)i * H + o] += xin[i] * delta[o];
  free(dy);
}

/*
 * Loss of R rows and, if grad != NULL, its gradient with respect to params
 * (policy net then value net, layout of msrl_ref.c); grad is overwritten.
 * actions_i: int32 [R] (categorical) or actions_f: double [R, out_dim/2] (Gaussian).
 * stats (may be NULL): [0] mean policy term, [1] mean value term (without c_v),
 * [2] mean entropy, [3] fraction of rows whose clipped branch is active,
 * [4] mean (logp_old - logp_new).
 */
double ref_ppo_loss(const ref_policy_cfg* p, const ref_ppo_cfg* c, const double* params, int64_t R,
                    const double* obs, const int32_t* actions_i, const double* actions_f,
                    const double* logp_old, const double* adv, const double* ret, double* grad,
                    double* stats) {
  const int in = p->in_dim, H = p->hidden, O = p->out_dim, bf = p->bf16;
  const int L = p->hidden_layers > 0 ? p->hidden_layers : 2;
  const int in_v = p->value_in_dim > 0 ? p->value_in_dim : in; /* input width of the value net */
  const int G = in_v / in;                                     /* rows per value-net input */
  const size_t np_pi = ref_net_param_count_l(in, H, O, L), np_v = ref_net_param_count_l(in_v, H, 1, L);
  const double* Ppi = params;
  const double* Pv = params + np_pi;
  double* xin = (double*)malloc(sizeof(double) * (size_t)in_v);
  double* act = (double*)malloc(sizeof(double) * (size_t)H * L);
  double* delta = (double*)malloc(sizeof(double) * (size_t)H * L);
  double* y = (double*)malloc(sizeof(double) * (size_t)O);
  double* dy = (double*)malloc(sizeof(double) * (size_t)O);
  if (grad) memset(grad, 0, sizeof(double) * (np_pi + np_v));
  double s_pi = 0.0, s_v = 0.0, s_h = 0.0, s_clip = 0.0, s_kl = 0.0;
  const double invR = R > 0 ? 1.0 / (double)R : 0.0;
  for (int64_t n = 0; n < R; ++n) {
    const double* x = obs + (size_t)n * in;
    /* ---- policy */
    net_forward(in, H, O, L, Ppi, x, bf, xin, act, y);
    double logp, ent;
    if (p->dist == REF_CATEGORICAL) {
      double mx = y[0], z = 0.0;
      for (int k = 1; k < O; ++k)
        if (y[k] > mx) mx = y[k];
      for (int k = 0; k < O; ++k) z += exp(y[k] - mx);
      const double lse = mx + log(z);
      const int a = actions_i[n];
      logp = y[a] - lse;
      ent = 0.0;
      for (int k = 0; k < O; ++k) {
        const double lp = y[k] - lse;
        ent -= exp(lp) * lp;
      }
      /* d logp / dy_k = [k == a] - p_k;  dH / dy_k = -p_k (log p_k + H) */
      for (int k = 0; k < O; ++k) {
        const double pk = exp(y[k] - lse);
        dy[k] = (k == a ? 1.0 : 0.0) - pk; /* holds dlogp/dy for now */
      }
    } else {
      const int K = O / 2;
      logp = 0.0;
      ent = 0.0;
      for (int d = 0; d < K; ++d) {
        const double mu = y[d], ls = y[K + d], sg = exp(ls);
        const double e = (actions_f[(size_t)n * K + d] - mu) / sg;
        logp += -0.5 * e * e - ls - 0.91893853320467274178;
        ent += ls + 1.4189385332046727418; /* 1/2 ln(2 pi e) */
        dy[d] = e / sg;                    /* dlogp/dmu */
        dy[K + d] = e * e - 1.0;           /* dlogp/dlogstd */
      }
    }
    const double rho = exp(logp - logp_old[n]);
    const double A = adv[n];
    double rc = rho;
    if (rc < 1.0 - c->clip) rc = 1.0 - c->clip;
    if (rc > 1.0 + c->clip) rc = 1.0 + c->clip;
    const double un = rho * A, cl = rc * A;
    const int clipped = cl < un; /* the clipped branch is the strict minimum */
    s_pi += -(clipped ? cl : un);
    s_h += ent;
    s_clip += clipped ? 1.0 : 0.0;
    s_kl += logp_old[n] - logp;
    if (grad) {
      /* dL/dlogp = -A rho if the unclipped branch is active, else 0 */
      const double gl = clipped ? 0.0 : -A * rho;
      if (p->dist == REF_CATEGORICAL) {
        double mx = y[0], z = 0.0;
        for (int k = 1; k < O; ++k)
          if (y[k] > mx) mx = y[k];
        for (int k = 0; k < O; ++k) z += exp(y[k] - mx);
        const double lse = mx + log(z);
        for (int k = 0; k < O; ++k) {
          const double lp = y[k] - lse, pk = exp(lp);
          const double dH = -pk * (lp + ent);
          dy[k] = (gl * dy[k] - c->ent_coef * dH) * invR;
        }
      } else {
        const int K = O / 2;
        for (int d = 0; d < K; ++d) {
          dy[d] = gl * dy[d] * invR;
          dy[K + d] = (gl * dy[K + d] - c->ent_coef * 1.0) * invR;
        }
      }
      net_backward(in, H, O, L, Ppi, bf, xin, act, dy, grad, delta);
    }
  }
  /* ---- value: one evaluation per group of G rows (G = 1: per row) */
  const int64_t Rg = R / G;
  const double invRg = Rg > 0 ? 1.0 / (double)Rg : 0.0;
  for (int64_t g = 0; g < Rg; ++g) {
    double v;
    net_forward(in_v, H, 1, L, Pv, obs + (size_t)g * in_v, bf, xin, act, &v);
    const double err = v - ret[g * G];
    s_v += err * err;
    if (grad) {
      const double dv = c->vf_coef * 2.0 * err * invRg;
      net_backward(in_v, H, 1, L, Pv, bf, xin, act, &dv, grad + np_pi, delta);
    }
  }
  free(xin); free(act); free(delta); free(y); free(dy);
  if (stats) {
    stats[0] = s_pi * invR;
    stats[1] = s_v * invRg;
    stats[2] = s_h * invR;
    stats[3] = s_clip * invR;
    stats[4] = s_kl * invR;
  }
  return (s_pi - c->ent_coef * s_h) * invR + c->vf_coef * s_v * invRg;
}

/* One Adam step on n parameters; k is the 1-based step counter of this step. */
void ref_adam_step(const ref_ppo_cfg* c, double* params, double* m, double* v, const double* grad,
                   size_t n, int64_t k) {
  const double c1 = 1.0 - pow(c->beta1, (double)k), c2 = 1.0 - pow(c->beta2, (double)k);
  for (size_t i = 0; i < n; ++i) {
    m[i] = c->beta1 * m[i] + (1.0 - c->beta1) * grad[i];
    v[i] = c->beta2 * v[i] + (1.0 - c->beta2) * grad[i] * grad[i];
    params[i] -= c->lr * (m[i] / c1) / (sqrt(v[i] / c2) + c->adam_eps);
  }
}

/*
 * Learner.learn's training loop: `iters` passes over the R rows, each split into `minibatches`
 * consecutive blocks of rows (the last takes the remainder; with a centralised critic the blocks
 * hold whole groups), one Adam step per block.
 * step_counter: Adam steps taken before this call (0 for fresh moments); returns the mean of the
 * minibatch losses (the listing's loss / iter, per minibatch).
 */
double ref_ppo_update(const ref_policy_cfg* p, const ref_ppo_cfg* c, double* params, double* m,
                      double* v, int64_t* step_counter, int64_t R, int iters, int minibatches,
                      const double* obs, const int32_t* actions_i, const double* actions_f,
                      const double* logp_old, const double* adv, const double* ret) {
  const int L = p->hidden_layers > 0 ? p->hidden_layers : 2;
  const size_t np = ref_net_param_count_l(p->in_dim, p->hidden, p->out_dim, L) +
                    ref_net_param_count_l(p->value_in_dim > 0 ? p->value_in_dim : p->in_dim, p->hidden, 1, L);
  double* g = (double*)malloc(sizeof(double) * np);
  const int K = p->out_dim / 2;
  const int G = p->value_in_dim > p->in_dim ? p->value_in_dim / p->in_dim : 1;
  const int64_t block = R / minibatches / G * G; /* whole groups of rows (centralised critic) */
  double total = 0.0;
  for (int it = 0; it < iters; ++it)
    for (int b = 0; b < minibatches; ++b) {
      const int64_t r0 = (int64_t)b * block, r1 = b == minibatches - 1 ? R : r0 + block;
      total += ref_ppo_loss(p, c, params, r1 - r0, obs + (size_t)r0 * p->in_dim,
                            actions_i ? actions_i + r0 : NULL,
                            actions_f ? actions_f + (size_t)r0 * K : NULL, logp_old + r0, adv + r0,
                            ret + r0, g, NULL);
      *step_counter += 1;
      ref_adam_step(c, params, m, v, g, np, *step_counter);
    }
  free(g);
  return total / ((double)iters * minibatches);
}
