/*
 * msrl_learn_ref.c -- CPU oracle of the learner's policy update (next hot-path
 * row after rollout + GAE; no HIP path is checked against it yet).
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
 * bf16 rounding points in the forward pass).  In bf16 mode the derivative
 * treats every rounding as the identity (straight-through): dL/dW uses the
 * rounded layer input, dL/d(input) uses the rounded weight, nothing else is
 * rounded in the backward pass.  At rho exactly on a clip edge, or where both
 * branches of the min are equal, the unclipped branch gives the derivative.
 *
 * Adam (Kingma & Ba, 2015) with bias correction, step counter k >= 1:
 *   m <- b1 m + (1-b1) g;  v <- b2 v + (1-b2) g^2;
 *   theta <- theta - lr * (m / (1-b1^k)) / (sqrt(v / (1-b2^k)) + adam_eps)
 *
 * Pins (tests/test_oracle_learner.py): loss and every gradient against an
 * automatic-differentiation library on the same formulas (both distributions,
 * all clip regimes, bf16 straight-through), central finite differences of the
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
  int32_t hidden_layers; /* the learner is defined for two hidden layers only (0 or 2) */
} ref_policy_cfg;

typedef struct {
  double clip, vf_coef, ent_coef;
  double lr, beta1, beta2, adam_eps;
} ref_ppo_cfg;

double ref_bf16_round(double x); /* msrl_ref.c */
size_t ref_net_param_count(int in, int H, int out);

static double rnd(double x, int bf16) { return bf16 ? ref_bf16_round(x) : x; }

/* Forward pass of one in-H-H-out network on one row, keeping what the backward pass needs:
 * xin (rounded input), a1, a2 (tanh outputs, unrounded), y. */
static void net_forward(int in, int H, int out, const double* P, const double* x, int bf16,
                        double* xin, double* a1, double* a2, double* y) {
  const double* W1 = P;
  const double* b1 = W1 + (size_t)in * H;
  const double* W2 = b1 + H;
  const double* b2 = W2 + (size_t)H * H;
  const double* W3 = b2 + H;
  const double* b3 = W3 + (size_t)H * out;
  for (int i = 0; i < in; ++i) xin[i] = rnd(x[i], bf16);
  for (int o = 0; o < H; ++o) {
    double s = 0.0;
    for (int i = 0; i < in; ++i) s += xin[i] * rnd(W1[(size_t)i * H + o], bf16);
    a1[o] = tanh(s + b1[o]);
  }
  for (int o = 0; o < H; ++o) {
    double s = 0.0;
    for (int i = 0; i < H; ++i) s += rnd(a1[i], bf16) * rnd(W2[(size_t)i * H + o], bf16);
    a2[o] = tanh(s + b2[o]);
  }
  for (int o = 0; o < out; ++o) {
    double s = 0.0;
    for (int i = 0; i < H; ++i) s += rnd(a2[i], bf16) * rnd(W3[(size_t)i * out + o], bf16);
    y[o] = s + b3[o];
  }
}

/* Backward pass of one row: G += dL/dP given dy = dL/dy (straight-through across roundings). */
static void net_backward(int in, int H, int out, const double* P, int bf16, const double* xin,
                         const double* a1, const double* a2, const double* dy, double* G,
                         double* d1, double* d2) {
  const size_t oW1 = 0, ob1 = (size_t)in * H, oW2 = ob1 + H, ob2 = oW2 + (size_t)H * H,
               oW3 = ob2 + H, ob3 = oW3 + (size_t)H * out;
  /* layer 3 */
  for (int o = 0; o < out; ++o) G[ob3 + o] += dy[o];
  for (int i = 0; i < H; ++i) {
    double da = 0.0;
    const double in3 = rnd(a2[i], bf16);
    for (int o = 0; o < out; ++o) {
      G[oW3 + (size_t)i * out + o] += in3 * dy[o];
      da += rnd(P[oW3 + (size_t)i * out + o], bf16) * dy[o];
    }
    d2[i] = da * (1.0 - a2[i] * a2[i]); /* dL/dz2 */
  }
  /* layer 2 */
  for (int o = 0; o < H; ++o) G[ob2 + o] += d2[o];
  for (int i = 0; i < H; ++i) {
    double da = 0.0;
    const double in2 = rnd(a1[i], bf16);
    for (int o = 0; o < H; ++o) {
      G[oW2 + (size_t)i * H + o] += in2 * d2[o];
      da += rnd(P[oW2 + (size_t)i * H + o], bf16) * d2[o];
    }
    d1[i] = da * (1.0 - a1[i] * a1[i]); /* dL/dz1 */
  }
  /* layer 1 */
  for (int o = 0; o < H; ++o) G[ob1 + o] += d1[o];
  for (int i = 0; i < in; ++i)
    for (int o = 0; o < H; ++o) G[oW1 + (size_t)i * H + o] += xin[i] * d1[o];
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
  const size_t np_pi = ref_net_param_count(in, H, O), np_v = ref_net_param_count(in, H, 1);
  const double* Ppi = params;
  const double* Pv = params + np_pi;
  double* xin = (double*)malloc(sizeof(double) * (size_t)in);
  double* a1 = (double*)malloc(sizeof(double) * (size_t)H);
  double* a2 = (double*)malloc(sizeof(double) * (size_t)H);
  double* d1 = (double*)malloc(sizeof(double) * (size_t)H);
  double* d2 = (double*)malloc(sizeof(double) * (size_t)H);
  double* y = (double*)malloc(sizeof(double) * (size_t)O);
  double* dy = (double*)malloc(sizeof(double) * (size_t)O);
  if (grad) memset(grad, 0, sizeof(double) * (np_pi + np_v));
  double s_pi = 0.0, s_v = 0.0, s_h = 0.0, s_clip = 0.0, s_kl = 0.0;
  const double invR = R > 0 ? 1.0 / (double)R : 0.0;
  for (int64_t n = 0; n < R; ++n) {
    const double* x = obs + (size_t)n * in;
    /* ---- policy */
    net_forward(in, H, O, Ppi, x, bf, xin, a1, a2, y);
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
      net_backward(in, H, O, Ppi, bf, xin, a1, a2, dy, grad, d1, d2);
    }
    /* ---- value */
    double v;
    net_forward(in, H, 1, Pv, x, bf, xin, a1, a2, &v);
    const double err = v - ret[n];
    s_v += err * err;
    if (grad) {
      const double dv = c->vf_coef * 2.0 * err * invR;
      net_backward(in, H, 1, Pv, bf, xin, a1, a2, &dv, grad + np_pi, d1, d2);
    }
  }
  free(xin); free(a1); free(a2); free(d1); free(d2); free(y); free(dy);
  if (stats) {
    stats[0] = s_pi * invR;
    stats[1] = s_v * invR;
    stats[2] = s_h * invR;
    stats[3] = s_clip * invR;
    stats[4] = s_kl * invR;
  }
  return (s_pi + c->vf_coef * s_v - c->ent_coef * s_h) * invR;
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
 * consecutive blocks of rows (the last takes the remainder), one Adam step per block.
 * step_counter: Adam steps taken before this call (0 for fresh moments); returns the mean of the
 * minibatch losses (the listing's loss / iter, per minibatch).
 */
double ref_ppo_update(const ref_policy_cfg* p, const ref_ppo_cfg* c, double* params, double* m,
                      double* v, int64_t* step_counter, int64_t R, int iters, int minibatches,
                      const double* obs, const int32_t* actions_i, const double* actions_f,
                      const double* logp_old, const double* adv, const double* ret) {
  const size_t np = ref_net_param_count(p->in_dim, p->hidden, p->out_dim) +
                    ref_net_param_count(p->in_dim, p->hidden, 1);
  double* g = (double*)malloc(sizeof(double) * np);
  const int K = p->out_dim / 2;
  const int64_t block = R / minibatches;
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
