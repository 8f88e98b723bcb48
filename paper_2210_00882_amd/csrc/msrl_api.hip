// C ABI of the library (include/msrl.h): argument checks, state ownership,
// kernel selection and launches.  All arithmetic of the path runs in the HIP
// kernels; nothing here computes on the host.
#include "../../include/msrl.h"

#include <hip/hip_runtime.h>

#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "dev_common.h"
#include "packed.h"
#include "api_common.h"
#include "registry.h"
#include "tag_kernels.h"

namespace msrl {
hipError_t launch_pack(const PackJobs& jobs, hipStream_t stream);
hipError_t launch_gae(const float* rewards, const float* values, const uint8_t* dones, int T,
                      int64_t M, float gamma, float lambda, float* adv, float* ret,
                      hipStream_t stream);
}  // namespace msrl

using namespace msrl;

struct msrl_state {
  msrl_env_cfg env;
  msrl_policy_cfg pol;
  uint64_t seed;
  int device;
  int state_size;        // floats per env
  float* env_state;      // device [E, S]
  int64_t* g;            // device [E]
  uint8_t* packed;       // device, two packed networks
  uint8_t* dyn;          // device, lingauss dynamics tiles
  float* dyn_src;        // device copy of A then B (row-major), source of dyn
  NetLayout layout;
  NetLayout critic_layout;  // centralised critic: its image follows the policy network's in `packed`
  bool central;
  KernelEntry kernel;
  int cus;               // compute units of the device
  int in_used;           // leading observation features that can be non-zero (inputs of layer 1)
  int tag_tiles;         // pursuit env: 32-env tiles per workgroup (1 or 4)
  bool packed_valid;     // `packed` holds the image of the parameters of an earlier call
};

namespace {
thread_local char g_err[512] = "";
}

namespace msrl {
int fail(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}
}  // namespace msrl

namespace {

#define HIP_TRY(expr)                                                                       \
  do {                                                                                      \
    hipError_t e_ = (expr);                                                                 \
    if (e_ != hipSuccess)                                                                   \
      return fail(e_ == hipErrorOutOfMemory ? MSRL_ENOMEM : MSRL_EDEVICE, "%s failed: %s",  \
                  #expr, hipGetErrorString(e_));                                            \
  } while (0)

// the compiled rollout kernels (built once; find_kernel sits behind the per-step calls too)
const std::vector<KernelEntry>& all_kernels() {
  static const std::vector<KernelEntry> table = [] {
    std::vector<KernelEntry> t;
#define MSRL_CALL_FAMILY(NAME, N0, N1, H, BF16) particle_family_##NAME(t);
    MSRL_PARTICLE_FAMILIES(MSRL_CALL_FAMILY)
#undef MSRL_CALL_FAMILY
    const KernelEntry more[] = {entry_l17_6_h256(), entry_l17_6_h256_act(), entry_l17_6_h256_step(),
                                entry_l17_6_h256_deep(), entry_l17_6_h256_act_deep(),
                                entry_p10_h256_bf16_env(), entry_p10_h256_bf16_mlp(), entry_p10_h256_bf16_clocks(),
                                entry_p3_h64_f32_env()};
    t.insert(t.end(), more, more + sizeof(more) / sizeof(more[0]));
    return t;
  }();
  return table;
}

bool valid_policy(const msrl_policy_cfg* p) {
  return p && p->in_dim >= 1 && p->hidden >= 1 && p->out_dim >= 1 &&
         (p->dtype == MSRL_F32 || p->dtype == MSRL_BF16) &&
         (p->dist == MSRL_CATEGORICAL || p->dist == MSRL_DIAG_GAUSSIAN) &&
         (p->hidden_layers == 0 || (p->hidden_layers >= 2 && p->hidden_layers <= 8)) &&
         (p->roles >= 0 && p->roles <= 2) && p->value_in_dim >= 0;
}

// input width of the value network; wider than the policy's: a centralised critic on the joint observation
int value_in_of(const msrl_policy_cfg& p) { return p.value_in_dim > 0 ? p.value_in_dim : p.in_dim; }
bool central_of(const msrl_policy_cfg& p) { return value_in_of(p) != p.in_dim; }

int roles_of(const msrl_policy_cfg& p) { return p.roles == 0 ? 1 : p.roles; }

int layers_of(const msrl_policy_cfg& p) { return p.hidden_layers == 0 ? 2 : p.hidden_layers; }

bool valid_env_shape(const msrl_env_cfg* e) {
  if (!e || e->num_envs < 1 || e->num_agents < 1 || e->obs_dim < 1 || e->episode_len < 1) return false;
  if (e->kind == MSRL_ENV_PARTICLE)
    return e->num_landmarks >= 0 &&
           e->obs_dim == 4 + 2 * e->num_landmarks + 4 * (e->num_agents - 1);
  if (e->kind == MSRL_ENV_LINGAUSS)
    return e->num_agents == 1 && e->num_landmarks == 0 && e->act_dim >= 1;
  if (e->kind == MSRL_ENV_TAG)
    return e->num_landmarks >= 0 && e->num_chasers >= 1 && e->num_chasers < e->num_agents &&
           e->obs_dim == 4 + 2 * e->num_landmarks + 4 * (e->num_agents - 1) && e->contact_margin > 0.0f;
  return false;
}

// Pursuit env: 32-env tiles per workgroup.  Four tiles (16 waves behind one copy of the weights in LDS,
// four waves per SIMD) once that still gives most compute units a workgroup, one tile (more, smaller
// workgroups, two per compute unit) below.
// (four tiles x agents must fit the 16 waves of a workgroup: at most 4 agents per env.)
int choose_tag_tiles(int num_envs, int num_agents, int cus) {
  return num_agents * 4 <= 16 && (int64_t)(num_envs / 128) * 8 >= (int64_t)cus * 5 ? 4 : 1;
}

size_t net_params(int in, int h, int out, int layers) {
  return (size_t)in * h + h + (size_t)(layers - 1) * ((size_t)h * h + h) + (size_t)h * out + out;
}

// Initial state of episode 0: one thread per (env, entity).
__global__ void init_state_kernel(int kind, int E, int N, int L, int D, uint32_t seed_lo,
                                  uint32_t seed_hi, float* env_state, int64_t* g) {
  const int64_t tid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (kind == MSRL_ENV_PARTICLE) {
    const int per = N + L, S = 4 * N + 2 * L;
    if (tid >= (int64_t)E * per) return;
    const int env = (int)(tid / per), ent = (int)(tid % per);
    const Words4 w = draw(seed_lo, seed_hi, (uint32_t)env, (uint32_t)ent, 0, 1, 0);
    const float x = 2.0f * u01(w.w[0]) - 1.0f, y = 2.0f * u01(w.w[1]) - 1.0f;
    float* es = env_state + (size_t)env * S;
    if (ent < N) {
      es[4 * ent] = x;
      es[4 * ent + 1] = y;
      es[4 * ent + 2] = 0.0f;
      es[4 * ent + 3] = 0.0f;
    } else {
      es[4 * N + 2 * (ent - N)] = x;
      es[4 * N + 2 * (ent - N) + 1] = y;
    }
    if (ent == 0) g[env] = 0;
  } else {
    const int blocks = (D + 3) / 4;
    if (tid >= (int64_t)E * blocks) return;
    const int env = (int)(tid / blocks), b = (int)(tid % blocks);
    float e[4];
    normals4(seed_lo, seed_hi, (uint32_t)env, 0, 0, 1, (uint32_t)b, e);
    for (int c = 0; c < 4; ++c)
      if (4 * b + c < D) env_state[(size_t)env * D + 4 * b + c] = e[c];
    if (b == 0) g[env] = 0;
  }
}

PackJob weight_job(const void* src, void* dst, bool bf16, int n_in, int n_out, int nuc, int kt,
                   int in_map, int out_map, int gauss_k) {
  PackJob j;
  memset(&j, 0, sizeof(j));
  j.src = src; j.dst = dst; j.src_bf16 = bf16; j.is_bias = 0;
  j.n_in = n_in; j.n_out = n_out; j.src_out_major = 0;
  j.nuc = nuc; j.kt = kt; j.in_map = in_map; j.out_map = out_map; j.gauss_k = gauss_k;
  j.group = kt; j.chunk_stride = kt; j.slot_base = 0;  // plain (uc major, kt minor) order
  j.scale = 1.0f;
  return j;
}

PackJob bias_job(const void* src, void* dst, bool bf16, int n_out, int nuc, int out_map, int gauss_k) {
  PackJob j;
  memset(&j, 0, sizeof(j));
  j.src = src; j.dst = dst; j.src_bf16 = bf16; j.is_bias = 1;
  j.n_out = n_out; j.nuc = nuc; j.out_map = out_map; j.gauss_k = gauss_k;
  return j;
}

// Enqueue the re-ordering of the caller's parameter buffer into st->packed.
int pack_params(msrl_state* st, const void* params, hipStream_t stream) {
  const msrl_policy_cfg& p = st->pol;
  const bool bf16 = p.dtype == MSRL_BF16;
  const size_t esz = bf16 ? 2 : 4;
  const int in_map1 = st->env.kind == MSRL_ENV_LINGAUSS ? IN_CHAIN : (bf16 ? IN_LINEAR16 : IN_PAIRS);
  PackJobs jobs;
  jobs.n = 0;
  const uint8_t* src = (const uint8_t*)params;
  for (int net = 0; net < 2 * roles_of(p); ++net) {  // per role: policy, value
    const int out = net % 2 == 0 ? p.out_dim : 1;
    const int out_map = (net % 2 == 0 && p.dist == MSRL_DIAG_GAUSSIAN) ? OUT_GAUSS : OUT_NATURAL;
    const int gk = p.out_dim / 2;
    // a centralised critic has a layout of its own (more layer-1 tiles) behind the policy network
    const bool joint = st->central && net == 1;
    const NetLayout& L = joint ? st->critic_layout : st->layout;
    const int in_rows = net % 2 == 1 ? value_in_of(p) : p.in_dim;
    // joint observation: per agent a block of whole layer-1 tiles, the row's non-zero prefix at its start
    const int block = tiles_for_inputs(st->in_used + 1, bf16) * (bf16 ? 16 : 8);
    const int in_used = joint ? st->env.num_agents * block : st->in_used;
    uint8_t* dst = st->packed + (size_t)net * st->layout.bytes;
    const int layers = layers_of(p);
    const size_t hh = (size_t)p.hidden * p.hidden * esz, hb = (size_t)p.hidden * esz;
    const uint8_t* W1 = src;
    const uint8_t* b1 = W1 + (size_t)in_rows * p.hidden * esz;
    const uint8_t* Wmid = b1 + hb;                                  // hidden layers 2 .. layers-1: W b each
    const uint8_t* W2 = Wmid + (size_t)(layers - 2) * (hh + hb);   // the last hidden layer
    const uint8_t* b2 = W2 + hh;
    const uint8_t* W3 = b2 + hb;
    const uint8_t* b3 = W3 + (size_t)p.hidden * out * esz;
    // only the inputs that can be non-zero are packed (a prefix of the rows of W1)
    PackJob j1 = weight_job(W1, dst + L.w1, bf16, in_used, p.hidden, L.nuc, L.kt1, in_map1, OUT_NATURAL, 0);
    // fp32 hidden layers are stored times 2 log2(e): the kernels' tanh then starts at the exp2 (dev_common.h)
    const float hidden_scale = bf16 ? 1.0f : TANH_PRESCALE;
    j1.scale = hidden_scale;
    j1.bias = b1;  // the bias is the input after them; the kernels feed 1 there
    j1.bias_index = joint ? st->in_used : in_used;  // (joint: in the padding of the first agent's block)
    if (joint) {
      j1.in_block = block;
      j1.in_block_used = st->in_used;
      j1.in_block_stride = p.in_dim;
    }
    jobs.job[jobs.n++] = j1;
    // chunk blocks of the hidden layers before the last one: kt2 tiles of the chunk and its bias tile
    for (int l = 0; l < layers - 2; ++l) {
      const uint8_t* Wl = Wmid + (size_t)l * (hh + hb);
      PackJob jm = weight_job(Wl, dst + L.chunks + (size_t)l * L.nuc * L.chunk_bytes, bf16, p.hidden, p.hidden, L.nuc,
                              L.kt2 + 1, IN_CHAIN, OUT_NATURAL, 0);
      jm.scale = hidden_scale;
      jm.bias = Wl + hh;
      jm.bias_index = p.hidden;
      jm.chunk_stride = L.chunk_tiles;
      jobs.job[jobs.n++] = jm;
    }
    // chunk block uc of the last hidden layer: kt2 tiles of chunk uc, its bias tile, the tpc layer-3
    // tiles fed by chunk uc-1, the tpc layer-3 tiles fed by chunk uc
    uint8_t* last = dst + L.chunks + (size_t)(layers - 2) * L.nuc * L.chunk_bytes;
    PackJob j2 = weight_job(W2, last, bf16, p.hidden, p.hidden, L.nuc, L.kt2 + 1, IN_CHAIN, OUT_NATURAL, 0);
    j2.scale = hidden_scale;
    j2.bias = b2;
    j2.bias_index = p.hidden;
    j2.chunk_stride = L.chunk_tiles;
    jobs.job[jobs.n++] = j2;
    PackJob j3 = weight_job(W3, last, bf16, p.hidden, out, 1, L.kt2, IN_CHAIN, out_map, gk);
    j3.group = L.tpc;
    j3.chunk_stride = L.chunk_tiles;
    j3.slot_base = L.kt2 + 1 + L.tpc;  // own chunk's copy
    jobs.job[jobs.n++] = j3;
    if (L.nuc > 1) {
      PackJob j3b = j3;               // copy for the following chunk's stage: tiles of chunks 0 .. nuc-2
      j3b.dst = last + L.chunk_bytes;
      j3b.kt = L.kt2 - L.tpc;
      j3b.slot_base = L.kt2 + 1;
      jobs.job[jobs.n++] = j3b;
    }
    jobs.job[jobs.n++] = bias_job(b3, dst + L.b3, bf16, out, 1, out_map, gk);
    src = b3 + (size_t)out * esz;
  }
  HIP_TRY(launch_pack(jobs, stream));
  return MSRL_OK;
}

int check_traj(const msrl_state* st, const msrl_traj* out, bool need_gae) {
  if (!out) return fail(MSRL_EINVAL, "trajectory struct is NULL");
  if (!out->obs || !out->actions || !out->logp || !out->rewards || !out->dones || !out->values)
    return fail(MSRL_EINVAL, "a required trajectory pointer is NULL");
  if (need_gae && (!out->adv || !out->ret)) return fail(MSRL_EINVAL, "adv / ret pointer is NULL");
  (void)st;
  return MSRL_OK;
}

// the compiled kernel for this state's configuration and the given phase variant, or null
// (several instances of a phase differ in the row blocks per workgroup: pick < 0 takes the one with the fewest,
// pick > 0 the one with the most, 0 the first)
bool find_kernel(const msrl_env_cfg& env, const msrl_policy_cfg& pol, int phase, KernelEntry* out, int pick = 0) {
  const bool bf16 = pol.dtype == MSRL_BF16;
  // networks with more than two hidden layers, and a centralised critic, have kernels of their own for the
  // full rollout and for the actor fragment, and no measurement variants; the environment-only variant
  // runs no network
  if (layers_of(pol) > 2) {
    if (central_of(pol)) return false;
    if (phase == PHASE_ALL) phase = PHASE_DEEP;
    else if (phase == PHASE_ACT) phase = PHASE_ACT_DEEP;
    else if (phase != PHASE_STEP) return false;
  } else if (central_of(pol)) {
    if (phase == PHASE_ALL) phase = PHASE_CENTRAL;
    else if (phase == PHASE_ACT) phase = PHASE_ACT_CENTRAL;
    else if (phase != PHASE_STEP) return false;
  }
  bool found = false;
  for (const KernelEntry& k : all_kernels()) {
    if (k.phase != phase || k.kind != env.kind || k.hidden != pol.hidden || (k.bf16 != 0) != bf16) continue;

    if (env.kind == MSRL_ENV_PARTICLE) {
      if (k.n != env.num_agents || env.num_landmarks != env.num_agents) continue;
    } else {
      if (k.n != env.obs_dim || k.k != env.act_dim) continue;
    }
    if (!found || (pick < 0 && k.row_waves < out->row_waves) || (pick > 0 && k.row_waves > out->row_waves)) *out = k;
    found = true;
    if (pick == 0) break;
  }
  return found;
}

// Envs per workgroup of a launch of `kernel`.  Every workgroup runs all T steps, so the launch takes
// ceil(blocks / CUs) rounds.  The block is shrunk to the smallest size that needs no more rounds than
// the largest one: equal work per workgroup instead of a short last round.  (Rounds are counted per CU
// even where several workgroups fit one: they would share its SIMDs, and a wave with fewer rows costs
// the same.)  Computed per launch: the kernels of a state (full rollout, actor fragment, env step,
// measurement variants) differ in the row blocks a workgroup holds.
int envs_per_block(const KernelEntry& kernel, int64_t num_envs, int cus) {
  const int64_t max_epb = (int64_t)kernel.envs_per_wave * (kernel.row_waves ? kernel.row_waves : kernel.waves);
  const int64_t blocks_max = (num_envs + max_epb - 1) / max_epb;
  const int64_t rounds = (blocks_max + cus - 1) / cus;
  int64_t epb = (num_envs + rounds * cus - 1) / (rounds * cus);
  if (epb < 1) epb = 1;
  if (epb > max_epb) epb = max_epb;
  return (int)epb;
}

// params may be null for the variants that run no network; obs_in / actions_in feed the
// step-granular variants
int enqueue_rollout(msrl_state* st, const KernelEntry& kernel, const void* params, int32_t T, msrl_traj* out,
                    hipStream_t stream, const float* obs_in = nullptr, const void* actions_in = nullptr) {
  if (params) {
    int rc = pack_params(st, params, stream);
    if (rc != MSRL_OK) return rc;
    st->packed_valid = true;
  }
  RolloutArgs a;
  memset(&a, 0, sizeof(a));
  a.env_state = st->env_state;
  a.g = st->g;
  a.packed = st->packed;
  a.dyn = st->dyn;
  a.E = st->env.num_envs;
  a.T = T;
  a.ep = st->env.episode_len;
  a.dt = st->env.dt;
  a.keep = 1.0f - st->env.damping;
  a.fdt = st->env.force * st->env.dt;
  a.coll2 = (2.0f * st->env.radius) * (2.0f * st->env.radius);
  a.noise_std = st->env.noise_std;
  a.act_cost = st->env.act_cost;
  a.seed_lo = (uint32_t)st->seed;
  a.seed_hi = (uint32_t)(st->seed >> 32);
  a.obs = out->obs;
  a.actions = out->actions;
  a.logp = out->logp;
  a.rewards = out->rewards;
  a.dones = out->dones;
  a.values = out->values;
  a.logits = out->logits;
  a.M = (int64_t)st->env.num_envs * st->env.num_agents;
  a.obs_in = obs_in;
  a.actions_in = actions_in;
  a.envs_per_block = envs_per_block(kernel, st->env.num_envs, st->cus);
  a.layers = layers_of(st->pol);
  a.critic = st->central ? st->packed + st->layout.bytes : nullptr;
  int64_t blocks = ((int64_t)a.E + a.envs_per_block - 1) / a.envs_per_block;
  // (the actor fragment's kernel walks over the row blocks itself: one workgroup per compute unit at most)
  if (kernel.kind == MSRL_ENV_PARTICLE && kernel.phase == PHASE_ACT && blocks > st->cus) blocks = st->cus;
  void* args[] = {&a};
  HIP_TRY(hipLaunchKernel(kernel.fn, dim3((unsigned)blocks), dim3(64 * kernel.waves), args, 0, stream));
  return MSRL_OK;
}

// the pursuit env has a kernel family of its own (tag_kernels.h)
int enqueue_tag(msrl_state* st, const void* params, int32_t T, msrl_traj* out, hipStream_t stream,
                int phase = TAG_ALL, const float* obs_in = nullptr, const void* actions_in = nullptr) {
  if (params) {  // (the environment-only variant runs no network)
    int rc = pack_params(st, params, stream);
    if (rc != MSRL_OK) return rc;
    st->packed_valid = true;
  }
  const msrl_env_cfg& e = st->env;
  TagArgs a;
  memset(&a, 0, sizeof(a));
  a.env_state = st->env_state;
  a.g = st->g;
  a.packed = st->packed;
  a.E = e.num_envs;
  a.T = T;
  a.ep = e.episode_len;
  a.dt = e.dt;
  a.keep = 1.0f - e.damping;
  a.accel[0] = e.accel_c; a.accel[1] = e.accel_r;
  a.vmax[0] = e.vmax_c; a.vmax[1] = e.vmax_r;
  a.rad[0] = e.radius_c; a.rad[1] = e.radius_r;
  a.cforce = e.contact_force;
  a.cmargin = e.contact_margin;
  a.seed_lo = (uint32_t)st->seed;
  a.seed_hi = (uint32_t)(st->seed >> 32);
  a.obs = out->obs;
  a.actions = (int32_t*)out->actions;
  a.logp = out->logp;
  a.rewards = out->rewards;
  a.dones = out->dones;
  a.values = out->values;
  a.logits = out->logits;
  a.M = (int64_t)e.num_envs * e.num_agents;
  a.obs_in = obs_in;
  a.actions_in = (const int32_t*)actions_in;
  HIP_TRY(launch_tag_rollout(e.num_chasers, e.num_agents - e.num_chasers, e.num_landmarks, st->pol.hidden,
                             st->pol.dtype == MSRL_BF16, st->tag_tiles, phase, a, stream));
  return MSRL_OK;
}

// Host-side set-up of a state for (env, policy): argument checks, kernel selection, launch shape and
// the layout of the packed parameters.  Touches no device memory: every device pointer of *st is
// left null and *packed_bytes says how large the packed image is.  `who` names the caller in messages.
int configure_state(msrl_state* st, const char* who, const msrl_env_cfg* env, const msrl_policy_cfg* policy,
                    uint64_t seed, size_t* packed_bytes) {
  if (!valid_env_shape(env))
    return fail(MSRL_EINVAL, "%s: inconsistent environment configuration "
                             "(kind %d, envs %d, agents %d, landmarks %d, obs_dim %d, episode_len %d)",
                who, env->kind, env->num_envs, env->num_agents, env->num_landmarks, env->obs_dim, env->episode_len);
  if (!valid_policy(policy)) return fail(MSRL_EINVAL, "%s: invalid policy configuration", who);
  if (policy->in_dim != env->obs_dim)
    return fail(MSRL_EINVAL, "%s: policy in_dim %d != obs_dim %d", who, policy->in_dim, env->obs_dim);
  if (roles_of(*policy) != (env->kind == MSRL_ENV_TAG ? 2 : 1))
    return fail(MSRL_EINVAL, "%s: the pursuit env takes two parameter sets (roles = 2), the others one", who);
  if (env->kind == MSRL_ENV_PARTICLE || env->kind == MSRL_ENV_TAG) {
    if (policy->dist != MSRL_CATEGORICAL || policy->out_dim != 5)
      return fail(MSRL_EINVAL, "%s: the particle envs need a categorical policy with out_dim 5", who);
  } else {
    if (policy->dist != MSRL_DIAG_GAUSSIAN || policy->out_dim != 2 * env->act_dim)
      return fail(MSRL_EINVAL, "%s: the lingauss env needs a Gaussian policy with out_dim 2*act_dim", who);
  }
  if (central_of(*policy) &&
      (env->kind != MSRL_ENV_PARTICLE || policy->value_in_dim != env->num_agents * policy->in_dim ||
       layers_of(*policy) != 2))
    return fail(MSRL_EINVAL, "%s: value_in_dim %d: a centralised critic takes num_agents * in_dim = %d "
                             "inputs (particle env, two hidden layers)",
                who, policy->value_in_dim, env->num_agents * policy->in_dim);
  if (env->tag_tiles != 0 && (env->kind != MSRL_ENV_TAG || (env->tag_tiles != 1 && env->tag_tiles != 4) ||
                              (env->tag_tiles == 4 && env->num_agents > 4)))
    return fail(MSRL_EINVAL, "%s: tag_tiles %d (0 lets the library choose; 1, or 4 with at most 4 agents per env; "
                             "pursuit env only)", who, env->tag_tiles);
  if (env->wave_roles != 0 && (env->kind != MSRL_ENV_PARTICLE || env->wave_roles < 0 || env->wave_roles > 2))
    return fail(MSRL_EINVAL, "%s: wave_roles %d (0 lets the library choose, 1 or 2 waves per row block; "
                             "particle env only)", who, env->wave_roles);
  // kernel selection
  KernelEntry found;
  memset(&found, 0, sizeof(found));
  found.envs_per_wave = 32;
  found.waves = 1;
  const bool ok = env->kind == MSRL_ENV_TAG
                      ? layers_of(*policy) == 2 &&
                            tag_rollout_compiled(env->num_chasers, env->num_agents - env->num_chasers,
                                                 env->num_landmarks, policy->hidden, policy->dtype == MSRL_BF16,
                                                 env->tag_tiles == 4 ? 4 : 1)
                      : find_kernel(*env, *policy, PHASE_ALL, &found);
  if (!ok)
    return fail(MSRL_EUNSUPPORTED,
                "%s: no kernel compiled for kind %d, agents %d, landmarks %d, obs_dim %d, "
                "act_dim %d, hidden %d, dtype %d",
                who, env->kind, env->num_agents, env->num_landmarks, env->obs_dim, env->act_dim, policy->hidden,
                policy->dtype);

  int cus = 256;
  int device = 0;
  if (hipGetDevice(&device) != hipSuccess ||
      hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, device) != hipSuccess || cus < 1)
    return fail(MSRL_EDEVICE, "%s: cannot query the current device", who);
  if (env->kind == MSRL_ENV_PARTICLE) {
    // Two waves per row block, one per network, where that shape is compiled: the two networks of a step do
    // not depend on each other, a step is then half as long a chain of instructions, and with every weight
    // tile resident it has no stage barriers.  64-unit networks: measured faster at every env count (1.1x to
    // 1.9x); two row blocks per workgroup - one wave per SIMD - as long as that gives every SIMD at most one
    // wave anyway, else four where compiled (fp32: 1.2x at 16k envs and more; bf16: no gain).  128-unit bf16
    // networks: 1.8x as long as its workgroups run in one round, the same or a little slower beyond.
    const int64_t row_blocks = ((int64_t)env->num_envs + found.envs_per_wave - 1) / found.envs_per_wave;
    KernelEntry split;
    const bool have = find_kernel(*env, *policy, PHASE_SPLIT, &split, row_blocks > 2 * (int64_t)cus ? 1 : -1);
    if (env->wave_roles == 2 && !have)
      return fail(MSRL_EUNSUPPORTED, "%s: wave_roles 2 is compiled for 64-unit networks and 128-unit bf16 networks "
                                     "of two hidden layers with a per-agent critic", who);
    const bool pays = policy->hidden == 64 || row_blocks <= (int64_t)split.row_waves * cus;
    if (have && (env->wave_roles == 2 || (env->wave_roles == 0 && pays))) found = split;
  }

  memset(st, 0, sizeof(*st));
  st->env = *env;
  st->env.A = nullptr;
  st->env.B = nullptr;
  st->pol = *policy;
  st->seed = seed;
  st->kernel = found;
  st->device = device;
  st->cus = cus;
  // Pursuit env: tiles of 32 envs per workgroup (msrl_env_cfg.tag_tiles, 0 = chosen here).
  st->tag_tiles = env->tag_tiles != 0 ? env->tag_tiles : choose_tag_tiles(env->num_envs, env->num_agents, cus);
  if (env->kind == MSRL_ENV_TAG && st->tag_tiles == 4 &&
      !tag_rollout_compiled(env->num_chasers, env->num_agents - env->num_chasers, env->num_landmarks, policy->hidden,
                            policy->dtype == MSRL_BF16, 4))
    st->tag_tiles = 1;  // (fp32 networks: one tile per workgroup only)
  st->state_size = (int)msrl_env_state_size(env);
  // The particle observation ends in 2 (N - 1) slots that are always zero: layer 1 skips them.
  st->in_used = env->kind == MSRL_ENV_PARTICLE ? 4 * env->num_agents + 2 : policy->in_dim;
  const int n_nets = 2 * roles_of(*policy);
  st->layout = net_layout(st->in_used, policy->hidden, policy->dtype == MSRL_BF16, layers_of(*policy));
  st->central = central_of(*policy);
  // (joint observation: num_agents blocks of whole layer-1 tiles, see pack_params)
  {
    const bool bf16 = policy->dtype == MSRL_BF16;
    st->critic_layout = net_layout(env->num_agents * tiles_for_inputs(st->in_used + 1, bf16) * (bf16 ? 16 : 8) - 1,
                                   policy->hidden, bf16);
  }
  // (behind a centralised critic's image: the memory its kernel's tile fetches may read past the end)
  *packed_bytes = st->central ? st->layout.bytes + st->critic_layout.bytes + (size_t)CRITIC_FETCH_PAD_TILES * 1024
                              : n_nets * st->layout.bytes;
  return MSRL_OK;
}

}  // namespace

// ------------------------------------------------------------------ the entry point that allocates nothing
// msrl_rollout_gae_static keeps the packed parameter image (the buffer msrl_rollout_init would
// allocate) in this array.  Every GPU holds its own copy at its own address; in host code the name
// below is only a handle for hipGetSymbolAddress, never a device address.
static __device__ __align__(256) uint8_t scratch[MSRL_STATIC_SCRATCH_BYTES];

namespace {

constexpr int MAX_DEVICES = 64;
std::mutex g_scratch_mutex;
uint8_t* g_scratch_ptr[MAX_DEVICES];  // device address of `scratch` on device d, looked up on first use

// address of the scratch array on the current device (looked up once per device, with it current)
int scratch_of_current_device(uint8_t** out) {
  int dev = -1;
  HIP_TRY(hipGetDevice(&dev));
  if (dev < 0 || dev >= MAX_DEVICES)
    return fail(MSRL_EUNSUPPORTED, "msrl_rollout_gae_static: device index %d is beyond the %d devices it keeps track of",
                dev, MAX_DEVICES);
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (!p) return fail(MSRL_EDEVICE, "msrl_rollout_gae_static: the scratch array has no address on device %d", dev);
    g_scratch_ptr[dev] = (uint8_t*)p;
  }
  *out = g_scratch_ptr[dev];
  return MSRL_OK;
}

// p[0 .. n) <- 0 in 16-byte pieces (a kernel rather than a memset node: the call may be captured into a graph)
__global__ void zero16_kernel(uint4* p, size_t n) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = make_uint4(0u, 0u, 0u, 0u);
}

}  // namespace

extern "C" {

const char* msrl_last_error(void) { return g_err; }

size_t msrl_param_count(const msrl_policy_cfg* cfg) {
  if (!valid_policy(cfg)) return 0;
  const int L = layers_of(*cfg);
  return (size_t)roles_of(*cfg) *
         (net_params(cfg->in_dim, cfg->hidden, cfg->out_dim, L) + net_params(value_in_of(*cfg), cfg->hidden, 1, L));
}

size_t msrl_env_state_size(const msrl_env_cfg* cfg) {
  if (!valid_env_shape(cfg)) return 0;
  return cfg->kind != MSRL_ENV_LINGAUSS ? (size_t)4 * cfg->num_agents + 2 * cfg->num_landmarks
                                        : (size_t)cfg->obs_dim;
}

int msrl_rollout_init(const msrl_env_cfg* env, const msrl_policy_cfg* policy, uint64_t seed,
                      msrl_state** out) {
  if (!env || !policy || !out) return fail(MSRL_EINVAL, "msrl_rollout_init: NULL argument");
  *out = nullptr;
  msrl_state* st = new (std::nothrow) msrl_state;
  if (!st) return fail(MSRL_ENOMEM, "msrl_rollout_init: host allocation failed");
  size_t packed_bytes = 0;
  int rc = configure_state(st, "msrl_rollout_init", env, policy, seed, &packed_bytes);
  if (rc != MSRL_OK) {
    delete st;
    return rc;
  }
  if (env->kind == MSRL_ENV_LINGAUSS && (!env->A || !env->B)) {
    delete st;
    return fail(MSRL_EINVAL, "msrl_rollout_init: lingauss needs A and B");
  }
  auto cleanup = [&](int code) {
    msrl_rollout_destroy(st);
    return code;
  };
#define INIT_TRY(expr)                                                                         \
  do {                                                                                         \
    hipError_t e_ = (expr);                                                                    \
    if (e_ != hipSuccess) {                                                                    \
      rc = fail(e_ == hipErrorOutOfMemory ? MSRL_ENOMEM : MSRL_EDEVICE, "%s failed: %s", #expr, \
                hipGetErrorString(e_));                                                        \
      return cleanup(rc);                                                                      \
    }                                                                                          \
  } while (0)

  const size_t E = (size_t)env->num_envs;
  INIT_TRY(hipMalloc((void**)&st->env_state, E * st->state_size * sizeof(float)));
  INIT_TRY(hipMalloc((void**)&st->g, E * sizeof(int64_t)));
  INIT_TRY(hipMalloc((void**)&st->packed, packed_bytes));
  INIT_TRY(hipMemset(st->packed, 0, packed_bytes));
  if (env->kind == MSRL_ENV_LINGAUSS) {
    const int D = env->obs_dim, K = env->act_dim;
    const int ktA = tiles_for_inputs(D + 1, false), ktB = tiles_for_inputs(K, false);  // as the kernel counts them
    INIT_TRY(hipMalloc((void**)&st->dyn_src, ((size_t)D * D + (size_t)D * K) * sizeof(float)));
    INIT_TRY(hipMalloc((void**)&st->dyn, (size_t)(ktA + ktB) * 1024));
    INIT_TRY(hipMemcpy(st->dyn_src, env->A, (size_t)D * D * sizeof(float), hipMemcpyHostToDevice));
    INIT_TRY(hipMemcpy(st->dyn_src + (size_t)D * D, env->B, (size_t)D * K * sizeof(float), hipMemcpyHostToDevice));
    PackJobs jobs;
    jobs.n = 2;
    jobs.job[0] = weight_job(st->dyn_src, st->dyn, false, D, D, 1, ktA, IN_CHAIN, OUT_NATURAL, 0);
    jobs.job[0].src_out_major = 1;  // A[out, in]
    jobs.job[1] = weight_job(st->dyn_src + (size_t)D * D, st->dyn + (size_t)ktA * 1024, false, K, D, 1, ktB,
                             IN_CHAIN, OUT_NATURAL, 0);
    jobs.job[1].src_out_major = 1;  // B[out, in]
    INIT_TRY(launch_pack(jobs, nullptr));
  }
  {
    const int64_t items = env->kind != MSRL_ENV_LINGAUSS
                              ? (int64_t)E * (env->num_agents + env->num_landmarks)
                              : (int64_t)E * ((env->obs_dim + 3) / 4);
    // (the pursuit env starts an episode like the particle env)
    hipLaunchKernelGGL(init_state_kernel, dim3((unsigned)((items + 255) / 256)), dim3(256), 0, nullptr,
                       env->kind == MSRL_ENV_TAG ? (int)MSRL_ENV_PARTICLE : env->kind, env->num_envs, env->num_agents, env->num_landmarks, env->obs_dim,
                       (uint32_t)seed, (uint32_t)(seed >> 32), st->env_state, st->g);
    INIT_TRY(hipGetLastError());
    INIT_TRY(hipDeviceSynchronize());
  }
#undef INIT_TRY
  *out = st;
  return MSRL_OK;
}

void msrl_rollout_destroy(msrl_state* st) {
  if (!st) return;
  if (st->env_state) (void)hipFree(st->env_state);
  if (st->g) (void)hipFree(st->g);
  if (st->packed) (void)hipFree(st->packed);
  if (st->dyn) (void)hipFree(st->dyn);
  if (st->dyn_src) (void)hipFree(st->dyn_src);
  delete st;
}

int msrl_rollout_step(msrl_state* st, const void* params, int32_t T, msrl_traj* out, void* hip_stream) {
  if (!st || !params) return fail(MSRL_EINVAL, "msrl_rollout_step: NULL argument");
  if (T <= 0) return fail(MSRL_EINVAL, "msrl_rollout_step: T must be positive (got %d)", T);
  int rc = check_traj(st, out, false);
  if (rc != MSRL_OK) return rc;
  if (st->env.kind == MSRL_ENV_TAG) return enqueue_tag(st, params, T, out, (hipStream_t)hip_stream);
  return enqueue_rollout(st, st->kernel, params, T, out, (hipStream_t)hip_stream);
}

int msrl_gae(const float* rewards, const float* values, const uint8_t* dones, int32_t T, int64_t M,
             float gamma, float lambda, float* adv, float* ret, void* hip_stream) {
  if (T < 0 || M < 0) return fail(MSRL_EINVAL, "msrl_gae: negative size (T %d, M %lld)", T, (long long)M);
  if (T == 0 || M == 0) return MSRL_OK;
  if (!rewards || !values || !dones || !adv || !ret) return fail(MSRL_EINVAL, "msrl_gae: NULL argument");
  HIP_TRY(launch_gae(rewards, values, dones, T, M, gamma, lambda, adv, ret, (hipStream_t)hip_stream));
  return MSRL_OK;
}

int msrl_rollout_gae(msrl_state* st, const void* params, int32_t T, float gamma, float lambda,
                     msrl_traj* out, void* hip_stream) {
  if (!st || !params) return fail(MSRL_EINVAL, "msrl_rollout_gae: NULL argument");
  if (T <= 0) return fail(MSRL_EINVAL, "msrl_rollout_gae: T must be positive (got %d)", T);
  int rc = check_traj(st, out, true);
  if (rc != MSRL_OK) return rc;
  rc = st->env.kind == MSRL_ENV_TAG ? enqueue_tag(st, params, T, out, (hipStream_t)hip_stream)
                                    : enqueue_rollout(st, st->kernel, params, T, out, (hipStream_t)hip_stream);
  if (rc != MSRL_OK) return rc;
  const int64_t M = (int64_t)st->env.num_envs * st->env.num_agents;
  HIP_TRY(launch_gae(out->rewards, out->values, out->dones, T, M, gamma, lambda, out->adv, out->ret,
                     (hipStream_t)hip_stream));
  return MSRL_OK;
}

int msrl_rollout_gae_static(const msrl_env_cfg* env, const msrl_policy_cfg* policy, uint64_t seed,
                            float* env_state, int64_t* step_counters, const void* params, int32_t T,
                            float gamma, float lambda, msrl_traj* out, void* hip_stream) {
  if (!env || !policy || !env_state || !step_counters || !params)
    return fail(MSRL_EINVAL, "msrl_rollout_gae_static: NULL argument");
  if (T <= 0) return fail(MSRL_EINVAL, "msrl_rollout_gae_static: T must be positive (got %d)", T);
  if (env->kind == MSRL_ENV_LINGAUSS)
    return fail(MSRL_EUNSUPPORTED, "msrl_rollout_gae_static: the lingauss env is not supported (its dynamics "
                                   "matrices need a device copy, which msrl_rollout_init makes)");
  msrl_state st;  // lives for this call only; every device pointer in it is the caller's or the scratch array
  size_t packed_bytes = 0;
  int rc = configure_state(&st, "msrl_rollout_gae_static", env, policy, seed, &packed_bytes);
  if (rc != MSRL_OK) return rc;
  if (packed_bytes > (size_t)MSRL_STATIC_SCRATCH_BYTES)
    return fail(MSRL_EUNSUPPORTED, "msrl_rollout_gae_static: the packed parameters of this configuration take %zu "
                                   "bytes, the static scratch array holds %zu; use msrl_rollout_init + msrl_rollout_gae",
                packed_bytes, (size_t)MSRL_STATIC_SCRATCH_BYTES);
  rc = check_traj(&st, out, true);
  if (rc != MSRL_OK) return rc;
  uint8_t* sp = nullptr;
  rc = scratch_of_current_device(&sp);
  if (rc != MSRL_OK) return rc;
  st.env_state = env_state;
  st.g = step_counters;
  st.packed = sp;
  hipStream_t stream = (hipStream_t)hip_stream;
  // The array keeps the image of the last call, whatever its configuration was: clear the part this
  // call uses (the packing kernel writes the weights and leaves the padding tiles alone).
  const size_t pieces = (packed_bytes + 15) / 16;
  hipLaunchKernelGGL(zero16_kernel, dim3((unsigned)((pieces + 255) / 256)), dim3(256), 0, stream, (uint4*)sp, pieces);
  HIP_TRY(hipGetLastError());
  rc = env->kind == MSRL_ENV_TAG ? enqueue_tag(&st, params, T, out, stream)
                                 : enqueue_rollout(&st, st.kernel, params, T, out, stream);
  if (rc != MSRL_OK) return rc;
  const int64_t M = (int64_t)env->num_envs * env->num_agents;
  HIP_TRY(launch_gae(out->rewards, out->values, out->dones, T, M, gamma, lambda, out->adv, out->ret, stream));
  return MSRL_OK;
}

int msrl_measure_phase(msrl_state* st, const void* params, int32_t T, msrl_traj* out, int32_t phase,
                       void* hip_stream) {
  if (!st || !params) return fail(MSRL_EINVAL, "msrl_measure_phase: NULL argument");
  if (T <= 0) return fail(MSRL_EINVAL, "msrl_measure_phase: T must be positive (got %d)", T);
  if (phase != MSRL_PHASE_ENV && phase != MSRL_PHASE_MLP && phase != MSRL_PHASE_CLOCKS)
    return fail(MSRL_EINVAL, "msrl_measure_phase: unknown phase %d", phase);
  int rc = check_traj(st, out, false);
  if (rc != MSRL_OK) return rc;
  if (phase == MSRL_PHASE_CLOCKS && !out->logits)
    return fail(MSRL_EINVAL, "msrl_measure_phase: the clock stamps go to out->logits, which is NULL");
  KernelEntry k;
  if (!find_kernel(st->env, st->pol, phase, &k))
    return fail(MSRL_EUNSUPPORTED, "msrl_measure_phase: phase %d is not compiled for this configuration", phase);
  return enqueue_rollout(st, k, params, T, out, (hipStream_t)hip_stream);
}

int msrl_rollout_shape(const msrl_state* st, int32_t* workgroups, int32_t* waves, int32_t* row_waves) {
  if (!st) return fail(MSRL_EINVAL, "msrl_rollout_shape: NULL state");
  int64_t wg;
  int w, rw;
  if (st->env.kind == MSRL_ENV_TAG) {
    wg = ((int64_t)st->env.num_envs + 32 * st->tag_tiles - 1) / (32 * st->tag_tiles);
    w = rw = st->env.num_agents * st->tag_tiles;
  } else {
    const int epb = envs_per_block(st->kernel, st->env.num_envs, st->cus);
    wg = ((int64_t)st->env.num_envs + epb - 1) / epb;
    w = st->kernel.waves;
    rw = st->kernel.row_waves ? st->kernel.row_waves : st->kernel.waves;
  }
  if (workgroups) *workgroups = (int32_t)wg;
  if (waves) *waves = w;
  if (row_waves) *row_waves = rw;
  return MSRL_OK;
}

int msrl_observe(msrl_state* st, float* obs, void* hip_stream) {
  if (!st || !obs) return fail(MSRL_EINVAL, "msrl_observe: NULL argument");
  if (st->env.kind == MSRL_ENV_TAG) {
    msrl_traj out;
    memset(&out, 0, sizeof(out));
    out.obs = obs;
    return enqueue_tag(st, nullptr, 0, &out, (hipStream_t)hip_stream, TAG_STEP);
  }
  KernelEntry k;
  if (!find_kernel(st->env, st->pol, PHASE_STEP, &k))
    return fail(MSRL_EUNSUPPORTED, "msrl_observe: not compiled for this configuration");
  msrl_traj out;
  memset(&out, 0, sizeof(out));
  out.obs = obs;
  return enqueue_rollout(st, k, nullptr, 0, &out, (hipStream_t)hip_stream);
}

int msrl_act(msrl_state* st, const void* params, const float* obs, void* actions, float* logp, float* values,
             float* logits, void* hip_stream) {
  if (!st || !obs || !actions || !logp || !values) return fail(MSRL_EINVAL, "msrl_act: NULL argument");
  if (!params && !st->packed_valid)
    return fail(MSRL_EINVAL, "msrl_act: params is NULL and no earlier call on this state passed parameters");
  if (st->env.kind == MSRL_ENV_TAG) {
    msrl_traj out;
    memset(&out, 0, sizeof(out));
    out.actions = actions;
    out.logp = logp;
    out.values = values;
    out.logits = logits;
    return enqueue_tag(st, params, 0, &out, (hipStream_t)hip_stream, TAG_ACT, obs, nullptr);
  }
  KernelEntry k;
  if (!find_kernel(st->env, st->pol, PHASE_ACT, &k))
    return fail(MSRL_EUNSUPPORTED, "msrl_act: not compiled for this configuration");
  msrl_traj out;
  memset(&out, 0, sizeof(out));
  out.actions = actions;
  out.logp = logp;
  out.values = values;
  out.logits = logits;
  return enqueue_rollout(st, k, params, 0, &out, (hipStream_t)hip_stream, obs, nullptr);
}

int msrl_env_step(msrl_state* st, const void* actions, float* rewards, uint8_t* dones, float* next_obs,
                  void* hip_stream) {
  if (!st || !actions || !rewards || !dones || !next_obs)
    return fail(MSRL_EINVAL, "msrl_env_step: NULL argument");
  if (st->env.kind == MSRL_ENV_TAG) {
    msrl_traj out;
    memset(&out, 0, sizeof(out));
    out.obs = next_obs;
    out.rewards = rewards;
    out.dones = dones;
    return enqueue_tag(st, nullptr, 1, &out, (hipStream_t)hip_stream, TAG_STEP, nullptr, actions);
  }
  KernelEntry k;
  if (!find_kernel(st->env, st->pol, PHASE_STEP, &k))
    return fail(MSRL_EUNSUPPORTED, "msrl_env_step: not compiled for this configuration");
  msrl_traj out;
  memset(&out, 0, sizeof(out));
  out.obs = next_obs;
  out.rewards = rewards;
  out.dones = dones;
  return enqueue_rollout(st, k, nullptr, 1, &out, (hipStream_t)hip_stream, nullptr, actions);
}

int msrl_state_get(msrl_state* st, float* env_state, int64_t* step_counters) {
  if (!st) return fail(MSRL_EINVAL, "msrl_state_get: NULL state");
  HIP_TRY(hipDeviceSynchronize());
  const size_t E = (size_t)st->env.num_envs;
  if (env_state)
    HIP_TRY(hipMemcpy(env_state, st->env_state, E * st->state_size * sizeof(float), hipMemcpyDeviceToHost));
  if (step_counters) HIP_TRY(hipMemcpy(step_counters, st->g, E * sizeof(int64_t), hipMemcpyDeviceToHost));
  return MSRL_OK;
}

int msrl_state_set(msrl_state* st, const float* env_state, const int64_t* step_counters) {
  if (!st) return fail(MSRL_EINVAL, "msrl_state_set: NULL state");
  const size_t E = (size_t)st->env.num_envs;
  if (step_counters)
    for (size_t e = 0; e < E; ++e)
      if (step_counters[e] < 0) return fail(MSRL_EINVAL, "msrl_state_set: negative step counter");
  HIP_TRY(hipDeviceSynchronize());
  if (env_state)
    HIP_TRY(hipMemcpy(st->env_state, env_state, E * st->state_size * sizeof(float), hipMemcpyHostToDevice));
  if (step_counters) HIP_TRY(hipMemcpy(st->g, step_counters, E * sizeof(int64_t), hipMemcpyHostToDevice));
  HIP_TRY(hipDeviceSynchronize());
  return MSRL_OK;
}

}  // extern "C"
