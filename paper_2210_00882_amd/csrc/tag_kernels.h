// Fused actor + environment rollout for the pursuit ("tag") env: heterogeneous agents with one
// parameter set per role (interface header, MSRL_ENV_TAG; the task of the paper's GPU-only
// experiment, section 7.3, Fig. 10, as a synthetic stand-in).
//
// Layout: a workgroup owns TILES tiles of 32 envs and has one wave per tile and agent slot; lane n of
// a wave is env n of its tile, so the 32 rows of a wave's MFMA tile all have the same role and use
// the same weights.  (TILES = 4 puts 16 waves on a compute unit behind one copy of the weights: the
// kernel is bound by vector-ALU issue, and four waves per SIMD hide more of its latencies than the
// two that the LDS leaves room for with one tile per workgroup.)  The
// networks are small (bf16, 64 units), so the four of them (chasers' and runners' policy and
// value) stay resident in LDS for the whole kernel: no weight streaming, and the only barriers are
// those of the env step (two per step), where the agents of an env (one per wave) exchange
// positions through LDS.
// The MLP itself is the chained MFMA form of mlp.h, reading its tiles from the resident images.
#pragma once
#include <type_traits>
#include <vector>

#include "rollout_kernels.h"

namespace msrl {

struct TagArgs {
  float* env_state;       // [E, 4N + 2L]
  int64_t* g;             // [E]
  const uint8_t* packed;  // four packed networks (packed.h): role 0 policy, value, role 1 policy, value
  int E, T, ep;
  float dt, keep;
  float accel[2], vmax[2], rad[2];  // per role: 0 chasers, 1 runners
  float cforce, cmargin;
  uint32_t seed_lo, seed_hi;
  float* obs;
  int32_t* actions;
  float* logp;
  float* rewards;
  uint8_t* dones;
  float* values;
  float* logits;  // may be null
  int64_t M;
  const float* obs_in;        // TAG_ACT: observation rows [M, D] to act on
  const int32_t* actions_in;  // TAG_STEP: actions [M] to apply
};

// Variants (the step-granular calls of the library, as for the other envs):
//   TAG_ACT   both networks of the row's role and the sampling on observation rows given by the caller, with the
//             noise the fused kernel would draw at the state's step counters; writes values, actions, logp
//             (and logits) of one evaluation; the state is not changed;
//   TAG_STEP  applies the caller's actions for T = 1 (move, contact forces, rewards, done, reset, counters + 1;
//             writes rewards[0], dones[0]) and writes the observation of the resulting state to obs[0]; with
//             T = 0 it only writes the observation of the current state.  No network runs.
enum : int { TAG_ALL = 0, TAG_ACT = 1, TAG_STEP = 2 };

// layer-1 tiles of an observation of D features (+ the constant-1 input that carries the bias): 16 inputs
// per bf16 tile, 8 per fp32 tile
constexpr int tag_kt1(int D, bool bf16) { return bf16 ? (D + 1 + 15) / 16 : (D + 1 + 7) / 8; }
// LDS of a workgroup: the four resident networks, their output biases, the state tables of its tiles
constexpr int tag_lds_bytes(int N, int L, int H, bool bf16, int tiles) {
  const int kt1 = tag_kt1(4 + 2 * L + 4 * (N - 1), bf16), nuc = H / 32, kt2 = bf16 ? H / 16 : H / 8;
  const int net_tiles = nuc * kt1 + nuc * (kt2 + 1 + kt2 / nuc);
  return 4 * net_tiles * 1024 + 4 * 32 * 4 + tiles * (2 * 2 * 32 * N * 8 + 2 * 32 * (L > 0 ? L : 1) * 8 + 32 * N * 8 + 32 * N * 4);
}

template <int NC, int NR, int L, int H, bool BF16 = true, int TILES = 1, int PHASE = TAG_ALL>
__global__ __launch_bounds__(64 * (NC + NR) * TILES) void tag_rollout_kernel(TagArgs a) {
  constexpr int N = NC + NR;
  constexpr bool ACT = PHASE == TAG_ACT, STEP = PHASE == TAG_STEP;
  static_assert(64 * N * TILES <= 1024, "one wave per tile and agent slot");
  constexpr int D = 4 + 2 * L + 4 * (N - 1);
  constexpr int S = 4 * N + 2 * L;
  constexpr int KT1 = tag_kt1(D, BF16);
  typedef Mlp<H, BF16, 1, KT1> Net;
  typedef typename Net::Op Op;
  constexpr int PT = Net::PT;
  // Resident image of a network: its layer-1 tiles, then per 32-unit chunk the layer-2 tiles, the
  // bias tile and the layer-3 tiles the chunk feeds (the second copy of the layer-3 tiles that the
  // streaming kernels keep in the following block is left out: 72 KiB for the four networks, so
  // that two workgroups fit a compute unit).
  constexpr int BLOCK = Net::KT2 + 1 + Net::TPC;
  constexpr int NET_TILES = Net::L1_TILES + Net::NUC * BLOCK;
  static_assert(L <= N && N <= 16, "a landmark is handled by the wave of the agent with its index");

  __shared__ __attribute__((aligned(16))) u32x4 s_net[4][NET_TILES * 64];
  __shared__ __attribute__((aligned(16))) float s_b3[4][32];
  // State tables of the workgroup's envs, double-buffered over the steps: step t reads buffer t % 2
  // and writes the state of step t + 1 (moved, or reset after a done) into the other one, so that
  // two barriers per step suffice (new state visible; contact counts visible).  s_pm holds the
  // positions after the move, which the rewards are computed on.
  __shared__ float2 t_p[TILES][2][32][N], t_v[TILES][2][32][N], t_lm[TILES][2][32][L > 0 ? L : 1], t_pm[TILES][32][N];
  __shared__ float t_cnt[TILES][32][N];

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int tile = wave / N;      // env tile of this wave
  const int j = wave - tile * N;  // ... and its agent slot
  const int n = lane & 31, h = lane >> 5;
  // the tables of this wave's tile
  float2(&s_p)[2][32][N] = t_p[tile];
  float2(&s_v)[2][32][N] = t_v[tile];
  float2(&s_lm)[2][32][L > 0 ? L : 1] = t_lm[tile];
  float2(&s_pm)[32][N] = t_pm[tile];
  float(&s_cnt)[32][N] = t_cnt[tile];
  const int role = j < NC ? 0 : 1;
  const NetLayout ly = net_layout(D, H, BF16);
  for (int net = 0; net < (STEP ? 0 : 4); ++net) {
    const u32x4* src = (const u32x4*)(a.packed + (size_t)net * ly.bytes + ly.w1);
    for (int i = threadIdx.x; i < NET_TILES * 64; i += blockDim.x) {
      const int tile = i >> 6;
      int from = tile;  // layer-1 tiles keep their place
      if (tile >= Net::L1_TILES) {
        const int c = (tile - Net::L1_TILES) / BLOCK, r = (tile - Net::L1_TILES) % BLOCK;
        // layer-2 and bias tiles, then the chunk's own layer-3 tiles (behind the copy for the chunk before)
        from = Net::L1_TILES + c * Net::CHUNK_TILES + (r <= Net::KT2 ? r : r + Net::TPC);
      }
      s_net[net][i] = src[from * 64 + (i & 63)];
    }
    if (threadIdx.x < 32)
      s_b3[net][threadIdx.x] = *(const float*)(a.packed + (size_t)net * ly.bytes + ly.b3 + threadIdx.x * 4);
  }

  const int64_t env64 = ((int64_t)blockIdx.x * TILES + tile) * 32 + n;
  const bool valid = env64 < a.E;
  const uint32_t env = (uint32_t)(valid ? env64 : a.E - 1);
  const float* es = a.env_state + (size_t)env * S;
  float2 p = make_float2(es[4 * j], es[4 * j + 1]);
  float2 v = make_float2(es[4 * j + 2], es[4 * j + 3]);
  const int64_t g64 = a.g[env];
  uint32_t g32 = (uint32_t)g64;
  int tau = (int)(g64 % a.ep);
  uint32_t episode = (uint32_t)(g64 / a.ep);
  float2 lm_own = make_float2(0.0f, 0.0f);  // landmark j, kept by wave j < L
  if (j < L) lm_own = make_float2(es[4 * N + 2 * j], es[4 * N + 2 * j + 1]);
  if (h == 0) {
    s_p[0][n][j] = p;
    s_v[0][n][j] = v;
    if (j < L) s_lm[0][n][j] = lm_own;
  }
  const float my_rad = a.rad[role];
  const float inv_margin = 1.0f / a.cmargin;
  __syncthreads();

  for (int t = 0; t <= a.T; ++t) {
    const int cur = t & 1, nxt = cur ^ 1;
    // ---------------- observation row of (env n, agent j)
    // Feature IDX of the row; the index is a compile-time constant, so that each feature is one LDS
    // read and a subtraction (a lane needs the features 16 kt + 8 h + s: both halves are evaluated
    // and the lane keeps its own).
    auto feature = [&](auto IDX) -> float {
      constexpr int idx = decltype(IDX)::value;
      if constexpr (idx > D) {
        return 0.0f;
      } else if constexpr (idx == D) {
        return 1.0f;  // input D carries the bias
      } else if constexpr (ACT) {
        return valid ? a.obs_in[((size_t)env * N + j) * D + idx] : 0.0f;  // the caller's row
      } else if constexpr (idx < 4) {
        return idx == 0 ? v.x : idx == 1 ? v.y : idx == 2 ? p.x : p.y;
      } else if constexpr ((idx - 4) / 2 < L) {
        const float2 lm = s_lm[cur][n][(idx - 4) / 2];
        return idx % 2 ? lm.y - p.y : lm.x - p.x;
      } else {
        constexpr int q0 = (idx - 4) / 2 - L;
        constexpr bool vel = q0 >= N - 1;
        constexpr int q = vel ? q0 - (N - 1) : q0;
        const int o = q + (q >= j ? 1 : 0);  // the q-th other agent (j is wave-uniform)
        const float2 w = vel ? s_v[cur][n][o] : s_p[cur][n][o];
        return vel ? (idx % 2 ? w.y : w.x) : (idx % 2 ? w.y - p.y : w.x - p.x);
      }
    };
    Op x[1][KT1 * PT];
    // (TAG_STEP stores one observation, that of the last state, to step slot 0, and runs no network)
    float* const orow = a.obs + ((size_t)(STEP ? 0 : t) * a.M + (size_t)env * N + j) * D;
    const bool observe = !STEP || t == a.T;
    if constexpr (!BF16) {
      // fp32 operands: operand mm of the layer-1 contraction is feature 2 mm + h (one k step of two inputs per
      // MFMA); the lane with h = mm % 2 stores the pair (2 mm, 2 mm + 1) of the observation row
      auto pair_at = [&](auto MM) {
        constexpr int mm = decltype(MM)::value;
        if constexpr (mm < KT1 * 4) {
          const float lo = feature(std::integral_constant<int, 2 * mm>{});
          const float hi = feature(std::integral_constant<int, 2 * mm + 1>{});
          x[0][mm] = h ? hi : lo;
          if (valid && !ACT && 2 * mm + 2 <= D && h == (mm & 1)) *(f32x2*)(orow + 2 * mm) = f32x2{lo, hi};
        }
      };
      auto pairs8 = [&](auto B) {
        constexpr int b = decltype(B)::value;
        pair_at(std::integral_constant<int, b>{}); pair_at(std::integral_constant<int, b + 1>{});
        pair_at(std::integral_constant<int, b + 2>{}); pair_at(std::integral_constant<int, b + 3>{});
        pair_at(std::integral_constant<int, b + 4>{}); pair_at(std::integral_constant<int, b + 5>{});
        pair_at(std::integral_constant<int, b + 6>{}); pair_at(std::integral_constant<int, b + 7>{});
      };
      static_assert(KT1 * 4 <= 32, "layer-1 operands of the observation");
      if (observe) {
        pairs8(std::integral_constant<int, 0>{});
        pairs8(std::integral_constant<int, 8>{});
        pairs8(std::integral_constant<int, 16>{});
        pairs8(std::integral_constant<int, 24>{});
      }
    }
#pragma unroll
    for (int kt = 0; kt < (BF16 ? KT1 : 0); ++kt) {
      if (!observe) break;
      f32x8 f;
      auto fill = [&](auto KT, auto S8) {
        constexpr int k = decltype(KT)::value, s = decltype(S8)::value;
        const float lo = feature(std::integral_constant<int, 16 * k + s>{});
        const float hi = feature(std::integral_constant<int, 16 * k + 8 + s>{});
        f[s] = h ? hi : lo;
      };
      auto fill_all = [&](auto KT) {
        fill(KT, std::integral_constant<int, 0>{}); fill(KT, std::integral_constant<int, 1>{});
        fill(KT, std::integral_constant<int, 2>{}); fill(KT, std::integral_constant<int, 3>{});
        fill(KT, std::integral_constant<int, 4>{}); fill(KT, std::integral_constant<int, 5>{});
        fill(KT, std::integral_constant<int, 6>{}); fill(KT, std::integral_constant<int, 7>{});
      };
      static_assert(!BF16 || KT1 <= 4, "layer-1 tiles of the observation");
      if (kt == 0) fill_all(std::integral_constant<int, 0>{});
      if (kt == 1) fill_all(std::integral_constant<int, 1>{});
      if (kt == 2) fill_all(std::integral_constant<int, 2>{});
      if (kt == 3) fill_all(std::integral_constant<int, 3>{});
      if (valid && !ACT) {
        float* dst = orow + 16 * kt + 8 * h;
        const int i0 = 16 * kt + 8 * h;
        // rows are D floats apart: 16-byte pieces when D % 4 == 0, 8-byte pieces otherwise (D is even)
        constexpr int PW = D % 4 == 0 ? 4 : 2;
#pragma unroll
        for (int q = 0; q < 8 / PW; ++q) {
          if (i0 + PW * q + PW <= D) {
            if constexpr (PW == 4)
              *(f32x4*)(dst + 4 * q) = f32x4{f[4 * q], f[4 * q + 1], f[4 * q + 2], f[4 * q + 3]};
            else
              *(f32x2*)(dst + 2 * q) = f32x2{f[2 * q], f[2 * q + 1]};
          }
        }
      }
      if constexpr (BF16) x[0][kt] = __builtin_convertvector(f, bf16x8);
    }

    // ---------------- networks of this wave's role, from the resident images
    f32x16 out_p[1], out_v[1];
    out_p[0] = out_v[0] = zero16();
#pragma unroll
    for (int net = 0; net < (STEP ? 0 : 2); ++net) {
      f32x16(&out)[1] = net == 0 ? out_p : out_v;
      const u32x4* base = &s_net[2 * role + net][0] + lane;
      Op h1[1][Net::KT2 * PT];
      Net::layer1(base, x, h1);
      out[0] = bias_init(s_b3[2 * role + net], h);
      // layer 2 chunk by chunk; the tanh of chunk c-1 and its layer-3 MFMAs run among those of chunk c
      f32x16 acc = zero16(), prev = zero16();
#pragma unroll
      for (int c = 0; c <= Net::NUC; ++c) {
        const u32x4* blk = base + (Net::L1_TILES + c * BLOCK) * 64;
        float tt[16];
        if (c < Net::NUC) {
          acc = zero16();
#pragma unroll
          for (int kt = 0; kt < Net::KT2; ++kt) {
            u32x4 raw = blk[kt * 64];
            if (c > 0) pin(raw);
            mma_tile<BF16>(raw, &h1[0][kt * PT], acc);
            if (c > 0) tanh_range<!BF16>(prev, tt, kt * 16 / Net::KT2, (kt + 1) * 16 / Net::KT2, true);
          }
          mma_bias_tile<BF16>(blk[Net::KT2 * 64], Operand<BF16>::one(h), acc);
        } else {
          tanh_range<!BF16>(prev, tt, 0, 16, false);
        }
        if (c > 0) {
          Op h2[Net::PC];
          to_operands<BF16>(tt, h2);
          const u32x4* l3 = base + (Net::L1_TILES + (c - 1) * BLOCK + Net::KT2 + 1) * 64;
#pragma unroll
          for (int i = 0; i < Net::TPC; ++i) mma_tile<BF16>(l3[i * 64], &h2[i * PT], out[0]);
        }
        prev = acc;
      }
    }
    const size_t o = (size_t)t * a.M + (size_t)env * N + j;
    if (valid && h == 0 && !STEP) a.values[o] = out_v[0][0];
    if (!ACT && t == a.T) break;

    // ---------------- sampling
    float l[5];
    l[0] = out_p[0][0];
    l[1] = out_p[0][1];
    l[2] = out_p[0][2];
    l[3] = out_p[0][3];
    l[4] = __shfl_xor(out_p[0][0], 32);  // logit 4 sits in register 0 of the partner lane
    const Words4 w = draw(a.seed_lo, a.seed_hi, env, (uint32_t)j, g32, 0, 0);
    float lp;
    int act;
    sample_categorical5(l, u01(w.w[0]), act, lp);
    act = __shfl(act, n);  // the h = 0 lane of the row decides
    if constexpr (STEP) act = valid ? a.actions_in[(size_t)env * N + j] : 0;
    if (valid && h == 0 && !STEP) {
      a.actions[o] = act;
      a.logp[o] = lp;
      if (a.logits) {
#pragma unroll
        for (int k = 0; k < 5; ++k) a.logits[o * 5 + k] = l[k];
      }
    }

    if constexpr (ACT) break;  // one evaluation, no move

    // ---------------- move: action force and contact forces, from the positions before the move
    float fx = a.accel[role] * ((act == 1 ? 1.0f : 0.0f) - (act == 2 ? 1.0f : 0.0f));
    float fy = a.accel[role] * ((act == 3 ? 1.0f : 0.0f) - (act == 4 ? 1.0f : 0.0f));
#pragma unroll
    for (int q = 0; q < N; ++q) {
      if (q == j) continue;  // uniform
      const float2 po = s_p[cur][n][q];
      const float dx = p.x - po.x, dy = p.y - po.y;
      const float d = __builtin_amdgcn_sqrtf(dx * dx + dy * dy);
      const float z = (my_rad + a.rad[q < NC ? 0 : 1] - d) * inv_margin;
      // smooth max(0, overlap): max(z, 0) + log(1 + exp(-|z|)), on the exp2 / log2 units
      const float pen = a.cmargin * (fmaxf(z, 0.0f) + __logf(1.0f + __expf(-fabsf(z))));
      if (d > 0.0f) {
        const float k = a.cforce * pen * __builtin_amdgcn_rcpf(d);
        fx += k * dx;
        fy += k * dy;
      }
    }
    v.x = v.x * a.keep + fx * a.dt;
    v.y = v.y * a.keep + fy * a.dt;
    const float sp = __builtin_amdgcn_sqrtf(v.x * v.x + v.y * v.y);
    if (sp > a.vmax[role]) {
      const float k = a.vmax[role] * __builtin_amdgcn_rcpf(sp);
      v.x *= k;
      v.y *= k;
    }
    p.x += v.x * a.dt;
    p.y += v.y * a.dt;
    const float2 moved = p;
    // the state of the next step: the moved one, or the first of the next episode after a done
    const bool done = tau + 1 == a.ep;
    g32 += 1;
    tau = done ? 0 : tau + 1;
    if (done) {
      episode += 1;
      const Words4 wa = draw(a.seed_lo, a.seed_hi, env, (uint32_t)j, episode, 1, 0);
      p = make_float2(2.0f * u01(wa.w[0]) - 1.0f, 2.0f * u01(wa.w[1]) - 1.0f);
      v = make_float2(0.0f, 0.0f);
      if (j < L) {
        const Words4 wl = draw(a.seed_lo, a.seed_hi, env, (uint32_t)(N + j), episode, 1, 0);
        lm_own = make_float2(2.0f * u01(wl.w[0]) - 1.0f, 2.0f * u01(wl.w[1]) - 1.0f);
      }
    }
    if (h == 0) {
      s_pm[n][j] = moved;
      s_p[nxt][n][j] = p;
      s_v[nxt][n][j] = v;
      if (j < L) s_lm[nxt][n][j] = lm_own;
    }
    __syncthreads();  // moved positions and the next state are visible

    // ---------------- rewards on the moved positions: contacts between chasers and runners
    float cnt = 0.0f;
    const float dmin = a.rad[0] + a.rad[1];
#pragma unroll
    for (int q = 0; q < N; ++q) {
      if ((q < NC) == (j < NC)) continue;  // uniform: only the other role
      const float2 po = s_pm[n][q];
      const float dx = moved.x - po.x, dy = moved.y - po.y;
      cnt += dx * dx + dy * dy < dmin * dmin ? 1.0f : 0.0f;
    }
    if (h == 0) s_cnt[n][j] = cnt;
    __syncthreads();  // contact counts are visible
    float rew;
    if (role == 0) {
      float total = 0.0f;
#pragma unroll
      for (int q = 0; q < NC; ++q) total += s_cnt[n][q];
      rew = 10.0f * total;
    } else {
      rew = -10.0f * cnt - 10.0f * (fmaxf(fabsf(moved.x) - 1.0f, 0.0f) + fmaxf(fabsf(moved.y) - 1.0f, 0.0f));
    }
    if (valid && h == 0) {
      a.rewards[o] = rew;
      a.dones[o] = done ? 1 : 0;
    }
  }

  if constexpr (ACT) return;  // the env state did not move

  // ---------------- write the env state back
  if (valid && h == 0) {
    float* eo = a.env_state + (size_t)env * S;
    eo[4 * j] = p.x;
    eo[4 * j + 1] = p.y;
    eo[4 * j + 2] = v.x;
    eo[4 * j + 3] = v.y;
    if (j < L) {
      eo[4 * N + 2 * j] = lm_own.x;
      eo[4 * N + 2 * j + 1] = lm_own.y;
    }
    if (j == 0) a.g[env] = g64 + a.T;
  }
}

// ---- the compiled instances, by construction: every (chasers, runners) with at most 8 agents in all and
// up to 4 landmarks (never more than agents), 64 hidden units, bf16 networks and - where the four networks
// still fit the LDS at twice the size - fp32 ones; per shape the full rollout with one env tile per workgroup
// and (bf16), while 4 tiles x agents fit the 16 waves of a workgroup, with four; the actor fragment; the env
// step.
struct TagEntry {
  int nc, nr, landmarks, hidden, bf16, tiles, phase;
  const void* fn;  // __global__ void (*)(TagArgs)
};
constexpr int TAG_MAX_AGENTS = 8, TAG_MAX_LANDMARKS = 4;

template <int NC, int NR, int L, bool BF16>
void add_tag_shape_typed(std::vector<TagEntry>& out) {
  // (fp32 networks are twice the size: the four of them must still fit the 160 KiB of LDS)
  if constexpr (tag_lds_bytes(NC + NR, L, 64, BF16, 1) <= 160 * 1024) {
    const int b = BF16 ? 1 : 0;
    out.push_back(TagEntry{NC, NR, L, 64, b, 1, TAG_ALL, (const void*)&tag_rollout_kernel<NC, NR, L, 64, BF16, 1, TAG_ALL>});
    out.push_back(TagEntry{NC, NR, L, 64, b, 1, TAG_ACT, (const void*)&tag_rollout_kernel<NC, NR, L, 64, BF16, 1, TAG_ACT>});
    out.push_back(TagEntry{NC, NR, L, 64, b, 1, TAG_STEP, (const void*)&tag_rollout_kernel<NC, NR, L, 64, BF16, 1, TAG_STEP>});
    if constexpr (BF16 && 4 * (NC + NR) <= 16)
      out.push_back(TagEntry{NC, NR, L, 64, b, 4, TAG_ALL, (const void*)&tag_rollout_kernel<NC, NR, L, 64, BF16, 4, TAG_ALL>});
  }
}
template <int NC, int NR, int L>
void add_tag_shape(std::vector<TagEntry>& out) {
  add_tag_shape_typed<NC, NR, L, true>(out);
  add_tag_shape_typed<NC, NR, L, false>(out);
}
template <int NC, int NR, int L = 0>
void add_tag_landmarks(std::vector<TagEntry>& out) {
  if constexpr (L <= TAG_MAX_LANDMARKS && L <= NC + NR) {
    add_tag_shape<NC, NR, L>(out);
    add_tag_landmarks<NC, NR, L + 1>(out);
  }
}
// all shapes with NC chasers (one translation unit per NC: inst_tag_c*.hip)
template <int NC, int NR = 1>
void add_tag_chasers(std::vector<TagEntry>& out) {
  if constexpr (NC + NR <= TAG_MAX_AGENTS) {
    add_tag_landmarks<NC, NR>(out);
    add_tag_chasers<NC, NR + 1>(out);
  }
}
#define MSRL_TAG_FAMILIES(X) X(1) X(2) X(3) X(4) X(5) X(6) X(7)
#define MSRL_DECLARE_TAG_FAMILY(NC) void tag_family_c##NC(std::vector<TagEntry>& out);
MSRL_TAG_FAMILIES(MSRL_DECLARE_TAG_FAMILY)
#undef MSRL_DECLARE_TAG_FAMILY
#define MSRL_TAG_FAMILY_BODY(NC) \
  void tag_family_c##NC(std::vector<TagEntry>& out) { add_tag_chasers<NC>(out); }

// launcher of the compiled instances; returns hipErrorInvalidValue when no instance matches.
// tiles: env tiles per workgroup, 1 or 4 (the step-granular variants always take 1); phase: TAG_*.
hipError_t launch_tag_rollout(int nc, int nr, int landmarks, int hidden, bool bf16, int tiles, int phase,
                              const TagArgs& a, hipStream_t stream);
bool tag_rollout_compiled(int nc, int nr, int landmarks, int hidden, bool bf16, int tiles = 1);

}  // namespace msrl
