// The fused actor + environment rollout kernels.
//
// One launch runs all T steps (Listing 1 of the paper: the `duration` loop of
// Trainer.train around Actor.act).  Environments are independent, so a wave
// owns a fixed group of environments for the whole call and keeps their state in
// registers / LDS: per step it builds the observation rows, stores them, runs
// both networks on MFMA (mlp.h), samples the action with Philox, moves the
// environment, computes reward and done, resets finished episodes and stores
// the step's trajectory entries.  The waves of a workgroup share the weight
// stream (the network parameters pass through a double-buffered LDS window, one
// barrier per stage, and every wave multiplies its own rows with the stage that
// is resident) and the way out of the per-row outputs.
//
// Row <-> lane mapping: a wave handles 32*NB rows; row 32*q + n lives on lanes n
// and n + 32 (the two k-halves of the MFMA operands).  Both lanes keep a copy of
// the row's state and execute the same arithmetic.
//
// Stores.  A store instruction whose 64 lanes hit 64 different cache lines costs
// the memory pipeline about as much as 64 stores, and a cache line written in
// pieces by different waves reaches HBM in pieces.  So nothing is stored in row
// layout: observation rows pass through a per-wave LDS staging area and leave as
// consecutive 16-byte pieces of the wave's contiguous block, and the per-row
// scalars (value, action, logp, reward, done) of all waves are collected in LDS
// and written by one wave per array, after a barrier of the following step.
#pragma once
#include "dev_common.h"
#include "mlp.h"
#include "packed.h"

namespace msrl {

struct RolloutArgs {
  float* env_state;       // [E, S] snapshot layout of msrl_state_get
  int64_t* g;             // [E] step counters
  const uint8_t* packed;  // policy network, then value network (packed.h)
  const uint8_t* dyn;     // lingauss: tiles of A, then one tile of B
  int E, T, ep;
  int envs_per_block;     // envs owned by one workgroup (<= WAVES * envs per wave)
  float dt, keep, fdt, coll2;  // particle: dt, 1 - damping, force * dt, (2 radius)^2
  float noise_std, act_cost;   // lingauss
  uint32_t seed_lo, seed_hi;
  float* obs;
  void* actions;
  float* logp;
  float* rewards;
  uint8_t* dones;
  float* values;
  float* logits;  // may be null
  int64_t M;
  const float* obs_in;     // PHASE_ACT: observation rows [M, D] to act on
  const void* actions_in;  // PHASE_STEP: actions [M] to apply
  int layers;              // hidden layers of both networks (>= 2; kernels other than PHASE_DEEP take 2)
  const uint8_t* critic;   // PHASE_CENTRAL: packed value network on the joint observation (NetLayout of N * NZ inputs)
};

// Copies the layer-1 tiles and the output biases of both packed networks into LDS (once per kernel).
__device__ __forceinline__ void load_resident(u32x4* l1, float* b3, const uint8_t* packed,
                                              const NetLayout& ly, int l1_tiles) {
  for (int net = 0; net < 2; ++net) {
    const u32x4* src = (const u32x4*)(packed + (size_t)net * ly.bytes + ly.w1);
    for (int i = threadIdx.x; i < l1_tiles * 64; i += blockDim.x) l1[net * l1_tiles * 64 + i] = src[i];
    if (threadIdx.x < 32)
      b3[net * 32 + threadIdx.x] = *(const float*)(packed + (size_t)net * ly.bytes + ly.b3 + threadIdx.x * 4);
  }
}

// Categorical draw by inverse CDF in fp32, in index order; logp = z_a - log(sum exp z).
__device__ __forceinline__ void sample_categorical5(const float (&l)[5], float u, int& action,
                                                    float& logp) {
  float mx = l[0];
#pragma unroll
  for (int k = 1; k < 5; ++k) mx = fmaxf(mx, l[k]);
  float z[5], e[5], s = 0.0f;
#pragma unroll
  for (int k = 0; k < 5; ++k) {
    z[k] = l[k] - mx;
    e[k] = __expf(z[k]);
    s += e[k];
  }
  const float inv = __builtin_amdgcn_rcpf(s);  // 1 ulp; a draw that close to a bin edge is exempt anyway
  float c = 0.0f;
  int a = 4;
  bool found = false;
#pragma unroll
  for (int k = 0; k < 5; ++k) {
    c += e[k] * inv;
    if (!found && u < c) {
      a = k;
      found = true;
    }
  }
  float za = z[0];
#pragma unroll
  for (int k = 1; k < 5; ++k) za = (a == k) ? z[k] : za;
  action = a;
  logp = za - __logf(s);  // s is in [1, 5]: absolute error of the fast log ~1e-7
}

// Measurement variants of the same kernel (phase rooflines):
//   PHASE_ENV  the networks are skipped; logits and values are 0, which is what an all-zero parameter
//              buffer gives, so every output is still defined and checked against the full kernel;
//   PHASE_MLP  T evaluations of both networks on the current observation, no env step and no
//              trajectory stores (a checksum of the outputs goes to rewards[0, :] to keep them live).
//   PHASE_CLOCKS  the full kernel; in addition lane 0 of every wave of workgroup 0 reads the shader
//              clock at the phase boundaries of step T/2 and writes the cycles since the start of
//              that step to the logits buffer (which then holds no logits): wave w, stamp i at
//              float 32 w + i, i = CLK_* below.
// The two halves of a step as kernels of their own (step-granular calls of the library):
//   PHASE_ACT   both networks and the sampling on observation rows given by the caller (obs_in),
//              with the noise the fused kernel would draw at the state's step counters; writes
//              actions, logp, values (and logits); the state is not changed;
//   PHASE_STEP  applies the caller's actions (actions_in) for T = 1: move, reward, done, reset,
//              counters + 1; writes rewards[0], dones[0] and the observation of the new state to
//              obs[0].  With T = 0 it only writes the observation of the current state.
//   PHASE_DEEP  the full kernel for networks with more than two hidden layers (RolloutArgs::layers):
//              the further hidden layers run between layer 1 and the last hidden layer, their chunk
//              blocks coming through the same LDS window.
//   PHASE_CENTRAL  the full kernel with a centralised critic (bf16 networks): the policy network as
//              usual; the value network takes the joint observation of an env (RolloutArgs::critic
//              holds its tiles) and is evaluated once per env by the workgroup as a whole: the
//              joint observations of its envs are the columns of one MFMA tile, and wave w computes
//              the 32-unit chunk w of each layer, the layers meeting in LDS.
//   PHASE_ACT_DEEP, PHASE_ACT_CENTRAL  PHASE_ACT for networks with more than two hidden layers / with a
//              centralised critic (the joint observation is then built from the caller's rows).
// tiles of 1 KiB a fetch of the centralised critic's weights may read past the end of its image
constexpr int CRITIC_FETCH_PAD_TILES = 32;

enum : int { PHASE_ALL = 0, PHASE_ENV = 1, PHASE_MLP = 2, PHASE_CLOCKS = 3, PHASE_ACT = 4, PHASE_STEP = 5,
             PHASE_DEEP = 6, PHASE_CENTRAL = 7, PHASE_ACT_DEEP = 8, PHASE_ACT_CENTRAL = 9, PHASE_SPLIT = 10 };
// stamps: start of the step, observation rows built and stored, policy layer 1 done (after the
// stage barrier that precedes it), policy stage s done (s < 5), same for the value network,
// logits and values ready, sampling and move done, end of the step
enum : int { CLK_START = 0, CLK_OBS = 1, CLK_P_L1 = 2, CLK_P_STAGE = 3, CLK_V_L1 = 8, CLK_V_STAGE = 9,
             CLK_NETS = 14, CLK_SAMPLE = 15, CLK_END = 16, CLK_COUNT = 17,
             CLK_WAIT = 20 };  // slot 20: cycles of the step spent in the waits at the stage barriers

// ------------------------------------------------------------------ particle env
template <int N, int H, bool BF16, int NB, int WAVES, int PHASE = PHASE_ALL>
__global__ __launch_bounds__(64 * WAVES) void particle_rollout_kernel(RolloutArgs a) {
  constexpr int ROWS = 32 * NB;
  constexpr int EPW = ROWS / N;  // envs per wave
  constexpr int VR = EPW * N;    // rows in use
  constexpr int L = N;
  constexpr int D = 6 * N;
  constexpr int S = 4 * N + 2 * L;
  // Only the first NZ observation features can be non-zero (the remaining 2(N-1) are the zero
  // padding of the layout), so layer 1 contracts over NZ inputs plus the constant 1 that carries
  // the bias, which sits at input index NZ.
  constexpr int NZ = 4 * N + 2;
  constexpr int KT1 = BF16 ? (NZ + 1 + 15) / 16 : (NZ + 1 + 7) / 8;
  constexpr bool ACT = PHASE == PHASE_ACT || PHASE == PHASE_ACT_DEEP || PHASE == PHASE_ACT_CENTRAL;
  constexpr bool CENTRAL = PHASE == PHASE_CENTRAL || PHASE == PHASE_ACT_CENTRAL;
  // chunk blocks per stage (fewer barriers when they fit; the centralised critic needs the LDS)
  constexpr int CPS = BF16 && H >= 64 && !CENTRAL ? 2 : 1;
  // (fp32 operand mm of layer 1 is the input pair 2 mm + h: the NZ + 1 inputs end in MFMA L1_LAST of the last tile)
  constexpr int L1_LAST = BF16 ? 0 : (NZ + 1 - 8 * (KT1 - 1) + 1) / 2;
  // fp32 networks of 256 units run one wave per SIMD (four per workgroup): their layer-1 outputs live in the
  // accumulation registers that would otherwise lie idle, which leaves room for the output layer on the VALU
  // (the full rollout and the actor fragment alike: they must agree bit for bit)
  constexpr bool H1_ACC = !BF16 && H >= 256 && WAVES == 4 && (PHASE == PHASE_ALL || PHASE == PHASE_ACT);
  typedef Mlp<H, BF16, NB, KT1, L1_LAST, H1_ACC> Net;
  // PHASE_SPLIT: waves [0, RW) evaluate the policy network of row blocks 0 .. RW-1, waves [RW, 2 RW) the value
  // network of the same row blocks (role 1); every stage of both networks is resident in LDS
  constexpr bool SPLIT = PHASE == PHASE_SPLIT;
  static_assert(!SPLIT || WAVES % 2 == 0, "two waves per row block");
  constexpr int RW = SPLIT ? WAVES / 2 : WAVES;  // row blocks of a workgroup
  // LDS window: the stage in use and the one being copied; PHASE_SPLIT: all stages of a step
  constexpr int NBUF = SPLIT ? 2 * Net::NUC / CPS : 2;
  typedef WeightStream<Net, WAVES, NBUF, CPS> Stream;
  typedef typename Net::Op Op;
  static_assert(EPW >= 1, "a wave must hold at least one env");
  constexpr bool DEEP = PHASE == PHASE_DEEP || PHASE == PHASE_ACT_DEEP;
  constexpr bool FULL = (PHASE == PHASE_ALL || PHASE == PHASE_CLOCKS || DEEP || CENTRAL || SPLIT) && !ACT;
  static_assert(!CENTRAL || WAVES == Net::NUC, "centralised critic: one wave per 32-unit chunk");
  // The joint observation is laid out as one block of KT1 tiles per agent, the agent's row exactly as the
  // policy's layer 1 takes it (its constant 1 at input NZ included: agent 0's carries the critic's bias).
  constexpr int KT1C = N * KT1;
  constexpr int JCOLS = WAVES * EPW;            // envs of a workgroup = columns of the critic's tile
  static_assert(!CENTRAL || JCOLS <= 32, "the envs of a workgroup are the columns of one tile");
  constexpr bool HAS_NETS = PHASE != PHASE_ENV && PHASE != PHASE_STEP;     // the variant runs the networks
  constexpr bool STORES_OBS = PHASE != PHASE_MLP && !ACT;                  // ... stores observation rows
  static_assert(NB == 1, "the observation staging below assumes one 32-row block per wave");

  // Observation rows leave through a per-wave LDS staging area: the lanes write their features
  // in row layout, then the wave stores the same bytes as consecutive 16-byte (8-byte when D is
  // not a multiple of 4) pieces, so that one store instruction covers whole cache lines instead
  // of 64 separate rows.  SE envs (SR rows) are staged per pass: all of the wave's when they take at most
  // STG_ALL bytes, else as many as fit STG_SOME (networks of 256 units fill the LDS with their resident
  // layer-1 tiles and the window, fp32 ones the more, so their staging areas are smaller).
  constexpr bool TIGHT = SPLIT && H >= 128;  // (all weights resident: little LDS left)
  constexpr int STG_ALL = (!BF16 && H >= 256) || TIGHT ? 2048 : 4608;
  constexpr int STG_SOME = H >= 256 ? (BF16 ? 2560 : 2048) : (TIGHT ? 2048 : 3072);
  constexpr int SE = EPW * N * D * 4 <= STG_ALL ? EPW : (STG_SOME / (N * D * 4) >= 1 ? STG_SOME / (N * D * 4) : 1);
  constexpr int SR = SE * N;
  constexpr int PASSES = (EPW + SE - 1) / SE;
  constexpr int PW = D % 4 == 0 ? 4 : 2;  // floats per piece
  constexpr int STG = STORES_OBS ? SR * D : 4;

  // (the variants without networks hold no weights, so that as many of their workgroups fit a CU
  // as their registers allow)
  constexpr int L1_SLOTS = HAS_NETS ? Net::L1_TILES * 64 : 1;
  constexpr int W_SLOTS = HAS_NETS ? NBUF * Stream::BUF_SLOTS : 1;
  __shared__ __attribute__((aligned(16))) u32x4 s_l1[CENTRAL ? 1 : 2][L1_SLOTS];  // resident layer-1 tiles
  // centralised critic: joint observations as B-operand tiles, the layer outputs as tiles, partial values
  __shared__ __attribute__((aligned(16))) u32x4 s_j[CENTRAL ? KT1C * 64 : 1];
  __shared__ __attribute__((aligned(16))) u32x4 s_hc[CENTRAL ? Net::KT2 * 64 : 1];
  __shared__ __attribute__((aligned(16))) u32x4 s_w3c[CENTRAL ? WAVES * Net::TPC * 64 : 1];  // its output-layer tiles
  __shared__ float s_vpart[CENTRAL ? WAVES : 1][32];
  __shared__ __attribute__((aligned(16))) u32x4 s_w[W_SLOTS];       // chunk-block window
  __shared__ __attribute__((aligned(16))) float s_b3[2][32];
  __shared__ __attribute__((aligned(16))) float s_stg[WAVES][STG];
  __shared__ float2 s_tab[WAVES][2 * ROWS];  // [0,ROWS) landmarks, [ROWS,2ROWS) agents
  // Per-row outputs of a step (value, action, logp, reward, done) are collected for the whole
  // workgroup and written one array per wave after the next barrier: WAVES * VR consecutive rows
  // per store instead of VR, so that all but the edge cache lines are written whole.
  constexpr int WGR = PHASE == PHASE_MLP ? 1 : RW * VR;
  constexpr int PF = D < (BF16 ? 16 : 8) * KT1 ? D : (BF16 ? 16 : 8) * KT1;  // features every write fills
  constexpr bool PART_IN_STG = PF >= 32 && SR >= 2 && STORES_OBS && H >= 256;
  __shared__ float s_part[WAVES][PART_IN_STG ? 1 : 2 * ROWS];
  // (PHASE_SPLIT: two copies, used in turn by the steps, since the step has no barrier between the
  // store of the collected outputs and the first write of the next ones)
  constexpr int PAR = SPLIT ? 2 : 1;
  __shared__ float s_out[PAR][4][WGR];
  __shared__ __attribute__((aligned(4))) uint8_t s_done[PAR][WGR];
  __shared__ int s_act[SPLIT ? RW : 1][32];  // PHASE_SPLIT: the sampled actions, policy wave -> value wave

  int lane = threadIdx.x & 63;  // (not const: the centralised-critic variant hides it from the optimiser once per step)
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);  // uniform: lives in a scalar register
  const int role = SPLIT ? wave / RW : 0;     // which network this wave evaluates (PHASE_SPLIT)
  const int rset = SPLIT ? wave % RW : wave;  // its row block within the workgroup
  // Both waves of a row block step their own copy of its envs (the same arithmetic on the same actions);
  // the policy wave samples and stores actions, log-probabilities and the final state, the value wave
  // stores the observation rows and computes the reward (2 % faster than everything on the policy wave,
  // whose chain of instructions is the step's critical path).
  const bool writer = role == 0;
  const bool obs_writer = !SPLIT || role == 1;
  const bool rew_writer = !SPLIT || role == 1;
  const int n = lane & 31, h = lane >> 5;
  const int layers = DEEP ? a.layers : 2;
  const NetLayout ly = net_layout(NZ, H, BF16, layers);
  Stream ws;
  ws.lds = s_w;
  ws.packed = a.packed;
  ws.net_bytes = ly.bytes;
  ws.chunks_off = ly.chunks;
  ws.chunk_bytes = ly.chunk_bytes;
  ws.wave = wave;
  ws.lane = lane;
  if constexpr (DEEP) ws.stages_per_net = (layers - 1) * Stream::STAGES_PER_NET;
  // the critic's image (PHASE_CENTRAL): KT1C layer-1 tiles of 16 (bf16) or 8 (fp32) inputs
  const NetLayout lyc = net_layout(KT1C * (BF16 ? 16 : 8) - 1, H, BF16);
  if constexpr (HAS_NETS) {
#pragma unroll
    for (int s = 0; s < Stream::AHEAD; ++s) ws.issue(s, s);
    if constexpr (SPLIT) ws.issue(NBUF - 1, NBUF - 1);  // all of them: nothing is copied inside the step loop
    if constexpr (CENTRAL) {
      const u32x4* src = (const u32x4*)(a.packed + ly.w1);
      for (int i = threadIdx.x; i < Net::L1_TILES * 64; i += blockDim.x) s_l1[0][i] = src[i];
      if (threadIdx.x < 32) {
        s_b3[0][threadIdx.x] = *(const float*)(a.packed + ly.b3 + threadIdx.x * 4);
        s_b3[1][threadIdx.x] = *(const float*)(a.critic + lyc.b3 + threadIdx.x * 4);
      }
#pragma unroll
      for (int i = 0; i < Net::TPC; ++i)  // every wave keeps the output-layer tiles of its own chunk
        s_w3c[(wave * Net::TPC + i) * 64 + lane] =
            ((const u32x4*)(a.critic + lyc.chunks + ((size_t)wave * Net::CHUNK_TILES + Net::L3_OWN + i) * 1024))[lane];
      // joint observations: columns without an env stay zero
      for (int i = threadIdx.x; i < KT1C * 64 * 4; i += blockDim.x) ((uint32_t*)s_j)[i] = 0u;
    } else {
      load_resident(&s_l1[0][0], &s_b3[0][0], a.packed, ly, Net::L1_TILES);
    }
  }
  // features the lanes never write (>= the layer-1 tile range) stay zero for the whole kernel
  for (int i = threadIdx.x; i < WAVES * STG; i += blockDim.x) (&s_stg[0][0])[i] = 0.0f;
  if constexpr (SPLIT)
    ws.wait_all();
  else
    __syncthreads();
  int gs = 0;  // stages consumed so far: stage gs sits in buffer gs % NBUF
  // PHASE_ACT is persistent: the launch has at most one workgroup per compute unit, and a workgroup walks over
  // the row blocks vb = blockIdx.x, blockIdx.x + gridDim.x, ... with one copy of the resident weights and one
  // running weight stream (the set-up above is a tenth of a one-block pass).  Every other variant runs all its
  // steps on one block (the grid covers the blocks).  The walk is a jump back to this label: what is declared
  // below is set up again for the next block.
  constexpr bool PERSIST = PHASE == PHASE_ACT;
  int64_t vb = blockIdx.x;
next_row_block:
  // envs of this workgroup: [blk0, blk0 + envs_per_block); of this wave: EPW of them
  const int64_t blk0 = vb * a.envs_per_block;
  const int64_t blk_end = min(blk0 + (int64_t)a.envs_per_block, (int64_t)a.E);
  const int64_t env0 = blk0 + (int64_t)rset * EPW;
  float2* tab = s_tab[wave];
  float* stg = s_stg[wave];
  // Reward partials (2 x 32 floats, used only between the env move and the end of the step): when the
  // LDS is full they live in staging positions that the next observation write fills again (the
  // first 32 features of staging rows 0 and 1), otherwise in an array of their own.
  float* part0 = PART_IN_STG ? stg : s_part[wave];
  float* part1 = PART_IN_STG ? stg + D : s_part[wave] + ROWS;
  // rows of this wave that hold an env (the same for every lane)
  const int live_rows =
      __builtin_amdgcn_readfirstlane((int)max((int64_t)0, min((int64_t)EPW, blk_end - env0))) * N;

  int row[NB], base[NB], ag[NB];
  uint32_t env[NB];
  bool valid[NB];
  float2 p[NB], v[NB];
  uint32_t g32[NB];
  int tau[NB];
  uint32_t episode[NB];
  int64_t g64[NB];
#pragma unroll
  for (int q = 0; q < NB; ++q) {
    row[q] = 32 * q + n;
    int le = row[q] / N;
    ag[q] = row[q] - le * N;
    valid[q] = row[q] < VR && env0 + le < blk_end;
    if (!valid[q]) {
      le = 0;
      ag[q] = 0;
    }
    base[q] = le * N;
    env[q] = (uint32_t)(valid[q] ? env0 + le : blk0);
    const float* es = a.env_state + (size_t)env[q] * S;
    p[q] = make_float2(es[4 * ag[q]], es[4 * ag[q] + 1]);
    v[q] = make_float2(es[4 * ag[q] + 2], es[4 * ag[q] + 3]);
    const float2 lm = make_float2(es[4 * N + 2 * ag[q]], es[4 * N + 2 * ag[q] + 1]);
    g64[q] = a.g[env[q]];
    g32[q] = (uint32_t)g64[q];
    tau[q] = (int)(g64[q] % a.ep);
    episode[q] = (uint32_t)(g64[q] / a.ep);
    if (h == 0 && valid[q]) {
      tab[base[q] + ag[q]] = lm;
      tab[ROWS + base[q] + ag[q]] = p[q];
    }
  }
  wave_lds_sync();

  const int64_t m0 = env0 * N;  // first trajectory row of this wave
  const int wrow0 = rset * VR;  // ... and its first row within the workgroup
  // stores the collected per-row outputs of step ts; bit k of `arrays` selects array k (value,
  // action, logp, reward, done), which goes out through wave k % WAVES, 64 consecutive rows per
  // store instruction
  auto flush = [&](int ts, int arrays) {
    const int wg_rows = __builtin_amdgcn_readfirstlane((int)(blk_end - blk0)) * N;
    const size_t o0 = (size_t)ts * a.M + (size_t)blk0 * N;
    const int fp = SPLIT ? (ts & 1) : 0;
    constexpr int J = (WGR + 63) / 64;
    for (int arr = wave; arr < 5; arr += WAVES) {
      if (!((arrays >> arr) & 1)) continue;
      if (arr < 4) {
        float vv[J];
#pragma unroll
        for (int j = 0; j < J; ++j) vv[j] = s_out[fp][arr][min(lane + 64 * j, WGR - 1)];
        float* dst = arr == 0 ? a.values : arr == 1 ? (float*)a.actions : arr == 2 ? a.logp : a.rewards;
#pragma unroll
        for (int j = 0; j < J; ++j)
          if (lane + 64 * j < wg_rows) dst[o0 + lane + 64 * j] = vv[j];
      } else {
        uint8_t vv[J];
#pragma unroll
        for (int j = 0; j < J; ++j) vv[j] = s_done[fp][min(lane + 64 * j, WGR - 1)];
#pragma unroll
        for (int j = 0; j < J; ++j)
          if (lane + 64 * j < wg_rows) a.dones[o0 + lane + 64 * j] = vv[j];
      }
    }
  };


  // Outputs of a network as a bit mask (5 logits; the value network uses the first).  Only the fp32 output
  // layer's code depends on it: few outputs run on the VALU (Mlp::l3v).  All 16 bits keep the output layer on
  // the MFMA (bf16 kernels).
  constexpr uint32_t OUTS = BF16 ? 0xFFFFu : 0x1Fu;

  // Centralised critic (PHASE_CENTRAL).  The joint observations of the workgroup's envs are the
  // columns of one tile, and this wave computes the 32-unit chunk `wave` of each hidden layer.  Those
  // weight tiles are nobody else's, so they come straight from global memory (L2) into registers, one
  // policy stage ahead of the MFMAs that use them: every stage barrier already waits for all loads of
  // the wave, and the stage in between covers their latency.  The value is no input of the env step,
  // so nothing waits for it, and the critic rides on the policy's stages with one accumulator and
  // RING tile registers:
  //   step t,   stages S2 .. SPN-1  layer 1 on the joint observation of step t (the barrier of stage 1
  //                                 is the first one behind its writes);
  //   end of the policy stages      tanh, outputs to LDS (s_hc);
  //   step t+1, stages 0 .. S2-1    layer 2;
  //   step t+1, stage S2            tanh, output layer (tiles resident in LDS): the chunk's share of
  //                                 the value to s_vpart;
  //   step t+2, top                 every wave adds the shares of its envs; the values go out with the
  //                                 other per-row outputs at the barrier of stage 1.
  // The last step's layers 2 and 3 run behind the loop.
  constexpr int SPN = Stream::STAGES_PER_NET;
  static_assert(!CENTRAL || SPN >= 2, "the critic rides on the policy stages");
  constexpr int L2T = Net::KT2 + 1;  // layer-2 tiles of a chunk, the bias tile included
  constexpr int S2_ = (SPN * L2T + (L2T + KT1C) / 2) / (L2T + KT1C);  // stages in proportion to the tiles
  constexpr int S2 = S2_ < 1 ? 1 : (S2_ > SPN - 1 ? SPN - 1 : S2_);
  constexpr int S1 = SPN - S2;
  constexpr int RING = !CENTRAL ? 1 : ((L2T + S2 - 1) / S2 > (KT1C + S1 - 1) / S1 ? (L2T + S2 - 1) / S2 : (KT1C + S1 - 1) / S1);
  // uniform base addresses (scalar registers) of the chunk's layer-1 tiles and of its chunk block; the
  // lanes add 16 lane.  A fetch of RING tiles may reach past the tiles of its layer, by fewer than
  // CRITIC_FETCH_PAD_TILES tiles: the surplus is not used, and the host keeps that much memory behind
  // the critic's image so that the last wave's fetches stay inside the allocation.
  static_assert(!CENTRAL || (S2 * RING - L2T <= CRITIC_FETCH_PAD_TILES && S1 * RING - KT1C <= CRITIC_FETCH_PAD_TILES),
                "fetch range");
  const uint8_t* t1 = a.critic + (size_t)wave * KT1C * 1024;
  const uint8_t* t2 = a.critic + lyc.chunks + (size_t)wave * Net::CHUNK_TILES * 1024;
  const uint32_t lane16 = (uint32_t)lane * 16u;
  // Fetch of tiles [0, CNT) behind a base address into dst[0 .. CNT).  Left alone, the compiler
  // computes 64-bit vector addresses and keeps them in registers.  So the lane offset and the scalar
  // address of every group of four tiles (the reach of the immediate offset) are made opaque at every
  // fetch: a load then takes a scalar base, one 32-bit lane offset and an immediate.
  auto fetch_tiles = [&](const uint8_t* base, auto cnt, u32x4* dst) {
    typedef __attribute__((address_space(1))) const u32x4 global_u32x4;
    constexpr int CNT = decltype(cnt)::value;
    uint32_t off = lane16;
    asm volatile("" : "+v"(off));
#pragma unroll
    for (int g = 0; g < (CNT + 3) / 4; ++g) {
      uint64_t gb = (uint64_t)(uintptr_t)base + (uint64_t)(4 * g) * 1024;
      // (uniform: make it scalar; the builtin returns a signed int, which must not sign-extend into the high half)
      gb = (uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)gb) |
           (uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(gb >> 32)) << 32;
      asm volatile("" : "+s"(gb));
#pragma unroll
      for (int i = 4 * g; i < 4 * g + 4 && i < CNT; ++i) dst[i] = *(global_u32x4*)(gb + (uint64_t)(i - 4 * g) * 1024 + off);
    }
  };
  f32x16 cacc = zero16();
  u32x4 cring[RING];
  // layer-2 tile kt of the chunk times the layer-1 outputs in s_hc (the bias tile times the constant 1)
  // (a tile of B operands in LDS is 16 bytes per lane for both types: one bf16 operand or the four fp32 ones)
  auto lds_operands = [&](const u32x4& raw, Op (&b)[Net::PT]) {
    if constexpr (BF16) {
      b[0] = __builtin_bit_cast(bf16x8, raw);
    } else {
      const f32x4 f = __builtin_bit_cast(f32x4, raw);
#pragma unroll
      for (int i = 0; i < 4; ++i) b[i] = f[i];
    }
  };
  auto critic_l2_tile = [&](const u32x4& w, int kt, f32x16& c) {
    if (kt < Net::KT2) {
      Op b[Net::PT];
      lds_operands(s_hc[kt * 64 + lane], b);
      mma_tile<BF16>(w, b, c);
    } else {
      mma_bias_tile<BF16>(w, Operand<BF16>::one(h), c);
    }
  };
  // tanh of the chunk's layer-2 sums and the output layer: the chunk's share of the value of column lane % 32
  auto critic_l3 = [&](const f32x16& c) {
    float tt[16];
    Op h2c[Net::PC];
    tanh_range<!BF16>(c, tt, 0, 16, false);
    to_operands<BF16>(tt, h2c);
    f32x16 ov = zero16();
#pragma unroll
    for (int i = 0; i < Net::TPC; ++i) mma_tile<BF16>(s_w3c[(wave * Net::TPC + i) * 64 + lane], &h2c[i * Net::PT], ov);
    if (h == 0) s_vpart[wave][n] = ov[0];  // output 0: register 0 of the h = 0 lanes
  };
  // tanh of the chunk's layer-1 sums; outputs (as the next layer's operand tiles) to s_hc
  auto critic_l1_publish = [&](const f32x16& c) {
    float tt[16];
    Op hc[Net::PC];
    tanh_range<!BF16>(c, tt, 0, 16, false);
    to_operands<BF16>(tt, hc);
    // the chunk's 32 units are TPC tiles of the next layer's contraction
#pragma unroll
    for (int i = 0; i < Net::TPC; ++i) {
      u32x4 raw;
      if constexpr (BF16)
        raw = __builtin_bit_cast(u32x4, hc[i]);
      else
        raw = __builtin_bit_cast(u32x4, f32x4{hc[4 * i], hc[4 * i + 1], hc[4 * i + 2], hc[4 * i + 3]});
      s_hc[(Net::TPC * wave + i) * 64 + lane] = raw;
    }
  };
  // value of the rows' envs from the shares in s_vpart
  auto collect_values = [&]() {
#pragma unroll
    for (int q = 0; q < NB; ++q) {
      const int col = wave * EPW + base[q] / N;
      float vsum = s_b3[1][0];
#pragma unroll
      for (int w = 0; w < WAVES; ++w) vsum += s_vpart[w][col];
      if (h == 0 && valid[q]) s_out[0][0][wrow0 + row[q]] = vsum;
    }
  };
  float checksum[NB] = {};      // PHASE_MLP only

  long long clk0 = 0;
  for (int t = 0; t <= a.T; ++t) {
    const int par = SPLIT ? (t & 1) : 0;
    auto stamp = [&](int i) {
      if constexpr (PHASE == PHASE_CLOCKS) {
        if (blockIdx.x == 0 && t == a.T / 2 && lane == 0) {
          const long long now = clock64();
          if (i == CLK_START) clk0 = now;
          a.logits[32 * wave + i] = (float)(now - clk0);
        }
      }
    };
    stamp(CLK_START);
    // PHASE_CLOCKS: the wait for a stage (copies landed + workgroup barrier), timed
    long long clk_wait = 0;
    auto stage_wait = [&]() {
      if constexpr (PHASE == PHASE_CLOCKS) {
        const long long w0 = clock64();
        ws.wait_oldest();
        clk_wait += clock64() - w0;
      } else {
        ws.wait_oldest();
      }
    };
    if constexpr (CENTRAL || DEEP) {
      // The compiler moves every address and constant that does not change over the steps in front of
      // the loop; with the registers of these variants on top they no longer fit and would be reloaded from
      // scratch memory step by step.  Hiding the lane's indices from it once per step keeps that
      // arithmetic (a few dozen integer operations) inside the step.  (n, h and the wave's
      // scalars stay where they are.)
      asm volatile("" : "+v"(ag[0]), "+v"(base[0]), "+v"(row[0]), "+v"(env[0]), "+v"(lane));
    }
    if constexpr (!HAS_NETS) {  // (no stage barriers in these variants)
      __syncthreads();
      if (t > 0) flush(t - 1, PHASE == PHASE_STEP ? 0x18 : 0x1f);
      __syncthreads();
    } else if constexpr (SPLIT) {
      // every wave has finished step t-1: its collected outputs (in the other copy of s_out) go out
      __syncthreads();
      if (t > 0) flush(t - 1, 0x1f);
    } else {
      // The barrier of the policy network's first stage comes first in the step: its copies went out
      // during the last stage of the step before, and the wait for them also waits for every store
      // the wave still has in flight, so it must not sit behind the observation stores below.
      stage_wait();
      if constexpr (CENTRAL) {
        if (t > 1) collect_values();  // of step t - 2
      }
    }
    // ---------------- observation rows: build, store (through the staging area), convert to MFMA operands
    Op x[NB][KT1 * Net::PT];
    {
      constexpr int q = 0;
      auto pair_value = [&](int gp) -> float2 {
        // pair 0: v, 1: p, [2, 2+L): landmark - p, [2+L, 1+L+N): other agent - p, rest 0
        const int jj = gp - 2 - L;
        const int j = jj + (jj >= ag[q] ? 1 : 0);
        int idx = gp < 2 + L ? base[q] + gp - 2 : ROWS + base[q] + j;
        idx = min(max(idx, 0), 2 * ROWS - 1);
        const float2 tv = tab[idx];
        float2 o = make_float2(tv.x - p[q].x, tv.y - p[q].y);
        if (gp >= 1 + L + N) o = make_float2(0.0f, 0.0f);
        if (gp == 1) o = p[q];
        if (gp == 0) o = v[q];
        return o;
      };
      // pairs this lane contributes to the stored row: bf16 tiles hold 4 consecutive pairs per lane,
      // f32 tiles hold pair mm on both half-waves, of which half-wave mm % 2 stores it
      constexpr int NP = BF16 ? 4 * KT1 : 2 * KT1;
      float2 pr[NP];
      // PHASE_ACT takes the pair from the caller's row instead (zero beyond the row and for idle rows)
      auto pair_in = [&](int gp) -> float2 {
        if constexpr (ACT) {
          if (!valid[q] || 2 * gp + 2 > D) return make_float2(0.0f, 0.0f);
          return *(const float2*)(a.obs_in + (size_t)(m0 + row[q]) * D + 2 * gp);
        } else {
          return pair_value(gp);
        }
      };
      const bool build = PHASE != PHASE_STEP || t == a.T;  // PHASE_STEP needs rows only to store them
      if (!build) {
#pragma unroll
        for (int i = 0; i < NP; ++i) pr[i] = make_float2(0.0f, 0.0f);
#pragma unroll
        for (int i = 0; i < KT1 * Net::PT; ++i) x[q][i] = Op{};
      } else if constexpr (BF16) {
#pragma unroll
        for (int i = 0; i < NP; ++i) pr[i] = pair_in(8 * (i / 4) + 4 * h + i % 4);
      } else {
#pragma unroll
        for (int mm = 0; mm < KT1 * 4; ++mm) {
          const float2 o = pair_in(mm);
          if ((mm & 1) == 0) pr[mm / 2] = o;
          if ((mm & 1) == 1 && h == 1) pr[mm / 2] = o;
          x[q][mm] = h ? o.y : o.x;
          if (2 * mm == NZ) x[q][mm] = h ? 0.0f : 1.0f;  // input NZ carries the bias
        }
        if constexpr (CENTRAL) {
          // the same operands, four to a tile, are the agent's block of column (env) `col` of the joint observation
          if (valid[q]) {
            u32x4* dst = s_j + (ag[q] * KT1) * 64 + h * 32 + wave * EPW + base[q] / N;
#pragma unroll
            for (int kt = 0; kt < KT1; ++kt)
              dst[kt * 64] = __builtin_bit_cast(u32x4, f32x4{x[q][4 * kt], x[q][4 * kt + 1], x[q][4 * kt + 2], x[q][4 * kt + 3]});
          }
        }
      }
      // feature index of pr[i]
      auto feat = [&](int i) { return BF16 ? 16 * (i / 4) + 8 * h + 2 * (i % 4) : 4 * i + 2 * h; };
      if (STORES_OBS && build) {
#pragma unroll
        for (int ps = 0; ps < PASSES; ++ps) {
          const int r0 = ps * SR;
          const int lr = row[q] - r0;
          if (valid[q] && lr >= 0 && lr < SR) {
            float* dst = stg + lr * D;
            if constexpr (BF16 && D % 4 == 0) {
#pragma unroll
              for (int i = 0; i < NP; i += 2)
                if (feat(i) + 4 <= D)
                  *(float4*)(dst + feat(i)) = make_float4(pr[i].x, pr[i].y, pr[i + 1].x, pr[i + 1].y);
            } else {
#pragma unroll
              for (int i = 0; i < NP; ++i)
                if (feat(i) + 2 <= D) *(float2*)(dst + feat(i)) = pr[i];
            }
          }
          wave_lds_sync();
          const int pieces = obs_writer ? min(SR, live_rows - r0) * (D / PW) : 0;
          float* gdst = a.obs + ((size_t)(PHASE == PHASE_STEP ? 0 : t) * a.M + m0 + r0) * D;
#pragma unroll
          for (int j = 0; j * 64 < SR * (D / PW); ++j) {
            const int i = j * 64 + lane;
            if (i < pieces) {
              if constexpr (PW == 4)
                *(float4*)(gdst + 4 * i) = *(const float4*)(stg + 4 * i);
              else
                *(float2*)(gdst + 2 * i) = *(const float2*)(stg + 2 * i);
            }
          }
          wave_lds_sync();
        }
      }
      if constexpr (BF16) {
#pragma unroll
        for (int kt = 0; kt < KT1; ++kt) {
          f32x8 f;
#pragma unroll
          for (int pi = 0; pi < 4; ++pi) {
            f[2 * pi] = pr[4 * kt + pi].x;
            f[2 * pi + 1] = pr[4 * kt + pi].y;
          }
          if (NZ / 16 == kt && (NZ % 16) / 8 == h) f[NZ % 8] = 1.0f;  // input NZ carries the bias
          x[q][kt] = __builtin_convertvector(f, bf16x8);
        }
        if constexpr (CENTRAL) {
          // the same operands are the agent's block of column (env) `col` of the joint observation
          if (valid[q]) {
            u32x4* dst = s_j + (ag[q] * KT1) * 64 + h * 32 + wave * EPW + base[q] / N;
#pragma unroll
            for (int kt = 0; kt < KT1; ++kt) dst[kt * 64] = __builtin_bit_cast(u32x4, x[q][kt]);
          }
        }
      }
    }

    stamp(CLK_OBS);
    // ---------------- networks: policy, then value; chunk blocks come through the LDS window
    f32x16 out_p[NB], out_v[NB];
    if constexpr (!HAS_NETS) {
#pragma unroll
      for (int q = 0; q < NB; ++q) out_p[q] = out_v[q] = zero16();
    } else {
      Op h1[NB][Net::KT2 * Net::PT];
      if constexpr (DEEP) {
        const int spn = ws.stages_per_net;
#pragma unroll 1
        for (int net = 0; net < 2; ++net) {
          f32x16(&out)[NB] = net == 0 ? out_p : out_v;
          if (net == 1) {
            ws.wait_oldest();
            if (t > 0) flush(t - 1, 0x1f);
          }
          Net::layer1(&s_l1[net][0] + lane, x, h1);
          int sn = 0;  // stage within the network
          auto prefetch_target = [&](int& next, int& nbuf) {
            next = net * spn + sn + Stream::AHEAD;
            if (next >= 2 * spn) next -= 2 * spn;
            nbuf = (gs + Stream::AHEAD) % NBUF;
          };
          f32x16 acc[NB];
          // hidden layers 2 .. layers-1: h1 <- tanh(W h1 + b), one 32-unit chunk per block
#pragma unroll 1
          for (int layer = 2; layer < layers; ++layer) {
            Op hb[NB][Net::KT2 * Net::PT];
#pragma unroll 1
            for (int sc = 0; sc < Stream::STAGES_PER_NET; ++sc) {
              if (sn != 0) ws.wait_oldest();
              int next, nbuf;
              prefetch_target(next, nbuf);
              Op hn[CPS][NB][Net::PC];
#pragma unroll
              for (int c = 0; c < CPS; ++c) {
                const u32x4* tiles = ws.tiles(gs % NBUF, c);
                auto tick = [&](int kt) {
#pragma unroll
                  for (int i = 0; i < Stream::PER_WAVE; ++i)
                    if (i * (CPS * Net::KT2) / Stream::PER_WAVE == c * Net::KT2 + kt) ws.issue_part(next, nbuf, i);
                };
                if (c == 0 && sc == 0)
                  Net::template hidden_chunk<false>(tiles, h1, acc, hn[c], h, tick);
                else
                  Net::template hidden_chunk<true>(tiles, h1, acc, hn[c], h, tick);
              }
              // file the finished chunks (register indices are compile-time constants inside each branch)
#pragma unroll
              for (int k = 0; k < Stream::STAGES_PER_NET; ++k)
                if (sc == k) {
#pragma unroll
                  for (int c = 0; c < CPS; ++c) {
                    const int idx = k * CPS + c - 1;
                    if (idx >= 0) {
#pragma unroll
                      for (int q = 0; q < NB; ++q)
#pragma unroll
                        for (int j = 0; j < Net::PC; ++j) hb[q][idx * Net::PC + j] = hn[c][q][j];
                    }
                  }
                }
              ++gs;
              ++sn;
            }
            {
              Op hl[NB][Net::PC];
              Net::hidden_drain(acc, hl);
#pragma unroll
              for (int q = 0; q < NB; ++q)
#pragma unroll
                for (int j = 0; j < Net::PC; ++j) hb[q][(Net::NUC - 1) * Net::PC + j] = hl[q][j];
            }
#pragma unroll
            for (int q = 0; q < NB; ++q)
#pragma unroll
              for (int j = 0; j < Net::KT2 * Net::PT; ++j) h1[q][j] = hb[q][j];
          }
          // last hidden layer and output layer
          {
            const f32x16 b = Net::template out_init<OUTS>(s_b3[net], h);
#pragma unroll
            for (int q = 0; q < NB; ++q) out[q] = b;
          }
#pragma unroll 1
          for (int sc = 0; sc < Stream::STAGES_PER_NET; ++sc) {
            if (sn != 0) ws.wait_oldest();
            int next, nbuf;
            prefetch_target(next, nbuf);
#pragma unroll
            for (int c = 0; c < CPS; ++c) {
              const u32x4* tiles = ws.tiles(gs % NBUF, c);
              auto tick = [&](int kt) {
#pragma unroll
                for (int i = 0; i < Stream::PER_WAVE; ++i)
                  if (i * (CPS * Net::KT2) / Stream::PER_WAVE == c * Net::KT2 + kt) ws.issue_part(next, nbuf, i);
              };
              if (c == 0 && sc == 0)
                Net::template layer2_chunk<false, OUTS>(tiles, h1, acc, out, h, 16, tick);
              else
                Net::template layer2_chunk<true, OUTS>(tiles, h1, acc, out, h, 16, tick);
              if (c == CPS - 1 && sc == Stream::STAGES_PER_NET - 1)
                Net::template layer2_drain<OUTS>(tiles, acc, out, h, 16);
            }
            ++gs;
            ++sn;
          }
          Net::template out_finish<OUTS>(out, s_b3[net], h);
        }
      } else if constexpr (SPLIT) {
        // ---------------- this wave's network; all its stages are resident: no copies, waits or barriers
        f32x16 out[NB], acc[NB];
        Net::layer1(&s_l1[role][0] + lane, x, h1);
        auto tick = [&](int, int) {};
        {
          const f32x16 b = Net::template out_init<OUTS>(s_b3[role], h);
#pragma unroll
          for (int q = 0; q < NB; ++q) out[q] = b;
        }
        // (the value wave computes all five sums too: its output-layer rows beyond the first are zero)
#pragma unroll
        for (int sc = 0; sc < Stream::STAGES_PER_NET; ++sc) {
          const int buf = role * Stream::STAGES_PER_NET + sc;
          if (sc == 0)
            Net::template layer2_chunks<false, CPS, OUTS>(ws.tiles(buf, 0), h1, acc, out, h, 16, tick);
          else
            Net::template layer2_chunks<true, CPS, OUTS>(ws.tiles(buf, 0), h1, acc, out, h, 16, tick);
          if (sc == Stream::STAGES_PER_NET - 1)
            Net::template layer2_drain<OUTS>(ws.tiles(buf, CPS - 1), acc, out, h, 16);
        }
        Net::template out_finish<OUTS>(out, s_b3[role], h);
#pragma unroll
        for (int q = 0; q < NB; ++q) out_p[q] = out_v[q] = out[q];
      } else if constexpr (CENTRAL) {
        // ---------------- policy network through the window, the critic riding on its stages
        Net::layer1(&s_l1[0][0] + lane, x, h1);
        f32x16 acc[NB];
        {
          const f32x16 b = Net::template out_init<OUTS>(s_b3[0], h);
#pragma unroll
          for (int q = 0; q < NB; ++q) out_p[q] = b;
        }
#pragma unroll 1
        for (int sc = 0; sc < SPN; ++sc) {
          if (sc != 0) {
            ws.wait_oldest();
            if (sc == 1 && t > 0) {
              flush(t - 1, 0x1e);
              if (t > 1) flush(t - 2, 0x01);
            }
          }
          // critic: the tiles fetched during the stage before
          if (sc < S2) {
            if (t > 0) {
#pragma unroll
              for (int i = 0; i < RING; ++i)
                if (sc * RING + i < L2T) critic_l2_tile(cring[i], sc * RING + i, cacc);
            }
          } else {
            if (sc == S2) {
              if (t > 0) critic_l3(cacc);  // of the step before
              cacc = zero16();
            }
#pragma unroll
            for (int i = 0; i < RING; ++i) {
              const int kt = (sc - S2) * RING + i;
              if (kt < KT1C) {
                Op b[Net::PT];
                lds_operands(s_j[kt * 64 + lane], b);
                mma_tile<BF16>(cring[i], b, cacc);
              }
            }
          }
          {
            // ... and the fetch for the next stage (in the last stage, for stage 0 of the next step)
            const uint8_t* nb = sc + 1 < S2 ? t2 + (size_t)(sc + 1) * RING * 1024
                                : sc + 1 < SPN ? t1 + (size_t)(sc + 1 - S2) * RING * 1024 : t2;
            fetch_tiles(nb, std::integral_constant<int, RING>{}, cring);
          }
          int next = sc + Stream::AHEAD;  // AHEAD stages ahead, cyclic over the step
          if (next >= SPN) next -= SPN;
          const int nbuf = (gs + Stream::AHEAD) % NBUF;
          const u32x4* tiles = ws.tiles(gs % NBUF, 0);
          auto tick = [&](int kt) {
#pragma unroll
            for (int i = 0; i < Stream::PER_WAVE; ++i)
              if (i * Net::KT2 / Stream::PER_WAVE == kt) ws.issue_part(next, nbuf, i);
          };
          if (sc == 0)
            Net::template layer2_chunk<false, OUTS>(tiles, h1, acc, out_p, h, 16, tick);
          else
            Net::template layer2_chunk<true, OUTS>(tiles, h1, acc, out_p, h, 16, tick);
          if (sc == SPN - 1) Net::template layer2_drain<OUTS>(tiles, acc, out_p, h, 16);
          ++gs;
        }
        Net::template out_finish<OUTS>(out_p, s_b3[0], h);

        critic_l1_publish(cacc);
        cacc = zero16();  // layer 2 starts from zero in stage 0 of the next step
#pragma unroll
        for (int q = 0; q < NB; ++q) out_v[q] = zero16();
      } else {
  #pragma unroll
        for (int net = 0; net < 2; ++net) {
          f32x16(&out)[NB] = net == 0 ? out_p : out_v;
          // The first stage of the value network landed long ago, so its barrier can come before
          // layer 1.  Every wave has left the previous step long since and the store path is idle
          // (the observation stores went out at the start of the step): the collected per-row
          // outputs of the previous step go out here.
          if (net == 1) {
            stage_wait();
            if (FULL && t > 0) flush(t - 1, 0x1f);
            // The flush reads s_out / s_done of step t-1; the next writes to them are this step's values,
            // behind the value network.  A network of several stages has a stage barrier in between; one
            // that fits a single stage has none, so the order is made explicit here.
            if constexpr (Stream::STAGES_PER_NET == 1) __syncthreads();
          }
          Net::layer1(&s_l1[net][0] + lane, x, h1);
          stamp(net == 0 ? CLK_P_L1 : CLK_V_L1);
          f32x16 acc[NB];
          const int nout = net == 0 ? 5 : 1;  // (a constant once the loop over the networks is unrolled)
          {
            const f32x16 b = Net::template out_init<OUTS>(s_b3[net], h);
  #pragma unroll
            for (int q = 0; q < NB; ++q) out[q] = b;
          }
  #pragma unroll 1
          for (int sc = 0; sc < Stream::STAGES_PER_NET; ++sc) {
            if (sc != 0) stage_wait();
            int next = net * Stream::STAGES_PER_NET + sc + Stream::AHEAD;  // AHEAD stages ahead, cyclic over the step
            if (next >= Stream::STAGES_PER_STEP) next -= Stream::STAGES_PER_STEP;
            const int nbuf = (gs + Stream::AHEAD) % NBUF;
            {
              // the copies of the stage AHEAD stages later, spread over this stage's tile loops
              auto tick = [&](int c, int kt) {
  #pragma unroll
                for (int i = 0; i < Stream::PER_WAVE; ++i)
                  if (i * (CPS * Net::KT2) / Stream::PER_WAVE == c * Net::KT2 + kt) ws.issue_part(next, nbuf, i);
                if (kt == 0 && c == 0) stage_priority(sc, wave, WAVES);  // (1 % of the call at the benchmark's shape)
              };
              if (sc == 0)
                Net::template layer2_chunks<false, CPS, OUTS>(ws.tiles(gs % NBUF, 0), h1, acc, out, h, nout, tick);
              else
                Net::template layer2_chunks<true, CPS, OUTS>(ws.tiles(gs % NBUF, 0), h1, acc, out, h, nout, tick);
              if (sc == Stream::STAGES_PER_NET - 1)
                Net::template layer2_drain<OUTS>(ws.tiles(gs % NBUF, CPS - 1), acc, out, h, nout);
            }
            ++gs;
            if (sc < 5) stamp((net == 0 ? CLK_P_STAGE : CLK_V_STAGE) + sc);
          }
          Net::template out_finish<OUTS>(out, s_b3[net], h);
        }
      }
    }
    stamp(CLK_NETS);
    if constexpr (PHASE == PHASE_MLP) {
#pragma unroll
      for (int q = 0; q < NB; ++q)
        checksum[q] += out_v[q][0] + out_p[q][0] + out_p[q][1] + out_p[q][2] + out_p[q][3];
      continue;
    }
    if constexpr (!CENTRAL) {
#pragma unroll
      for (int q = 0; q < NB; ++q)
        if (h == 0 && valid[q] && (!SPLIT || role == 1)) s_out[par][0][wrow0 + row[q]] = out_v[q][0];
    }
    if (!ACT && t == a.T) break;

    // ---------------- sampling, physics
    float rew_term[NB];
    int action[NB];
#pragma unroll
    for (int q = 0; q < NB; ++q) {
      float l[5];
      l[0] = out_p[q][0];
      l[1] = out_p[q][1];
      l[2] = out_p[q][2];
      l[3] = out_p[q][3];
      l[4] = __shfl_xor(out_p[q][0], 32);  // logit 4 sits in register 0 of the partner lane
      float lp = 0.0f;
      int act = 0;
      if (writer) {  // (uniform)
        const Words4 w = draw(a.seed_lo, a.seed_hi, env[q], (uint32_t)ag[q], g32[q], 0, 0);
        sample_categorical5(l, u01(w.w[0]), act, lp);
        act = __shfl(act, n);  // the h = 0 lane of the row decides
      }
      if constexpr (SPLIT) {
        // the value wave of the row block moves its copy of the envs with the policy wave's actions
        if (writer && h == 0) s_act[rset][n] = act;
        __syncthreads();
        if (!writer) act = s_act[rset][n];
      }
      if constexpr (PHASE == PHASE_STEP) act = valid[q] ? ((const int32_t*)a.actions_in)[m0 + row[q]] : 0;
      action[q] = act;
      const size_t o = (size_t)t * a.M + m0 + row[q];
      if (h == 0 && valid[q] && writer) {
        s_out[par][1][wrow0 + row[q]] = __int_as_float(act);
        s_out[par][2][wrow0 + row[q]] = lp;
        if (PHASE != PHASE_CLOCKS && a.logits) {
#pragma unroll
          for (int k = 0; k < 5; ++k) a.logits[o * 5 + k] = l[k];
        }
      }
      const float fx = (act == 1 ? 1.0f : 0.0f) - (act == 2 ? 1.0f : 0.0f);
      const float fy = (act == 3 ? 1.0f : 0.0f) - (act == 4 ? 1.0f : 0.0f);
      v[q].x = v[q].x * a.keep + fx * a.fdt;
      v[q].y = v[q].y * a.keep + fy * a.fdt;
      p[q].x += v[q].x * a.dt;
      p[q].y += v[q].y * a.dt;
      if (h == 0 && valid[q]) tab[ROWS + base[q] + ag[q]] = p[q];
    }
    wave_lds_sync();
    stamp(CLK_SAMPLE);
    if constexpr (ACT) break;  // one evaluation, no move

    // ---------------- shared reward: lane h = 0 takes landmark ag (distance of the nearest agent),
    // lane h = 1 agent ag (collisions with the agents after it): one distance per lane and agent
#pragma unroll
    for (int q = 0; q < NB; ++q) {
      if (!rew_writer) break;  // (uniform)
      const float2 lm = tab[base[q] + ag[q]];
      const float2 ref = h ? p[q] : lm;
      float mn = 3.0e38f, cnt = 0.0f;
#pragma unroll
      for (int j = 0; j < N; ++j) {
        const float2 pj = tab[ROWS + base[q] + j];
        const float dx = pj.x - ref.x, dy = pj.y - ref.y;
        const float d2 = dx * dx + dy * dy;
        mn = fminf(mn, d2);
        cnt += (j > ag[q] && d2 < a.coll2) ? 1.0f : 0.0f;
      }
      rew_term[q] = h ? -cnt : -__builtin_amdgcn_sqrtf(mn);
      if (valid[q]) (h ? part1 : part0)[base[q] + ag[q]] = rew_term[q];
    }
    wave_lds_sync();
#pragma unroll
    for (int q = 0; q < NB; ++q) {
      // each half-wave sums its own kind of term over the env's agents; the halves are then added
      float r = 0.0f;
      if (rew_writer) {  // (uniform)
        const float* mine = h ? part1 : part0;
#pragma unroll
        for (int j = 0; j < N; ++j) r += mine[base[q] + j];
        r += __shfl_xor(r, 32);
      }
      const bool done = tau[q] + 1 == a.ep;
      if (h == 0 && valid[q] && rew_writer) {
        s_out[par][3][wrow0 + row[q]] = r;
        s_done[par][wrow0 + row[q]] = done ? 1 : 0;
      }
      g32[q] += 1;
      tau[q] = done ? 0 : tau[q] + 1;
      if (done) {
        episode[q] += 1;
        const Words4 wa = draw(a.seed_lo, a.seed_hi, env[q], (uint32_t)ag[q], episode[q], 1, 0);
        p[q] = make_float2(2.0f * u01(wa.w[0]) - 1.0f, 2.0f * u01(wa.w[1]) - 1.0f);
        v[q] = make_float2(0.0f, 0.0f);
        const Words4 wl = draw(a.seed_lo, a.seed_hi, env[q], (uint32_t)(N + ag[q]), episode[q], 1, 0);
        if (h == 0 && valid[q]) {
          tab[base[q] + ag[q]] = make_float2(2.0f * u01(wl.w[0]) - 1.0f, 2.0f * u01(wl.w[1]) - 1.0f);
          tab[ROWS + base[q] + ag[q]] = p[q];
        }
      }
    }
    wave_lds_sync();
    stamp(CLK_END);
    if constexpr (PHASE == PHASE_CLOCKS) {
      if (blockIdx.x == 0 && t == a.T / 2 && lane == 0) a.logits[32 * wave + CLK_WAIT] = (float)clk_wait;
    }
  }

  if constexpr (PERSIST) {
    __syncthreads();  // every wave's outputs of this row block are in s_out
    flush(0, 0x07);   // values, actions, logp (the next block writes s_out behind several stage barriers)
    vb += gridDim.x;
    if (vb * a.envs_per_block < a.E) goto next_row_block;
    ws.wait_all();  // copies issued ahead for a block that will not come
    return;
  }
  if constexpr (HAS_NETS) ws.wait_all();  // copies issued ahead for stages that will not run
  if constexpr (!HAS_NETS) __syncthreads();
  if constexpr (ACT && !CENTRAL) {
    flush(0, 0x07);  // values, actions, logp of the one evaluation
    return;          // the env state did not move
  }
  if constexpr (CENTRAL) {
    // values of the last two steps: the shares of step T-1 are in s_vpart; layers 2 and 3 of step T
    // have no policy stages left to ride on and run here
    u32x4 wl[L2T];
    fetch_tiles(t2, std::integral_constant<int, L2T>{}, wl);
    if (a.T > 0) collect_values();
    cacc = zero16();
#pragma unroll
    for (int kt = 0; kt < L2T; ++kt) critic_l2_tile(wl[kt], kt, cacc);
    __syncthreads();  // s_out[0] holds the values of step T-1, and nobody reads s_vpart any more
    if (a.T > 0) flush(a.T - 1, 0x01);
    critic_l3(cacc);
    __syncthreads();
    collect_values();
    __syncthreads();
    if constexpr (ACT) {
      flush(0, 0x07);  // values (just collected), actions, logp of the one evaluation
      return;          // the env state did not move
    }
  }
  if constexpr (PHASE != PHASE_MLP && PHASE != PHASE_STEP)
    flush(a.T, 0x01);  // values[T]; every earlier step went out inside the loop
  if constexpr (PHASE == PHASE_MLP) {
#pragma unroll
    for (int q = 0; q < NB; ++q)
      if (valid[q]) a.rewards[m0 + row[q]] = checksum[q];
    return;  // the env state did not move
  }

  // ---------------- write the env state back
#pragma unroll
  for (int q = 0; q < NB; ++q) {
    if (h == 0 && valid[q] && writer) {
      float* es = a.env_state + (size_t)env[q] * S;
      es[4 * ag[q]] = p[q].x;
      es[4 * ag[q] + 1] = p[q].y;
      es[4 * ag[q] + 2] = v[q].x;
      es[4 * ag[q] + 3] = v[q].y;
      const float2 lm = tab[base[q] + ag[q]];
      es[4 * N + 2 * ag[q]] = lm.x;
      es[4 * N + 2 * ag[q] + 1] = lm.y;
      if (ag[q] == 0) a.g[env[q]] = g64[q] + a.T;
    }
  }
}

// ------------------------------------------------------------------ linear-Gaussian env
// State unit u of a row lives in accumulator layout: lane (n, h), register r with
// u = 8*(r/4) + 4*h + r%4, so s' = A s + B a is one more MFMA chain on the same
// registers and its result is already the next step's layer-1 operand.
// PHASE: PHASE_ALL, or one of the step-granular variants PHASE_ACT / PHASE_STEP (see above; here
// actions_in is float [M, K]).
template <int D, int K, int H, int WAVES, int PHASE = PHASE_ALL>
__global__ __launch_bounds__(64 * WAVES) void lingauss_rollout_kernel(RolloutArgs a) {
  static_assert(PHASE == PHASE_ALL || PHASE == PHASE_ACT || PHASE == PHASE_STEP || PHASE == PHASE_DEEP ||
                    PHASE == PHASE_ACT_DEEP,
                "no measurement variants here");
  constexpr bool HAS_NETS = PHASE != PHASE_STEP;
  constexpr bool DEEP = PHASE == PHASE_DEEP || PHASE == PHASE_ACT_DEEP;
  constexpr bool ACT = PHASE == PHASE_ACT || PHASE == PHASE_ACT_DEEP;
  constexpr int KT1 = (D + 1 + 7) / 8;  // + the constant-1 input that carries the bias
  constexpr int NR = 4 * KT1;           // state registers per lane
  constexpr int NBUF = 2, CPS = 1;
  // (the state sits in accumulator layout: MFMA j of a layer-1 tile multiplies inputs 8 kt + j and 8 kt + 4 + j,
  // so the D + 1 inputs, the constant 1 included, reach MFMA min(4, inputs in the last tile) of the last tile)
  constexpr int L1_REST = D + 1 - 8 * (KT1 - 1);
  // (one wave per SIMD: the layer-1 outputs live in accumulation registers, 151 vector registers instead of 256)
  typedef Mlp<H, false, 1, KT1, L1_REST < 4 ? L1_REST : 4, true> Net;
  typedef WeightStream<Net, WAVES, NBUF, CPS> Stream;
  static_assert(D <= 31 && K <= 8, "one MFMA chunk of state (plus the constant input), one tile of action");

  __shared__ __attribute__((aligned(16))) u32x4 s_l1[2][HAS_NETS ? Net::L1_TILES * 64 : 1];
  __shared__ __attribute__((aligned(16))) u32x4 s_w[HAS_NETS ? NBUF * Stream::BUF_SLOTS : 1];
  __shared__ __attribute__((aligned(16))) float s_b3[2][32];

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);  // uniform: lives in a scalar register
  const int n = lane & 31, h = lane >> 5;
  const int layers = DEEP ? a.layers : 2;
  const NetLayout ly = net_layout(D, H, false, layers);
  Stream ws;
  ws.lds = s_w;
  ws.packed = a.packed;
  ws.net_bytes = ly.bytes;
  ws.chunks_off = ly.chunks;
  ws.chunk_bytes = ly.chunk_bytes;
  ws.wave = wave;
  ws.lane = lane;
  if constexpr (DEEP) ws.stages_per_net = (layers - 1) * Stream::STAGES_PER_NET;
  if constexpr (HAS_NETS) {
#pragma unroll
    for (int s = 0; s < Stream::AHEAD; ++s) ws.issue(s, s);
    load_resident(&s_l1[0][0], &s_b3[0][0], a.packed, ly, Net::L1_TILES);
  }
  __syncthreads();

  const int64_t blk0 = (int64_t)blockIdx.x * a.envs_per_block;
  const int64_t blk_end = min(blk0 + (int64_t)a.envs_per_block, (int64_t)a.E);
  const int64_t env0 = blk0 + (int64_t)wave * 32;
  const bool valid = env0 + n < blk_end;
  const uint32_t env = (uint32_t)(valid ? env0 + n : blk0);
  // the dynamics tiles are read once per step by every wave: they stay in registers
  u32x4 dynA[KT1], dynB;
#pragma unroll
  for (int kt = 0; kt < KT1; ++kt) dynA[kt] = ((const u32x4*)a.dyn)[kt * 64 + lane];
  dynB = ((const u32x4*)a.dyn)[KT1 * 64 + lane];
  int gs = 0;

  float s[1][NR];
#pragma unroll
  for (int r = 0; r < NR; ++r) {
    const int u = 8 * (r >> 2) + 4 * h + (r & 3);
    const float* src = ACT ? a.obs_in : a.env_state;  // PHASE_ACT works on the caller's rows
    s[0][r] = u < D ? src[(size_t)env * D + u] : 0.0f;
  }
  const int64_t g64 = a.g[env];
  uint32_t g32 = (uint32_t)g64;
  int tau = (int)(g64 % a.ep);
  uint32_t episode = (uint32_t)(g64 / a.ep);

  for (int t = 0; t <= a.T; ++t) {
    const size_t o = (size_t)t * a.M + env;
    // PHASE_STEP writes one observation, that of the last state, to row block 0
    if (valid && !ACT && (PHASE != PHASE_STEP || t == a.T)) {
      const size_t oo = PHASE == PHASE_STEP ? (size_t)env : o;
#pragma unroll
      for (int r = 0; r < NR; ++r) {
        const int u = 8 * (r >> 2) + 4 * h + (r & 3);
        if (u < D) a.obs[oo * D + u] = s[0][r];
      }
    }
    f32x16 out_p[1], out_v[1];
    if constexpr (!HAS_NETS) {
      out_p[0] = out_v[0] = zero16();
    } else {
      float h1[1][Net::KT2 * Net::PT];
      float x[1][NR];  // the state with the constant 1 at input D
#pragma unroll
      for (int r = 0; r < NR; ++r) {
        const int u = 8 * (r >> 2) + 4 * h + (r & 3);
        x[0][r] = u == D ? 1.0f : s[0][r];
      }
#pragma unroll
      for (int net = 0; net < 2; ++net) {
        f32x16(&out)[1] = net == 0 ? out_p : out_v;
        Net::layer1(&s_l1[net][0] + lane, x, h1);
        f32x16 acc[1];
        const int spn = ws.stages_per_net;
        int sn = 0;  // stage within the network
        if constexpr (DEEP) {
          // hidden layers 2 .. layers-1 (see the particle kernel): h1 <- tanh(W h1 + b)
#pragma unroll 1
          for (int layer = 2; layer < layers; ++layer) {
            float hb[1][Net::KT2 * Net::PT];
#pragma unroll 1
            for (int sc = 0; sc < Stream::STAGES_PER_NET; ++sc) {
              ws.wait_oldest();
              int next = net * spn + sn + Stream::AHEAD;
              if (next >= 2 * spn) next -= 2 * spn;
              const int nbuf = (gs + Stream::AHEAD) % NBUF;
              float hn[1][Net::PC];
              const u32x4* tiles = ws.tiles(gs % NBUF, 0);
              auto tick = [&](int kt) {
#pragma unroll
                for (int i = 0; i < Stream::PER_WAVE; ++i)
                  if (i * Net::KT2 / Stream::PER_WAVE == kt) ws.issue_part(next, nbuf, i);
              };
              if (sc == 0)
                Net::template hidden_chunk<false>(tiles, h1, acc, hn, h, tick);
              else
                Net::template hidden_chunk<true>(tiles, h1, acc, hn, h, tick);
#pragma unroll
              for (int k = 1; k < Stream::STAGES_PER_NET; ++k)
                if (sc == k) {
#pragma unroll
                  for (int j = 0; j < Net::PC; ++j) hb[0][(k - 1) * Net::PC + j] = hn[0][j];
                }
              ++gs;
              ++sn;
            }
            {
              float hl[1][Net::PC];
              Net::hidden_drain(acc, hl);
#pragma unroll
              for (int j = 0; j < Net::PC; ++j) hb[0][(Net::NUC - 1) * Net::PC + j] = hl[0][j];
            }
#pragma unroll
            for (int j = 0; j < Net::KT2 * Net::PT; ++j) h1[0][j] = hb[0][j];
          }
        }
        // Output layer: the policy's 2 K outputs on the MFMA (all 16 bits), the one value on the VALU (`net` is a
        // constant once the loop over the networks is unrolled).  Measured at the benchmark's shape: both on the
        // MFMA 21.64 ms, the value on the VALU 21.27, both on the VALU 21.62 (12 sums per activation are too many).
        constexpr uint32_t OUTS_P = 0xFFFFu, OUTS_V = 0x1u;
        out[0] = net == 0 ? Net::template out_init<OUTS_P>(s_b3[net], h) : Net::template out_init<OUTS_V>(s_b3[net], h);
#pragma unroll 1
        for (int sc = 0; sc < Stream::STAGES_PER_NET; ++sc) {
          ws.wait_oldest();
          int next = net * spn + sn + Stream::AHEAD;  // AHEAD stages ahead, cyclic over the step
          if (next >= 2 * spn) next -= 2 * spn;
          ++sn;
          const int nbuf = (gs + Stream::AHEAD) % NBUF;
#pragma unroll
          for (int c = 0; c < CPS; ++c) {
            const u32x4* tiles = ws.tiles(gs % NBUF, c);
            // the copies of the stage AHEAD stages later, spread over this stage's tile loops
            auto tick = [&](int kt) {
#pragma unroll
              for (int i = 0; i < Stream::PER_WAVE; ++i)
                if (i * (CPS * Net::KT2) / Stream::PER_WAVE == c * Net::KT2 + kt) ws.issue_part(next, nbuf, i);
            };
            const bool first = c == 0 && sc == 0, last = c == CPS - 1 && sc == Stream::STAGES_PER_NET - 1;
            if (net == 0) {
              if (first)
                Net::template layer2_chunk<false, OUTS_P>(tiles, h1, acc, out, h, 16, tick);
              else
                Net::template layer2_chunk<true, OUTS_P>(tiles, h1, acc, out, h, 16, tick);
              if (last) Net::template layer2_drain<OUTS_P>(tiles, acc, out, h, 16);
            } else {
              if (first)
                Net::template layer2_chunk<false, OUTS_V>(tiles, h1, acc, out, h, 16, tick);
              else
                Net::template layer2_chunk<true, OUTS_V>(tiles, h1, acc, out, h, 16, tick);
              if (last) Net::template layer2_drain<OUTS_V>(tiles, acc, out, h, 16);
            }
          }
          ++gs;
        }
        if (net == 0)
          Net::template out_finish<OUTS_P>(out, s_b3[net], h);
        else
          Net::template out_finish<OUTS_V>(out, s_b3[net], h);
      }
    }
    if (valid && h == 0 && PHASE != PHASE_STEP) a.values[o] = out_v[0][0];
    if (!ACT && t == a.T) break;

    // action dims 4h + c: mean in register c, log-std in register 4 + c
    float eps[4], act[4], lp = 0.0f, cost = 0.0f;
    normals4(a.seed_lo, a.seed_hi, env, 0, g32, 0, (uint32_t)h, eps);
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const int d = 4 * h + c;
      const float mean = out_p[0][c], logstd = out_p[0][4 + c];
      act[c] = 0.0f;
      if (d < K) {
        act[c] = mean + __expf(logstd) * eps[c];
        if constexpr (PHASE == PHASE_STEP) act[c] = valid ? ((const float*)a.actions_in)[(size_t)env * K + d] : 0.0f;
        lp += -0.5f * eps[c] * eps[c] - logstd - 0.9189385332046727f;
        cost += act[c] * act[c];
        if (valid && PHASE != PHASE_STEP) {
          ((float*)a.actions)[o * K + d] = act[c];
          if (a.logits) {
            a.logits[o * (2 * K) + d] = mean;
            a.logits[o * (2 * K) + K + d] = logstd;
          }
        }
      }
    }
    lp += __shfl_xor(lp, 32);
    float ss = 0.0f;
#pragma unroll
    for (int r = 0; r < NR; ++r) ss += s[0][r] * s[0][r];
    float rew = ss + a.act_cost * cost;
    rew += __shfl_xor(rew, 32);
    const bool done = tau + 1 == a.ep;
    if (valid && h == 0) {
      if (PHASE != PHASE_STEP) a.logp[o] = lp;
      if (!ACT) {
        a.rewards[o] = -rew;
        a.dones[o] = done ? 1 : 0;
      }
    }
    if constexpr (ACT) break;  // one evaluation, no move

    // s' = A s + B a + noise_std * eps
    f32x16 acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0.0f;
#pragma unroll
    for (int kt = 0; kt < KT1; ++kt) mma_tile<false>(dynA[kt], &s[0][4 * kt], acc);
    mma_tile<false>(dynB, act, acc);
#pragma unroll
    for (int b = 0; b < KT1; ++b) {
      float e[4];  // reset draw (stream 1, new episode) or step noise (stream 2, step counter)
      normals4(a.seed_lo, a.seed_hi, env, 0, done ? episode + 1 : g32, done ? 1u : 2u,
               (uint32_t)(2 * b + h), e);
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const int u = 8 * b + 4 * h + c;
        const float nv = done ? e[c] : acc[4 * b + c] + a.noise_std * e[c];
        s[0][4 * b + c] = u < D ? nv : 0.0f;
      }
    }
    g32 += 1;
    tau = done ? 0 : tau + 1;
    if (done) episode += 1;
  }

  if constexpr (HAS_NETS) ws.wait_all();  // copies issued ahead for stages that will not run
  if constexpr (ACT) return;  // the env state did not move

  if (valid) {
#pragma unroll
    for (int r = 0; r < NR; ++r) {
      const int u = 8 * (r >> 2) + 4 * h + (r & 3);
      if (u < D) a.env_state[(size_t)env * D + u] = s[0][r];
    }
    if (h == 0) a.g[env] = g64 + a.T;
  }
}

}  // namespace msrl
