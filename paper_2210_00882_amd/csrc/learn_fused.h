// Learner's gradient pass with the activations kept on chip (bf16 networks, categorical policy).
//
// ppo_rows_kernel runs forward pass, per-row loss and backward pass through the activations for a
// tile of 32 rows per wave, in the transposed "chained" form of the rollout kernels (mlp.h): a
// layer's accumulators (units x rows) are the next layer's B operand, so h1, h2, dL/dz2 and dL/dz1
// never leave the register file.  What the weight gradients need -- the layer inputs and the
// pre-activation gradients with the rows as contraction index -- is written once, as bf16, in a
// tiled unit-major layout:
//     tensor[tile][g][unit][8 rows],   tile = row / 32, g = (row % 32) / 8,
// i.e. the 16 KiB a wave produces per tensor and tile are contiguous, and a lane of the weight
// gradient kernel (wgrad_tiled_kernel) fetches the 8 rows of its MFMA fragment with one 16-byte
// load, the lanes of a wave reading consecutive pieces.  Weights reach the row kernel as MFMA A-operand tiles (packed.h) through the LDS window of
// WeightStream: per 32-row tile the forward chunk blocks (W2 by output chunk, W3), then the
// backward chunk blocks (W2 by input chunk); the layer-1 tiles and the tiles of W3 for the backward
// pass stay resident.
//
// Per-row loss (Listing 1 of the paper, mappo_net_train; the definition is that of the clipped
// surrogate objective stated with msrl_ppo_grad in the interface header).
#pragma once
#include "mlp.h"
#include "row_sel.h"

namespace msrl {

// ---------------------------------------------------------------- row kernel
struct RowsArgs {
  const uint8_t* packed;  // this network: forward image (NetLayout), then backward image of the same size:
                          // W3 tiles for dL/dz2 in the layer-1 area, W2 tiles by input chunk in the chunk blocks
  const float* b3;        // output bias [out_dim] (fp32 master)
  const float* obs;       // [R, D]
  const void* actions;    // int32 [R]
  const float* logp_old;
  const float* adv;
  const float* ret;
  int64_t R, n_tiles;     // n_tiles = ceil(R / 32)
  int D, out_dim;
  int obs_vec4;           // rows of obs may be read as 16-byte pieces (D % 4 == 0, base aligned)
  float clip, vf_coef, ent_coef, inv_R;
  // tiled unit-major outputs (bf16): xt has 16 KT1 units, h1t .. dz1t have H, dyt has 16
  __bf16 *xt, *h1t, *h2t, *dz2t, *dz1t, *dyt;
  float* stats;  // bins as in LossArgs
  RowSel sel;    // where row r of this call lies in obs, actions, logp_old, adv, ret
  // 64-unit networks: the weight gradients are formed inside the row kernel (no tiled tensors are written);
  // workgroup b stores its share as copy b (copies part_stride floats apart) of the gradient vector in `part`,
  // the six tensors of this network at the offsets o*
  float* part;
  int64_t part_stride;
  int32_t oW1, ob1, oW2, ob2, oW3, ob3;
};

__device__ __forceinline__ uint32_t quad_swap1(uint32_t x) {  // value of lane ^ 1
  return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0xB1, 0xF, 0xF, false);
}

// Tiled unit-major layout of the tensors the weight gradients read (bf16):
//     tensor[tile = row / 32][g = (row % 32) / 8][unit][row % 8]
// The 8 rows of one unit and group are the 16 bytes a lane of the weight-gradient kernel feeds to
// an MFMA, and the lanes of that kernel (one unit each) read consecutive 16-byte pieces.
//
// Results leave the wave through a staging area in LDS (one per wave), so that the global stores
// are runs of 16 bytes per lane (512 bytes per group for a chunk of 32 units): the memory pipeline
// takes about as long for a 64-lane store of 4 bytes per lane as for one of 16.  Values are held
// one row per lane and two consecutive units per 32-bit register; neighbouring lanes trade halves,
// so that a lane holds two consecutive rows of one unit, and write the staging area in the order
// [g][unit][4 row pairs] (32-bit LDS writes; the groups are 8 words apart modulo the banks).
struct Stager {
  static constexpr int GS = 136;  // words per group in the staging area (32 units x 4, + 8)
  static constexpr int WORDS = 4 * GS;
  uint32_t* stg;     // this wave's staging area
  uint32_t sel;      // byte selector of the exchange
  int w_chain;       // word offset of this lane for chunk values
  int w_lin;         // ... for observation values (linear input map)
  int lane;
  __device__ __forceinline__ Stager(uint32_t* s, int lane_, int n, int h)
      : stg(s), sel((n & 1) ? 0x03020706u : 0x05040100u),
        w_chain((n >> 3) * GS + (4 * h + (n & 1)) * 4 + ((n >> 1) & 3)),
        w_lin((n >> 3) * GS + (8 * h + (n & 1)) * 4 + ((n >> 1) & 3)), lane(lane_) {}
  __device__ __forceinline__ uint32_t trade(uint32_t x) const {
    return __builtin_amdgcn_perm(quad_swap1(x), x, sel);
  }
  // staged values of NU units (32: two pieces per lane, 16: one) -> units unit0 .. of a tile with U units
  template <int NU>
  __device__ __forceinline__ void flush(__bf16* tile, int U, int unit0) const {
    constexpr int K = NU / 16;
    wave_lds_sync();
    u32x4 v[K];
    int at[K];
#pragma unroll
    for (int k = 0; k < K; ++k) {
      const int idx = 64 * k + lane, g = idx / NU, u = idx % NU;
      v[k] = *(const u32x4*)(stg + g * GS + u * 4);
      at[k] = g * U + unit0 + u;
    }
#pragma unroll
    for (int k = 0; k < K; ++k) ((u32x4*)tile)[at[k]] = v[k];
    wave_lds_sync();
  }
  // one 32-unit chunk in operand form into the staging area (units 0 .. 31)
  __device__ __forceinline__ void stage_chunk(const bf16x8 (&op)[2]) const {
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const u32x4 w = __builtin_bit_cast(u32x4, op[j]);
#pragma unroll
      for (int d = 0; d < 4; ++d) {
        const int r = 8 * j + 2 * d;  // accumulator register of the low half
        stg[(8 * (r / 4) + r % 4) * 4 + w_chain] = trade(w[d]);
      }
    }
  }
  // the first 16 units of a chunk (operand 0) into the staging area (units 0 .. 15)
  __device__ __forceinline__ void stage_half(const bf16x8& op) const {
    const u32x4 w = __builtin_bit_cast(u32x4, op);
#pragma unroll
    for (int d = 0; d < 4; ++d) stg[(8 * (d / 2) + 2 * (d % 2)) * 4 + w_chain] = trade(w[d]);
  }
  // 16 observation inputs (one layer-1 operand) into the staging area, units slot0 .. slot0 + 15 (slot0 = 0 or 16)
  __device__ __forceinline__ void stage_inputs16(const bf16x8& op, int slot0) const {
    const u32x4 w = __builtin_bit_cast(u32x4, op);
#pragma unroll
    for (int d = 0; d < 4; ++d) stg[(2 * d + slot0) * 4 + w_lin] = trade(w[d]);
  }
  // one 32-unit chunk in operand form -> units unit0 .. unit0 + 31 of a tile
  __device__ __forceinline__ void chunk(__bf16* tile, int U, int unit0, const bf16x8 (&op)[2]) const {
    stage_chunk(op);
    flush<32>(tile, U, unit0);
  }
  // the first 16 units of a chunk (operand 0) -> units 0 .. 15 of a tile with 16 units
  __device__ __forceinline__ void half_chunk(__bf16* tile, const bf16x8& op) const {
    stage_half(op);
    flush<16>(tile, 16, 0);
  }
  // 16 observation inputs (one layer-1 operand) -> units unit0 .. unit0 + 15 of a tile
  __device__ __forceinline__ void inputs16(__bf16* tile, int U, int unit0, const bf16x8& op) const {
    stage_inputs16(op, 0);
    flush<16>(tile, U, unit0);
  }
  // The staged values as operands of a contraction over the rows (the weight gradients): for MFMA step k
  // (rows 16 k .. 16 k + 15 of the tile) lane (i, h) takes rows 8 (2 k + h) .. + 7 of unit i -- the same 16
  // bytes a lane of the weight-gradient kernels fetches from a tile in memory.
  __device__ __forceinline__ void frags32(bf16x8 (&f)[2]) const {
    wave_lds_sync();
#pragma unroll
    for (int k = 0; k < 2; ++k) f[k] = __builtin_bit_cast(bf16x8, *(const u32x4*)(stg + (2 * k + (lane >> 5)) * GS + (lane & 31) * 4));
    wave_lds_sync();
  }
  // ... when only units 0 .. 15 are staged: the lanes of units 16 .. 31 get zero
  __device__ __forceinline__ void frags16(bf16x8 (&f)[2]) const {
    wave_lds_sync();
#pragma unroll
    for (int k = 0; k < 2; ++k) {
      u32x4 v = {0, 0, 0, 0};
      if ((lane & 31) < 16) v = *(const u32x4*)(stg + (2 * k + (lane >> 5)) * GS + (lane & 31) * 4);
      f[k] = __builtin_bit_cast(bf16x8, v);
    }
    wave_lds_sync();
  }
  // The way back, for a chunk the wave wrote earlier: its 2 KiB into registers as they lie in
  // memory (fetch; issued early), then through the staging area into operand form (unstage).
  __device__ __forceinline__ void fetch(const __bf16* tile, int U, int unit0, u32x4 (&raw)[2]) const {
#pragma unroll
    for (int k = 0; k < 2; ++k) {
      const int idx = 64 * k + lane, g = idx / 32, u = idx % 32;
      raw[k] = ((const u32x4*)tile)[g * U + unit0 + u];
    }
  }
  __device__ __forceinline__ void unstage(const u32x4 (&raw)[2], bf16x8 (&op)[2]) const {
    wave_lds_sync();
#pragma unroll
    for (int k = 0; k < 2; ++k) {
      const int idx = 64 * k + lane, g = idx / 32, u = idx % 32;
      *(u32x4*)(stg + g * GS + u * 4) = raw[k];
    }
    wave_lds_sync();
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      u32x4 w;
#pragma unroll
      for (int d = 0; d < 4; ++d) {
        const int r = 8 * j + 2 * d;
        w[d] = trade(stg[(8 * (r / 4) + r % 4) * 4 + w_chain]);  // the 2 x 2 exchange is its own inverse
      }
      op[j] = __builtin_bit_cast(bf16x8, w);
    }
    wave_lds_sync();
  }
};

// acc * (1 - a^2) for accumulator registers [r0, r1), a = the stored (rounded) activation
__device__ __forceinline__ void dtanh_range(const f32x16& acc, const bf16x8 (&hp)[2], float (&t)[16], int r0,
                                            int r1, bool pinned) {
  float v[16];
#pragma unroll
  for (int r = 0; r < 16; ++r)
    if (r >= r0 && r < r1) {
      v[r] = acc[r];
      if (pinned) pin(v[r]);
    }
#pragma unroll
  for (int r = 0; r < 16; ++r)
    if (r >= r0 && r < r1) {
      const float a = (float)hp[r / 8][r % 8];
      t[r] = v[r] * (1.0f - a * a);
    }
#pragma unroll
  for (int r = 0; r < 16; ++r)
    if (r >= r0 && r < r1 && pinned) pin(t[r]);
}

// One chunk block of the forward pass: acc <- layer-2 pre-activations of the block's 32 units (bias
// included); if PIPE, `acc` holds those of the chunk before on entry: they get tanh, feed layer 3
// (out) and are returned as operands in hprev.  tick(kt) runs once per layer-2 tile.
template <class Net, bool PIPE, class Tick>
__device__ __forceinline__ void fwd_chunk(const u32x4* tiles, const bf16x8 (&h1)[1][Net::KT2], f32x16& acc,
                                          f32x16& out, int h, bf16x8 (&hprev)[2], Tick&& tick) {
  constexpr int KT2 = Net::KT2, TPC = Net::TPC, G = Net::G, LAST = Net::L3_PREV + TPC;
  u32x4 ring[G];
#pragma unroll
  for (int i = 0; i < G; ++i) ring[i] = tiles[i * 64];
  const f32x16 prev = acc;
  float t[16];
  acc = zero16();
  if constexpr (PIPE && KT2 % 2 == 0) {
    // two tiles per round, the tanh chains of both side by side in three pinned groups (as in Mlp::layer2_chunk)
    float w[16];
#pragma unroll
    for (int kt = 0; kt < KT2; kt += 2) {
      const int r0 = kt * 16 / KT2, r1 = (kt + 2) * 16 / KT2;
      u32x4 raw = ring[kt % G];
      if (kt + G < LAST) ring[kt % G] = tiles[(kt + G) * 64];
      pin(raw);
      acc = mma(__builtin_bit_cast(bf16x8, raw), h1[0][kt], acc);
      tanh_stage1(prev, w, r0, r1);
      u32x4 raw2 = ring[(kt + 1) % G];
      if (kt + 1 + G < LAST) ring[(kt + 1) % G] = tiles[(kt + 1 + G) * 64];
      pin(raw2);
      acc = mma(__builtin_bit_cast(bf16x8, raw2), h1[0][kt + 1], acc);
      tanh_stage2(w, r0, r1);
      tanh_stage3(w, t, r0, r1);
      tick(kt);
      tick(kt + 1);
    }
  } else {
#pragma unroll
    for (int kt = 0; kt < KT2; ++kt) {
      u32x4 raw = ring[kt % G];
      if (kt + G < LAST) ring[kt % G] = tiles[(kt + G) * 64];
      if (PIPE) pin(raw);
      acc = mma(__builtin_bit_cast(bf16x8, raw), h1[0][kt], acc);
      if (PIPE) tanh_range(prev, t, kt * 16 / KT2, (kt + 1) * 16 / KT2, true);
      tick(kt);
    }
  }
  {
    bf16x8 one = {0, 0, 0, 0, 0, 0, 0, 0};  // the two parts of the bias sit at k slots 0 and 1 of h = 0
    one[0] = (__bf16)(h == 0 ? 1.0f : 0.0f);
    one[1] = one[0];
    const u32x4 raw = ring[KT2 % G];
    if (KT2 + G < LAST) ring[KT2 % G] = tiles[(KT2 + G) * 64];
    acc = mma(__builtin_bit_cast(bf16x8, raw), one, acc);
  }
  if (PIPE) {
    to_operands<true>(t, hprev);
#pragma unroll
    for (int i = 0; i < TPC; ++i)
      out = mma(__builtin_bit_cast(bf16x8, ring[(Net::L3_PREV + i) % G]), hprev[i], out);
  }
}

// One chunk block of the backward pass: acc <- W2 dz2 for the block's 32 layer-1 units; if PIPE, the
// result of the chunk before (in `acc` on entry) is multiplied by 1 - h1^2 (hp: that chunk's
// activations) and returned as operands in dprev.
template <class Net, bool PIPE, class Tick>
__device__ __forceinline__ void bwd_chunk(const u32x4* tiles, const bf16x8 (&dz2)[Net::KT2], f32x16& acc,
                                          const bf16x8 (&hp)[2], bf16x8 (&dprev)[2], Tick&& tick) {
  constexpr int KT2 = Net::KT2, G = Net::G;
  u32x4 ring[G];
#pragma unroll
  for (int i = 0; i < G; ++i) ring[i] = tiles[i * 64];
  const f32x16 prev = acc;
  float t[16];
  acc = zero16();
#pragma unroll
  for (int kt = 0; kt < KT2; ++kt) {
    u32x4 raw = ring[kt % G];
    if (kt + G < KT2) ring[kt % G] = tiles[(kt + G) * 64];
    if (PIPE) pin(raw);
    acc = mma(__builtin_bit_cast(bf16x8, raw), dz2[kt], acc);
    if (PIPE) dtanh_range(prev, hp, t, kt * 16 / KT2, (kt + 1) * 16 / KT2, true);
    tick(kt);
  }
  if (PIPE) to_operands<true>(t, dprev);
}

// waves per workgroup of the row kernel = row tiles per group: eight, two per SIMD; four (one per SIMD, with
// the whole register file) for 64-unit networks, which keep their weight-gradient tiles in registers
constexpr int rows_waves(int H) { return H <= 64 ? 4 : 8; }
constexpr int ROWS_STAT_BINS = 64;  // bins per statistic in RowsArgs::stats (after 8 result slots)

// workgroups of the row kernel that share a compute unit: two for 64-unit networks (their registers are
// held to 128 per lane for that, and 60 KiB of LDS each leave the room), one above
constexpr int rows_workgroups_per_cu(int H) { return 1; }

template <int H, int KT1, int NET, int WAVES>
__global__ __launch_bounds__(64 * WAVES) __attribute__((amdgpu_waves_per_eu(WAVES / 4 * rows_workgroups_per_cu(H))))
void ppo_rows_kernel(RowsArgs a) {
  constexpr int NBUF = 2;
  typedef Mlp<H, true, 1, KT1> Net;
  constexpr int NUC = Net::NUC, KT2 = Net::KT2, TPC = Net::TPC, G = Net::G;
  constexpr int CPS = NUC % 2 == 0 ? 2 : 1;
  typedef WeightStream<Net, WAVES, NBUF, CPS> Stream;
  constexpr int SPN = Stream::STAGES_PER_NET;
  typedef bf16x8 Op;
  static_assert(KT2 >= G && TPC <= 2, "ring prefetch depth; layer-3 tiles per chunk");
  // Up to 128 units all 2 SPN stages of a tile (forward, then backward chunk blocks) fit the LDS at once:
  // they are copied there once, and the tile loop has no waits for copies and no barriers, so the waves of
  // a workgroup drift apart and cover each other's memory latencies.  (The wait for a streamed stage,
  // s_waitcnt vmcnt, also waits for every store the wave has in flight - two KiB per row here.)
  constexpr bool RESIDENT = H <= 128;
  constexpr int WBUFS = RESIDENT ? 2 * SPN : NBUF;
  // 64-unit networks: the weight gradients are formed here too.  What the other widths write as tiles is, on
  // its way through the staging area, already in the operand form of a contraction over the tile's 32 rows; a
  // wave keeps those operands (x, h1, h2; then dy, dz2, dz1 as they appear) and adds the products to gradient
  // tiles it holds for the whole launch: XT x 2 (W1; its rows in_dim, in_dim + 1 meet the constant-1 inputs
  // and so are the bias gradient), 2 x 2 (W2), 2 (W3), and a ones-row product each for the biases of layers
  // 2 and 3 -- 11 or 13 tiles of 16 registers, which is why these kernels run one wave per SIMD.  At the end
  // the waves of a workgroup add their tiles up in wave order and store one copy per workgroup.
  constexpr bool ONCHIP = H <= 64;
  constexpr int XT = ONCHIP ? KT1 / 2 : 1;  // 32-unit tiles of the observation operand
  static_assert(!ONCHIP || (KT1 % 2 == 0 && NUC == 2 && WAVES >= 2), "two layer-1 operands per 32-unit tile; 64 hidden units");

  __shared__ __attribute__((aligned(16))) u32x4 s_l1[Net::L1_TILES * 64];
  __shared__ __attribute__((aligned(16))) u32x4 s_w3t[NUC * 64];
  __shared__ __attribute__((aligned(16))) u32x4 s_w[WBUFS * Stream::BUF_SLOTS];
  __shared__ __attribute__((aligned(16))) float s_b3[32];
  __shared__ __attribute__((aligned(16))) uint32_t s_stg[WAVES][Stager::WORDS];
  __shared__ float s_red[ONCHIP ? (WAVES - 1) * 16 * 64 : 1];  // the other waves' copy of one gradient tile

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int n = lane & 31, h = lane >> 5;
  const Stager sg(s_stg[wave], lane, n, h);
  const int O = NET == 0 ? a.out_dim : 1;
  const NetLayout ly = net_layout(16 * KT1 - 1, H, true);
  Stream ws;
  ws.lds = s_w;
  ws.packed = a.packed;
  ws.net_bytes = ly.bytes;  // "network 1" of the stream = the backward image
  ws.chunks_off = ly.chunks;
  ws.chunk_bytes = ly.chunk_bytes;
  ws.wave = wave;
  ws.lane = lane;
  if constexpr (RESIDENT) {
#pragma unroll
    for (int sgi = 0; sgi < 2 * SPN; ++sgi) ws.issue(sgi, sgi);
  } else {
    ws.issue(0, 0);
  }
  {
    const u32x4* src = (const u32x4*)(a.packed + ly.w1);
    for (int i = threadIdx.x; i < Net::L1_TILES * 64; i += blockDim.x) s_l1[i] = src[i];
    const u32x4* src3 = (const u32x4*)(a.packed + ly.bytes + ly.w1);
    for (int i = threadIdx.x; i < NUC * 64; i += blockDim.x) s_w3t[i] = src3[i];
    if (threadIdx.x < 32) s_b3[threadIdx.x] = (int)threadIdx.x < O ? a.b3[threadIdx.x] : 0.0f;
  }
  if constexpr (RESIDENT) ws.wait_all(); else __syncthreads();

  float st[5] = {0.0f, 0.0f, 0.0f, 0.0f, 0.0f};  // per-lane sums: policy term, value term, entropy, clipped, kl
  // ONCHIP: gradient tiles (C[m][n]: register r of lane (i, h) <-> m = 8 (r / 4) + 4 h + r % 4, n = i) ...
  f32x16 gW1[XT][2], gW2[2][2], gW3[2], gB2[2], gB3;
  // ... and the operands kept from the forward pass
  bf16x8 fx[XT][2], fh1[2][2], fh2[2][2];
  Op h2keep[ONCHIP ? KT2 : 1];  // layer-2 activations in chained operand form (the other widths read them back)
  bf16x8 ones;
#pragma unroll
  for (int e = 0; e < 8; ++e) ones[e] = (__bf16)1.0f;
  if constexpr (ONCHIP) {
    gB3 = zero16();
#pragma unroll
    for (int c = 0; c < 2; ++c) {
      gW3[c] = gB2[c] = zero16();
#pragma unroll
      for (int m = 0; m < 2; ++m) gW2[m][c] = zero16();
#pragma unroll
      for (int m = 0; m < XT; ++m) gW1[m][c] = zero16();
    }
  }
  int gs = 0;  // stages consumed so far: stage gs sits in buffer gs % WBUFS
  const int64_t groups = (a.n_tiles + WAVES - 1) / WAVES;
  // copies of stage `next` into buffer `nbuf`, spread over the tile loops of the current stage
  auto spread = [&](int next, int nbuf, int c, int kt) {
    if constexpr (RESIDENT) return;
#pragma unroll
    for (int i = 0; i < Stream::PER_WAVE; ++i)
      if (i * (CPS * KT2) / Stream::PER_WAVE == c * KT2 + kt) ws.issue_part(next, nbuf, i);
  };
  // ONCHIP: chunk c of dL/dz1 (operand form) times the observation operands -> W1's gradient tiles
  auto dz1_product = [&](int c, const Op (&dz)[2]) {
    bf16x8 fdz[2];
    sg.stage_chunk(dz);
    sg.frags32(fdz);
#pragma unroll
    for (int k = 0; k < 2; ++k)
#pragma unroll
      for (int m = 0; m < XT; ++m) {
        if (c == 0) gW1[m][0] = mma(fx[m][k], fdz[k], gW1[m][0]);
        else gW1[m][1] = mma(fx[m][k], fdz[k], gW1[m][1]);
      }
  };
  // What a tile reads per row: this lane's 8 observation inputs of every layer-1 operand and the inputs of
  // the loss; zeros for rows beyond the end.  ONCHIP kernels (one wave per SIMD, nothing to cover a load's
  // latency with) fetch them one tile ahead where the registers allow (two layer-1 operands).
  constexpr bool AHEAD = ONCHIP && KT1 <= 2;
  struct RowInputs {
    f32x8 f[KT1];
    int act;
    float lpo, adv, ret;
  };
  auto load_rows = [&](int64_t grp) -> RowInputs {
    RowInputs in;
    const int64_t row = (grp * WAVES + wave) * 32 + n;
    const bool valid = grp < groups && row < a.R;
    const int64_t prow = valid ? a.sel.at(row) : 0;  // the row inside the caller's arrays
    in.act = 0;
    in.lpo = in.adv = in.ret = 0.0f;
    if (valid) {
      if constexpr (NET == 0) {
        in.act = ((const int32_t*)a.actions)[prow];
        in.lpo = a.logp_old[prow];
        in.adv = a.adv[prow];
      } else {
        in.ret = a.ret[prow];
      }
    }
#pragma unroll
    for (int kt = 0; kt < KT1; ++kt) {
      const int i0 = 16 * kt + 8 * h;
      if (valid && a.obs_vec4 && i0 + 8 <= a.D) {
        const f32x4 u = *(const f32x4*)(a.obs + prow * a.D + i0), w = *(const f32x4*)(a.obs + prow * a.D + i0 + 4);
        in.f[kt] = f32x8{u[0], u[1], u[2], u[3], w[0], w[1], w[2], w[3]};
      } else {
#pragma unroll
        for (int s = 0; s < 8; ++s) in.f[kt][s] = (valid && i0 + s < a.D) ? a.obs[prow * a.D + i0 + s] : 0.0f;
      }
    }
    return in;
  };
  RowInputs ahead;
  if constexpr (AHEAD) ahead = load_rows(blockIdx.x);
#pragma unroll 1
  for (int64_t grp = blockIdx.x; grp < groups; grp += gridDim.x) {
    const int64_t tile = grp * WAVES + wave;
    const bool live = tile < a.n_tiles;  // uniform over the wave
    const int64_t row = tile * 32 + n;
    const bool valid = live && row < a.R;
    if constexpr (!RESIDENT) ws.wait_oldest();  // forward stage 0 is in; every wave has left the previous tile
    RowInputs in;
    if constexpr (AHEAD) {
      in = ahead;
      ahead = load_rows(grp + gridDim.x);
    } else {
      in = load_rows(grp);
    }
    const int act = in.act;
    const float lpo = in.lpo, adv = in.adv, ret = in.ret;

    // ---------------- observation row -> layer-1 operands (inputs D and D + 1 carry the two bias parts)
    Op x[1][KT1];
#pragma unroll
    for (int kt = 0; kt < KT1; ++kt) {
      f32x8 f = in.f[kt];
      const int i0 = 16 * kt + 8 * h;
#pragma unroll
      for (int s = 0; s < 8; ++s)
        if (i0 + s == a.D || i0 + s == a.D + 1) f[s] = 1.0f;
      x[0][kt] = __builtin_convertvector(f, bf16x8);
    }
    if constexpr (ONCHIP) {
      if (live) {
#pragma unroll
        for (int m = 0; m < XT; ++m) {
          sg.stage_inputs16(x[0][2 * m], 0);
          sg.stage_inputs16(x[0][2 * m + 1], 16);
          sg.frags32(fx[m]);
        }
      }
    } else if (NET == 0 && live) {
      __bf16* xt = a.xt + (size_t)tile * (16 * KT1) * 32;
#pragma unroll
      for (int kt = 0; kt < KT1; ++kt) sg.inputs16(xt, 16 * KT1, 16 * kt, x[0][kt]);
    }

    // ---------------- forward.  The activations go to their tiles as they are produced.  Layer 1's
    // stay in registers for the backward pass; layer 2's are read back from their tile (by the wave
    // that wrote them) where dL/dz2 needs them: holding both layers to the end of the tile would
    // leave room for one wave per SIMD only.
    __bf16* t1 = a.h1t + (size_t)tile * H * 32;
    __bf16* t2 = a.h2t + (size_t)tile * H * 32;
    f32x16 out = bias_init(s_b3, h);
    Op h1[1][KT2];  // layer-1 activations: kept for the backward pass
    {
      Net::layer1(s_l1 + lane, x, h1);
      if (live) {
#pragma unroll
        for (int c = 0; c < NUC; ++c) {
          const Op pr[2] = {h1[0][2 * c], h1[0][2 * c + 1]};
          if constexpr (ONCHIP) {
            sg.stage_chunk(pr);
            sg.frags32(fh1[c]);
          } else {
            sg.chunk(t1, H, 32 * c, pr);
          }
        }
      }
      f32x16 acc = zero16();
#pragma unroll 1
      for (int sc = 0; sc < SPN; ++sc) {
        if constexpr (!RESIDENT) {
          if (sc != 0) ws.wait_oldest();
        }
        const int next = sc + 1;  // the first backward stage follows the last forward stage
        const int nbuf = (gs + 1) % NBUF;
#pragma unroll
        for (int c = 0; c < CPS; ++c) {
          const u32x4* tiles = ws.tiles(gs % WBUFS, c);
          auto tick = [&](int kt) { spread(next, nbuf, c, kt); };
          Op hn[2];
          if (c == 0 && sc == 0) {  // the first chunk of a tile has no chunk before it
            fwd_chunk<Net, false>(tiles, h1, acc, out, h, hn, tick);
          } else {
            fwd_chunk<Net, true>(tiles, h1, acc, out, h, hn, tick);
            if constexpr (ONCHIP) {
              // (64 units: one stage of two chunks, so this is chunk 0, finished while chunk 1 was summed)
              h2keep[0] = hn[0];
              h2keep[1] = hn[1];
              if (live) {
                sg.stage_chunk(hn);
                sg.frags32(fh2[0]);
              }
            } else {
              if (live) sg.chunk(t2, H, 32 * (sc * CPS + c - 1), hn);
            }
          }
        }
        ++gs;
      }
      // last chunk: its tanh and layer-3 contribution (tiles of the last stage, still resident)
      {
        const u32x4* tiles = ws.tiles((gs - 1) % WBUFS, CPS - 1);
        float t[16];
        Op hl[2];
        tanh_range(acc, t, 0, 16, false);
        to_operands<true>(t, hl);
#pragma unroll
        for (int i = 0; i < TPC; ++i)
          out = mma(__builtin_bit_cast(bf16x8, tiles[(Net::L3_OWN + i) * 64]), hl[i], out);
        if constexpr (ONCHIP) {
          h2keep[2] = hl[0];
          h2keep[3] = hl[1];
          if (live) {
            sg.stage_chunk(hl);
            sg.frags32(fh2[1]);
          }
        } else {
          if (live) sg.chunk(t2, H, 32 * (NUC - 1), hl);
        }
      }
    }

    // ---------------- per-row loss and dL/dy in accumulator layout (register r <-> output 8 (r/4) + 4 h + r % 4)
    float dyr[16];
#pragma unroll
    for (int r = 0; r < 16; ++r) dyr[r] = 0.0f;
    if constexpr (NET == 0) {
      float l[16];
#pragma unroll
      for (int k = 0; k < 16; ++k) {
        const int r = 4 * (k >> 3) + (k & 3);
        const float own = out[r], oth = __shfl_xor(own, 32);
        l[k] = (((k >> 2) & 1) == h) ? own : oth;
      }
      float mx = l[0];
#pragma unroll
      for (int k = 1; k < 16; ++k) mx = k < O ? fmaxf(mx, l[k]) : mx;
      float z = 0.0f;
#pragma unroll
      for (int k = 0; k < 16; ++k) z += k < O ? __expf(l[k] - mx) : 0.0f;
      const float lse = mx + __logf(z);
      float ent = 0.0f, logp = 0.0f;
#pragma unroll
      for (int k = 0; k < 16; ++k) {
        const float lp = l[k] - lse;
        ent -= k < O ? __expf(lp) * lp : 0.0f;
        if (k == act) logp = lp;
      }
      const float rho = __expf(logp - lpo);
      const float rc = fminf(fmaxf(rho, 1.0f - a.clip), 1.0f + a.clip);
      const float un = rho * adv, cl = rc * adv;
      const bool clipped = cl < un;
      const float gl = clipped ? 0.0f : -adv * rho;
      // each lane differentiates with respect to its own eight outputs
#pragma unroll
      for (int r = 0; r < 8; ++r) {
        const int k = 8 * (r / 4) + 4 * h + r % 4;
        const float lp = out[r] - lse, pk = __expf(lp);
        const float dlp = (k == act ? 1.0f : 0.0f) - pk, dH = -pk * (lp + ent);
        dyr[r] = (valid && k < O) ? (gl * dlp - a.ent_coef * dH) * a.inv_R : 0.0f;
      }
      if (valid && h == 0) {
        st[0] += -(clipped ? cl : un);
        st[2] += ent;
        st[3] += clipped ? 1.0f : 0.0f;
        st[4] += lpo - logp;
      }
    } else {
      const float v = __shfl(out[0], n);  // output 0 sits in register 0 of the h = 0 lane
      const float err = v - ret;
      if (valid && h == 0) {
        dyr[0] = a.vf_coef * 2.0f * err * a.inv_R;
        st[1] += err * err;
      }
    }
    Op dyo[2];
    to_operands<true>(dyr, dyo);
    if constexpr (ONCHIP) {
      if (live) {
        bf16x8 fdy[2];
        sg.stage_half(dyo[0]);
        sg.frags16(fdy);
#pragma unroll
        for (int k = 0; k < 2; ++k) {
#pragma unroll
          for (int m = 0; m < 2; ++m) gW3[m] = mma(fh2[m][k], fdy[k], gW3[m]);
          gB3 = mma(ones, fdy[k], gB3);
        }
      }
    } else {
      if (live) sg.half_chunk(a.dyt + (size_t)tile * 16 * 32, dyo[0]);
    }

    // ---------------- dL/dz2 = (W3 dy) * (1 - h2^2), chunk by chunk
    Op dz2[KT2];
    {
      __bf16* tz2 = a.dz2t + (size_t)tile * H * 32;
      u32x4 raw[2] = {u32x4{0, 0, 0, 0}, u32x4{0, 0, 0, 0}};
      if constexpr (!ONCHIP) {
        if (live) sg.fetch(t2, H, 0, raw);
      }
#pragma unroll
      for (int c = 0; c < NUC; ++c) {
        Op hp[2];
        if constexpr (ONCHIP) {
          hp[0] = h2keep[2 * c];
          hp[1] = h2keep[2 * c + 1];
        } else {
          sg.unstage(raw, hp);
          if (live && c + 1 < NUC) sg.fetch(t2, H, 32 * (c + 1), raw);
        }
        const f32x16 g = mma(__builtin_bit_cast(bf16x8, s_w3t[c * 64 + lane]), dyo[0], zero16());
        float t[16];
        dtanh_range(g, hp, t, 0, 16, false);
        Op dz[2];
        to_operands<true>(t, dz);
        dz2[2 * c] = dz[0];
        dz2[2 * c + 1] = dz[1];
        if constexpr (ONCHIP) {
          if (live) {
            bf16x8 fdz[2];
            sg.stage_chunk(dz);
            sg.frags32(fdz);
#pragma unroll
            for (int k = 0; k < 2; ++k) {
#pragma unroll
              for (int m = 0; m < 2; ++m) gW2[m][c] = mma(fh1[m][k], fdz[k], gW2[m][c]);
              gB2[c] = mma(ones, fdz[k], gB2[c]);
            }
          }
        } else {
          if (live) sg.chunk(tz2, H, 32 * c, dz);
        }
      }
    }

    // ---------------- dL/dz1 = (W2 dz2) * (1 - h1^2): chunk blocks of the backward image
    {
      __bf16* tz1 = a.dz1t + (size_t)tile * H * 32;
      f32x16 acc = zero16();
      Op hp[2] = {Op{0, 0, 0, 0, 0, 0, 0, 0}, Op{0, 0, 0, 0, 0, 0, 0, 0}};  // layer-1 activations of the chunk before
#pragma unroll 1
      for (int sc = 0; sc < SPN; ++sc) {
        if constexpr (!RESIDENT) ws.wait_oldest();
        int next = SPN + sc + 1;  // the next tile's first forward stage follows the last backward stage
        if (next >= 2 * SPN) next -= 2 * SPN;
        const int nbuf = (gs + 1) % NBUF;
#pragma unroll
        for (int c = 0; c < CPS; ++c) {
          const u32x4* tiles = ws.tiles(gs % WBUFS, c);
          auto tick = [&](int kt) { spread(next, nbuf, c, kt); };
          const int chunk = sc * CPS + c;
          Op dz[2];
          if (c == 0 && sc == 0) {
            bwd_chunk<Net, false>(tiles, dz2, acc, hp, dz, tick);
          } else {
            bwd_chunk<Net, true>(tiles, dz2, acc, hp, dz, tick);
            if constexpr (ONCHIP) {
              if (live) dz1_product(0, dz);  // (one stage of two chunks: this is chunk 0)
            } else {
              if (live) sg.chunk(tz1, H, 32 * (chunk - 1), dz);
            }
          }
          // activations of this chunk, for the epilogue that runs during the next one (register indices
          // are compile-time constants inside each branch)
#pragma unroll
          for (int k = 0; k < SPN; ++k)
            if (sc == k) {
              hp[0] = h1[0][2 * (k * CPS + c)];
              hp[1] = h1[0][2 * (k * CPS + c) + 1];
            }
        }
        ++gs;
      }
      {
        float t[16];
        dtanh_range(acc, hp, t, 0, 16, false);
        Op dz[2];
        to_operands<true>(t, dz);
        if constexpr (ONCHIP) {
          if (live) dz1_product(NUC - 1, dz);
        } else {
          if (live) sg.chunk(tz1, H, 32 * (NUC - 1), dz);
        }
      }
    }
  }
  if constexpr (ONCHIP) {
    // The waves' tiles are added in wave order (through LDS, a tile at a time) and wave 0 stores the sum as
    // this workgroup's copy: tile (mt, nt) of a tensor holds C[32 mt + m][32 nt + i], m as above.
    const int64_t copy = (int64_t)blockIdx.x * a.part_stride;
    auto reduce_tile = [&](f32x16& g) {
      __syncthreads();  // the tile before has been read
      if (wave > 0) {
#pragma unroll
        for (int r = 0; r < 16; ++r) s_red[((wave - 1) * 16 + r) * 64 + lane] = g[r];
      }
      __syncthreads();
      if (wave == 0) {
#pragma unroll
        for (int w = 0; w < WAVES - 1; ++w)
#pragma unroll
          for (int r = 0; r < 16; ++r) g[r] += s_red[(w * 16 + r) * 64 + lane];
      }
    };
    // rows m < M of C into a row-major tensor at offset oC with `ldc` columns, of which N are in use
    auto store_tile = [&](const f32x16& g, int mt, int nt, int M, int N, int32_t oC, int ldc) {
      const int nn = 32 * nt + n;
      if (wave != 0 || nn >= N) return;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int m = 32 * mt + 8 * (r / 4) + 4 * h + r % 4;
        if (m < M) a.part[copy + oC + (int64_t)m * ldc + nn] = g[r];
      }
    };
    // row `row` of C (a bias gradient) into a vector at offset ob
    auto store_row = [&](const f32x16& g, int mt, int nt, int row, int N, int32_t ob) {
      const int nn = 32 * nt + n;
      if (wave != 0 || nn >= N) return;
#pragma unroll
      for (int r = 0; r < 16; ++r)
        if (32 * mt + 8 * (r / 4) + 4 * h + r % 4 == row) a.part[copy + ob + nn] = g[r];
    };
#pragma unroll
    for (int c = 0; c < 2; ++c) {
#pragma unroll
      for (int m = 0; m < XT; ++m) {
        reduce_tile(gW1[m][c]);
        store_tile(gW1[m][c], m, c, a.D, H, a.oW1, H);
        store_row(gW1[m][c], m, c, a.D, H, a.ob1);  // the constant-1 input at index D: the sum over the rows
      }
#pragma unroll
      for (int m = 0; m < 2; ++m) {
        reduce_tile(gW2[m][c]);
        store_tile(gW2[m][c], m, c, H, H, a.oW2, H);
      }
      reduce_tile(gB2[c]);
      store_row(gB2[c], 0, c, 0, H, a.ob2);  // every row of a ones-product is the sum over the rows
      reduce_tile(gW3[c]);
      store_tile(gW3[c], c, 0, H, O, a.oW3, O);
    }
    reduce_tile(gB3);
    store_row(gB3, 0, 0, 0, O, a.ob3);
  }
  if constexpr (!RESIDENT) ws.wait_all();  // the copy issued ahead for a tile that does not exist

  // sums of the wave -> one atomic per statistic and wave, spread over the bins
#pragma unroll
  for (int q = 0; q < 5; ++q) {
    if ((NET == 0) == (q == 1)) continue;  // the value term belongs to the value network's launch
    float s = st[q];
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o);
    if (lane == 0) atomicAdd(a.stats + 8 + q * ROWS_STAT_BINS + (blockIdx.x * WAVES + wave) % ROWS_STAT_BINS, s);
  }
}

// launchers of the instantiated row kernels (one translation unit per hidden size)
hipError_t launch_ppo_rows_h64(int kt1, int net, const RowsArgs& a, unsigned grid, hipStream_t s);
hipError_t launch_ppo_rows_h128(int kt1, int net, const RowsArgs& a, unsigned grid, hipStream_t s);
hipError_t launch_ppo_rows_h256(int kt1, int net, const RowsArgs& a, unsigned grid, hipStream_t s);

#define MSRL_ROWS_LAUNCHER(HID)                                                                             \
  hipError_t launch_ppo_rows_h##HID(int kt1, int net, const RowsArgs& a, unsigned grid, hipStream_t s) {    \
    if (kt1 == 2 && net == 0) hipLaunchKernelGGL((ppo_rows_kernel<HID, 2, 0, rows_waves(HID)>), dim3(grid), dim3(64 * rows_waves(HID)), 0, s, a);      \
    else if (kt1 == 2) hipLaunchKernelGGL((ppo_rows_kernel<HID, 2, 1, rows_waves(HID)>), dim3(grid), dim3(64 * rows_waves(HID)), 0, s, a);    \
    else if (kt1 == 4 && net == 0) hipLaunchKernelGGL((ppo_rows_kernel<HID, 4, 0, rows_waves(HID)>), dim3(grid), dim3(64 * rows_waves(HID)), 0, s, a); \
    else if (kt1 == 4) hipLaunchKernelGGL((ppo_rows_kernel<HID, 4, 1, rows_waves(HID)>), dim3(grid), dim3(64 * rows_waves(HID)), 0, s, a);    \
    else return hipErrorInvalidValue;                                                                       \
    return hipGetLastError();                                                                               \
  }

}  // namespace msrl
