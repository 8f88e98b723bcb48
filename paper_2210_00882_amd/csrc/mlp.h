// Policy / value network forward pass on MFMA, one wave per group of 32*NB rows.
//
// Every layer is computed transposed (units x rows), so a layer's accumulators
//   lane (n = lane % 32, h = lane / 32), register r  <->  row n, unit 32*uc + 8*(r/4) + 4*h + r%4
// are, after bias + tanh (+ rounding to bf16), exactly the B operand of the next
// layer's MFMAs: activations never leave the register file.  The weights are
// the A operand; the workgroup streams them through LDS in stages (the layer-1
// tiles, then one block per 32-unit chunk of layer 2 together with the layer-3
// tiles of that chunk and of the one before; see packed.h), and every wave of
// the workgroup reads the same stage.  Layer 3 is accumulated as the layer-2
// chunks complete, so h2 is consumed as soon as it is produced.
#pragma once
#include "dev_common.h"
#include "packed.h"

namespace msrl {

typedef float f32x8 __attribute__((ext_vector_type(8)));

__device__ __forceinline__ f32x16 mma(bf16x8 a, bf16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}
__device__ __forceinline__ f32x16 mma(float a, float b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c, 0, 0, 0);
}

template <bool BF16> struct Operand;
template <> struct Operand<true> {
  typedef bf16x8 T;                    // one B operand: 8 k-slots of one MFMA
  static constexpr int PER_TILE = 1;   // MFMAs (B operands) per weight tile
  static constexpr int PER_CHUNK = 2;  // B operands made from one 32-unit accumulator
};
template <> struct Operand<false> {
  typedef float T;
  static constexpr int PER_TILE = 4;
  static constexpr int PER_CHUNK = 16;
};

// acc += tile * operands, for one weight tile held as raw 16 bytes per lane
template <bool BF16>
__device__ __forceinline__ void mma_tile(const u32x4& raw, const typename Operand<BF16>::T* b,
                                         f32x16& acc) {
#ifdef MSRL_X_NO_MFMA
  acc[0] += __builtin_bit_cast(f32x4, raw)[0];
  return;
#endif
  if constexpr (BF16) {
    acc = mma(__builtin_bit_cast(bf16x8, raw), b[0], acc);
  } else {
    const f32x4 a = __builtin_bit_cast(f32x4, raw);
#pragma unroll
    for (int j = 0; j < 4; ++j) acc = mma(a[j], b[j], acc);
  }
}

// bias for the 16 accumulator registers of chunk uc: units 32uc + 8b + 4h + c
__device__ __forceinline__ f32x16 bias_init(const float* lds_bias, int uc, int h) {
  f32x16 acc;
#pragma unroll
  for (int b = 0; b < 4; ++b) {
    const f32x4 v = *(const f32x4*)(lds_bias + 32 * uc + 8 * b + 4 * h);
#pragma unroll
    for (int c = 0; c < 4; ++c) acc[4 * b + c] = v[c];
  }
  return acc;
}

// Program-order pins.  The compiler is free to move pure arithmetic anywhere, and left alone it
// puts all MFMAs of a block first and all tanh work last, so nothing overlaps inside a wave.  An
// empty volatile asm on a value fixes the point in program order where the value must exist; the
// pins keep "MFMAs of tile k, tanh slice k, MFMAs of tile k+1, ..." in the order written below.
__device__ __forceinline__ void pin(float& v) { asm volatile("" : "+v"(v)); }
__device__ __forceinline__ void pin(f32x16& v) { asm volatile("" : "+v"(v)); }

// tanh of accumulator registers [r0, r1) of a 32-unit chunk into a scratch array.  When pinned,
// the whole group is computed between two pins, so its independent chains can be interleaved
// with each other but stay between the neighbouring MFMAs.
__device__ __forceinline__ void tanh_range(const f32x16& acc, float (&t)[16], int r0, int r1, bool pinned) {
  float v[16];
#pragma unroll
  for (int r = 0; r < 16; ++r)
    if (r >= r0 && r < r1) {
      v[r] = acc[r];
      if (pinned) pin(v[r]);
    }
#pragma unroll
  for (int r = 0; r < 16; ++r)
    if (r >= r0 && r < r1) t[r] = fast_tanh(v[r]);
#pragma unroll
  for (int r = 0; r < 16; ++r)
    if (r >= r0 && r < r1 && pinned) pin(t[r]);
}

// the 16 activated values of a chunk as the next layer's B operands
template <bool BF16>
__device__ __forceinline__ void to_operands(const float (&t)[16], typename Operand<BF16>::T* out) {
  if constexpr (BF16) {
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      f32x8 v;
#pragma unroll
      for (int s = 0; s < 8; ++s) v[s] = t[8 * j + s];
      out[j] = __builtin_convertvector(v, bf16x8);  // round to nearest even
    }
  } else {
#pragma unroll
    for (int r = 0; r < 16; ++r) out[r] = t[r];
  }
}

// Software pipeline inside a wave: while the MFMAs of chunk c run, the VALU
// applies bias-free tanh to the accumulators of chunk c-1 (the bias is the
// accumulator's initial value), so both pipes are busy from one instruction
// stream.  In a layer-2 stage the layer-3 MFMAs of chunk c-1 follow.
template <int H, bool BF16, int NB, int KT1>
struct Mlp {
#ifdef MSRL_X_NO_TILE_READ
#define TILE_AT(p, i) (u32x4{(uint32_t)(i), 1u, 2u, 3u})
#else
#define TILE_AT(p, i) ((p)[(i) * 64])
#endif
  typedef typename Operand<BF16>::T Op;
  static constexpr int PT = Operand<BF16>::PER_TILE;
  static constexpr int PC = Operand<BF16>::PER_CHUNK;
  static constexpr int NUC = H / 32;
  static constexpr int KT2 = BF16 ? H / 16 : H / 8;
  static constexpr int TPC = KT2 / NUC;              // layer-3 tiles fed by one 32-unit chunk
  static constexpr int L1_TILES = NUC * KT1;         // stage 0 of a network
  static constexpr int CHUNK_TILES = KT2 + 2 * TPC;  // stages 1..NUC: layer-2 tiles of chunk c,
                                                     // layer-3 tiles of chunk c-1, of chunk c
  static constexpr int STAGES = 1 + NUC;
  static constexpr int MAX_STAGE_TILES = L1_TILES > CHUNK_TILES ? L1_TILES : CHUNK_TILES;
  static constexpr int G = 4;  // LDS reads run G tiles ahead of the MFMAs that consume them
  // tanh of the previous chunk, spread over the NT tiles of the current one
#ifndef MSRL_GS
#define MSRL_GS 1
#endif
  // tiles per tanh group: after every GS-th tile the tanh of GS tiles' share of values is issued
  static constexpr int GS = MSRL_GS;
  template <int NT>
  __device__ static __forceinline__ void tanh_slice(const f32x16 (&prev)[NB], float (&t)[NB][16], int kt) {
    constexpr int gs = GS < NT ? GS : NT;
    if (kt % gs != gs - 1) return;
    const int k0 = kt - (gs - 1);
    const int r0 = k0 * 16 / NT, r1 = (kt + 1) * 16 / NT;
#pragma unroll
    for (int q = 0; q < NB; ++q) tanh_range(prev[q], t[q], r0, r1, true);
  }

  // tiles: this lane's slot of tile 0 of the stage in LDS (tile t is at tiles[64 t]).
  __device__ static __forceinline__ void layer1(const u32x4* tiles, const float* lds_b1,
                                                const Op (&x)[NB][KT1 * PT],
                                                Op (&h1)[NB][KT2 * PT], int h) {
    u32x4 ring[G];
#pragma unroll
    for (int i = 0; i < G && i < L1_TILES; ++i) ring[i] = TILE_AT(tiles, i);
    f32x16 prev[NB];
#pragma unroll
    for (int uc = 0; uc <= NUC; ++uc) {
      f32x16 acc[NB];
      float t[NB][16];
      if (uc < NUC) {
        const f32x16 b = bias_init(lds_b1, uc, h);
#pragma unroll
        for (int q = 0; q < NB; ++q) acc[q] = b;
      }
#pragma unroll
      for (int kt = 0; kt < KT1; ++kt) {
        if (uc < NUC) {
          const int idx = uc * KT1 + kt;
          const u32x4 raw = ring[idx % G];
          if (idx + G < L1_TILES) ring[idx % G] = TILE_AT(tiles, idx + G);
#pragma unroll
          for (int q = 0; q < NB; ++q) {
            mma_tile<BF16>(raw, &x[q][kt * PT], acc[q]);
            if (uc > 0) pin(acc[q]);
          }
        }
        if (uc > 0) tanh_slice<KT1>(prev, t, kt);
      }
      if (uc > 0) {
#pragma unroll
        for (int q = 0; q < NB; ++q) to_operands<BF16>(t[q], &h1[q][(uc - 1) * PC]);
      }
#pragma unroll
      for (int q = 0; q < NB; ++q) prev[q] = acc[q];
    }
  }

  __device__ static __forceinline__ void out_init(const float* lds_b3, f32x16 (&out)[NB], int h) {
    const f32x16 b = bias_init(lds_b3, 0, h);
#pragma unroll
    for (int q = 0; q < NB; ++q) out[q] = b;
  }

  // Stage of chunk uc: acc <- layer-2 pre-activations of chunk uc; if PIPE, `acc` holds
  // those of chunk uc-1 on entry, which get tanh and feed layer 3 meanwhile.
  template <bool PIPE>
  __device__ static __forceinline__ void layer2_chunk(const u32x4* tiles, const float* lds_b2, int uc,
                                                      const Op (&h1)[NB][KT2 * PT],
                                                      f32x16 (&acc)[NB], f32x16 (&out)[NB], int h) {
    u32x4 ring[G];
#pragma unroll
    for (int i = 0; i < G; ++i) ring[i] = TILE_AT(tiles, i);
    f32x16 prev[NB];
    float t[NB][16];
    const f32x16 b = bias_init(lds_b2, uc, h);
#pragma unroll
    for (int q = 0; q < NB; ++q) {
      prev[q] = acc[q];
      acc[q] = b;
    }
#pragma unroll
    for (int kt = 0; kt < KT2; ++kt) {
      const u32x4 raw = ring[kt % G];
      if (kt + G < KT2 + TPC) ring[kt % G] = TILE_AT(tiles, kt + G);
#pragma unroll
      for (int q = 0; q < NB; ++q) {
        mma_tile<BF16>(raw, &h1[q][kt * PT], acc[q]);
        if (PIPE) pin(acc[q]);
      }
      if (PIPE) tanh_slice<KT2>(prev, t, kt);
    }
    if (PIPE) {
      Op h2[NB][PC];
#pragma unroll
      for (int q = 0; q < NB; ++q) to_operands<BF16>(t[q], h2[q]);
#pragma unroll
      for (int i = 0; i < TPC; ++i) {
        const u32x4 raw = ring[(KT2 + i) % G];
#pragma unroll
        for (int q = 0; q < NB; ++q) mma_tile<BF16>(raw, &h2[q][i * PT], out[q]);
      }
    }
  }

  // after the last chunk stage: its tanh and layer-3 contribution (tiles of the same stage)
  __device__ static __forceinline__ void layer2_drain(const u32x4* tiles, const f32x16 (&acc)[NB],
                                                      f32x16 (&out)[NB]) {
    u32x4 w3[TPC];
#pragma unroll
    for (int i = 0; i < TPC; ++i) w3[i] = TILE_AT(tiles, KT2 + TPC + i);
    float t[NB][16];
    Op h2[NB][PC];
#pragma unroll
    for (int q = 0; q < NB; ++q) {
      tanh_range(acc[q], t[q], 0, 16, false);
      to_operands<BF16>(t[q], h2[q]);
    }
#pragma unroll
    for (int i = 0; i < TPC; ++i) {
#pragma unroll
      for (int q = 0; q < NB; ++q) mma_tile<BF16>(w3[i], &h2[q][i * PT], out[q]);
    }
  }
};

// Weight stream of a workgroup: stage g of the endless sequence (policy stages,
// value stages, policy stages, ...) lives in LDS buffer g % 3 and is copied there
// two stages ahead by direct global->LDS loads (no registers involved).
//
// The copy instruction is issued from inline assembly on purpose: issued through
// the compiler builtin, every later LDS read of the *resident* stage would be
// made to wait for the copies still in flight (the compiler cannot tell the
// buffers apart), which serialises the L2 latency with the compute.  The price
// is that the wait is written by hand: each wave issues exactly PER_WAVE copies
// per stage, loads complete in order, so "at most PER_WAVE vector-memory
// operations outstanding" means the copies of the stage before the newest one
// have landed.  Vector-memory operations the compiler issues itself only add to
// the outstanding count, which makes the wait longer, never shorter.
template <class Net, int WAVES>
struct WeightStream {
  static constexpr int STAGES_PER_STEP = 2 * Net::STAGES;
  static constexpr int PER_WAVE = (Net::MAX_STAGE_TILES + WAVES - 1) / WAVES;  // copies per wave and stage
  static constexpr int BUF_TILES = PER_WAVE * WAVES;                            // incl. padding tiles
  static constexpr int BUF_SLOTS = BUF_TILES * 64;                              // u32x4 slots per buffer
  static constexpr int NBUF = 3;
  static_assert(PER_WAVE <= 15, "the hand-written wait encodes the count in 4 bits");
  u32x4* lds;  // NBUF * BUF_SLOTS slots
  const uint8_t* packed;
  size_t net_bytes, chunks_off, chunk_bytes;
  int wave, lane;

  // start copying stage s (0 .. STAGES_PER_STEP-1) into buffer `buf`
  mutable int x_issued = 0;
  __device__ __forceinline__ void issue(int s, int buf) const {
#ifdef MSRL_X_NO_RELOAD
    if (x_issued >= MSRL_X_NO_RELOAD) return;
    ++x_issued;
#endif
    const int net = s >= Net::STAGES ? 1 : 0;
    const int ls = s - net * Net::STAGES;
    const uint8_t* src = packed + (size_t)net * net_bytes +
                         (ls == 0 ? 0 : chunks_off + (size_t)(ls - 1) * chunk_bytes);
    const int n_tiles = ls == 0 ? Net::L1_TILES : Net::CHUNK_TILES;
    typedef __attribute__((address_space(3))) u32x4 lds_u32x4;
    const uint32_t base = (uint32_t)(uintptr_t)(lds_u32x4*)(lds + buf * BUF_SLOTS);
#pragma unroll
    for (int i = 0; i < PER_WAVE; ++i) {
      const int t = wave + i * WAVES;
      // a wave with no tile left repeats tile 0 into its padding tile: every wave issues PER_WAVE copies
      const uint8_t* g = src + (size_t)(t < n_tiles ? t : 0) * 1024 + (size_t)lane * 16;
      const uint32_t m0 = __builtin_amdgcn_readfirstlane(base + (uint32_t)t * 1024u);
      asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(g), "s"(m0) : "memory", "m0");
    }
  }
  // wait until only the newest stage's copies may be outstanding, then for every wave
  __device__ __forceinline__ void wait_older() const {
    // s_waitcnt vmcnt(PER_WAVE): simm16 = vmcnt[3:0] | expcnt(7) << 4 | lgkmcnt(15) << 8
#ifndef MSRL_X_NO_WAIT
    __builtin_amdgcn_s_waitcnt(0x0F70 | PER_WAVE);
#endif
    sync();
  }
  __device__ __forceinline__ void wait_all() const {
    __builtin_amdgcn_s_waitcnt(0x0F70);
    sync();
  }
  __device__ __forceinline__ void sync() const {
#ifndef MSRL_X_NO_BARRIER
    __syncthreads();
#endif
  }
  __device__ __forceinline__ const u32x4* tiles(int buf) const { return lds + buf * BUF_SLOTS + lane; }
};

}  // namespace msrl
