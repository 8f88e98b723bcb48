// Policy / value network forward pass on MFMA, one wave per group of 32*NB rows.
//
// Every layer is computed transposed (units x rows), so a layer's accumulators
//   lane (n = lane % 32, h = lane / 32), register r  <->  row n, unit 32*uc + 8*(r/4) + 4*h + r%4
// are, after bias + tanh (+ rounding to bf16), exactly the B operand of the next
// layer's MFMAs: activations never leave the register file.  The weights are
// the A operand; the workgroup streams them through LDS in stages (the layer-1
// tiles, then one block per 32-unit chunk of layer 2 with the layer-3 tiles that
// consume it; see packed.h), and every wave of the workgroup reads the same
// stage.  Layer 3 is accumulated inside the layer-2 chunk stage, so h2 is
// consumed as soon as it is produced.
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

// tanh of a 32-unit accumulator, stored as the next layer's B operands
template <bool BF16>
__device__ __forceinline__ void activate(const f32x16& acc, typename Operand<BF16>::T* out) {
  if constexpr (BF16) {
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      f32x8 t;
#pragma unroll
      for (int s = 0; s < 8; ++s) t[s] = fast_tanh(acc[8 * j + s]);
      out[j] = __builtin_convertvector(t, bf16x8);  // round to nearest even
    }
  } else {
#pragma unroll
    for (int r = 0; r < 16; ++r) out[r] = fast_tanh(acc[r]);
  }
}

template <int H, bool BF16, int NB, int KT1>
struct Mlp {
  typedef typename Operand<BF16>::T Op;
  static constexpr int PT = Operand<BF16>::PER_TILE;
  static constexpr int PC = Operand<BF16>::PER_CHUNK;
  static constexpr int NUC = H / 32;
  static constexpr int KT2 = BF16 ? H / 16 : H / 8;
  static constexpr int TPC = KT2 / NUC;            // layer-3 tiles fed by one 32-unit chunk
  static constexpr int L1_TILES = NUC * KT1;       // stage 0 of a network
  static constexpr int CHUNK_TILES = KT2 + TPC;    // stages 1..NUC of a network
  static constexpr int STAGES = 1 + NUC;
  static constexpr int MAX_STAGE_TILES = L1_TILES > CHUNK_TILES ? L1_TILES : CHUNK_TILES;

  // tiles: this lane's slot of tile 0 of the stage in LDS (tile t is at tiles[64 t]).
  __device__ static __forceinline__ void layer1(const u32x4* tiles, const float* lds_b1,
                                                const Op (&x)[NB][KT1 * PT],
                                                Op (&h1)[NB][KT2 * PT], int h) {
#pragma unroll
    for (int uc = 0; uc < NUC; ++uc) {
      f32x16 acc[NB];
      const f32x16 b = bias_init(lds_b1, uc, h);
#pragma unroll
      for (int q = 0; q < NB; ++q) acc[q] = b;
#pragma unroll
      for (int kt = 0; kt < KT1; ++kt) {
        const u32x4 raw = tiles[(uc * KT1 + kt) * 64];
#pragma unroll
        for (int q = 0; q < NB; ++q) mma_tile<BF16>(raw, &x[q][kt * PT], acc[q]);
      }
#pragma unroll
      for (int q = 0; q < NB; ++q) activate<BF16>(acc[q], &h1[q][uc * PC]);
    }
  }

  __device__ static __forceinline__ void out_init(const float* lds_b3, f32x16 (&out)[NB], int h) {
    const f32x16 b = bias_init(lds_b3, 0, h);
#pragma unroll
    for (int q = 0; q < NB; ++q) out[q] = b;
  }

  // one 32-unit chunk of layer 2 and its contribution to layer 3
  __device__ static __forceinline__ void layer2_chunk(const u32x4* tiles, const float* lds_b2, int uc,
                                                      const Op (&h1)[NB][KT2 * PT],
                                                      f32x16 (&out)[NB], int h) {
    f32x16 acc[NB];
    const f32x16 b = bias_init(lds_b2, uc, h);
#pragma unroll
    for (int q = 0; q < NB; ++q) acc[q] = b;
#pragma unroll
    for (int kt = 0; kt < KT2; ++kt) {
      const u32x4 raw = tiles[kt * 64];
#pragma unroll
      for (int q = 0; q < NB; ++q) mma_tile<BF16>(raw, &h1[q][kt * PT], acc[q]);
    }
    Op h2[NB][PC];
#pragma unroll
    for (int q = 0; q < NB; ++q) activate<BF16>(acc[q], h2[q]);
#pragma unroll
    for (int i = 0; i < TPC; ++i) {
      const u32x4 raw = tiles[(KT2 + i) * 64];
#pragma unroll
      for (int q = 0; q < NB; ++q) mma_tile<BF16>(raw, &h2[q][i * PT], out[q]);
    }
  }
};

// Double-buffered weight stream of a workgroup: stage g of the endless sequence
// (policy stages, value stages, policy stages, ...) lives in buffer g % 2.
template <class Net, int WAVES>
struct WeightStream {
  static constexpr int STAGES_PER_STEP = 2 * Net::STAGES;
  static constexpr int BUF_SLOTS = Net::MAX_STAGE_TILES * 64;  // u32x4 slots per buffer
  u32x4* lds;            // 2 * BUF_SLOTS slots
  const uint8_t* packed;
  size_t net_bytes, chunks_off, chunk_bytes;
  int wave, lane;

  // start the copy of stage s (0 .. STAGES_PER_STEP-1) into buffer `parity`
  __device__ __forceinline__ void issue(int s, int parity) const {
    const int net = s >= Net::STAGES ? 1 : 0;
    const int ls = s - net * Net::STAGES;
    const uint8_t* src = packed + (size_t)net * net_bytes +
                         (ls == 0 ? 0 : chunks_off + (size_t)(ls - 1) * chunk_bytes);
    const int n_tiles = ls == 0 ? Net::L1_TILES : Net::CHUNK_TILES;
    u32x4* dst = lds + parity * BUF_SLOTS;
    for (int t = wave; t < n_tiles; t += WAVES)
      __builtin_amdgcn_global_load_lds((const u32x4*)(src + (size_t)t * 1024) + lane, dst + t * 64, 16, 0, 0);
  }
  // wait for this wave's copies, then for every wave of the workgroup
  __device__ __forceinline__ void wait() const {
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
  }
  __device__ __forceinline__ const u32x4* tiles(int parity) const { return lds + parity * BUF_SLOTS + lane; }
};

}  // namespace msrl
