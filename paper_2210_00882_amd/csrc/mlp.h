// Policy / value network forward pass on MFMA, one wave per group of 32*NB rows.
//
// Every layer is computed transposed (units x rows), so a layer's accumulators
//   lane (n = lane % 32, h = lane / 32), register r  <->  row n, unit 32*uc + 8*(r/4) + 4*h + r%4
// are, after bias + tanh (+ rounding to bf16), exactly the B operand of the next
// layer's MFMAs: activations never leave the register file.  The weights are
// the A operand and stream in as 1 KiB tiles in the order written by the
// packing kernel (packed.h).  Layer 3 is accumulated inside the layer-2 chunk
// loop, so h2 is consumed as soon as it is produced.
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
  typedef bf16x8 T;                 // one B operand: 8 k-slots of one MFMA
  static constexpr int PER_TILE = 1;  // MFMAs (B operands) per weight tile
  static constexpr int PER_CHUNK = 2; // B operands made from one 32-unit accumulator
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
  static constexpr int TPC = KT2 / NUC;  // layer-3 tiles fed by one 32-unit chunk

  // net: packed network in global memory; lds_bias: b1[H] b2[H] b3[32];
  // x: layer-1 B operands; out: layer-3 accumulators (32 physical outputs x rows).
  __device__ static __forceinline__ void forward(const uint8_t* __restrict__ net,
                                                 const float* lds_bias, const Op (&x)[NB][KT1 * PT],
                                                 f32x16 (&out)[NB], int lane) {
    const int h = lane >> 5;
    const u32x4* w1 = (const u32x4*)net + lane;
    const u32x4* w2 = (const u32x4*)(net + (size_t)NUC * KT1 * 1024) + lane;
    const u32x4* w3 = (const u32x4*)(net + (size_t)NUC * KT1 * 1024 + (size_t)NUC * KT2 * 1024) + lane;
    Op h1[NB][KT2 * PT];

#pragma unroll
    for (int uc = 0; uc < NUC; ++uc) {
      f32x16 acc[NB];
      const f32x16 b = bias_init(lds_bias, uc, h);
#pragma unroll
      for (int q = 0; q < NB; ++q) acc[q] = b;
#pragma unroll
      for (int kt = 0; kt < KT1; ++kt) {
        const u32x4 raw = w1[(uc * KT1 + kt) * 64];
#pragma unroll
        for (int q = 0; q < NB; ++q) mma_tile<BF16>(raw, &x[q][kt * PT], acc[q]);
      }
#pragma unroll
      for (int q = 0; q < NB; ++q) activate<BF16>(acc[q], &h1[q][uc * PC]);
    }

    {
      const f32x16 b = bias_init(lds_bias + 2 * H, 0, h);
#pragma unroll
      for (int q = 0; q < NB; ++q) out[q] = b;
    }
#pragma unroll 1
    for (int uc = 0; uc < NUC; ++uc) {
      f32x16 acc[NB];
      const f32x16 b = bias_init(lds_bias + H, uc, h);
#pragma unroll
      for (int q = 0; q < NB; ++q) acc[q] = b;
      const u32x4* w = w2 + (size_t)uc * KT2 * 64;
#pragma unroll
      for (int kt = 0; kt < KT2; ++kt) {
        const u32x4 raw = w[kt * 64];
#pragma unroll
        for (int q = 0; q < NB; ++q) mma_tile<BF16>(raw, &h1[q][kt * PT], acc[q]);
      }
      Op h2[NB][PC];
#pragma unroll
      for (int q = 0; q < NB; ++q) activate<BF16>(acc[q], h2[q]);
      const u32x4* w3c = w3 + (size_t)uc * TPC * 64;
#pragma unroll
      for (int i = 0; i < TPC; ++i) {
        const u32x4 raw = w3c[i * 64];
#pragma unroll
        for (int q = 0; q < NB; ++q) mma_tile<BF16>(raw, &h2[q][i * PT], out[q]);
      }
    }
  }
};

}  // namespace msrl
