// Policy / value network forward pass on MFMA, one wave per group of 32*NB rows.
//
// Every layer is computed transposed (units x rows), so a layer's accumulators
//   lane (n = lane % 32, h = lane / 32), register r  <->  row n, unit 32*uc + 8*(r/4) + 4*h + r%4
// are, after tanh (+ rounding to bf16), exactly the B operand of the next
// layer's MFMAs: activations never leave the register file.  The weights are
// the A operand and come from LDS: the layer-1 tiles stay resident, the layer-2
// and layer-3 tiles stream through an LDS window in one stage per 32-unit chunk
// (packed.h), and every wave of the workgroup reads the same stage.  Biases are
// one more input of the contraction (the constant 1), so an accumulator starts
// at zero.  Layer 3 is accumulated as the layer-2 chunks complete, so h2 is
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
  // B operand of a bias tile: the constant 1 at input slot (h = 0, s = 0)
  static __device__ __forceinline__ T one(int h) {
    T v = {0, 0, 0, 0, 0, 0, 0, 0};
    v[0] = (__bf16)(h == 0 ? 1.0f : 0.0f);
    return v;
  }
};
template <> struct Operand<false> {
  typedef float T;
  static constexpr int PER_TILE = 4;
  static constexpr int PER_CHUNK = 16;
  static __device__ __forceinline__ T one(int h) { return h == 0 ? 1.0f : 0.0f; }
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

// the same for the first NM of the tile's MFMAs (fp32 tiles are four MFMAs of two inputs each: a layer-1 tile
// whose last inputs do not exist needs fewer; the products left out are zero weight times zero input)
template <bool BF16, int NM>
__device__ __forceinline__ void mma_tile_first(const u32x4& raw, const typename Operand<BF16>::T* b, f32x16& acc) {
  if constexpr (BF16) {
    mma_tile<BF16>(raw, b, acc);
  } else {
    const f32x4 a = __builtin_bit_cast(f32x4, raw);
#pragma unroll
    for (int j = 0; j < NM; ++j) acc = mma(a[j], b[j], acc);
  }
}

// acc += bias tile * 1: only input slot (h = 0, first k) of the tile is populated
template <bool BF16>
__device__ __forceinline__ void mma_bias_tile(const u32x4& raw, const typename Operand<BF16>::T& one,
                                              f32x16& acc) {
  if constexpr (BF16)
    acc = mma(__builtin_bit_cast(bf16x8, raw), one, acc);
  else
    acc = mma(__builtin_bit_cast(f32x4, raw)[0], one, acc);
}

__device__ __forceinline__ f32x16 zero16() {
  f32x16 z;
#pragma unroll
  for (int r = 0; r < 16; ++r) z[r] = 0.0f;
  return z;
}

// the 16 accumulator registers of the output chunk from a bias vector in LDS (units 8b + 4h + c)
__device__ __forceinline__ f32x16 bias_init(const float* lds_bias, int h) {
  f32x16 acc;
#pragma unroll
  for (int b = 0; b < 4; ++b) {
    const f32x4 v = *(const f32x4*)(lds_bias + 8 * b + 4 * h);
#pragma unroll
    for (int c = 0; c < 4; ++c) acc[4 * b + c] = v[c];
  }
  return acc;
}

// Program-order pins.  The compiler is free to move pure arithmetic anywhere, and left alone it
// puts all MFMAs of a block first and all tanh work last, so nothing overlaps inside a wave.  An
// empty volatile asm on a value fixes the point in program order where the value must exist; the
// pins keep "MFMAs of tile k, tanh slice k, MFMAs of tile k+1, ..." in the order written below.
// The MFMAs are held in place through their weight tile, not through the accumulator: where the
// compiler keeps accumulators in the accumulation registers, a pin on one would cost a round trip
// through vector registers and a wait for the matrix pipe at every tile.
__device__ __forceinline__ void pin(float& v) { asm volatile("" : "+v"(v)); }
__device__ __forceinline__ void pin(u32x4& v) { asm volatile("" : "+v"(v)); }

// tanh of accumulator registers [r0, r1) of a 32-unit chunk into a scratch array.  When pinned,
// the whole group is computed between two pins, so it stays between the neighbouring MFMAs.
// PRESCALED: the accumulators hold 2 log2(e) times the pre-activation (fp32 networks, see fast_tanh_prescaled).
template <bool PRESCALED = false>
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
    if (r >= r0 && r < r1) t[r] = PRESCALED ? fast_tanh_prescaled(v[r]) : fast_tanh(v[r]);
#pragma unroll
  for (int r = 0; r < 16; ++r)
    if (r >= r0 && r < r1 && pinned) pin(t[r]);
}

// tanh of accumulator registers [r0, r1) in three stages, each closed by pins, so that a caller can put
// an MFMA between the stages: the independent chains of a stage follow one another (no dependent
// instruction directly behind a transcendental one, so no wait states), and the matrix pipe gets its
// next instruction while the chains are half way.
//   stage 1: w = 2^(c x) + 1     stage 2: w = 1 / w     stage 3: t = 1 - 2 w
__device__ __forceinline__ void tanh_stage1(const f32x16& acc, float (&w)[16], int r0, int r1) {
#pragma unroll
  for (int r = 0; r < 16; ++r)
    if (r >= r0 && r < r1) {
      w[r] = acc[r];
      pin(w[r]);
    }
#pragma unroll
  for (int r = 0; r < 16; ++r)
    if (r >= r0 && r < r1) w[r] = __builtin_amdgcn_exp2f(w[r] * 2.8853900817779268f);
#pragma unroll
  for (int r = 0; r < 16; ++r)
    if (r >= r0 && r < r1) w[r] = w[r] + 1.0f;
#pragma unroll
  for (int r = 0; r < 16; ++r)
    if (r >= r0 && r < r1) pin(w[r]);
}
__device__ __forceinline__ void tanh_stage2(float (&w)[16], int r0, int r1) {
#pragma unroll
  for (int r = 0; r < 16; ++r)
    if (r >= r0 && r < r1) w[r] = __builtin_amdgcn_rcpf(w[r]);
#pragma unroll
  for (int r = 0; r < 16; ++r)
    if (r >= r0 && r < r1) pin(w[r]);
}
__device__ __forceinline__ void tanh_stage3(const float (&w)[16], float (&t)[16], int r0, int r1) {
#pragma unroll
  for (int r = 0; r < 16; ++r)
    if (r >= r0 && r < r1) t[r] = 1.0f - 2.0f * w[r];
#pragma unroll
  for (int r = 0; r < 16; ++r)
    if (r >= r0 && r < r1) pin(t[r]);
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

// Software pipeline inside a wave: while the MFMAs of chunk c run, the VALU applies tanh to the
// accumulators of chunk c-1, so both pipes are busy from one instruction stream.  In a layer-2
// stage the layer-3 MFMAs of chunk c-1 follow.
// L1_LAST: fp32 only, the MFMAs of the last layer-1 tile that meet an existing input (0: all four); which inputs
// an MFMA of a tile multiplies depends on the operand layout of the kernel's observation
// H1_ACC: fp32 only, the layer-1 outputs are parked in accumulation registers (a kernel with one wave per SIMD
// has 256 of them beside its 256 vector registers, and an MFMA takes its B operand from either file)
template <int H, bool BF16, int NB, int KT1, int L1_LAST = 0, bool H1_ACC = false>
struct Mlp {
  typedef typename Operand<BF16>::T Op;
  static constexpr int PT = Operand<BF16>::PER_TILE;
  static constexpr int PC = Operand<BF16>::PER_CHUNK;
  static constexpr int NUC = H / 32;
  static constexpr int KT2 = BF16 ? H / 16 : H / 8;
  static constexpr int TPC = KT2 / NUC;                  // layer-3 tiles fed by one 32-unit chunk
  static constexpr int L1_TILES = NUC * KT1;             // resident
  static constexpr int CHUNK_TILES = KT2 + 1 + 2 * TPC;  // one stage: layer-2 tiles of chunk c, its bias
                                                         // tile, layer-3 tiles of chunk c-1, of chunk c
  static constexpr int L3_PREV = KT2 + 1, L3_OWN = KT2 + 1 + TPC;
  static constexpr int G = 4;  // LDS reads run G tiles ahead of the MFMAs that consume them
  // bf16: one MFMA per tile and (with 256 units) one activation per tile, so the tanh chains are taken two
  // tiles at a time (see tanh_stage1); fp32 tiles are four MFMAs long and hide a chain each as they are
  static constexpr bool PAIRED = BF16 && KT2 % 2 == 0;
  // fp32 networks: the output layer runs on the VALU.  Its few outputs (5 logits, 1 value, 2 K Gaussian
  // parameters) would fill 32 rows of an MFMA that takes 64 cycles per 2 inputs - a sixth of the matrix
  // work of a 128-unit network - while the VALU of these kernels is mostly idle.  Each lane multiplies the
  // activations it holds (16 per chunk) with their weights as the tanh slices complete, between the MFMAs of
  // the next chunk; `out` then holds the lane's partial sum of output o in register o, and out_finish adds the
  // two lanes of a row and the bias and puts the result where the MFMA would have (the accumulator layout).
  // bf16 networks keep the MFMA (2 instructions of 32 cycles per chunk; their VALU is the busy unit), and so do
  // output layers with more than 6 outputs - more than one for 256-unit networks whose layer-1 outputs are not
  // parked in accumulation registers (H1_ACC): those kernels have few registers to spare.
  // OUTS: bit o set <-> output o exists.
  template <uint32_t OUTS>
  static constexpr bool l3v() {
    return !BF16 && __builtin_popcount(OUTS) <= (H <= 128 || H1_ACC ? 6 : 1);
  }
  // layer-3 tiles of a chunk that pass through the ring of LDS reads
  template <uint32_t OUTS>
  static constexpr int l3s() { return l3v<OUTS>() ? 0 : TPC; }

  __device__ static __forceinline__ int lane_id() {
    return (int)__builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u));
  }
  // start value of the output accumulators: the bias (MFMA path), or zero (the bias comes in out_finish)
  template <uint32_t OUTS>
  __device__ static __forceinline__ f32x16 out_init(const float* lds_bias, int h) {
    if constexpr (l3v<OUTS>()) return zero16();
    else return bias_init(lds_bias, h);
  }
  // out[o] += sum over registers r in [r0, r1) of t[r] * W3[unit of (r, h)][o] for the outputs o whose bit is set
  // in OUTS and that are below nout (a network with fewer outputs than the kernel's mask: a constant where the
  // caller's loop over the networks is unrolled).  w3h: the layer-3 tiles
  // of the chunk as floats, at the slot of lane 32 h: register r = 4 i + j meets component j of slot o + 32 h of
  // tile i (the A operand of the MFMA that would multiply it), the same address for every lane of a half-wave.
  template <uint32_t OUTS>
  __device__ static __forceinline__ void l3_slice(const float* w3h, const float (&t)[16], f32x16& out, int r0, int r1,
                                                  int nout, f32x4 (&wg)[16]) {
    static_assert(OUTS != 0 && OUTS < 65536u, "one register per output");
#pragma unroll
    for (int r = 0; r < 16; ++r)
      if (r >= r0 && r < r1) {
        if (r % 4 == 0) {
          // the weights of registers r .. r+3, 16 bytes per output, fetched as the group starts (as single
          // words the compiler fetches them far ahead and the 128-unit kernel spills 29 registers)
#pragma unroll
          for (int o = 0; o < 16; ++o)
            if (((OUTS >> o) & 1u) && o < nout) wg[o] = *(const f32x4*)(w3h + ((r / 4) * 64 + o) * 4);
        }
#pragma unroll
        for (int o = 0; o < 16; ++o)
          if (((OUTS >> o) & 1u) && o < nout) out[o] = __builtin_fmaf(t[r], wg[o][r % 4], out[o]);
      }
  }
  // this half-wave's view of layer-3 tile `first` of the chunk block whose lane slots start at `tiles`
  __device__ static __forceinline__ const float* l3_weights(const u32x4* tiles, int first, int h) {
    return (const float*)(tiles + first * 64 - lane_id() + 32 * h);
  }
  // after the last chunk: (VALU path) partial sums of the two lanes of a row + bias, into the accumulator layout
  template <uint32_t OUTS>
  __device__ static __forceinline__ void out_finish(f32x16 (&out)[NB], const float* lds_bias, int h) {
    if constexpr (l3v<OUTS>()) {
#pragma unroll
      for (int q = 0; q < NB; ++q) {
        float tot[16];
#pragma unroll
        for (int o = 0; o < 16; ++o)
          tot[o] = (OUTS >> o) & 1u ? out[q][o] + __shfl_xor(out[q][o], 32) + lds_bias[o] : 0.0f;
        f32x16 res;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int u0 = 8 * (r / 4) + r % 4, u1 = u0 + 4;  // the register's output on the lanes h = 0 / h = 1
          res[r] = h ? (u1 < 16 ? tot[u1 < 16 ? u1 : 0] : 0.0f) : (u0 < 16 ? tot[u0 < 16 ? u0 : 0] : 0.0f);
        }
        out[q] = res;
      }
    }
  }

  // tanh of the previous chunk, spread over the NT tiles of the current one
  template <int NT>
  __device__ static __forceinline__ void tanh_slice(const f32x16 (&prev)[NB], float (&t)[NB][16], int kt) {
    const int r0 = kt * 16 / NT, r1 = (kt + 1) * 16 / NT;
#pragma unroll
    for (int q = 0; q < NB; ++q) tanh_range<!BF16>(prev[q], t[q], r0, r1, true);
  }

  // Layer 1.  tiles: this lane's slot of tile 0 in LDS (tile t is at tiles[64 t]); x holds the
  // observation with the constant 1 at input index in_dim.
  __device__ static __forceinline__ void layer1(const u32x4* tiles, const Op (&x)[NB][KT1 * PT],
                                                Op (&h1)[NB][KT2 * PT]) {
    u32x4 ring[G];
#pragma unroll
    for (int i = 0; i < G && i < L1_TILES; ++i) ring[i] = tiles[i * 64];
    f32x16 prev[NB];
#pragma unroll
    for (int uc = 0; uc <= NUC; ++uc) {
      f32x16 acc[NB];
      float t[NB][16];
#pragma unroll
      for (int q = 0; q < NB; ++q) acc[q] = zero16();
#pragma unroll
      for (int kt = 0; kt < KT1; ++kt) {
        if (uc < NUC) {
          const int idx = uc * KT1 + kt;
          u32x4 raw = ring[idx % G];
          if (idx + G < L1_TILES) ring[idx % G] = tiles[(idx + G) * 64];
          if (uc > 0) pin(raw);
          constexpr int LAST = BF16 || L1_LAST == 0 ? PT : L1_LAST;
          static_assert(LAST >= 1 && LAST <= PT, "one to four MFMAs");
#pragma unroll
          for (int q = 0; q < NB; ++q) {
            if (kt == KT1 - 1)
              mma_tile_first<BF16, LAST>(raw, &x[q][kt * PT], acc[q]);
            else
              mma_tile<BF16>(raw, &x[q][kt * PT], acc[q]);
          }
        }
        if (uc > 0) tanh_slice<KT1>(prev, t, kt);
      }
      if (uc > 0) {
#pragma unroll
        for (int q = 0; q < NB; ++q) {
          if constexpr (H1_ACC && !BF16) {
#pragma unroll
            for (int r = 0; r < 16; ++r)
              asm volatile("v_accvgpr_write_b32 %0, %1" : "=a"(h1[q][(uc - 1) * PC + r]) : "v"(t[q][r]));
          } else {
            to_operands<BF16>(t[q], &h1[q][(uc - 1) * PC]);
          }
        }
      }
#pragma unroll
      for (int q = 0; q < NB; ++q) prev[q] = acc[q];
    }
  }

  // Stage of chunk uc: acc <- layer-2 pre-activations of chunk uc; if PIPE, `acc` holds those of
  // chunk uc-1 on entry, which get tanh and feed layer 3 meanwhile.
  // tick(kt) is called once per layer-2 tile: the caller spreads the copies of a later stage over
  // the loop, so that they queue behind the MFMAs instead of stalling every wave at the stage start.
  template <bool PIPE, uint32_t OUTS, class Tick>
  __device__ static __forceinline__ void layer2_chunk(const u32x4* tiles, const Op (&h1)[NB][KT2 * PT],
                                                      f32x16 (&acc)[NB], f32x16 (&out)[NB], int h, int nout,
                                                      Tick&& tick) {
    constexpr bool L3V = l3v<OUTS>();
    constexpr int L3S = l3s<OUTS>();
    const float* w3h = L3V ? l3_weights(tiles, L3_PREV, h) : nullptr;
    f32x4 wg[16];
    u32x4 ring[G];
#pragma unroll
    for (int i = 0; i < G; ++i) ring[i] = tiles[i * 64];
    f32x16 prev[NB];
    float t[NB][16];
#pragma unroll
    for (int q = 0; q < NB; ++q) {
      prev[q] = acc[q];
      acc[q] = zero16();
    }
    if constexpr (PIPE && PAIRED) {
      // two tiles per round: the tanh chains of both tiles' share of the chunk before run side by side,
      // the second tile's MFMAs sit between their first and second stage
      float w[NB][16];
#pragma unroll
      for (int kt = 0; kt < KT2; kt += 2) {
        const int r0 = kt * 16 / KT2, r1 = (kt + 2) * 16 / KT2;
        u32x4 raw = ring[kt % G];
        if (kt + G < L3_PREV + L3S) ring[kt % G] = tiles[(kt + G) * 64];
        pin(raw);
#pragma unroll
        for (int q = 0; q < NB; ++q) mma_tile<BF16>(raw, &h1[q][kt * PT], acc[q]);
#pragma unroll
        for (int q = 0; q < NB; ++q) tanh_stage1(prev[q], w[q], r0, r1);
        u32x4 raw2 = ring[(kt + 1) % G];
        if (kt + 1 + G < L3_PREV + L3S) ring[(kt + 1) % G] = tiles[(kt + 1 + G) * 64];
        pin(raw2);
#pragma unroll
        for (int q = 0; q < NB; ++q) mma_tile<BF16>(raw2, &h1[q][(kt + 1) * PT], acc[q]);
#pragma unroll
        for (int q = 0; q < NB; ++q) {
          tanh_stage2(w[q], r0, r1);
          tanh_stage3(w[q], t[q], r0, r1);
        }
        tick(kt);
        tick(kt + 1);
      }
    } else {
#pragma unroll
    for (int kt = 0; kt < KT2; ++kt) {
      u32x4 raw = ring[kt % G];
      if (kt + G < L3_PREV + L3S) ring[kt % G] = tiles[(kt + G) * 64];
      if (PIPE) pin(raw);
#pragma unroll
      for (int q = 0; q < NB; ++q) mma_tile<BF16>(raw, &h1[q][kt * PT], acc[q]);
      if (PIPE) {
        tanh_slice<KT2>(prev, t, kt);
        if constexpr (l3v<OUTS>()) {
#pragma unroll
          for (int q = 0; q < NB; ++q) l3_slice<OUTS>(w3h, t[q], out[q], kt * 16 / KT2, (kt + 1) * 16 / KT2, nout, wg);
        }
      }
      tick(kt);
    }
    }
    {
      const Op one = Operand<BF16>::one(h);
      const u32x4 raw = ring[KT2 % G];
      if (KT2 + G < L3_PREV + L3S) ring[KT2 % G] = tiles[(KT2 + G) * 64];
#pragma unroll
      for (int q = 0; q < NB; ++q) mma_bias_tile<BF16>(raw, one, acc[q]);
    }
    if (PIPE && !L3V) {
      Op h2[NB][PC];
#pragma unroll
      for (int q = 0; q < NB; ++q) to_operands<BF16>(t[q], h2[q]);
#pragma unroll
      for (int i = 0; i < TPC; ++i) {
        const u32x4 raw = ring[(L3_PREV + i) % G];
#pragma unroll
        for (int q = 0; q < NB; ++q) mma_tile<BF16>(raw, &h2[q][i * PT], out[q]);
      }
    }
  }

  // The CPS chunk blocks of one stage (consecutive in the LDS buffer) as one stream of tiles: the ring of
  // LDS reads runs on across the chunk boundaries, so the latency of the first reads is paid once per
  // stage (behind its barrier) and not once per chunk.  Chunk 0 is piped (its predecessor's tanh and
  // layer-3 share run beside it) iff PIPE0; the later chunks always are.  tick(c, kt) once per layer-2 tile.
  template <bool PIPE0, int CPS, uint32_t OUTS, class Tick>
  __device__ static __forceinline__ void layer2_chunks(const u32x4* tiles, const Op (&h1)[NB][KT2 * PT],
                                                       f32x16 (&acc)[NB], f32x16 (&out)[NB], int h, int nout,
                                                       Tick&& tick) {
    // tiles a chunk consumes, in order: its KT2 layer-2 tiles, its bias tile and, if piped, the TPC
    // layer-3 tiles fed by the chunk before it; they are consecutive inside the chunk block
    // (the layer-3 tiles only where the MFMA multiplies them)
    constexpr bool L3V = l3v<OUTS>();
    constexpr int L3S = l3s<OUTS>();
    constexpr int PER0 = KT2 + 1 + (PIPE0 ? L3S : 0), PERN = KT2 + 1 + L3S;
    constexpr int TOTAL = PER0 + (CPS - 1) * PERN;
    auto tile_at = [](int p) -> int {  // position in the stream -> tile index in the buffer
      if (p < PER0) return p;
      const int q = p - PER0;
      return (1 + q / PERN) * CHUNK_TILES + q % PERN;
    };
    u32x4 ring[G];
#pragma unroll
    for (int i = 0; i < G; ++i) ring[i] = tiles[tile_at(i) * 64];
    // next tile of the stream; the slot it leaves is refilled G positions ahead
    auto pop = [&](int p) -> u32x4 {
      const u32x4 raw = ring[p % G];
      if (p + G < TOTAL) ring[p % G] = tiles[tile_at(p + G) * 64];
      return raw;
    };
#pragma unroll
    for (int c = 0; c < CPS; ++c) {
      const bool pipe = PIPE0 || c > 0;
      const int p0 = c == 0 ? 0 : PER0 + (c - 1) * PERN;  // position of the chunk's first tile
      const float* w3h = L3V ? l3_weights(tiles, c * CHUNK_TILES + L3_PREV, h) : nullptr;
      f32x4 wg[16];
      f32x16 prev[NB];
      float t[NB][16];
#pragma unroll
      for (int q = 0; q < NB; ++q) {
        prev[q] = acc[q];
        acc[q] = zero16();
      }
      if (pipe && PAIRED) {
        // two tiles per round: the tanh chains of both tiles' share of the chunk before run side by
        // side, the second tile's MFMAs sit between their first and second stage
        float w[NB][16];
#pragma unroll
        for (int kt = 0; kt < KT2; kt += 2) {
          const int r0 = kt * 16 / KT2, r1 = (kt + 2) * 16 / KT2;
          u32x4 raw = pop(p0 + kt);
          pin(raw);
#pragma unroll
          for (int q = 0; q < NB; ++q) mma_tile<BF16>(raw, &h1[q][kt * PT], acc[q]);
#pragma unroll
          for (int q = 0; q < NB; ++q) tanh_stage1(prev[q], w[q], r0, r1);
          u32x4 raw2 = pop(p0 + kt + 1);
          pin(raw2);
#pragma unroll
          for (int q = 0; q < NB; ++q) mma_tile<BF16>(raw2, &h1[q][(kt + 1) * PT], acc[q]);
#pragma unroll
          for (int q = 0; q < NB; ++q) {
            tanh_stage2(w[q], r0, r1);
            tanh_stage3(w[q], t[q], r0, r1);
          }
          tick(c, kt);
          tick(c, kt + 1);
        }
      } else {
#pragma unroll
        for (int kt = 0; kt < KT2; ++kt) {
          u32x4 raw = pop(p0 + kt);
          if (pipe) pin(raw);
#pragma unroll
          for (int q = 0; q < NB; ++q) mma_tile<BF16>(raw, &h1[q][kt * PT], acc[q]);
          if (pipe) {
            tanh_slice<KT2>(prev, t, kt);
            if constexpr (l3v<OUTS>()) {
#pragma unroll
              for (int q = 0; q < NB; ++q) l3_slice<OUTS>(w3h, t[q], out[q], kt * 16 / KT2, (kt + 1) * 16 / KT2, nout, wg);
            }
          }
          tick(c, kt);
        }
      }
      {
        const Op one = Operand<BF16>::one(h);
        const u32x4 raw = pop(p0 + KT2);
#pragma unroll
        for (int q = 0; q < NB; ++q) mma_bias_tile<BF16>(raw, one, acc[q]);
      }
      if (pipe && !L3V) {
        Op h2[NB][PC];
#pragma unroll
        for (int q = 0; q < NB; ++q) to_operands<BF16>(t[q], h2[q]);
#pragma unroll
        for (int i = 0; i < TPC; ++i) {
          const u32x4 raw = pop(p0 + KT2 + 1 + i);
#pragma unroll
          for (int q = 0; q < NB; ++q) mma_tile<BF16>(raw, &h2[q][i * PT], out[q]);
        }
      }
    }
  }

  // A chunk block of a hidden layer that is not the last one: acc <- pre-activations of chunk uc
  // (bias included); if PIPE, `acc` holds those of chunk uc-1 on entry, which get tanh meanwhile and
  // are returned as operands of the following layer in hprev.
  template <bool PIPE, class Tick>
  __device__ static __forceinline__ void hidden_chunk(const u32x4* tiles, const Op (&hin)[NB][KT2 * PT],
                                                      f32x16 (&acc)[NB], Op (&hprev)[NB][PC], int h,
                                                      Tick&& tick) {
    u32x4 ring[G];
#pragma unroll
    for (int i = 0; i < G; ++i) ring[i] = tiles[i * 64];
    f32x16 prev[NB];
    float t[NB][16];
#pragma unroll
    for (int q = 0; q < NB; ++q) {
      prev[q] = acc[q];
      acc[q] = zero16();
    }
    if constexpr (PIPE && PAIRED) {
      // two tiles per round, the tanh chains of both side by side (as in layer2_chunk)
      float w[NB][16];
#pragma unroll
      for (int kt = 0; kt < KT2; kt += 2) {
        const int r0 = kt * 16 / KT2, r1 = (kt + 2) * 16 / KT2;
        u32x4 raw = ring[kt % G];
        if (kt + G < KT2 + 1) ring[kt % G] = tiles[(kt + G) * 64];
        pin(raw);
#pragma unroll
        for (int q = 0; q < NB; ++q) mma_tile<BF16>(raw, &hin[q][kt * PT], acc[q]);
#pragma unroll
        for (int q = 0; q < NB; ++q) tanh_stage1(prev[q], w[q], r0, r1);
        u32x4 raw2 = ring[(kt + 1) % G];
        if (kt + 1 + G < KT2 + 1) ring[(kt + 1) % G] = tiles[(kt + 1 + G) * 64];
        pin(raw2);
#pragma unroll
        for (int q = 0; q < NB; ++q) mma_tile<BF16>(raw2, &hin[q][(kt + 1) * PT], acc[q]);
#pragma unroll
        for (int q = 0; q < NB; ++q) {
          tanh_stage2(w[q], r0, r1);
          tanh_stage3(w[q], t[q], r0, r1);
        }
        tick(kt);
        tick(kt + 1);
      }
    } else {
#pragma unroll
      for (int kt = 0; kt < KT2; ++kt) {
        u32x4 raw = ring[kt % G];
        if (kt + G < KT2 + 1) ring[kt % G] = tiles[(kt + G) * 64];
        if (PIPE) pin(raw);
#pragma unroll
        for (int q = 0; q < NB; ++q) mma_tile<BF16>(raw, &hin[q][kt * PT], acc[q]);
        if (PIPE) tanh_slice<KT2>(prev, t, kt);
        tick(kt);
      }
    }
    {
      const Op one = Operand<BF16>::one(h);
      const u32x4 raw = ring[KT2 % G];
#pragma unroll
      for (int q = 0; q < NB; ++q) mma_bias_tile<BF16>(raw, one, acc[q]);
    }
    if (PIPE) {
#pragma unroll
      for (int q = 0; q < NB; ++q) to_operands<BF16>(t[q], hprev[q]);
    }
  }
  // the last chunk of such a layer
  __device__ static __forceinline__ void hidden_drain(const f32x16 (&acc)[NB], Op (&hlast)[NB][PC]) {
#pragma unroll
    for (int q = 0; q < NB; ++q) {
      float t[16];
      tanh_range<!BF16>(acc[q], t, 0, 16, false);
      to_operands<BF16>(t, hlast[q]);
    }
  }

  // after the last chunk stage: its tanh and layer-3 contribution (tiles of the same stage)
  template <uint32_t OUTS>
  __device__ static __forceinline__ void layer2_drain(const u32x4* tiles, const f32x16 (&acc)[NB],
                                                      f32x16 (&out)[NB], int h, int nout) {
    if constexpr (l3v<OUTS>()) {
      const float* w3h = l3_weights(tiles, L3_OWN, h);
      f32x4 wg[16];
#pragma unroll
      for (int q = 0; q < NB; ++q) {
        float t[16];
        tanh_range<!BF16>(acc[q], t, 0, 16, false);
        l3_slice<OUTS>(w3h, t, out[q], 0, 16, nout, wg);
      }
      return;
    }
    u32x4 w3[TPC];
#pragma unroll
    for (int i = 0; i < TPC; ++i) w3[i] = tiles[(L3_OWN + i) * 64];
    float t[NB][16];
    Op h2[NB][PC];
#pragma unroll
    for (int q = 0; q < NB; ++q) {
      tanh_range<!BF16>(acc[q], t[q], 0, 16, false);
      to_operands<BF16>(t[q], h2[q]);
    }
#pragma unroll
    for (int i = 0; i < TPC; ++i) {
#pragma unroll
      for (int q = 0; q < NB; ++q) mma_tile<BF16>(w3[i], &h2[q][i * PT], out[q]);
    }
  }
};

// Of the two waves that share a SIMD the older one wins the issue arbitration, runs ahead and then waits at
// the stage barrier while the other finishes alone.  Handing the higher priority to the other half of the
// workgroup stage by stage keeps the pair closer together.
__device__ __forceinline__ void stage_priority(int stage, int wave, int waves) {
  if ((stage & 1) == (wave >= waves / 2 ? 1 : 0))
    __builtin_amdgcn_s_setprio(1);
  else
    __builtin_amdgcn_s_setprio(0);
}

// Weight stream of a workgroup: stage g of the endless sequence (groups of CPS
// policy chunk blocks, then of value chunk blocks, then policy again, ...) lives
// in LDS buffer g % NBUF and is copied there NBUF - 1 stages ahead by direct global->LDS loads
// (no registers involved).
//
// The copy instruction is issued from inline assembly on purpose: issued through
// the compiler builtin, every later LDS read of the *resident* stage would be
// made to wait for the copies still in flight (the compiler cannot tell the
// buffers apart), which serialises the L2 latency with the compute.  The price
// is that the wait is written by hand: each wave issues exactly PER_WAVE copies
// per stage, loads complete in order, so "at most (NBUF - 2) * PER_WAVE vector
// memory operations outstanding" means the copies of the stage about to be used
// have landed.  Vector-memory operations the compiler issues itself only add to
// the outstanding count, which makes the wait longer, never shorter.
template <class Net, int WAVES, int NBUF, int CPS>
struct WeightStream {
  // a stage = CPS consecutive chunk blocks of one network
  static_assert(Net::NUC % CPS == 0, "stages must not straddle networks");
  static constexpr int STAGES_PER_NET = Net::NUC / CPS;
  static constexpr int STAGES_PER_STEP = 2 * STAGES_PER_NET;
  static constexpr int STAGE_TILES = CPS * Net::CHUNK_TILES;
  static constexpr int PER_WAVE = (STAGE_TILES + WAVES - 1) / WAVES;  // copies per wave and stage
  static constexpr int BUF_SLOTS = STAGE_TILES * 64;                   // u32x4 slots per buffer
  static constexpr int AHEAD = NBUF - 1;
  static_assert(NBUF >= 2, "a stage in use and one in flight");
  u32x4* lds;  // NBUF * BUF_SLOTS slots
  const uint8_t* packed;
  size_t net_bytes, chunks_off, chunk_bytes;
  int wave, lane;
  int stages_per_net = STAGES_PER_NET;  // more with more than two hidden layers (set by the kernel)

  // copy number i (0 .. PER_WAVE-1) of this wave for stage s (0 .. 2 stages_per_net - 1) into buffer `buf`
  __device__ __forceinline__ void issue_part(int s, int buf, int i) const {
    const int net = s >= stages_per_net ? 1 : 0;
    const uint8_t* src = packed + (size_t)net * net_bytes + chunks_off +
                         (size_t)(s - net * stages_per_net) * CPS * chunk_bytes;
    typedef __attribute__((address_space(3))) u32x4 lds_u32x4;
    const uint32_t base = (uint32_t)(uintptr_t)(lds_u32x4*)(lds + buf * BUF_SLOTS);
    // a wave with no tile left copies tile 0 once more (same bytes to the same place), so that
    // every wave issues exactly PER_WAVE copies per stage
    int t = wave + i * WAVES;
    t = t < STAGE_TILES ? t : 0;
    // Scalar base address + per-lane byte offset: no vector registers are tied up by addresses
    // (`wave` must be wave-uniform; the kernels read it with readfirstlane).  The address is copied
    // by a scalar instruction inside the asm block: that is the one wait state the hardware wants
    // between the write of M0 and the copy instruction, and it makes the address register
    // scalar-written whatever produced the operand (a memory instruction may not read a scalar
    // register a vector instruction wrote less than 5 cycles earlier, and the compiler cannot
    // see into the block to keep that distance).
    const uint64_t sbase = (uint64_t)(uintptr_t)(src + (size_t)t * 1024);
    const uint32_t m0 = base + (uint32_t)t * 1024u;
    uint64_t tmp;
    asm volatile("s_mov_b32 m0, %3\n\ts_mov_b64 %0, %2\n\tglobal_load_lds_dwordx4 %1, %0"
                 : "=&s"(tmp)
                 : "v"(lane * 16), "s"(sbase), "s"(m0)
                 : "memory", "m0");
  }
  __device__ __forceinline__ void issue(int s, int buf) const {
#pragma unroll
    for (int i = 0; i < PER_WAVE; ++i) issue_part(s, buf, i);
  }
  // wait until the oldest stage in flight has landed, then for every wave of the workgroup
  __device__ __forceinline__ void wait_oldest() const {
    static_assert((NBUF - 2) * PER_WAVE <= 15, "the hand-written wait encodes the count in 4 bits");
    // s_waitcnt vmcnt(n): simm16 = vmcnt[3:0] | expcnt(7) << 4 | lgkmcnt(15) << 8
    __builtin_amdgcn_s_waitcnt(0x0F70 | ((NBUF - 2) * PER_WAVE));
    __syncthreads();
  }
  __device__ __forceinline__ void wait_all() const {
    __builtin_amdgcn_s_waitcnt(0x0F70);
    __syncthreads();
  }
  // this lane's slot of tile 0 of chunk block c of the stage in buffer `buf`
  __device__ __forceinline__ const u32x4* tiles(int buf, int c) const {
    return lds + buf * BUF_SLOTS + c * Net::CHUNK_TILES * 64 + lane;
  }
};

}  // namespace msrl
