// Kernels around the learner's row kernel (learn_fused.h): packing of the fp32 master weights into
// bf16 MFMA tiles, and the weight gradients from the tiled unit-major tensors the row kernel writes.
// Included by one translation unit only (the kernels here are not templates).
#pragma once
#include "learn_fused.h"

namespace msrl {

// ---------------------------------------------------------------- packing (fp32 master -> bf16 tiles)
struct LearnPackJob {
  const float* src;
  const float* bias;  // or null: split into a bf16 high and low part at input indices bias_index, +1
  u32x4* dst;
  int n_in, n_out;
  int64_t s_in, s_out;  // element (in, out) is src[in * s_in + out * s_out]
  int bias_index;
  int nuc, kt;  // output chunks of 32, tiles per chunk
  int group, chunk_stride, slot_base;  // destination tile as in PackJob (packed.h)
  int linear;   // input map: 1 = 16 kt + 8 h + s (observation), 0 = chained
};
struct LearnPackJobs {
  int n;
  LearnPackJob job[12];
  float* clear;   // or null: floats [0, n_clear) are set to zero (the statistics bins of the pass)
  int n_clear;
};

__device__ __forceinline__ uint32_t bf16_bits(float v) {
  const __bf16 b = (__bf16)v;  // round to nearest even
  return (uint32_t)__builtin_bit_cast(uint16_t, b);
}

__global__ void learn_pack_kernel(LearnPackJobs jobs) {
  const LearnPackJob& j = jobs.job[blockIdx.y];
  const int tid = blockIdx.x * blockDim.x + threadIdx.x;
  if (jobs.clear && blockIdx.y == 0)
    for (int i = tid; i < jobs.n_clear; i += gridDim.x * blockDim.x) jobs.clear[i] = 0.0f;
  if (tid >= j.nuc * j.kt * 64) return;
  const int tile = tid >> 6, lane = tid & 63;
  const int uc = tile / j.kt, kt = tile % j.kt;
  const int dst_slot = ((uc + kt / j.group) * j.chunk_stride + j.slot_base + kt % j.group) * 64 + lane;
  const int m = lane & 31, h = lane >> 5;
  const int o = 32 * uc + m;
  float v[8];
  for (int e = 0; e < 8; ++e) {
    const int i = j.linear ? 16 * kt + 8 * h + e : 32 * (kt >> 1) + 16 * (kt & 1) + 8 * (e >> 2) + 4 * h + (e & 3);
    v[e] = 0.0f;
    if (o < j.n_out) {
      if (i < j.n_in) {
        v[e] = j.src[(int64_t)i * j.s_in + (int64_t)o * j.s_out];
      } else if (j.bias && (i == j.bias_index || i == j.bias_index + 1)) {
        const float b = j.bias[o];
        const float hi = (float)(__bf16)b;
        v[e] = i == j.bias_index ? hi : b - hi;
      }
    }
  }
  u32x4 w;
  for (int p = 0; p < 4; ++p) w[p] = bf16_bits(v[2 * p]) | (bf16_bits(v[2 * p + 1]) << 16);
  j.dst[dst_slot] = w;
}

// ---------------------------------------------------------------- weight gradients from the tiled layout
struct WgradTArgs {
  const __bf16* A;  // [tiles][4][UA][8]: left operand, its units are the rows of C
  const __bf16* B;  // [tiles][4][UB][8]: right operand, its units are the columns of C
  int UA, UB;
  int M, N;         // units that take part (M <= min(UA, 256), N <= min(UB, 256))
  int m_out;        // rows m < m_out of C are written
  int64_t n_tiles;
  int tiles_per_slice;  // row tiles per workgroup, even
  float* C;         // [slice][m_out, ldc] = the slice's A^T-contraction; the copies are slice_stride floats apart
  int64_t ldc;
  float* bias;      // [slice][N] = the slice's sums of B over the rows, or null
  int64_t slice_stride;
};

// Output-stationary like wgrad_kernel (learn_kernels.h): workgroup z takes the row tiles
// [z tiles_per_slice, (z+1) tiles_per_slice), wave w the units 32 w .. 32 w + 31 of A and all NTW
// column tiles of 32; the B fragments of a step (two row tiles = four k tiles) are shared through
// LDS.  Both operands are fetched DEPTH steps ahead into registers: the kernel does little
// arithmetic per byte, so what it needs is enough loads in flight per compute unit to cover the
// memory latency (NTW = 1, the output layer, has the registers for a deeper queue).
// The bias gradient is one more contraction with a left operand of ones: wave w adds it up for
// column tile w.
// Every slice stores its own copy of the result; reduce_partials_kernel (learn_kernels.h) adds the
// copies up in slice order, so the gradient does not depend on the order the workgroups finish in.
// Several such contractions in one launch (blockIdx.y picks the job): the launches of one gradient
// pass are short, so their tails and their memory latencies overlap when the workgroups of all of
// them are resident together.
struct WgradTJobs {
  int n;
  WgradTArgs job[6];
};

template <int NTW, int DEPTH>
__global__ __launch_bounds__(512) void wgrad_tiled_kernel(WgradTJobs jobs) {
  const WgradTArgs& g = jobs.job[blockIdx.y];
  constexpr int FR = NTW * 4 * 64;                 // B fragments per step
  constexpr int PER = (FR + 511) / 512;            // ... per thread
  __shared__ __attribute__((aligned(16))) u32x4 s_b[FR];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int i = lane & 31, h = lane >> 5;
  const int64_t t_begin = (int64_t)blockIdx.x * g.tiles_per_slice;
  const int64_t t_end = min(g.n_tiles, t_begin + g.tiles_per_slice);
  if (t_begin >= t_end) return;  // whole workgroup
  const int ntiles = min(NTW, (g.N + 31) / 32);
  const int m0 = 32 * wave;
  const bool m_live = m0 < g.M;
  const bool a_ok = m0 + i < g.M;
  const bool b_live = g.bias != nullptr && wave < ntiles;
  const bf16x8 zero = {0, 0, 0, 0, 0, 0, 0, 0};
  auto panel_frag = [&](int f, int64_t T0) -> bf16x8 {
    const int slot = f * 512 + threadIdx.x;
    const int j = slot / 256, kk = (slot / 64) % 4, l = slot % 64;
    const int nn = 32 * j + (l & 31);
    const int64_t T = T0 + kk / 2;
    if (slot < FR && j < ntiles && nn < g.N && T < t_end)
      return ((const bf16x8*)g.B)[((size_t)T * 4 + 2 * (kk % 2) + (l >> 5)) * g.UB + nn];
    return zero;
  };
  auto a_frag = [&](int kk, int64_t T0) -> bf16x8 {
    const int64_t T = T0 + kk / 2;
    if (a_ok && T < t_end) return ((const bf16x8*)g.A)[((size_t)T * 4 + 2 * (kk % 2) + h) * g.UA + m0 + i];
    return zero;
  };
  f32x16 acc[NTW], accb = zero16();
#pragma unroll
  for (int j = 0; j < NTW; ++j) acc[j] = zero16();
  bf16x8 ones;
#pragma unroll
  for (int s = 0; s < 8; ++s) ones[s] = (__bf16)1.0f;
  // queue of DEPTH steps; slot d holds step (begin + 2 d) + 2 DEPTH k for k = 0, 1, ...
  bf16x8 qb[DEPTH][PER], qa[DEPTH][4];
#pragma unroll
  for (int d = 0; d < DEPTH; ++d) {
#pragma unroll
    for (int f = 0; f < PER; ++f) qb[d][f] = panel_frag(f, t_begin + 2 * d);
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) qa[d][kk] = a_frag(kk, t_begin + 2 * d);
  }
  for (int64_t T0 = t_begin; T0 < t_end; T0 += 2 * DEPTH) {
#pragma unroll
    for (int d = 0; d < DEPTH; ++d) {
      const int64_t Td = T0 + 2 * d;
      if (Td >= t_end) break;  // uniform
#pragma unroll
      for (int f = 0; f < PER; ++f)
        if (f * 512 + (int)threadIdx.x < FR) s_b[f * 512 + threadIdx.x] = __builtin_bit_cast(u32x4, qb[d][f]);
      __syncthreads();
      // refill the slot (fragments beyond the slice read as zero): the B part now, the A part once
      // the MFMAs below have been issued (they read the registers at issue)
#pragma unroll
      for (int f = 0; f < PER; ++f) qb[d][f] = panel_frag(f, Td + 2 * DEPTH);
      if (m_live) {
#pragma unroll
        for (int kk = 0; kk < 4; ++kk)
#pragma unroll
          for (int j = 0; j < NTW; ++j) {
            if (j >= ntiles) continue;  // uniform
            acc[j] = mma(qa[d][kk], __builtin_bit_cast(bf16x8, s_b[(j * 4 + kk) * 64 + lane]), acc[j]);
          }
      }
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) qa[d][kk] = a_frag(kk, Td + 2 * DEPTH);
      if (b_live) {
#pragma unroll
        for (int kk = 0; kk < 4; ++kk)
          accb = mma(ones, __builtin_bit_cast(bf16x8, s_b[(wave * 4 + kk) * 64 + lane]), accb);
      }
      __syncthreads();
    }
  }
  if (b_live && h == 0) {
    const int nn = 32 * wave + i;  // every row of the ones-contraction is the column sum: take row 0
    if (nn < g.N) g.bias[(int64_t)blockIdx.x * g.slice_stride + nn] = accb[0];
  }
  if (!m_live) return;
#pragma unroll
  for (int j = 0; j < NTW; ++j) {
    const int nn = 32 * j + i;
    if (j >= ntiles || nn >= g.N) continue;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int m = m0 + 8 * (r / 4) + 4 * h + r % 4;
      if (m < g.m_out && m < g.M) g.C[(int64_t)blockIdx.x * g.slice_stride + (int64_t)m * g.ldc + nn] = acc[j][r];
    }
  }
}

}  // namespace msrl
