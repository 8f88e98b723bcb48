// Kernels of the learner's policy update (PPO clipped surrogate, Listing 1 of
// the paper: mappo_net_train): forward and backward passes of the policy and
// value networks over a minibatch of stored rows, as plain dense contractions
// on MFMA with the activations kept in device memory, plus the per-row loss,
// the transposes the weight gradients need, and Adam.
//
// Every contraction has the form C[m][n] = sum_k A[m][k] * B[n][k] with both operands stored
// k-contiguous, so that a lane fetches its MFMA fragment with one 16-byte load.  Three kernels:
// rowgemm_kernel for the layers (many rows, few columns; weights resident in LDS; writes the
// result row-major and, for the weight gradients, unit-major, and sums the columns for the bias
// gradient), wgrad_kernel for the weight gradients (few outputs, the rows as contraction index;
// output-stationary with LDS panels), gemm_kernel as the general fallback.  Every global access
// is bounds-checked against the extents passed in.
#pragma once
#include "dev_common.h"
#include "row_sel.h"

namespace msrl {

// ---------------------------------------------------------------- fragments
// One "k tile" is 16 k-values in bf16 mode (one 32x32x16 MFMA) and 8 in fp32
// mode (four 32x32x2 MFMAs).  Lane (i = lane % 32, h = lane / 32) holds, for
// operand row i, k-values 8h..8h+7 of the tile (bf16) or 2j+h, j = 0..3 (fp32).
template <bool BF16> struct Frag;
template <> struct Frag<true> {
  typedef bf16x8 T;
  static constexpr int KT = 16;
};
template <> struct Frag<false> {
  typedef f32x4 T;
  static constexpr int KT = 8;
};

__device__ __forceinline__ bf16x8 frag_zero(bf16x8*) {
  bf16x8 z = {0, 0, 0, 0, 0, 0, 0, 0};
  return z;
}
__device__ __forceinline__ f32x4 frag_zero(f32x4*) {
  f32x4 z = {0.0f, 0.0f, 0.0f, 0.0f};
  return z;
}

// fragment of row `p` (k contiguous, element type S) at k offset k0; the row holds at least
// k0 + KT elements (extents are padded to whole tiles by the host)
__device__ __forceinline__ bf16x8 load_frag(const __bf16* p, int k0, int h, bf16x8*) {
  return *(const bf16x8*)(p + k0 + 8 * h);
}
__device__ __forceinline__ bf16x8 load_frag(const float* p, int k0, int h, bf16x8*) {
  const f32x4 a = *(const f32x4*)(p + k0 + 8 * h), b = *(const f32x4*)(p + k0 + 8 * h + 4);
  typedef float f32x8 __attribute__((ext_vector_type(8)));
  const f32x8 v = {a[0], a[1], a[2], a[3], b[0], b[1], b[2], b[3]};
  return __builtin_convertvector(v, bf16x8);  // round to nearest even
}
__device__ __forceinline__ f32x4 load_frag(const float* p, int k0, int h, f32x4*) {
  const f32x4 a = *(const f32x4*)(p + k0), b = *(const f32x4*)(p + k0 + 4);
  f32x4 r;
  r[0] = h ? a[1] : a[0];
  r[1] = h ? a[3] : a[2];
  r[2] = h ? b[1] : b[0];
  r[3] = h ? b[3] : b[2];
  return r;
}

__device__ __forceinline__ void mma_frag(const bf16x8& a, const bf16x8& b, f32x16& c) {
  c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}
__device__ __forceinline__ void mma_frag(const f32x4& a, const f32x4& b, f32x16& c) {
#pragma unroll
  for (int j = 0; j < 4; ++j) c = __builtin_amdgcn_mfma_f32_32x32x2f32(a[j], b[j], c, 0, 0, 0);
}

__device__ __forceinline__ void store_elem(float* p, float v) { *p = v; }
__device__ __forceinline__ void store_elem(__bf16* p, float v) { *p = (__bf16)v; }
__device__ __forceinline__ float load_elem(const float* p) { return *p; }
__device__ __forceinline__ float load_elem(const __bf16* p) { return (float)*p; }
// the value a store of element type S would hold (bf16: rounded to nearest even)
__device__ __forceinline__ float as_stored(float v, const float*) { return v; }
__device__ __forceinline__ float as_stored(float v, const __bf16*) { return (float)(__bf16)v; }

// 8 consecutive elements as 16-byte pieces (the address must be 16-byte aligned: ld and column
// offsets are multiples of 8 elements)
__device__ __forceinline__ void load8(const float* p, float (&v)[8]) {
  const f32x4 a = *(const f32x4*)p, b = *(const f32x4*)(p + 4);
#pragma unroll
  for (int e = 0; e < 4; ++e) { v[e] = a[e]; v[4 + e] = b[e]; }
}
__device__ __forceinline__ void load8(const __bf16* p, float (&v)[8]) {
  const bf16x8 a = *(const bf16x8*)p;
#pragma unroll
  for (int e = 0; e < 8; ++e) v[e] = (float)a[e];
}
__device__ __forceinline__ void store8(float* p, const float (&v)[8]) {
  *(f32x4*)p = f32x4{v[0], v[1], v[2], v[3]};
  *(f32x4*)(p + 4) = f32x4{v[4], v[5], v[6], v[7]};
}
__device__ __forceinline__ void store8(__bf16* p, const float (&v)[8]) {
  typedef float f32x8 __attribute__((ext_vector_type(8)));
  const f32x8 f = {v[0], v[1], v[2], v[3], v[4], v[5], v[6], v[7]};
  *(bf16x8*)p = __builtin_convertvector(f, bf16x8);
}

// ---------------------------------------------------------------- contraction
enum : int {
  EPI_BIAS_TANH = 0,  // C = tanh(acc + bias[n])
  EPI_BIAS = 1,       // C = acc + bias[n]
  EPI_DTANH = 2,      // C = acc * (1 - Hm[m][n]^2)
  EPI_PARTIAL = 3     // C[slice] = acc: the k range is split over blockIdx.z and every slice writes its own
                      // copy of C, slice_stride floats apart; reduce_partials_kernel adds the copies up in a
                      // fixed order (no float atomics: the gradient is the same bits on every run)
};

struct GemmArgs {
  const void* A;  // [M_alloc, lda], k contiguous
  const void* B;  // [N_alloc, ldb], k contiguous
  void* C;        // [M, ldc] row-major
  const float* bias;
  const void* Hm;  // EPI_DTANH: [M, ldh], same element type as C
  int64_t M, N;    // extent of C that is written
  int64_t M_alloc, N_alloc;  // rows of A / B that may be read (rows beyond read as zero)
  int64_t K;       // contraction length, a multiple of the k tile; both operands hold it
  int64_t lda, ldb, ldc, ldh;
  int64_t k_per_slice;  // EPI_PARTIAL: k values per blockIdx.z, a multiple of the k tile
  int64_t slice_stride; // EPI_PARTIAL: floats between the copies of C of consecutive slices
};

// 4 waves per workgroup; a wave owns 32 rows of C and NT = 4 column tiles of 32.
template <bool BF16, typename SA, typename SB, typename SC, int EPI>
__global__ __launch_bounds__(256) void gemm_kernel(GemmArgs g) {
  typedef typename Frag<BF16>::T F;
  constexpr int KT = Frag<BF16>::KT, NT = 4;
  __shared__ float s_c[EPI == EPI_PARTIAL ? 1 : 4][EPI == EPI_PARTIAL ? 1 : 32 * (32 * NT + 4)];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int i = lane & 31, h = lane >> 5;
  const int64_t m0 = ((int64_t)blockIdx.x * 4 + wave) * 32;
  const int64_t n0 = (int64_t)blockIdx.y * (32 * NT);
  if (m0 >= g.M) return;
  int64_t k_begin = 0, k_end = g.K;
  if (EPI == EPI_PARTIAL) {
    k_begin = (int64_t)blockIdx.z * g.k_per_slice;
    k_end = min(g.K, k_begin + g.k_per_slice);
    if (k_begin >= k_end) return;
  }
  const SA* arow = (const SA*)g.A + (m0 + i) * g.lda;
  const bool a_ok = m0 + i < g.M_alloc;
  const SB* brow[NT];
  bool b_ok[NT];
#pragma unroll
  for (int j = 0; j < NT; ++j) {
    brow[j] = (const SB*)g.B + (n0 + 32 * j + i) * g.ldb;
    b_ok[j] = n0 + 32 * j + i < g.N_alloc;
  }
  f32x16 acc[NT];
#pragma unroll
  for (int j = 0; j < NT; ++j)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[j][r] = 0.0f;
#pragma unroll 4
  for (int64_t k = k_begin; k < k_end; k += KT) {
    const F a = a_ok ? load_frag(arow, (int)k, h, (F*)nullptr) : frag_zero((F*)nullptr);
#pragma unroll
    for (int j = 0; j < NT; ++j) {
      if (n0 + 32 * j >= g.N) continue;  // uniform: no column of this tile is written
      const F b = b_ok[j] ? load_frag(brow[j], (int)k, h, (F*)nullptr) : frag_zero((F*)nullptr);
      mma_frag(a, b, acc[j]);
    }
  }
  // accumulator: lane (n = i, h), register r <-> row 8 (r / 4) + 4 h + r % 4 of the tile
  if constexpr (EPI == EPI_PARTIAL) {
#pragma unroll
    for (int j = 0; j < NT; ++j) {
      const int64_t n = n0 + 32 * j + i;
      if (n >= g.N) continue;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int64_t m = m0 + 8 * (r / 4) + 4 * h + r % 4;
        if (m < g.M) ((float*)g.C)[(int64_t)blockIdx.z * g.slice_stride + m * g.ldc + n] = acc[j][r];
      }
    }
  } else {
    // Through the wave's LDS tile into row layout: a lane then owns 8 consecutive columns of a row, so
    // C (and Hm) move as 16-byte pieces, 16 lanes per 128-column row, instead of one element per lane.
    float* t = &s_c[wave][0];
#pragma unroll
    for (int j = 0; j < NT; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) t[(8 * (r / 4) + 4 * h + r % 4) * (32 * NT + 4) + 32 * j + i] = acc[j][r];
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    const int c8 = (lane & 15) * 8;  // first of this lane's 8 columns
    const int64_t n = n0 + c8;
#pragma unroll
    for (int it = 0; it < 8; ++it) {
      const int rl = (lane >> 4) + 4 * it;
      const int64_t m = m0 + rl;
      if (m >= g.M || n >= g.N) continue;
      float v[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) v[e] = t[rl * (32 * NT + 4) + c8 + e];
      if (n + 8 <= g.N) {
        if (EPI == EPI_BIAS_TANH || EPI == EPI_BIAS) {
#pragma unroll
          for (int e = 0; e < 8; ++e) v[e] += g.bias[n + e];
        }
        if (EPI == EPI_BIAS_TANH) {
#pragma unroll
          for (int e = 0; e < 8; ++e) v[e] = tanhf(v[e]);
        }
        if (EPI == EPI_DTANH) {
          float hv[8];
          load8((const SC*)g.Hm + m * g.ldh + n, hv);
#pragma unroll
          for (int e = 0; e < 8; ++e) v[e] *= 1.0f - hv[e] * hv[e];
        }
        store8((SC*)g.C + m * g.ldc + n, v);
      } else {  // ragged last columns: one element at a time
        for (int e = 0; e < 8 && n + e < g.N; ++e) {
          float w = v[e];
          if (EPI == EPI_BIAS_TANH) w = tanhf(w + g.bias[n + e]);
          if (EPI == EPI_BIAS) w = w + g.bias[n + e];
          if (EPI == EPI_DTANH) {
            const float hv = load_elem((const SC*)g.Hm + m * g.ldh + n + e);
            w = w * (1.0f - hv * hv);
          }
          store_elem((SC*)g.C + m * g.ldc + n + e, w);
        }
      }
    }
  }
}

// ---------------------------------------------------------------- row-parallel contraction
// C[m][n] = epilogue(sum_k A[m][k] B[n][k]) for many rows m and few columns n (a layer of a
// network: B holds its weights).  A workgroup of 8 waves keeps the fragments of 32 NT columns of B
// in LDS for its whole life and walks over 256-row tiles of A: a wave fetches the fragments of its
// 32 rows straight from global memory and reads B from LDS.  The result passes through the
// wave's LDS tile, 64 columns at a time: once row-wise (16-byte pieces of C, and of Hm for the
// tanh derivative), then, if Ct is given, column-wise for the unit-major copy Ct[n][m] that the
// weight-gradient contraction reads (rows m in [M, M_pad) of it are written as zero); the column
// pass can also add up the columns (the bias gradient).  C itself may be null when only the
// unit-major copy is wanted.  Needs K <= KMAX (256; 704 with half as many columns per workgroup, for
// the joint observation in bf16) and N a multiple of 8.
struct RowGemmArgs {
  GemmArgs g;
  void* Ct;        // [N, ldt] or null
  int64_t ldt;
  int64_t M_pad;   // rows covered (>= M, a multiple of 16); tiles beyond are not visited
  int64_t tiles;   // 256-row tiles
  float* colsum;   // with Ct: colsum[workgroup blockIdx.y][n] = that workgroup's share of sum_m C[m][n] (the bias
                   // gradient of the layer; the shares are colsum_stride floats apart), or null
  int64_t colsum_stride;
};

template <bool BF16, typename SC, int EPI, int NT, int KMAX = 256>
__global__ __launch_bounds__(512) void rowgemm_kernel(RowGemmArgs ra) {
  typedef typename Frag<BF16>::T F;
  constexpr int KT = Frag<BF16>::KT, KK_MAX = KMAX / KT, TW = 64 + 4;
  static_assert(NT % 2 == 0, "the epilogue works on pairs of 32-column tiles");
  __shared__ __attribute__((aligned(16))) u32x4 s_b[NT * KK_MAX * 64];
  __shared__ float s_c[8][32 * TW];
  const GemmArgs& g = ra.g;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int i = lane & 31, h = lane >> 5;
  // (the column group is the fast grid index: the workgroups that read the same rows of A run at the same
  // time, so only the first of them fetches those rows from HBM)
  const int64_t n0 = (int64_t)blockIdx.x * (32 * NT);
  const int KK = (int)(g.K / KT);
  for (int idx = threadIdx.x; idx < NT * KK * 64; idx += 512) {
    const int j = idx / (KK * 64), rem = idx % (KK * 64), kk = rem / 64, l = rem % 64;
    const int64_t n = n0 + 32 * j + (l & 31);
    const F f = n < g.N_alloc ? load_frag((const SC*)g.B + n * g.ldb, kk * KT, l >> 5, (F*)nullptr)
                              : frag_zero((F*)nullptr);
    s_b[idx] = __builtin_bit_cast(u32x4, f);
  }
  __syncthreads();
  float* t = &s_c[wave][0];
  float csum[NT / 2];  // column sums of this lane's column of each 64-column chunk
#pragma unroll
  for (int c = 0; c < NT / 2; ++c) csum[c] = 0.0f;
  for (int64_t tile = blockIdx.y; tile < ra.tiles; tile += gridDim.y) {
    const int64_t m0 = (tile * 8 + wave) * 32;
    if (m0 >= ra.M_pad) continue;  // wave-uniform
    const SC* arow = (const SC*)g.A + (m0 + i) * g.lda;
    const bool a_ok = m0 + i < g.M_alloc;
    f32x16 acc[NT];
#pragma unroll
    for (int j = 0; j < NT; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[j][r] = 0.0f;
#pragma unroll 4
    for (int kk = 0; kk < KK; ++kk) {
      const F a = a_ok ? load_frag(arow, kk * KT, h, (F*)nullptr) : frag_zero((F*)nullptr);
#pragma unroll
      for (int j = 0; j < NT; ++j) {
        if (n0 + 32 * j >= g.N) continue;  // uniform
        mma_frag(a, __builtin_bit_cast(F, s_b[(j * KK + kk) * 64 + lane]), acc[j]);
      }
    }
#pragma unroll
    for (int c = 0; c < NT / 2; ++c) {
      const int64_t nc = n0 + 64 * c;
      if (nc >= g.N) continue;  // uniform
      // accumulator: lane (n = i, h), register r <-> row 8 (r / 4) + 4 h + r % 4
#pragma unroll
      for (int jj = 0; jj < 2; ++jj)
#pragma unroll
        for (int r = 0; r < 16; ++r) t[(8 * (r / 4) + 4 * h + r % 4) * TW + 32 * jj + i] = acc[2 * c + jj][r];
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      {
        const int c8 = (lane & 7) * 8;
        const int64_t n = nc + c8;
#pragma unroll
        for (int it = 0; it < 4; ++it) {
          const int rl = (lane >> 3) + 8 * it;
          const int64_t m = m0 + rl;
          float v[8];
#pragma unroll
          for (int e = 0; e < 8; ++e) v[e] = t[rl * TW + c8 + e];
          const bool live = m < g.M && n + 8 <= g.N;
          if (live) {
            if (EPI == EPI_BIAS_TANH || EPI == EPI_BIAS) {
#pragma unroll
              for (int e = 0; e < 8; ++e) v[e] += g.bias[n + e];
            }
            if (EPI == EPI_BIAS_TANH) {
#pragma unroll
              for (int e = 0; e < 8; ++e) v[e] = tanhf(v[e]);
            }
            if (EPI == EPI_DTANH) {
              float hv[8];
              load8((const SC*)g.Hm + m * g.ldh + n, hv);
#pragma unroll
              for (int e = 0; e < 8; ++e) v[e] *= 1.0f - hv[e] * hv[e];
            }
            if (g.C) store8((SC*)g.C + m * g.ldc + n, v);
          } else {
#pragma unroll
            for (int e = 0; e < 8; ++e) v[e] = 0.0f;
          }
          // final values for the column pass, as the stores hold them: the column sums (a bias gradient)
          // add up the same rounded values the weight-gradient contraction reads
#pragma unroll
          for (int e = 0; e < 8; ++e) t[rl * TW + c8 + e] = as_stored(v[e], (const SC*)nullptr);
        }
      }
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      if (ra.Ct) {
        const int64_t n = nc + lane;  // one column per lane
        if (n < g.N) {
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            if (m0 + 8 * q >= ra.M_pad) continue;
            float v[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) v[e] = t[(8 * q + e) * TW + lane];
            store8((SC*)ra.Ct + n * ra.ldt + m0 + 8 * q, v);
#pragma unroll
            for (int e = 0; e < 8; ++e) csum[c] += v[e];
          }
        }
      }
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
    }
  }
  if (ra.Ct && ra.colsum) {
    // the eight waves' sums are added in wave order, then one plain store per column: no float atomics
    float* red = &s_c[0][0];
    __syncthreads();  // every wave is past its last tile
#pragma unroll
    for (int c = 0; c < NT / 2; ++c) red[(wave * (NT / 2) + c) * 64 + lane] = csum[c];
    __syncthreads();
    if (wave == 0) {
#pragma unroll
      for (int c = 0; c < NT / 2; ++c) {
        const int64_t n = n0 + 64 * c + lane;
        float s = 0.0f;
#pragma unroll
        for (int w = 0; w < 8; ++w) s += red[(w * (NT / 2) + c) * 64 + lane];
        if (n < g.N) ra.colsum[(int64_t)blockIdx.y * ra.colsum_stride + n] = s;
      }
    }
  }
}

// ---------------------------------------------------------------- weight-gradient contraction
// C[slice][m][n] = sum_{k in slice} A[m][k] B[n][k] with few m, n (<= 256 each: the units of two layers) and a
// very long k (the rows of the minibatch).  Output-stationary: workgroup z takes the k range
// [z k_per_slice, (z+1) k_per_slice), wave w of its 8 waves the 32 rows m = 32 w .. 32 w + 31 of C
// and all columns (up to 128 accumulator registers); the B fragments of a chunk of 4 k tiles are
// shared through LDS (loaded once per workgroup, by all threads, one chunk ahead in registers), the
// A fragments are the wave's own and come straight from global memory.  Every slice writes its own
// copy of C (slice_stride floats apart); reduce_partials_kernel adds the copies in slice order.
template <bool BF16, typename S>
__global__ __launch_bounds__(512) void wgrad_kernel(GemmArgs g) {
  typedef typename Frag<BF16>::T F;
  constexpr int KT = Frag<BF16>::KT, KC = 4 * KT, NTW = 8, PER = NTW * 4 * 64 / 512;  // fragments per thread
  __shared__ __attribute__((aligned(16))) u32x4 s_b[NTW * 4 * 64];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int i = lane & 31, h = lane >> 5;
  const int64_t k_begin = (int64_t)blockIdx.x * g.k_per_slice, k_end = min(g.K, k_begin + g.k_per_slice);
  if (k_begin >= k_end) return;  // whole workgroup
  const int ntiles = (int)((g.N + 31) / 32);  // column tiles in use (<= NTW)
  const int64_t m0 = 32 * wave;
  const bool m_live = m0 < g.M;
  const S* arow = (const S*)g.A + (m0 + i) * g.lda;
  const bool a_ok = m_live && m0 + i < g.M_alloc;
  // fragment `f` of this thread in a chunk: slot = f * 512 + tid -> (column tile j, k tile kk, lane l)
  auto panel_frag = [&](int f, int64_t k0) -> F {
    const int slot = f * 512 + threadIdx.x;
    const int j = slot / 256, kk = (slot / 64) % 4, l = slot % 64;
    const int64_t n = 32 * j + (l & 31), k = k0 + kk * KT;
    if (j < ntiles && n < g.N_alloc && k < k_end)
      return load_frag((const S*)g.B + n * g.ldb, (int)k, l >> 5, (F*)nullptr);
    return frag_zero((F*)nullptr);
  };
  f32x16 acc[NTW];
#pragma unroll
  for (int j = 0; j < NTW; ++j)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[j][r] = 0.0f;
  F next[PER];
#pragma unroll
  for (int f = 0; f < PER; ++f) next[f] = panel_frag(f, k_begin);
  for (int64_t k0 = k_begin; k0 < k_end; k0 += KC) {
#pragma unroll
    for (int f = 0; f < PER; ++f) s_b[f * 512 + threadIdx.x] = __builtin_bit_cast(u32x4, next[f]);
    __syncthreads();
    if (k0 + KC < k_end) {
#pragma unroll
      for (int f = 0; f < PER; ++f) next[f] = panel_frag(f, k0 + KC);
    }
    F a[4];
#pragma unroll
    for (int kk = 0; kk < 4; ++kk)
      a[kk] = (a_ok && k0 + kk * KT < k_end) ? load_frag(arow, (int)(k0 + kk * KT), h, (F*)nullptr)
                                            : frag_zero((F*)nullptr);
    if (m_live) {
#pragma unroll
      for (int kk = 0; kk < 4; ++kk)
#pragma unroll
        for (int j = 0; j < NTW; ++j) {
          if (j >= ntiles) continue;  // uniform
          mma_frag(a[kk], __builtin_bit_cast(F, s_b[(j * 4 + kk) * 64 + lane]), acc[j]);
        }
    }
    __syncthreads();
  }
  if (!m_live) return;
#pragma unroll
  for (int j = 0; j < NTW; ++j) {
    const int64_t n = 32 * j + i;
    if (j >= ntiles || n >= g.N) continue;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int64_t m = m0 + 8 * (r / 4) + 4 * h + r % 4;
      if (m < g.M) ((float*)g.C)[(int64_t)blockIdx.x * g.slice_stride + m * g.ldc + n] = acc[j][r];
    }
  }
}

// ---------------------------------------------------------------- transposes, conversions
// dst[c][r] = src[r][c] for r < rows, c < cols; dst rows are ldd long and columns in
// [rows, rows_pad) are written as zero (the contraction over rows reads whole k tiles).
template <typename S, typename D>
__global__ __launch_bounds__(256) void transpose_kernel(const S* src, int64_t rows, int64_t cols, int64_t lds_,
                                                        D* dst, int64_t ldd, int64_t rows_pad, int64_t cols_out) {
  __shared__ float tile[32][33];
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;  // 32 x 8
  const int64_t r0 = (int64_t)blockIdx.x * 32, c0 = (int64_t)blockIdx.y * 32;
#pragma unroll
  for (int s = 0; s < 4; ++s) {
    const int64_t r = r0 + ty + 8 * s, c = c0 + tx;
    tile[ty + 8 * s][tx] = (r < rows && c < cols) ? load_elem(src + r * lds_ + c) : 0.0f;
  }
  __syncthreads();
#pragma unroll
  for (int s = 0; s < 4; ++s) {
    const int64_t c = c0 + ty + 8 * s, r = r0 + tx;
    if (c < cols_out && r < rows_pad) store_elem(dst + c * ldd + r, tile[tx][ty + 8 * s]);
  }
}

// dst[r][c] = src[r][c] converted, zero for c in [cols, ldd) and for r in [rows, rows_pad)
template <typename S, typename D>
__global__ void convert_pad_kernel(const S* src, int64_t rows, int64_t cols, int64_t lds_, D* dst, int64_t ldd,
                                   int64_t rows_pad) {
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= rows_pad * ldd) return;
  const int64_t r = idx / ldd, c = idx % ldd;
  store_elem(dst + idx, (r < rows && c < cols) ? load_elem(src + r * lds_ + c) : 0.0f);
}

// Both copies of the observations in one pass over the source: dst[r][c] = src[sel.at(r)][c] converted (zero for
// c in [cols, ldd) and for r in [rows, rows_pad)) and dstT[c][r] = the same values unit-major (rows of ldt
// elements; columns in [rows, rows_pad) zero), 64 x 64 tiles through LDS, a lane stores two neighbouring
// elements at once.  ldd, ldt and rows_pad are even.  Grid: (ceil(rows_pad / 64), ceil(ldd / 64)).
__device__ __forceinline__ void store_pair(float* p, float a, float b) { *(float2*)p = make_float2(a, b); }
__device__ __forceinline__ void store_pair(__bf16* p, float a, float b) {
  typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
  bf16x2 v;
  v[0] = (__bf16)a;
  v[1] = (__bf16)b;
  *(bf16x2*)p = v;
}
template <typename D>
__global__ __launch_bounds__(256) void gather_pad_transpose_kernel(const float* src, RowSel sel, int64_t rows,
                                                                    int64_t cols, int64_t lds_, D* dst, int64_t ldd,
                                                                    D* dstT, int64_t ldt, int64_t rows_pad) {
  __shared__ float tile[64][65];
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;  // 32 pairs x 8
  const int64_t r0 = (int64_t)blockIdx.x * 64, c0 = (int64_t)blockIdx.y * 64;
#pragma unroll
  for (int s = 0; s < 8; ++s) {
    const int64_t r = r0 + ty + 8 * s, c = c0 + 2 * tx;
    float v0 = 0.0f, v1 = 0.0f;
    if (r < rows) {
      const float* row = src + sel.at(r) * lds_;
      if (c < cols) v0 = row[c];
      if (c + 1 < cols) v1 = row[c + 1];
    }
    tile[ty + 8 * s][2 * tx] = v0;
    tile[ty + 8 * s][2 * tx + 1] = v1;
    if (r < rows_pad && c < ldd) store_pair(dst + r * ldd + c, v0, v1);
  }
  __syncthreads();
#pragma unroll
  for (int s = 0; s < 8; ++s) {
    const int64_t c = c0 + ty + 8 * s, r = r0 + 2 * tx;
    if (c < ldd && r < rows_pad) store_pair(dstT + c * ldt + r, tile[2 * tx][ty + 8 * s], tile[2 * tx + 1][ty + 8 * s]);
  }
}

__global__ void fill_kernel(float* p, int64_t n, float v) {
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx < n) p[idx] = v;
}

// out[slice][u] = sum_{r in slice} src[u][r], r < rows (src unit-major).  blockIdx.x = unit, blockIdx.y =
// slice of `per_slice` rows, whose sums lie slice_stride floats apart.
template <typename S>
__global__ __launch_bounds__(256) void rowsum_kernel(const S* src, int64_t units, int64_t rows, int64_t lds_,
                                                     int64_t per_slice, float* out, int64_t slice_stride) {
  __shared__ float part[4];
  const int64_t u = blockIdx.x;
  const int64_t r_begin = (int64_t)blockIdx.y * per_slice, r_end = min(rows, r_begin + per_slice);
  float s = 0.0f;
  if (u < units)
    for (int64_t r = r_begin + threadIdx.x; r < r_end; r += 256) s += load_elem(src + u * lds_ + r);
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o);
  if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = s;
  __syncthreads();
  if (threadIdx.x == 0 && u < units)
    out[(int64_t)blockIdx.y * slice_stride + u] = part[0] + part[1] + part[2] + part[3];
}

// ---------------------------------------------------------------- Adam
// One step on element idx (c1 = 1 - beta1^k, c2 = 1 - beta2^k for step k).  The kernel below and the
// reduction of the slices' gradients (which can apply the step to what it has just summed) share it.
struct AdamArgs {
  float *p, *m, *v;  // p null: no step
  float lr, b1, b2, eps, c1, c2;
};
__device__ __forceinline__ void adam_update(const AdamArgs& a, int64_t idx, float gi) {
  const float mi = a.b1 * a.m[idx] + (1.0f - a.b1) * gi;
  const float vi = a.b2 * a.v[idx] + (1.0f - a.b2) * gi * gi;
  a.m[idx] = mi;
  a.v[idx] = vi;
  a.p[idx] -= a.lr * (mi / a.c1) / (sqrtf(vi / a.c2) + a.eps);
}
__global__ void adam_kernel(AdamArgs a, const float* g, int64_t n) {
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx < n) adam_update(a, idx, g[idx]);
}

// stats[q] = sum of the bins of statistic q (the first wave of a workgroup)
constexpr int STAT_BINS = 64;
__device__ __forceinline__ void stats_reduce(float* stats) {
  if (threadIdx.x >= 64) return;
  for (int q = 0; q < 5; ++q) {
    float s = stats[8 + q * STAT_BINS + threadIdx.x];
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o);
    if (threadIdx.x == 0) stats[q] = s;
  }
}

// ---------------------------------------------------------------- sum of the slices' gradients
// grad[j.offset + i] = sum_{s < j.slices} part[s * slice_stride + j.offset + i] for every job j (one per
// parameter tensor: the kernels above split a tensor's contraction over a number of slices of its own).
// A workgroup takes REDUCE_ELEMS consecutive elements of a job, one per lane; wave w of its four adds the
// slices [w n / 4, (w + 1) n / 4) in ascending order (four chains, so that several loads are in flight),
// and the waves' sums are joined in wave order.  The order of the additions is fixed, so a gradient is the
// same bits every time.  With `adam.p` set the Adam step of each element follows at once; with `stats` set
// one more workgroup (the last) adds up the bins of the loss statistics.
constexpr int REDUCE_MAX_JOBS = 40, REDUCE_ELEMS = 64;
struct ReduceJobs {
  int32_t offset[REDUCE_MAX_JOBS];  // first float of the tensor in the parameter vector
  int32_t count[REDUCE_MAX_JOBS];
  int32_t slices[REDUCE_MAX_JOBS];
  int32_t first_block[REDUCE_MAX_JOBS + 1];  // prefix sums of ceil(count / REDUCE_ELEMS): block -> job
  int32_t jobs;
};
__global__ __launch_bounds__(256) void reduce_partials_kernel(const float* part, int64_t slice_stride, ReduceJobs j,
                                                              float* grad, AdamArgs adam, float* stats) {
  __shared__ float s_sum[3][REDUCE_ELEMS];
  if ((int)blockIdx.x >= j.first_block[j.jobs]) {
    if (stats) stats_reduce(stats);
    return;
  }
  int q = 0;
  while (q + 1 < j.jobs && (int)blockIdx.x >= j.first_block[q + 1]) ++q;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int i = ((int)blockIdx.x - j.first_block[q]) * REDUCE_ELEMS + lane;
  const bool live = i < j.count[q];
  const int n = j.slices[q];
  const int s_begin = wave * n / 4, s_end = (wave + 1) * n / 4;
  float s0 = 0.0f, s1 = 0.0f, s2 = 0.0f, s3 = 0.0f;
  if (live) {
    const float* p = part + j.offset[q] + i;
    int s = s_begin;
    for (; s + 4 <= s_end; s += 4) {
      s0 += p[(int64_t)(s + 0) * slice_stride];
      s1 += p[(int64_t)(s + 1) * slice_stride];
      s2 += p[(int64_t)(s + 2) * slice_stride];
      s3 += p[(int64_t)(s + 3) * slice_stride];
    }
    for (; s < s_end; ++s) s0 += p[(int64_t)s * slice_stride];
  }
  const float mine = (s0 + s1) + (s2 + s3);
  if (wave > 0) s_sum[wave - 1][lane] = mine;
  __syncthreads();
  if (wave != 0 || !live) return;
  const float gi = ((mine + s_sum[0][lane]) + s_sum[1][lane]) + s_sum[2][lane];
  grad[j.offset[q] + i] = gi;
  if (adam.p) adam_update(adam, j.offset[q] + i, gi);
}

// ---------------------------------------------------------------- per-row loss
struct LossArgs {
  const float* y;       // [R, 32] policy outputs (columns >= out_dim unused)
  const float* v;       // [R, 32] value output in column 0
  const void* actions;  // int32 [R] or float [R, K]
  const float* logp_old;
  const float* adv;
  const float* ret;
  void* dy;             // [R_pad, 32] dL/dy of the policy net, compute type; pad rows and columns zero
  void* dv;             // [R_pad, 32] dL/dv in column 0
  void* dyt;            // [32, ldt] unit-major copies of the two, columns [R, R_pad) zero
  void* dvt;
  int64_t ldt;
  float* stats;         // [8 + 5 * STAT_BINS]: bins at 8 + q * STAT_BINS += sum of statistic q: policy term,
                        // value term, entropy, clipped rows, logp_old - logp
  int64_t R, R_pad;
  int out_dim, dist;
  float clip, vf_coef, ent_coef, inv_R;
  // value network on groups of G consecutive rows (centralised critic; G = 1: on the row itself): v and dv
  // have Rv = R / G rows, the target of group g is ret[g G], the value term is a mean over the groups
  int G;
  int64_t Rv, Rv_pad;
  float inv_Rv;
  int policy, value;  // which of the two parts this launch computes (the other one's buffers are not touched)
  RowSel sel;         // where row n of this call lies in actions, logp_old, adv, ret
};

// One row per lane.  Every loop runs over the 32 padded columns with a predicate, so that the
// per-row arrays stay in registers.
template <typename SC>
__global__ __launch_bounds__(256) void loss_kernel(LossArgs a) {
  const int64_t n = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  float s_pi = 0.0f, s_v = 0.0f, s_h = 0.0f, s_c = 0.0f, s_kl = 0.0f;
  if (n < a.R_pad) {
    float dy[32];
#pragma unroll
    for (int k = 0; k < 32; ++k) dy[k] = 0.0f;
    float dv = 0.0f;
    if (n < a.R && a.policy) {
      const int O = a.out_dim;
      const int64_t pn = a.sel.at(n);
      float y[32];
#pragma unroll
      for (int k = 0; k < 32; k += 4) {
        const f32x4 t = *(const f32x4*)(a.y + n * 32 + k);
        y[k] = t[0]; y[k + 1] = t[1]; y[k + 2] = t[2]; y[k + 3] = t[3];
      }
      float logp = 0.0f, ent = 0.0f;
      float dlp[32];  // d logp / dy
      float dH[32];   // d entropy / dy
#pragma unroll
      for (int k = 0; k < 32; ++k) dlp[k] = dH[k] = 0.0f;
      if (a.dist == 0) {
        float mx = y[0];
#pragma unroll
        for (int k = 1; k < 32; ++k) mx = k < O ? fmaxf(mx, y[k]) : mx;
        float z = 0.0f;
#pragma unroll
        for (int k = 0; k < 32; ++k) z += k < O ? expf(y[k] - mx) : 0.0f;
        const float lse = mx + logf(z);
        const int act = ((const int32_t*)a.actions)[pn];
#pragma unroll
        for (int k = 0; k < 32; ++k) {
          const float lp = y[k] - lse;
          ent -= k < O ? expf(lp) * lp : 0.0f;
        }
#pragma unroll
        for (int k = 0; k < 32; ++k) {
          const float lp = y[k] - lse, pk = expf(lp);
          if (k == act) logp = lp;
          dlp[k] = k < O ? (k == act ? 1.0f : 0.0f) - pk : 0.0f;
          dH[k] = k < O ? -pk * (lp + ent) : 0.0f;
        }
      } else {
        const int K = O / 2;  // <= 16: mean d in column d, log-std in column K + d
#pragma unroll
        for (int d = 0; d < 16; ++d) {
          if (d < K) {
            float ls = 0.0f;
#pragma unroll
            for (int k = 0; k < 32; ++k) ls = k == K + d ? y[k] : ls;
            const float mu = y[d], sg = expf(ls);
            const float e = (((const float*)a.actions)[pn * K + d] - mu) / sg;
            logp += -0.5f * e * e - ls - 0.9189385332046727f;
            ent += ls + 1.4189385332046727f;
            dlp[d] = e / sg;
#pragma unroll
            for (int k = 0; k < 32; ++k) {
              dlp[k] = k == K + d ? e * e - 1.0f : dlp[k];
              dH[k] = k == K + d ? 1.0f : dH[k];
            }
          }
        }
      }
      const float rho = expf(logp - a.logp_old[pn]), A = a.adv[pn];
      const float rc = fminf(fmaxf(rho, 1.0f - a.clip), 1.0f + a.clip);
      const float un = rho * A, cl = rc * A;
      const bool clipped = cl < un;
      const float gl = clipped ? 0.0f : -A * rho;
#pragma unroll
      for (int k = 0; k < 32; ++k) dy[k] = (gl * dlp[k] - a.ent_coef * dH[k]) * a.inv_R;
      s_pi = -(clipped ? cl : un);
      s_h = ent;
      s_c = clipped ? 1.0f : 0.0f;
      s_kl = a.logp_old[pn] - logp;
    }
    if (n < a.Rv && a.value) {  // thread n also takes group n of the value network
      const float err = a.v[n * 32] - a.ret[a.sel.at(n * a.G)];
      dv = a.vf_coef * 2.0f * err * a.inv_Rv;
      s_v = err * err;
    }
    SC* pdy = (SC*)a.dy + n * 32;
    SC* pdv = (SC*)a.dv + n * 32;
#pragma unroll
    for (int k = 0; k < 32; k += 8) {
      const float v8[8] = {dy[k], dy[k + 1], dy[k + 2], dy[k + 3], dy[k + 4], dy[k + 5], dy[k + 6], dy[k + 7]};
      const float w8[8] = {k == 0 ? dv : 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f};
      if (a.policy) store8(pdy + k, v8);
      if (n < a.Rv_pad && a.value) store8(pdv + k, w8);
    }
#pragma unroll
    for (int k = 0; k < 32; ++k) {  // consecutive lanes write consecutive rows of a unit
      if (a.policy) store_elem((SC*)a.dyt + k * a.ldt + n, dy[k]);
      if (n < a.Rv_pad && a.value) store_elem((SC*)a.dvt + k * a.ldt + n, k == 0 ? dv : 0.0f);
    }
  }
  // sums of the workgroup -> one atomic per statistic, spread over STAT_BINS bins per statistic
  // (thousands of atomics on one address would serialise); stats_reduce_kernel adds the bins up
  __shared__ float part[4][5];
  float s[5] = {s_pi, s_v, s_h, s_c, s_kl};
#pragma unroll
  for (int q = 0; q < 5; ++q) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) s[q] += __shfl_xor(s[q], o);
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6][q] = s[q];
  }
  __syncthreads();
  if (threadIdx.x < 5)
    atomicAdd(a.stats + 8 + threadIdx.x * STAT_BINS + blockIdx.x % STAT_BINS,
              part[0][threadIdx.x] + part[1][threadIdx.x] + part[2][threadIdx.x] + part[3][threadIdx.x]);
}

__global__ __launch_bounds__(64) void stats_reduce_kernel(float* stats) { stats_reduce(stats); }

// out[0] += scale * sum of x[sel.at(r)], r < rows (one float atomic per workgroup; out cleared by the caller)
__global__ __launch_bounds__(256) void rows_sum_kernel(const float* x, RowSel sel, int64_t rows, float scale, float* out) {
  __shared__ float part[4];
  float s = 0.0f;
  for (int64_t r = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; r < rows; r += (int64_t)gridDim.x * blockDim.x)
    s += x[sel.at(r)];
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o);
  if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = s;
  __syncthreads();
  if (threadIdx.x == 0) atomicAdd(out, scale * (part[0] + part[1] + part[2] + part[3]));
}

}  // namespace msrl
