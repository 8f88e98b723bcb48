// Device-side building blocks shared by the HIP kernels: Philox4x32-10 streams,
// uniform / normal transforms, fast tanh, MFMA operand types.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace msrl {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// ---------------------------------------------------------------- Philox4x32-10
// Counter (env, entity, time, stream<<16 | block), key = 64-bit seed
// (Salmon et al., SC'11).  Streams: 0 action noise, 1 reset draws, 2 env noise.
struct Words4 {
  uint32_t w[4];
};

__device__ __forceinline__ Words4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                                 uint32_t k0, uint32_t k1) {
#pragma unroll
  for (int i = 0; i < 10; ++i) {
    const uint32_t hi0 = __umulhi(0xD2511F53u, c0), lo0 = 0xD2511F53u * c0;
    const uint32_t hi1 = __umulhi(0xCD9E8D57u, c2), lo1 = 0xCD9E8D57u * c2;
    const uint32_t n0 = hi1 ^ c1 ^ k0, n2 = hi0 ^ c3 ^ k1;
    c0 = n0; c1 = lo1; c2 = n2; c3 = lo0;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  Words4 r;
  r.w[0] = c0; r.w[1] = c1; r.w[2] = c2; r.w[3] = c3;
  return r;
}

__device__ __forceinline__ Words4 draw(uint32_t seed_lo, uint32_t seed_hi, uint32_t env,
                                       uint32_t entity, uint32_t time, uint32_t stream,
                                       uint32_t block) {
  return philox4x32_10(env, entity, time, (stream << 16) | block, seed_lo, seed_hi);
}

// u in [0,1) from the top 24 bits: exact in fp32.
__device__ __forceinline__ float u01(uint32_t w) { return (float)(w >> 8) * 5.9604644775390625e-08f; }

// Box-Muller pair; the radius uses a uniform in (0,1].
__device__ __forceinline__ void normal_pair(uint32_t w0, uint32_t w1, float& e0, float& e1) {
  const float u1 = (float)((w0 >> 8) + 1u) * 5.9604644775390625e-08f;
  const float u2 = (float)(w1 >> 8) * 5.9604644775390625e-08f;
  const float r = sqrtf(-2.0f * logf(u1));
  float s, c;
  sincosf(6.283185307179586f * u2, &s, &c);
  e0 = r * c;
  e1 = r * s;
}

// Four standard normals = block `block` of a stream (normals 4*block .. 4*block+3).
__device__ __forceinline__ void normals4(uint32_t seed_lo, uint32_t seed_hi, uint32_t env,
                                         uint32_t entity, uint32_t time, uint32_t stream,
                                         uint32_t block, float e[4]) {
  const Words4 w = draw(seed_lo, seed_hi, env, entity, time, stream, block);
  normal_pair(w.w[0], w.w[1], e[0], e[1]);
  normal_pair(w.w[2], w.w[3], e[2], e[3]);
}

// tanh(x) = 1 - 2 / (1 + e^(2x)) on the hardware exp2 / rcp units; absolute
// error about 2e-7, saturates cleanly to +-1 for large |x|.
__device__ __forceinline__ float fast_tanh(float x) {
  const float e = __builtin_amdgcn_exp2f(x * 2.8853900817779268f);
  return 1.0f - 2.0f * __builtin_amdgcn_rcpf(e + 1.0f);
}

// The same for an argument that already carries the factor 2 log2(e): the packed fp32 images hold their hidden
// layers' weights and biases times that factor (packed.h), so the fp32 kernels' pre-activations arrive scaled
// and the chain is one multiply shorter.
constexpr float TANH_PRESCALE = 2.8853900817779268f;
__device__ __forceinline__ float fast_tanh_prescaled(float x) {
  return 1.0f - 2.0f * __builtin_amdgcn_rcpf(__builtin_amdgcn_exp2f(x) + 1.0f);
}

// Keeps the compiler from moving LDS traffic of one wave across this point.
// A wave's own LDS operations complete in issue order, so data written by one
// lane is visible to the other lanes of the same wave afterwards.
__device__ __forceinline__ void wave_lds_sync() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

}  // namespace msrl
