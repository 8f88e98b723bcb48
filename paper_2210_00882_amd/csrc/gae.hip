// GAE advantage / return pass: a reverse-time scan, sequential in t and
// parallel over the M trajectory columns.  HBM-bound: 9 bytes read and 8 bytes
// written per (t, column).  Each lane owns VEC adjacent columns, so every load
// and store of a wave is one contiguous run; the loads of UNROLL time steps are
// issued as one batch, and the batch after it is already in flight while the
// dependent recurrence consumes this one, which keeps enough bytes in flight
// without any cross-lane communication.
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace msrl {

template <int VEC> struct VecT;
template <> struct VecT<1> { typedef float F; typedef uint8_t B; };
template <> struct VecT<4> { typedef float4 F; typedef uchar4 B; };

__device__ __forceinline__ float comp(const float& v, int) { return v; }
__device__ __forceinline__ float comp(const float4& v, int i) { return (&v.x)[i]; }
__device__ __forceinline__ float compb(const uint8_t& v, int) { return (float)v; }
__device__ __forceinline__ float compb(const uchar4& v, int i) { return (float)(&v.x)[i]; }
__device__ __forceinline__ float& comp_ref(float& v, int) { return v; }
__device__ __forceinline__ float& comp_ref(float4& v, int i) { return (&v.x)[i]; }

template <int VEC, int UNROLL>
__global__ __launch_bounds__(256) void gae_kernel(const float* __restrict__ rewards,
                                                  const float* __restrict__ values,
                                                  const uint8_t* __restrict__ dones, int T,
                                                  int64_t M, float gamma, float gl,
                                                  float* __restrict__ adv,
                                                  float* __restrict__ ret) {
  typedef typename VecT<VEC>::F F;
  typedef typename VecT<VEC>::B B;
  const int64_t col = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) * VEC;
  if (col >= M) return;
  const F* r = (const F*)(rewards + col);
  const F* v = (const F*)(values + col);
  const B* d = (const B*)(dones + col);
  F* a = (F*)(adv + col);
  F* q = (F*)(ret + col);
  const int64_t stride = M / VEC;  // rows are M elements apart

  float next_adv[VEC];
#pragma unroll
  for (int i = 0; i < VEC; ++i) next_adv[i] = 0.0f;
  F v_next = v[(int64_t)T * stride];

  // UNROLL time steps per batch; the loads of the next batch are in flight while this one runs
  auto load = [&](int tt, F (&rr)[UNROLL], F (&vv)[UNROLL], B (&dd)[UNROLL]) {
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
      const int64_t o = (int64_t)(tt - u) * stride;
      rr[u] = r[o];
      vv[u] = v[o];
      dd[u] = d[o];
    }
  };
  auto scan = [&](int tt, const F (&rr)[UNROLL], const F (&vv)[UNROLL], const B (&dd)[UNROLL]) {
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
      F oa, oq;
#pragma unroll
      for (int i = 0; i < VEC; ++i) {
        const float nd = 1.0f - compb(dd[u], i);
        const float vt = comp(vv[u], i);
        const float delta = comp(rr[u], i) + gamma * nd * comp(v_next, i) - vt;
        next_adv[i] = delta + gl * nd * next_adv[i];
        comp_ref(oa, i) = next_adv[i];
        comp_ref(oq, i) = next_adv[i] + vt;
      }
      const int64_t o = (int64_t)(tt - u) * stride;
      a[o] = oa;
      q[o] = oq;
      v_next = vv[u];
    }
  };
  int t = T - 1;
  if (t >= UNROLL - 1) {
    F ra[UNROLL], va[UNROLL], rb[UNROLL], vb[UNROLL];
    B da[UNROLL], db[UNROLL];
    load(t, ra, va, da);
    while (true) {
      bool more = t - UNROLL >= UNROLL - 1;  // a whole batch is left below this one
      if (more) load(t - UNROLL, rb, vb, db);
      scan(t, ra, va, da);
      t -= UNROLL;
      if (!more) break;
      more = t - UNROLL >= UNROLL - 1;
      if (more) load(t - UNROLL, ra, va, da);
      scan(t, rb, vb, db);
      t -= UNROLL;
      if (!more) break;
    }
  }
  for (; t >= 0; --t) {
    const int64_t o = (int64_t)t * stride;
    const F rr = r[o], vv = v[o];
    const B dd = d[o];
    F oa, oq;
#pragma unroll
    for (int i = 0; i < VEC; ++i) {
      const float nd = 1.0f - compb(dd, i);
      const float vt = comp(vv, i);
      const float delta = comp(rr, i) + gamma * nd * comp(v_next, i) - vt;
      next_adv[i] = delta + gl * nd * next_adv[i];
      comp_ref(oa, i) = next_adv[i];
      comp_ref(oq, i) = next_adv[i] + vt;
    }
    a[o] = oa;
    q[o] = oq;
    v_next = vv;
  }
}

hipError_t launch_gae(const float* rewards, const float* values, const uint8_t* dones, int T,
                      int64_t M, float gamma, float lambda, float* adv, float* ret,
                      hipStream_t stream) {
  if (T <= 0 || M <= 0) return hipSuccess;
  const float gl = gamma * lambda;
  const uintptr_t align = (uintptr_t)rewards | (uintptr_t)values | (uintptr_t)adv | (uintptr_t)ret;
  const bool vec4 = (M % 4 == 0) && (align % 16 == 0) && ((uintptr_t)dones % 4 == 0) &&
                    (M / 4 >= 64 * 1024);
  if (vec4) {
    const int64_t threads = M / 4;
    hipLaunchKernelGGL((gae_kernel<4, 8>), dim3((unsigned)((threads + 255) / 256)), dim3(256), 0,
                       stream, rewards, values, dones, T, M, gamma, gl, adv, ret);
  } else {
    hipLaunchKernelGGL((gae_kernel<1, 8>), dim3((unsigned)((M + 255) / 256)), dim3(256), 0, stream,
                       rewards, values, dones, T, M, gamma, gl, adv, ret);
  }
  return hipGetLastError();
}

}  // namespace msrl
