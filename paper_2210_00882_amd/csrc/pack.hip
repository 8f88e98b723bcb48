// Re-orders network parameters (and the linear-Gaussian dynamics matrices) into
// MFMA operand tiles; see packed.h for the layout.
#include "packed.h"

#include <hip/hip_runtime.h>

namespace msrl {

__device__ __forceinline__ int in_index(int map, bool bf16, int kt, int h, int e) {
  switch (map) {
    case IN_LINEAR16: return 16 * kt + 8 * h + e;
    case IN_PAIRS: return 8 * kt + 2 * e + h;
    default:
      return bf16 ? 32 * (kt >> 1) + 16 * (kt & 1) + 8 * (e >> 2) + 4 * h + (e & 3)
                  : 32 * (kt >> 2) + 8 * (kt & 3) + 4 * h + e;
  }
}

// physical output index -> logical output index, or -1 for padding
__device__ __forceinline__ int out_index(int map, int gauss_k, int phys, int n_out) {
  if (map == OUT_GAUSS) {
    if (phys < 8) return phys < gauss_k ? phys : -1;
    if (phys < 16) return (phys - 8) < gauss_k ? gauss_k + (phys - 8) : -1;
    return -1;
  }
  return phys < n_out ? phys : -1;
}

__device__ __forceinline__ float load_src(const void* src, int bf16, int idx) {
  if (bf16) {
    const uint32_t b = (uint32_t)((const uint16_t*)src)[idx] << 16;
    return __uint_as_float(b);
  }
  return ((const float*)src)[idx];
}

// grid: (blocks over work items, job); one thread per (tile, lane) or per bias slot.
__global__ void pack_kernel(PackJobs jobs) {
  const PackJob& j = jobs.job[blockIdx.y];
  const int tid = blockIdx.x * blockDim.x + threadIdx.x;
  if (j.is_bias) {
    if (tid >= 32 * j.nuc) return;
    const int o = out_index(j.out_map, j.gauss_k, tid, j.n_out);
    ((float*)j.dst)[tid] = o >= 0 ? load_src(j.src, j.src_bf16, o) : 0.0f;
    return;
  }
  const int n_tiles = j.nuc * j.kt;
  if (tid >= n_tiles * 64) return;
  const int tile = tid >> 6, lane = tid & 63;
  const int uc = tile / j.kt, kt = tile % j.kt;
  const int dst_slot = ((uc + kt / j.group) * j.chunk_stride + j.slot_base + kt % j.group) * 64 + lane;
  const int m = lane & 31, h = lane >> 5;
  const int o = out_index(j.out_map, j.gauss_k, 32 * uc + m, j.n_out);
  const bool bf16 = j.src_bf16 != 0;
  const int ne = bf16 ? 8 : 4;
  float v[8];
  for (int e = 0; e < ne; ++e) {
    const int i = in_index(j.in_map, bf16, kt, h, e);
    v[e] = 0.0f;
    bool weight = i < j.n_in;
    int li = i;
    if (j.in_block > 0) {
      weight = weight && i % j.in_block < j.in_block_used;
      li = (i / j.in_block) * j.in_block_stride + i % j.in_block;
    }
    if (o >= 0 && weight)
      v[e] = load_src(j.src, j.src_bf16, j.src_out_major ? o * j.n_in + li : li * j.n_out + o);
    else if (o >= 0 && j.bias && i == j.bias_index)
      v[e] = load_src(j.bias, j.src_bf16, o);
  }
  if (bf16) {
    // values are bfloat16-representable already: keep the top 16 bits
    uint32_t w[4];
    for (int p = 0; p < 4; ++p)
      w[p] = (__float_as_uint(v[2 * p]) >> 16) | (__float_as_uint(v[2 * p + 1]) & 0xFFFF0000u);
    ((uint4*)j.dst)[dst_slot] = make_uint4(w[0], w[1], w[2], w[3]);
  } else {
    ((float4*)j.dst)[dst_slot] = make_float4(v[0] * j.scale, v[1] * j.scale, v[2] * j.scale, v[3] * j.scale);
  }
}

hipError_t launch_pack(const PackJobs& jobs, hipStream_t stream) {
  if (jobs.n <= 0) return hipSuccess;
  int max_items = 0;
  for (int k = 0; k < jobs.n; ++k) {
    const PackJob& j = jobs.job[k];
    const int items = j.is_bias ? 32 * j.nuc : j.nuc * j.kt * 64;
    if (items > max_items) max_items = items;
  }
  dim3 grid((max_items + 255) / 256, jobs.n);
  hipLaunchKernelGGL(pack_kernel, grid, dim3(256), 0, stream, jobs);
  return hipGetLastError();
}

}  // namespace msrl
