// Table of the compiled rollout kernels.  Each instantiation lives in its own
// translation unit (inst_*.hip) so that they compile in parallel.
#pragma once
#include <vector>

#include "rollout_kernels.h"

namespace msrl {

struct KernelEntry {
  int kind;           // 0 particle, 1 lingauss
  int n;              // particle: agents per env; lingauss: state width
  int k;              // lingauss: action width; particle: 0
  int hidden;
  int bf16;
  const void* fn;     // __global__ void (*)(RolloutArgs)
  int envs_per_wave;
  int waves;          // waves per workgroup
  int phase;          // PHASE_ALL, or a measurement variant
  int row_waves;      // waves of a workgroup that own rows (PHASE_SPLIT: half of them; 0 stands for all)
};

// NB: 32-row blocks per wave; WAVES: waves per workgroup (they share the LDS weight window)
#define MSRL_PARTICLE_ENTRY_PHASE(NAME, N, H, BF16, NB, WAVES, PHASE)                       \
  KernelEntry NAME() {                                                                     \
    return KernelEntry{0, N, 0, H, BF16 ? 1 : 0,                                           \
                       (const void*)&particle_rollout_kernel<N, H, BF16, NB, WAVES, PHASE>, \
                       32 * NB / N, WAVES, PHASE};                                         \
  }
#define MSRL_PARTICLE_ENTRY(NAME, N, H, BF16, NB, WAVES) \
  MSRL_PARTICLE_ENTRY_PHASE(NAME, N, H, BF16, NB, WAVES, PHASE_ALL)

#define MSRL_LINGAUSS_ENTRY_PHASE(NAME, D, K, H, WAVES, PHASE)                                    \
  KernelEntry NAME() {                                                                            \
    return KernelEntry{1, D, K, H, 0, (const void*)&lingauss_rollout_kernel<D, K, H, WAVES, PHASE>, \
                       32, WAVES, PHASE};                                                         \
  }
#define MSRL_LINGAUSS_ENTRY(NAME, D, K, H, WAVES) MSRL_LINGAUSS_ENTRY_PHASE(NAME, D, K, H, WAVES, PHASE_ALL)

// ---- the particle env's kernel for every shape the design holds, by construction
// Agents per env N = 1 .. 10, hidden width 64 / 128 / 256, fp32 and bf16 networks; per shape the full
// rollout, the actor fragment, the env step, and the first two for networks with more than two hidden
// layers.  Waves per workgroup (they share one LDS copy of the weights): two for 64 units; eight above,
// but four where eight would not fit - fp32 networks of 256 units (their resident layer-1 tiles fill the
// LDS) and the deep fp32 kernels of 128 units (eight waves leave each 256 registers, which the deep
// kernel's state in fp32 exceeds; four waves run one per SIMD with twice that).
constexpr int particle_waves(int H, bool bf16, int phase) {
  const bool deep = phase == PHASE_DEEP || phase == PHASE_ACT_DEEP;
  return H == 64 ? 2 : (!bf16 && (H >= 256 || deep)) ? 4 : 8;
}
// fp32 networks of 256 units: the layer-1 tiles of both networks (ceil((4 N + 3) / 8) tiles of 8 inputs x
// 256 units x 4 bytes each) stay in LDS beside the two-stage window; beyond 7 agents they exceed 160 KB
constexpr bool particle_fits(int N, int H, bool bf16) { return bf16 || H < 256 || N <= 7; }

// Centralised critic: one wave per 32-unit chunk of the hidden layers, and the envs of a workgroup
// (waves x floor(32 / N)) are the at most 32 columns of the critic's tile: 64 units from 2 agents per env,
// 128 from 4, 256 from 7.  fp32 networks: 64 and 128 units with at most 8 agents per env (the joint
// observation, twice as many tiles, and the fp32 window must fit the LDS; the critic's ring of tile registers
// grows with the agents).
constexpr bool particle_central_fits(int N, int H, bool bf16) {
  return N >= 2 && (H / 32) * (32 / N) <= 32 && (bf16 || (H <= 128 && N <= 8));
}

// Two waves per row block (PHASE_SPLIT: one evaluates the policy network, the other the value network, and
// every weight tile of both stays in LDS).  Row blocks per workgroup of the narrow (which = 0) and the wide
// (which = 1) instance, 0 = not compiled: 64-unit networks two (one wave per SIMD), fp32 ones also four (two
// waves per SIMD: faster once every SIMD has a wave anyway); 128-unit bf16 networks four (88 KB of weights;
// fp32 ones would need 168 KB).
constexpr int particle_split_rows(int H, bool bf16, int which) {
  return H == 64 ? (which == 0 ? 2 : (bf16 ? 0 : 4)) : (H == 128 && bf16 && which == 0 ? 4 : 0);
}

// RWS: row blocks per workgroup of a PHASE_SPLIT instance
template <int N, int H, bool BF16, int PHASE, int RWS = 0>
KernelEntry particle_entry() {
  constexpr int RW = PHASE == PHASE_SPLIT ? RWS
                     : PHASE == PHASE_CENTRAL || PHASE == PHASE_ACT_CENTRAL ? H / 32 : particle_waves(H, BF16, PHASE);
  constexpr int W = PHASE == PHASE_SPLIT ? 2 * RW : RW;
  return KernelEntry{0, N, 0, H, BF16 ? 1 : 0, (const void*)&particle_rollout_kernel<N, H, BF16, 1, W, PHASE>,
                     32 / N, W, PHASE, RW};
}

template <int N0, int N1, int H, bool BF16>
void add_particle_family(std::vector<KernelEntry>& out) {
  if constexpr (N0 <= N1) {
    if constexpr (particle_fits(N0, H, BF16)) {
      out.push_back(particle_entry<N0, H, BF16, PHASE_ALL>());
      out.push_back(particle_entry<N0, H, BF16, PHASE_ACT>());
      out.push_back(particle_entry<N0, H, BF16, PHASE_STEP>());
      out.push_back(particle_entry<N0, H, BF16, PHASE_DEEP>());
      out.push_back(particle_entry<N0, H, BF16, PHASE_ACT_DEEP>());
      if constexpr (particle_split_rows(H, BF16, 0) != 0)
        out.push_back(particle_entry<N0, H, BF16, PHASE_SPLIT, particle_split_rows(H, BF16, 0)>());
      if constexpr (particle_split_rows(H, BF16, 1) != 0)
        out.push_back(particle_entry<N0, H, BF16, PHASE_SPLIT, particle_split_rows(H, BF16, 1)>());
    }
    if constexpr (particle_central_fits(N0, H, BF16)) {
      out.push_back(particle_entry<N0, H, BF16, PHASE_CENTRAL>());
      out.push_back(particle_entry<N0, H, BF16, PHASE_ACT_CENTRAL>());
    }
    add_particle_family<N0 + 1, N1, H, BF16>(out);
  }
}

// one translation unit per entry of this list (inst_family_*.hip): X(name, first N, last N, H, bf16)
#define MSRL_PARTICLE_FAMILIES(X)                                                   \
  X(h64_f32_a, 1, 5, 64, false)    X(h64_f32_b, 6, 10, 64, false)                   \
  X(h64_bf16_a, 1, 5, 64, true)    X(h64_bf16_b, 6, 10, 64, true)                   \
  X(h128_f32_a, 1, 5, 128, false)  X(h128_f32_b, 6, 10, 128, false)                 \
  X(h128_bf16_a, 1, 5, 128, true)  X(h128_bf16_b, 6, 10, 128, true)                 \
  X(h256_f32_a, 1, 4, 256, false)  X(h256_f32_b, 5, 7, 256, false)                  \
  X(h256_bf16_a, 1, 5, 256, true)  X(h256_bf16_b, 6, 10, 256, true)
#define MSRL_DECLARE_FAMILY(NAME, N0, N1, H, BF16) void particle_family_##NAME(std::vector<KernelEntry>& out);
MSRL_PARTICLE_FAMILIES(MSRL_DECLARE_FAMILY)
#undef MSRL_DECLARE_FAMILY
// in its translation unit: MSRL_DEFINE_FAMILY(name) with the list's numbers
#define MSRL_FAMILY_BODY(NAME, N0, N1, H, BF16) \
  void particle_family_##NAME(std::vector<KernelEntry>& out) { add_particle_family<N0, N1, H, BF16>(out); }

KernelEntry entry_l17_6_h256();
// measurement variants (phase rooflines)
KernelEntry entry_p10_h256_bf16_env();
KernelEntry entry_p10_h256_bf16_mlp();
KernelEntry entry_p10_h256_bf16_clocks();
KernelEntry entry_p3_h64_f32_env();

// step-granular variants (actor only, environment only)
KernelEntry entry_l17_6_h256_act();
KernelEntry entry_l17_6_h256_step();

// more than two hidden layers
KernelEntry entry_l17_6_h256_deep();
KernelEntry entry_l17_6_h256_act_deep();


}  // namespace msrl
