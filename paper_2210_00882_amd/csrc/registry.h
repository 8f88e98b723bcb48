// Table of the compiled rollout kernels.  Each instantiation lives in its own
// translation unit (inst_*.hip) so that they compile in parallel.
#pragma once
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

KernelEntry entry_p1_h64_f32();
KernelEntry entry_p2_h64_f32();
KernelEntry entry_p3_h64_f32();
KernelEntry entry_p3_h64_bf16();
KernelEntry entry_p6_h128_f32();
KernelEntry entry_p10_h256_bf16();
KernelEntry entry_l17_6_h256();
// measurement variants (phase rooflines)
KernelEntry entry_p10_h256_bf16_env();
KernelEntry entry_p10_h256_bf16_mlp();
KernelEntry entry_p10_h256_bf16_clocks();
KernelEntry entry_p3_h64_f32_env();

// step-granular variants (actor only, environment only)
KernelEntry entry_l17_6_h256_act();
KernelEntry entry_l17_6_h256_step();
KernelEntry entry_p1_h64_f32_act();
KernelEntry entry_p1_h64_f32_step();
KernelEntry entry_p2_h64_f32_act();
KernelEntry entry_p2_h64_f32_step();
KernelEntry entry_p3_h64_f32_act();
KernelEntry entry_p3_h64_f32_step();
KernelEntry entry_p3_h64_bf16_act();
KernelEntry entry_p3_h64_bf16_step();
KernelEntry entry_p6_h128_f32_act();
KernelEntry entry_p6_h128_f32_step();
KernelEntry entry_p10_h256_bf16_act();
KernelEntry entry_p10_h256_bf16_step();

// more than two hidden layers
KernelEntry entry_p3_h64_f32_deep();
KernelEntry entry_p3_h64_bf16_deep();
KernelEntry entry_p10_h256_bf16_deep();
KernelEntry entry_l17_6_h256_deep();

// centralised critic (value network on the joint observation of an env)
KernelEntry entry_p3_h64_bf16_central();
KernelEntry entry_p10_h256_bf16_central();

// the actor fragment for those
KernelEntry entry_p3_h64_f32_act_deep();
KernelEntry entry_p3_h64_bf16_act_deep();
KernelEntry entry_p10_h256_bf16_act_deep();
KernelEntry entry_l17_6_h256_act_deep();
KernelEntry entry_p3_h64_bf16_act_central();
KernelEntry entry_p10_h256_bf16_act_central();

}  // namespace msrl
