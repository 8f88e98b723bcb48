// Rollout kernels for networks with more than two hidden layers (see registry.h).
#include "registry.h"
namespace msrl {
MSRL_PARTICLE_ENTRY_PHASE(entry_p3_h64_f32_deep, 3, 64, false, 1, 2, PHASE_DEEP)
MSRL_PARTICLE_ENTRY_PHASE(entry_p3_h64_bf16_deep, 3, 64, true, 1, 2, PHASE_DEEP)
MSRL_PARTICLE_ENTRY_PHASE(entry_p3_h64_f32_act_deep, 3, 64, false, 1, 2, PHASE_ACT_DEEP)
MSRL_PARTICLE_ENTRY_PHASE(entry_p3_h64_bf16_act_deep, 3, 64, true, 1, 2, PHASE_ACT_DEEP)
}  // namespace msrl
