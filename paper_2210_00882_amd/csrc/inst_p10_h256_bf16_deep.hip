// Rollout kernel for networks with more than two hidden layers (see registry.h).
#include "registry.h"
namespace msrl {
MSRL_PARTICLE_ENTRY_PHASE(entry_p10_h256_bf16_deep, 10, 256, true, 1, 8, PHASE_DEEP)
MSRL_PARTICLE_ENTRY_PHASE(entry_p10_h256_bf16_act_deep, 10, 256, true, 1, 8, PHASE_ACT_DEEP)
}  // namespace msrl
