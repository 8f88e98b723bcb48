// Rollout kernel with a centralised critic (see registry.h).
#include "registry.h"
namespace msrl {
MSRL_PARTICLE_ENTRY_PHASE(entry_p10_h256_bf16_central, 10, 256, true, 1, 8, PHASE_CENTRAL)
MSRL_PARTICLE_ENTRY_PHASE(entry_p10_h256_bf16_act_central, 10, 256, true, 1, 8, PHASE_ACT_CENTRAL)
}  // namespace msrl
