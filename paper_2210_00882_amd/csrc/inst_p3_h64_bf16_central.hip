// Rollout kernel with a centralised critic (see registry.h).
#include "registry.h"
namespace msrl {
MSRL_PARTICLE_ENTRY_PHASE(entry_p3_h64_bf16_central, 3, 64, true, 1, 2, PHASE_CENTRAL)
MSRL_PARTICLE_ENTRY_PHASE(entry_p3_h64_bf16_act_central, 3, 64, true, 1, 2, PHASE_ACT_CENTRAL)
}  // namespace msrl
