// Step-granular variants of one rollout kernel: actor only, environment only (see registry.h).
#include "registry.h"
namespace msrl {
MSRL_PARTICLE_ENTRY_PHASE(entry_p10_h256_bf16_act, 10, 256, true, 1, 8, PHASE_ACT)
MSRL_PARTICLE_ENTRY_PHASE(entry_p10_h256_bf16_step, 10, 256, true, 1, 8, PHASE_STEP)
}  // namespace msrl
