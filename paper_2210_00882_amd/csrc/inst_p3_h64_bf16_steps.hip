// Step-granular variants of one rollout kernel: actor only, environment only (see registry.h).
#include "registry.h"
namespace msrl {
MSRL_PARTICLE_ENTRY_PHASE(entry_p3_h64_bf16_act, 3, 64, true, 1, 2, PHASE_ACT)
MSRL_PARTICLE_ENTRY_PHASE(entry_p3_h64_bf16_step, 3, 64, true, 1, 2, PHASE_STEP)
}  // namespace msrl
