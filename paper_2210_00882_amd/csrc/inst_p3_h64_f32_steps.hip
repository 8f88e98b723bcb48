// Step-granular variants of one rollout kernel: actor only, environment only (see registry.h).
#include "registry.h"
namespace msrl {
MSRL_PARTICLE_ENTRY_PHASE(entry_p3_h64_f32_act, 3, 64, false, 1, 2, PHASE_ACT)
MSRL_PARTICLE_ENTRY_PHASE(entry_p3_h64_f32_step, 3, 64, false, 1, 2, PHASE_STEP)
}  // namespace msrl
