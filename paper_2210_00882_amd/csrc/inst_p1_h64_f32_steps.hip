// Step-granular variants of one rollout kernel: actor only, environment only (see registry.h).
#include "registry.h"
namespace msrl {
MSRL_PARTICLE_ENTRY_PHASE(entry_p1_h64_f32_act, 1, 64, false, 1, 2, PHASE_ACT)
MSRL_PARTICLE_ENTRY_PHASE(entry_p1_h64_f32_step, 1, 64, false, 1, 2, PHASE_STEP)
}  // namespace msrl
