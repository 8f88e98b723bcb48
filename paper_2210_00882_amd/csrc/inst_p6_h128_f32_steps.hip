// Step-granular variants of one rollout kernel: actor only, environment only (see registry.h).
#include "registry.h"
namespace msrl {
MSRL_PARTICLE_ENTRY_PHASE(entry_p6_h128_f32_act, 6, 128, false, 1, 8, PHASE_ACT)
MSRL_PARTICLE_ENTRY_PHASE(entry_p6_h128_f32_step, 6, 128, false, 1, 8, PHASE_STEP)
}  // namespace msrl
