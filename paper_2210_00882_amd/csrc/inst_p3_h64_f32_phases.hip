// Measurement variant of one rollout kernel (see registry.h).
#include "registry.h"
namespace msrl {
MSRL_PARTICLE_ENTRY_PHASE(entry_p3_h64_f32_env, 3, 64, false, 1, 2, PHASE_ENV)
}  // namespace msrl
