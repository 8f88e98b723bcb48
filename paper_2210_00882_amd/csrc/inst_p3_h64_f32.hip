// One rollout-kernel instantiation (see registry.h).
#include "registry.h"
namespace msrl {
MSRL_PARTICLE_ENTRY(entry_p3_h64_f32, 3, 64, false, 1, 2)
}  // namespace msrl
