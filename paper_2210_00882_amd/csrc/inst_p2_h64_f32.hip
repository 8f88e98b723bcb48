// One rollout-kernel instantiation (see registry.h).
#include "registry.h"
namespace msrl {
MSRL_PARTICLE_ENTRY(entry_p2_h64_f32, 2, 64, false, 1, 2)
}  // namespace msrl
