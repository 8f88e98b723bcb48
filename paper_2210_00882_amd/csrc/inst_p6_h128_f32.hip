// One rollout-kernel instantiation (see registry.h).
#include "registry.h"
namespace msrl {
MSRL_PARTICLE_ENTRY(entry_p6_h128_f32, 6, 128, false, 1, 8)
}  // namespace msrl
