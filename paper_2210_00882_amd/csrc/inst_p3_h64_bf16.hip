// One rollout-kernel instantiation (see registry.h).
#include "registry.h"
namespace msrl {
MSRL_PARTICLE_ENTRY(entry_p3_h64_bf16, 3, 64, true, 1, 2)
}  // namespace msrl
