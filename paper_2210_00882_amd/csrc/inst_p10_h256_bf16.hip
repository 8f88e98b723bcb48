// One rollout-kernel instantiation (see registry.h).
#include "registry.h"
namespace msrl {
MSRL_PARTICLE_ENTRY(entry_p10_h256_bf16, 10, 256, true, 1, 8)
}  // namespace msrl
