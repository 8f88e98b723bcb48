// Particle-env rollout kernels for 1 .. 5 agents per env, 64 hidden units, bf16 networks
// (see MSRL_PARTICLE_FAMILIES in registry.h).
#include "registry.h"
namespace msrl {
MSRL_FAMILY_BODY(h64_bf16_a, 1, 5, 64, true)
}  // namespace msrl
