// Particle-env rollout kernels for 6 .. 10 agents per env, 64 hidden units, fp32 networks
// (see MSRL_PARTICLE_FAMILIES in registry.h).
#include "registry.h"
namespace msrl {
MSRL_FAMILY_BODY(h64_f32_b, 6, 10, 64, false)
}  // namespace msrl
