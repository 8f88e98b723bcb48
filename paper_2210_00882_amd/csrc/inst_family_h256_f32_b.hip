// Particle-env rollout kernels for 5 .. 7 agents per env, 256 hidden units, fp32 networks
// (see MSRL_PARTICLE_FAMILIES in registry.h).
#include "registry.h"
namespace msrl {
MSRL_FAMILY_BODY(h256_f32_b, 5, 7, 256, false)
}  // namespace msrl
