// Particle-env rollout kernels for 6 .. 10 agents per env, 128 hidden units, fp32 networks
// (see MSRL_PARTICLE_FAMILIES in registry.h).
#include "registry.h"
namespace msrl {
MSRL_FAMILY_BODY(h128_f32_b, 6, 10, 128, false)
}  // namespace msrl
