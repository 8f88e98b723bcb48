// Measurement variants of one rollout kernel (see registry.h).
#include "registry.h"
namespace msrl {
MSRL_PARTICLE_ENTRY_PHASE(entry_p10_h256_bf16_env, 10, 256, true, 1, 8, PHASE_ENV)
MSRL_PARTICLE_ENTRY_PHASE(entry_p10_h256_bf16_mlp, 10, 256, true, 1, 8, PHASE_MLP)
MSRL_PARTICLE_ENTRY_PHASE(entry_p10_h256_bf16_clocks, 10, 256, true, 1, 8, PHASE_CLOCKS)
}  // namespace msrl
