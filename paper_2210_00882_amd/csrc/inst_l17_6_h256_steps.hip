// Step-granular variants of one rollout kernel: actor only, environment only (see registry.h).
#include "registry.h"
namespace msrl {
MSRL_LINGAUSS_ENTRY_PHASE(entry_l17_6_h256_act, 17, 6, 256, 4, PHASE_ACT)
MSRL_LINGAUSS_ENTRY_PHASE(entry_l17_6_h256_step, 17, 6, 256, 4, PHASE_STEP)
}  // namespace msrl
