// Rollout kernel for networks with more than two hidden layers (see registry.h).
#include "registry.h"
namespace msrl {
MSRL_LINGAUSS_ENTRY_PHASE(entry_l17_6_h256_deep, 17, 6, 256, 4, PHASE_DEEP)
MSRL_LINGAUSS_ENTRY_PHASE(entry_l17_6_h256_act_deep, 17, 6, 256, 4, PHASE_ACT_DEEP)
}  // namespace msrl
