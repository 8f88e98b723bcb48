// One rollout-kernel instantiation (see registry.h).
#include "registry.h"
namespace msrl {
MSRL_LINGAUSS_ENTRY(entry_l17_6_h256, 17, 6, 256, 4)
}  // namespace msrl
