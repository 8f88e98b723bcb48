// Pursuit-env rollout kernels with 1 chaser (see MSRL_TAG_FAMILIES in tag_kernels.h).
#include "tag_kernels.h"
namespace msrl {
MSRL_TAG_FAMILY_BODY(1)
}  // namespace msrl
