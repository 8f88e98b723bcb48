// row kernels of the learner for hidden size 64
#include "learn_fused.h"

namespace msrl {
MSRL_ROWS_LAUNCHER(64)
}  // namespace msrl
