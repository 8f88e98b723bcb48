// row kernels of the learner for hidden size 128
#include "learn_fused.h"

namespace msrl {
MSRL_ROWS_LAUNCHER(128)
}  // namespace msrl
