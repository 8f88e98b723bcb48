// row kernels of the learner for hidden size 256
#include "learn_fused.h"

namespace msrl {
MSRL_ROWS_LAUNCHER(256)
}  // namespace msrl
