// Compiled instances of the pursuit-env rollout kernel (tag_kernels.h).
#include "tag_kernels.h"

namespace msrl {

namespace {
template <int NC, int NR, int L, int H>
hipError_t launch(const TagArgs& a, hipStream_t stream) {
  const unsigned blocks = (unsigned)((a.E + 31) / 32);
  hipLaunchKernelGGL((tag_rollout_kernel<NC, NR, L, H>), dim3(blocks), dim3(64 * (NC + NR)), 0, stream, a);
  return hipGetLastError();
}
}  // namespace

bool tag_rollout_compiled(int nc, int nr, int landmarks, int hidden) {
  return hidden == 64 && ((nc == 3 && nr == 1 && landmarks == 2) || (nc == 2 && nr == 2 && landmarks == 1));
}

hipError_t launch_tag_rollout(int nc, int nr, int landmarks, int hidden, const TagArgs& a, hipStream_t stream) {
  if (hidden == 64 && nc == 3 && nr == 1 && landmarks == 2) return launch<3, 1, 2, 64>(a, stream);
  if (hidden == 64 && nc == 2 && nr == 2 && landmarks == 1) return launch<2, 2, 1, 64>(a, stream);
  return hipErrorInvalidValue;
}

}  // namespace msrl
