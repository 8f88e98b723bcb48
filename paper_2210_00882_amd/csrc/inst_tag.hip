// Compiled instances of the pursuit-env rollout kernel (tag_kernels.h).
#include "tag_kernels.h"

namespace msrl {

namespace {
template <int NC, int NR, int L, int H>
hipError_t launch(int tiles, int phase, const TagArgs& a, hipStream_t stream) {
  if (phase == TAG_ACT || phase == TAG_STEP) {
    const unsigned blocks = (unsigned)((a.E + 31) / 32);
    if (phase == TAG_ACT)
      hipLaunchKernelGGL((tag_rollout_kernel<NC, NR, L, H, 1, TAG_ACT>), dim3(blocks), dim3(64 * (NC + NR)), 0, stream, a);
    else
      hipLaunchKernelGGL((tag_rollout_kernel<NC, NR, L, H, 1, TAG_STEP>), dim3(blocks), dim3(64 * (NC + NR)), 0, stream, a);
  } else if (tiles == 4) {
    const unsigned blocks = (unsigned)((a.E + 127) / 128);
    hipLaunchKernelGGL((tag_rollout_kernel<NC, NR, L, H, 4>), dim3(blocks), dim3(64 * (NC + NR) * 4), 0, stream, a);
  } else {
    const unsigned blocks = (unsigned)((a.E + 31) / 32);
    hipLaunchKernelGGL((tag_rollout_kernel<NC, NR, L, H, 1>), dim3(blocks), dim3(64 * (NC + NR)), 0, stream, a);
  }
  return hipGetLastError();
}
}  // namespace

bool tag_rollout_compiled(int nc, int nr, int landmarks, int hidden) {
  return hidden == 64 && ((nc == 3 && nr == 1 && landmarks == 2) || (nc == 2 && nr == 2 && landmarks == 1));
}

hipError_t launch_tag_rollout(int nc, int nr, int landmarks, int hidden, int tiles, int phase, const TagArgs& a,
                              hipStream_t stream) {
  if (tiles != 1 && tiles != 4) return hipErrorInvalidValue;
  if (phase != TAG_ALL && phase != TAG_ACT && phase != TAG_STEP) return hipErrorInvalidValue;
  if (hidden == 64 && nc == 3 && nr == 1 && landmarks == 2) return launch<3, 1, 2, 64>(tiles, phase, a, stream);
  if (hidden == 64 && nc == 2 && nr == 2 && landmarks == 1) return launch<2, 2, 1, 64>(tiles, phase, a, stream);
  return hipErrorInvalidValue;
}

}  // namespace msrl
