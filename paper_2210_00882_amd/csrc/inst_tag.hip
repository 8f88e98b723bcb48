// Table and launcher of the compiled instances of the pursuit-env rollout kernel (tag_kernels.h).
#include "tag_kernels.h"

namespace msrl {

namespace {
const std::vector<TagEntry>& tag_kernels() {
  static const std::vector<TagEntry> table = [] {
    std::vector<TagEntry> t;
#define MSRL_CALL_TAG_FAMILY(NC) tag_family_c##NC(t);
    MSRL_TAG_FAMILIES(MSRL_CALL_TAG_FAMILY)
#undef MSRL_CALL_TAG_FAMILY
    return t;
  }();
  return table;
}

const TagEntry* find_tag(int nc, int nr, int landmarks, int hidden, bool bf16, int tiles, int phase) {
  for (const TagEntry& k : tag_kernels())
    if (k.nc == nc && k.nr == nr && k.landmarks == landmarks && k.hidden == hidden && (k.bf16 != 0) == bf16 &&
        k.tiles == tiles && k.phase == phase)
      return &k;
  return nullptr;
}
}  // namespace

bool tag_rollout_compiled(int nc, int nr, int landmarks, int hidden, bool bf16, int tiles) {
  return find_tag(nc, nr, landmarks, hidden, bf16, tiles, TAG_ALL) != nullptr;
}

hipError_t launch_tag_rollout(int nc, int nr, int landmarks, int hidden, bool bf16, int tiles, int phase,
                              const TagArgs& a, hipStream_t stream) {
  if (phase == TAG_ACT || phase == TAG_STEP) tiles = 1;
  const TagEntry* k = find_tag(nc, nr, landmarks, hidden, bf16, tiles, phase);
  if (!k) return hipErrorInvalidValue;
  const unsigned blocks = (unsigned)((a.E + 32 * tiles - 1) / (32 * tiles));
  TagArgs args = a;
  void* params[] = {&args};
  return hipLaunchKernel(k->fn, dim3(blocks), dim3((unsigned)(64 * (nc + nr) * tiles)), params, 0, stream);
}

}  // namespace msrl
