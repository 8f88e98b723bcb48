// Table and launcher of the compiled instances of the pursuit-env rollout kernel (tag_kernels.h).
#include <unordered_map>

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

// (the table has about a thousand entries and the step-granular calls look one up per call: an index by
// shape, built once)
uint32_t tag_key(int nc, int nr, int landmarks, int hidden, bool bf16, int tiles, int phase) {
  return (uint32_t)nc | (uint32_t)nr << 4 | (uint32_t)landmarks << 8 | (uint32_t)(bf16 ? 1 : 0) << 12 |
         (uint32_t)tiles << 13 | (uint32_t)phase << 16 | (uint32_t)hidden << 20;
}
const TagEntry* find_tag(int nc, int nr, int landmarks, int hidden, bool bf16, int tiles, int phase) {
  static const std::unordered_map<uint32_t, const TagEntry*> index = [] {
    std::unordered_map<uint32_t, const TagEntry*> m;
    for (const TagEntry& k : tag_kernels())
      m.emplace(tag_key(k.nc, k.nr, k.landmarks, k.hidden, k.bf16 != 0, k.tiles, k.phase), &k);
    return m;
  }();
  if (nc < 0 || nc > 15 || nr < 0 || nr > 15 || landmarks < 0 || landmarks > 15 || tiles < 0 || tiles > 7 ||
      phase < 0 || phase > 15 || hidden < 0 || hidden > 4095)
    return nullptr;
  const auto it = index.find(tag_key(nc, nr, landmarks, hidden, bf16, tiles, phase));
  return it == index.end() ? nullptr : it->second;
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
