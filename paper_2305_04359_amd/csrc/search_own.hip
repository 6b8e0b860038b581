// The beam-search kernel variants in which every search has a start vertex of its own (the layers
// of the index of Sec. 4.2), without the (1 + eps) rule.
#include "ann_dispatch.hpp"
#include "search_kernel.hpp"

namespace annmi {

template <int KIND, int VEC, int NCH>
static hipError_t launch_own(const SearchArgs& a, const VecTable& T, hipStream_t s) {
  return launch_search_variant<KIND, VEC, NCH, false, true>(a, T, s);
}

hipError_t launch_search_own(const DistCfg& cfg, const SearchArgs& a, const VecTable& T, hipStream_t s) {
  ANN_DISPATCH_CFG(launch_own, a, T, s);
}

}  // namespace annmi
