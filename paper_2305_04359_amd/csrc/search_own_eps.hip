// The beam-search kernel variants with a start vertex per search and the (1 + eps) rule of
// Sec. 4.5 (queries on the bottom layer of the index of Sec. 4.2).
#include "ann_dispatch.hpp"
#include "search_kernel.hpp"

namespace annmi {

template <int KIND, int VEC, int NCH>
static hipError_t launch_own_eps(const SearchArgs& a, const VecTable& T, hipStream_t s) {
  return launch_search_variant<KIND, VEC, NCH, true, true>(a, T, s);
}

hipError_t launch_search_own_eps(const DistCfg& cfg, const SearchArgs& a, const VecTable& T, hipStream_t s) {
  ANN_DISPATCH_CFG(launch_own_eps, a, T, s);
}

}  // namespace annmi
