// The beam-search kernel variants with the (1 + eps) rule of Sec. 4.5 compiled in (queries
// through ann_search_eps).
#include "ann_dispatch.hpp"
#include "search_kernel.hpp"

namespace annmi {

template <int KIND, int VEC, int NCH>
static hipError_t launch_eps(const SearchArgs& a, const VecTable& T, hipStream_t s) {
  return launch_search_variant<KIND, VEC, NCH, true, false>(a, T, s);
}

hipError_t launch_search_eps(const DistCfg& cfg, const SearchArgs& a, const VecTable& T, hipStream_t s) {
  ANN_DISPATCH_CFG(launch_eps, a, T, s);
}

}  // namespace annmi
