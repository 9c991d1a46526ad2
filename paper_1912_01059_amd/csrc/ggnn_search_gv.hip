// User-query kernels whose visited set lives in global memory (searches of a thousand iterations and
// more, where a table in LDS would leave a compute unit with few wavefronts).
// Compiled a second time through ggnn_search_gv_wide.hip for vector arrays of 4 GiB and more.
#include "ggnn_search_kernels.h"

#ifndef GGNN_WIDE_OFFSETS
#define GGNN_WIDE_OFFSETS 0
#define GGNN_NAME(f) f
#else
#define GGNN_NAME(f) f##_wide
#endif

namespace ggnn {
hipError_t GGNN_NAME(launch_query_gv)(int slots, const GraphDev& G, int dtype, int metric, const void* queries, int64_t Q,
                                      int k, const SearchParams& sp, int every_layer, int32_t* ids, float* dists,
                                      uint32_t* counters, hipStream_t stream) {
  constexpr bool kWide = GGNN_WIDE_OFFSETS != 0;
  if (!sp.vis) return hipErrorInvalidValue;
  if (slots == 1) return launch_query_t<RegCacheT<1, true, false, kWide>>(G, dtype, metric, queries, Q, k, sp, every_layer, ids, dists, counters, stream);
  if (slots == 2) return launch_query_t<RegCacheT<2, true, false, kWide>>(G, dtype, metric, queries, Q, k, sp, every_layer, ids, dists, counters, stream);
  return hipErrorInvalidValue;
}
}  // namespace ggnn
