// The two launches of a large batch of user queries (upper layers; bottom layer in an order sorted by
// region), for the searches whose lists live in registers.
// Compiled a second time through ggnn_search_split_wide.hip for vector arrays of 4 GiB and more.
#include "ggnn_search_kernels.h"

#ifndef GGNN_WIDE_OFFSETS
#define GGNN_WIDE_OFFSETS 0
#define GGNN_NAME(f) f
#else
#define GGNN_NAME(f) f##_wide
#endif

namespace ggnn {
hipError_t GGNN_NAME(launch_query_split)(int slots, const GraphDev& G, int dtype, int metric, const void* queries, int64_t Q,
                                         int k, const SearchParams& sp, int32_t* ids, float* dists, uint32_t* counters,
                                         const SplitBufs& sb, hipStream_t stream) {
  constexpr bool kWide = GGNN_WIDE_OFFSETS != 0;
  if (slots == 1) return launch_query_split_t<RegCacheT<1, false, false, kWide>>(G, dtype, metric, queries, Q, k, sp, ids, dists, counters, sb, stream);
  if (slots == 2) return launch_query_split_t<RegCacheT<2, false, false, kWide>>(G, dtype, metric, queries, Q, k, sp, ids, dists, counters, sb, stream);
  return hipErrorInvalidValue;
}
}  // namespace ggnn
