// User-query kernels whose LDS table of visited and rejected ids has any multiple of 64 slots (searches
// of more than 384 iterations, where rounding the table up to a power of two would cost residency).
// Compiled a second time through ggnn_search_any_wide.hip for vector arrays of 4 GiB and more.
#include "ggnn_search_kernels.h"

#ifndef GGNN_WIDE_OFFSETS
#define GGNN_WIDE_OFFSETS 0
#define GGNN_NAME(f) f
#else
#define GGNN_NAME(f) f##_wide
#endif

namespace ggnn {
hipError_t GGNN_NAME(launch_query_any)(int slots, const GraphDev& G, int dtype, int metric, const void* queries, int64_t Q,
                                       int k, const SearchParams& sp, int every_layer, int32_t* ids, float* dists,
                                       uint32_t* counters, hipStream_t stream) {
  constexpr bool kWide = GGNN_WIDE_OFFSETS != 0;
  if (slots == 1) return launch_query_t<RegCacheT<1, false, true, kWide>>(G, dtype, metric, queries, Q, k, sp, every_layer, ids, dists, counters, stream);
  if (slots == 2) return launch_query_t<RegCacheT<2, false, true, kWide>>(G, dtype, metric, queries, Q, k, sp, every_layer, ids, dists, counters, stream);
  return hipErrorInvalidValue;
}
}  // namespace ggnn
