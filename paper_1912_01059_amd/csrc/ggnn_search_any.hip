// User-query kernels whose LDS table of visited and rejected ids has any multiple of 64 slots (searches
// of more than 384 iterations, where rounding the table up to a power of two would cost residency).
#include "ggnn_search_kernels.h"

namespace ggnn {
hipError_t launch_query_any(int slots, const GraphDev& G, int dtype, int metric, const void* queries, int64_t Q, int k,
                            const SearchParams& sp, int every_layer, int32_t* ids, float* dists, uint32_t* counters,
                            hipStream_t stream) {
  if (slots == 1) return launch_query_t<RegCacheAny>(G, dtype, metric, queries, Q, k, sp, every_layer, ids, dists, counters, stream);
  if (slots == 2) return launch_query_t<RegCache2Any>(G, dtype, metric, queries, Q, k, sp, every_layer, ids, dists, counters, stream);
  return hipErrorInvalidValue;
}
}  // namespace ggnn
