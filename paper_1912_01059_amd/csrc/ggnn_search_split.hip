// The two launches of a large batch of user queries (upper layers; bottom layer in an order sorted by
// region), for the searches whose lists live in registers.
#include "ggnn_search_kernels.h"

namespace ggnn {
hipError_t launch_query_split(int slots, const GraphDev& G, int dtype, int metric, const void* queries, int64_t Q, int k,
                              const SearchParams& sp, int32_t* ids, float* dists, uint32_t* counters,
                              const SplitBufs& sb, hipStream_t stream) {
  if (slots == 1) return launch_query_split_t<RegCache>(G, dtype, metric, queries, Q, k, sp, ids, dists, counters, sb, stream);
  if (slots == 2) return launch_query_split_t<RegCache2>(G, dtype, metric, queries, Q, k, sp, ids, dists, counters, sb, stream);
  return hipErrorInvalidValue;
}
}  // namespace ggnn
