// User-query kernels whose visited set lives in global memory (searches of a thousand iterations and
// more, where a table in LDS would leave a compute unit with few wavefronts).
#include "ggnn_search_kernels.h"

namespace ggnn {
hipError_t launch_query_gv(int slots, const GraphDev& G, int dtype, int metric, const void* queries, int64_t Q, int k,
                           const SearchParams& sp, int every_layer, int32_t* ids, float* dists, uint32_t* counters,
                           hipStream_t stream) {
  if (!sp.vis) return hipErrorInvalidValue;
  if (slots == 1) return launch_query_t<RegCacheGV>(G, dtype, metric, queries, Q, k, sp, every_layer, ids, dists, counters, stream);
  if (slots == 2) return launch_query_t<RegCache2GV>(G, dtype, metric, queries, Q, k, sp, every_layer, ids, dists, counters, stream);
  return hipErrorInvalidValue;
}
}  // namespace ggnn
