// Search kernels with best and prioq held in LDS (any capacities that fit one workgroup's LDS).
#include "ggnn_search_kernels.h"

namespace ggnn {
hipError_t launch_query_lds(const GraphDev& G, int dtype, int metric, const void* queries, int64_t Q, int k,
                            const SearchParams& sp, int every_layer, int32_t* ids, float* dists, uint32_t* counters,
                            hipStream_t stream) {
  return launch_query_t<LdsCache>(G, dtype, metric, queries, Q, k, sp, every_layer, ids, dists, counters, stream);
}
hipError_t launch_merge_lds(const GraphDev& G, int dtype, int metric, int l_top, int l_m, const SearchParams& sp,
                            int32_t* out_rows, float* dnn1, unsigned long long* work, hipStream_t stream) {
  return launch_merge_t<LdsCache>(G, dtype, metric, l_top, l_m, sp, out_rows, dnn1, work, stream);
}
hipError_t launch_sym_search_lds(const GraphDev& G, int dtype, int metric, int layer, int round, float w_mid,
                                 const SearchParams& sp, const SymBuffers& sb, unsigned long long* work,
                                 hipStream_t stream) {
  return launch_sym_search_t<LdsCache>(G, dtype, metric, layer, round, w_mid, sp, sb, work, stream);
}
}  // namespace ggnn
