// Search kernels with best and prioq held in registers (prioq of at most 64 entries, best of at
// most 64, or 128 for user queries).  Compiled twice: as it stands for vector arrays below 4 GiB, and
// through ggnn_search_reg_wide.hip (GGNN_WIDE_OFFSETS) with 64-bit row offsets for larger arrays.
#include "ggnn_search_kernels.h"

#ifndef GGNN_WIDE_OFFSETS
#define GGNN_WIDE_OFFSETS 0
#define GGNN_NAME(f) f
#else
#define GGNN_NAME(f) f##_wide
#endif

namespace ggnn {
namespace {
constexpr bool kWide = GGNN_WIDE_OFFSETS != 0;
using Cache1 = RegCacheT<1, false, false, kWide>;
using Cache2 = RegCacheT<2, false, false, kWide>;
}  // namespace
hipError_t GGNN_NAME(launch_query_reg)(const GraphDev& G, int dtype, int metric, const void* queries, int64_t Q, int k,
                                       const SearchParams& sp, int every_layer, int32_t* ids, float* dists,
                                       uint32_t* counters, hipStream_t stream) {
  return launch_query_t<Cache1>(G, dtype, metric, queries, Q, k, sp, every_layer, ids, dists, counters, stream);
}
hipError_t GGNN_NAME(launch_query_reg2)(const GraphDev& G, int dtype, int metric, const void* queries, int64_t Q, int k,
                                        const SearchParams& sp, int every_layer, int32_t* ids, float* dists,
                                        uint32_t* counters, hipStream_t stream) {
  return launch_query_t<Cache2>(G, dtype, metric, queries, Q, k, sp, every_layer, ids, dists, counters, stream);
}
hipError_t GGNN_NAME(launch_merge_reg)(const GraphDev& G, int dtype, int metric, int l_top, int l_m, const SearchParams& sp,
                                       int32_t* out_rows, float* dnn1, unsigned long long* work, hipStream_t stream) {
  return launch_merge_t<Cache1>(G, dtype, metric, l_top, l_m, sp, out_rows, dnn1, work, stream);
}
hipError_t GGNN_NAME(launch_sym_search_reg)(const GraphDev& G, int dtype, int metric, int layer, int round, float w_mid,
                                            const SearchParams& sp, const SymBuffers& sb, unsigned long long* work,
                                            hipStream_t stream) {
  return launch_sym_search_t<Cache1>(G, dtype, metric, layer, round, w_mid, sp, sb, work, stream);
}
}  // namespace ggnn
