// Search kernels with best and prioq held in registers (prioq of at most 64 entries, best of at
// most 64, or 128 for user queries).
#include "ggnn_search_kernels.h"

namespace ggnn {
hipError_t launch_query_reg(const GraphDev& G, int dtype, int metric, const void* queries, int64_t Q, int k,
                            const SearchParams& sp, int every_layer, int32_t* ids, float* dists, uint32_t* counters,
                            hipStream_t stream) {
  return launch_query_t<RegCache>(G, dtype, metric, queries, Q, k, sp, every_layer, ids, dists, counters, stream);
}
hipError_t launch_query_reg2(const GraphDev& G, int dtype, int metric, const void* queries, int64_t Q, int k,
                             const SearchParams& sp, int every_layer, int32_t* ids, float* dists, uint32_t* counters,
                             hipStream_t stream) {
  return launch_query_t<RegCache2>(G, dtype, metric, queries, Q, k, sp, every_layer, ids, dists, counters, stream);
}
hipError_t launch_merge_reg(const GraphDev& G, int dtype, int metric, int l_top, int l_m, const SearchParams& sp,
                            int32_t* out_rows, float* dnn1, unsigned long long* work, hipStream_t stream) {
  return launch_merge_t<RegCache>(G, dtype, metric, l_top, l_m, sp, out_rows, dnn1, work, stream);
}
hipError_t launch_sym_search_reg(const GraphDev& G, int dtype, int metric, int layer, int round, float w_mid,
                                 const SearchParams& sp, const SymBuffers& sb, unsigned long long* work,
                                 hipStream_t stream) {
  return launch_sym_search_t<RegCache>(G, dtype, metric, layer, round, w_mid, sp, sb, work, stream);
}
#ifdef GGNN_PHASE_TIMING
hipError_t read_phase_cycles(unsigned long long* out16, int reset) {
  hipError_t e = hipMemcpyFromSymbol(out16, HIP_SYMBOL(g_phase_cycles), sizeof(unsigned long long) * 16);
  if (e != hipSuccess) return e;
  if (reset) {
    unsigned long long z[16] = {0};
    e = hipMemcpyToSymbol(HIP_SYMBOL(g_phase_cycles), z, sizeof(z));
  }
  return e;
}
extern "C" int ggnn_debug_phase_cycles(unsigned long long* out16, int reset) { return (int)read_phase_cycles(out16, reset); }
#endif
}  // namespace ggnn
