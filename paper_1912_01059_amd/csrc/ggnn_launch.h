// Host-side launchers shared by the API translation unit and the kernel translation units.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "ggnn_device.h"

namespace ggnn {

// the work counters of the construction searches are spread over this many cache lines
constexpr int kWorkSlots = 1024;

// A dispatch counts the work-items of each grid dimension in 32 bits, so one launch of 64-lane
// workgroups holds fewer than 2^26 of them: a launch of 10^8 workgroups does not fit, and what the
// hardware then runs is not what was asked for.  Kernels that take one workgroup per item (query,
// point, segment) are launched in chunks of at most kMaxBlocksPerLaunch workgroups on the same stream;
// each launch is told its first item and the kernel adds blockIdx.x to it.  (A multiple of 8, so the
// workgroup -> XCD assignment continues across chunks.)
constexpr int64_t kMaxBlocksPerLaunch = (int64_t)1 << 24;
inline unsigned chunk_blocks(int64_t n_items, int64_t first) {
  const int64_t left = n_items - first;
  return (unsigned)(left < kMaxBlocksPerLaunch ? left : kMaxBlocksPerLaunch);
}

// state of one symmetric-linking pass over a layer (device buffers owned by the graph)
struct SymBuffers {
  int32_t* inv;       // n x ksym inverse links granted so far
  int32_t* ninv;      // n
  u64* pref;          // n x B candidate keys of the failed searches of the current round
  int32_t* npref;     // n
  int32_t* ptr;       // n  index of the candidate a request currently proposes to
  int32_t* state;     // n  0 = no request / settled nowhere, 1 = proposing, 2 = holds a slot
  int32_t* hold;      // n x ksym requests (their z) holding a slot of this row in this round
  int32_t* nhold;     // n
  int32_t* head;      // n  head of the list of requests proposing to this row
  int32_t* next;      // n  links of those lists
  int32_t* pending;   // 1  number of requests that still have to propose
};

// search kernels: best / prioq in registers (ggnn_search_reg.hip, capacities <= 64) or in LDS
// (ggnn_search_lds.hip); the API picks the register variant whenever the capacities allow it.
// Every register variant exists twice: plain for vector arrays below 4 GiB (32-bit row offsets) and
// `_wide` for larger arrays (64-bit row offsets; the *_wide.hip translation units).
#define GGNN_SEARCH_LAUNCHERS(SUFFIX)                                                                              \
  hipError_t launch_query##SUFFIX(const GraphDev& G, int dtype, int metric, const void* queries, int64_t Q, int k, \
                                  const SearchParams& sp, int every_layer, int32_t* ids, float* dists,             \
                                  uint32_t* counters, hipStream_t stream);                                         \
  hipError_t launch_merge##SUFFIX(const GraphDev& G, int dtype, int metric, int l_top, int l_m,                    \
                                  const SearchParams& sp, int32_t* out_rows, float* dnn1, unsigned long long* work, \
                                  hipStream_t stream);                                                             \
  hipError_t launch_sym_search##SUFFIX(const GraphDev& G, int dtype, int metric, int layer, int round, float w_mid,\
                                       const SearchParams& sp, const SymBuffers& sb, unsigned long long* work,  \
                                       hipStream_t stream);
GGNN_SEARCH_LAUNCHERS(_reg)
GGNN_SEARCH_LAUNCHERS(_reg_wide)
GGNN_SEARCH_LAUNCHERS(_lds)
#undef GGNN_SEARCH_LAUNCHERS
// slots = registers per lane of best (1 or 2)
#define GGNN_QUERY_LAUNCHERS(SUFFIX)                                                                               \
  /* best of up to 128 entries */                                                                                  \
  hipError_t launch_query_reg2##SUFFIX(const GraphDev& G, int dtype, int metric, const void* queries, int64_t Q,   \
                                       int k, const SearchParams& sp, int every_layer, int32_t* ids, float* dists, \
                                       uint32_t* counters, hipStream_t stream);                                    \
  /* ggnn_search_split.hip: launch sb.phase (1 or 2) of a large batch */                                           \
  hipError_t launch_query_split##SUFFIX(int slots, const GraphDev& G, int dtype, int metric, const void* queries,  \
                                        int64_t Q, int k, const SearchParams& sp, int32_t* ids, float* dists,      \
                                        uint32_t* counters, const SplitBufs& sb, hipStream_t stream);              \
  /* ggnn_search_gv.hip: visited ids in global memory (sp.vis: Q tables of RegCacheGV::vis_slots words) */        \
  hipError_t launch_query_gv##SUFFIX(int slots, const GraphDev& G, int dtype, int metric, const void* queries,     \
                                     int64_t Q, int k, const SearchParams& sp, int every_layer, int32_t* ids,      \
                                     float* dists, uint32_t* counters, hipStream_t stream);                        \
  /* ggnn_search_any.hip: LDS table of any multiple of 64 slots */                                                 \
  hipError_t launch_query_any##SUFFIX(int slots, const GraphDev& G, int dtype, int metric, const void* queries,    \
                                      int64_t Q, int k, const SearchParams& sp, int every_layer, int32_t* ids,     \
                                      float* dists, uint32_t* counters, hipStream_t stream);
GGNN_QUERY_LAUNCHERS()
GGNN_QUERY_LAUNCHERS(_wide)
#undef GGNN_QUERY_LAUNCHERS

// construction kernels (ggnn_build.hip)
hipError_t launch_gather_probe(const void* rows, int row_bytes, const int32_t* ids, int64_t n, int rows_per_wave,
                               uint32_t* out, hipStream_t stream);
hipError_t launch_merge_shards(int S, int64_t Q, int k, const int32_t* ids, const float* dists, const int32_t* offsets,
                               int32_t* out_ids, float* out_dists, hipStream_t stream);
hipError_t launch_fill_i32(int32_t* p, int64_t n, int32_t v, hipStream_t stream);
// order[0..Q) := the numbers 0..Q-1 sorted by key >> shift (a counting sort; the order within one value is
// not defined); bins: nbins + 1 ints of scratch, nbins <= kSortBins
constexpr int kSortBins = 65536;
hipError_t launch_sort_by_key(const int32_t* key, int64_t Q, int shift, int nbins, int32_t* bins, int32_t* order,
                              hipStream_t stream);
hipError_t launch_normalise(const void* base, int dtype, int64_t N, int D, float* out, hipStream_t stream);
hipError_t launch_select(const GraphDev& G, int l_top, const float* dnn1, int32_t* to_lower, int32_t* to_base,
                         hipStream_t stream);
// mean / max of x[0..n): partial holds 2*1024 doubles of scratch, out[0] = mean, out[1] = max
hipError_t launch_stats(const float* x, int64_t n, double* partial, float* out, hipStream_t stream);
hipError_t launch_sym_propose_first(const GraphDev& G, int layer, const SymBuffers& sb, int B, hipStream_t stream);
hipError_t launch_sym_propose(const GraphDev& G, int layer, const SymBuffers& sb, int B, hipStream_t stream);
hipError_t launch_sym_resolve(const GraphDev& G, int layer, const SymBuffers& sb, int B, hipStream_t stream);
hipError_t launch_sym_commit(const GraphDev& G, int layer, const SymBuffers& sb, hipStream_t stream);
hipError_t launch_sym_apply(const GraphDev& G, int layer, const SymBuffers& sb, int32_t* edges, int32_t* inv_count,
                            hipStream_t stream);

}  // namespace ggnn
