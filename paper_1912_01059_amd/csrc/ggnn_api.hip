// C ABI of the library (see include/ggnn.h): argument checks, device memory of the graph,
// and the sequencing of kernels for construction (Alg. 3, Alg. 6) and query (Alg. 1).
#include <math.h>
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <atomic>
#include <mutex>
#include <new>
#include <chrono>
#include <vector>

#include "ggnn.h"
#include "ggnn_geometry.h"
#include "ggnn_launch.h"
#include "ggnn_regcache.h"

using namespace ggnn;

static_assert(GGNN_ROW_LANES == kRowLanes && GGNN_WIDE_ROW_LANES == kWideRowLanes, "public constants and kernels disagree");
static_assert(GGNN_MAX_LEVELS == kMaxLevels, "public constant and kernels disagree");

// Workspace of ggnn_query_static (the two-launch path for callers that cannot allocate): one array per
// GPU, part of the loaded code object, held until the process ends.  In host code this name only
// stands for the symbol: the array's device address comes from hipGetSymbolAddress (scratch_ptr below).
constexpr size_t kScratchBytes = (size_t)GGNN_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

namespace {

thread_local char g_err[512] = "";

int fail(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

#define HIP_TRY(expr)                                                                              \
  do {                                                                                             \
    hipError_t e_ = (expr);                                                                        \
    if (e_ != hipSuccess) return fail(GGNN_ERR_HIP, "%s: %s", #expr, hipGetErrorString(e_));       \
  } while (0)

// device address of `scratch` on the current device, looked up once per device
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
unsigned char* g_scratch_ptr[kMaxDevices] = {nullptr};
int scratch_ptr(unsigned char** out) {
  int dev = -1;
  HIP_TRY(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return fail(GGNN_ERR_LIMIT, "device %d: this build keeps a workspace for devices 0..%d", dev, kMaxDevices - 1);
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (!p) return fail(GGNN_ERR_HIP, "hipGetSymbolAddress returned a null address for the workspace");
    g_scratch_ptr[dev] = (unsigned char*)p;
  }
  *out = g_scratch_ptr[dev];
  return GGNN_OK;
}

constexpr size_t kMaxLds = 160 * 1024;  // LDS of a compute unit on gfx950, all of which one workgroup may take

// How a search is dispatched.  Every call works on a snapshot of its own, taken once at the entry point
// (from the caller's ggnn_query_params, or from the process-wide defaults behind the ggnn_set_* calls,
// which are atomics): nothing on the dispatch path reads shared mutable state.
struct Tuning {
  int cache_mode;        // 0: best / prioq in registers whenever they fit, 1: always in LDS
  int64_t split_min;     // batches of at least this many every-layer queries take two launches
  int32_t vis_min_iter;  // iteration limit from which visited moves to global memory; <= 0: never
  bool vis_forced;       // ... whatever the batch size
};
constexpr int64_t kSplitMinQueries = 12288;  // smaller batches gain nothing from the two-launch path
constexpr int32_t kVisGlobalMinIter = 1100;
std::atomic<int> g_cache_mode{0};
std::atomic<int64_t> g_split_min_queries{kSplitMinQueries};
std::atomic<int32_t> g_vis_global_min_iter{kVisGlobalMinIter};
std::atomic<bool> g_vis_global_forced{false};
Tuning process_tuning() {
  return Tuning{g_cache_mode.load(), g_split_min_queries.load(), g_vis_global_min_iter.load(), g_vis_global_forced.load()};
}

// compute units of the current device (looked up once per device)
std::atomic<int> g_cu_count[64];
int cu_count() {
  int dev = 0, cus = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
  cus = g_cu_count[dev].load();
  if (cus > 0) return cus;
  if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0) {
    (void)hipGetLastError();
    cus = 256;
  }
  g_cu_count[dev].store(cus);
  return cus;
}

int next_pow2(int v) {
  int p = 1;
  while (p < v) p <<= 1;
  return p;
}

}  // namespace

struct ggnn_graph {
  int64_t N = 0;
  int D = 0, K = 0, L = 0, s = 0, g = 0;
  int dtype = 0, metric = 0;
  uint64_t seed = 0;
  int64_t n[kMaxLevels] = {0}, G[kMaxLevels] = {0};
  int32_t* edges[kMaxLevels] = {nullptr};
  int32_t* to_lower[kMaxLevels] = {nullptr};
  int32_t* to_base[kMaxLevels] = {nullptr};
  int32_t* inv_count[kMaxLevels] = {nullptr};
  int32_t* edge_tmp = nullptr;  // N*K, the buffer a merge writes before the swap
  float* dnn1 = nullptr;        // N
  float* stats_dev = nullptr;   // 2
  double* stats_partial = nullptr;
  unsigned long long* work_dev = nullptr;  // pops / rows gathered of merge and sym searches
  float stats[2] = {0.0f, 0.0f};
  const void* base = nullptr;   // borrowed
  float* norm = nullptr;        // cosine: owned unit-length copy
  hipStream_t stream = nullptr;
  // construction parameters
  float tau_build = 0.5f;
  int refinements = 2, pq_cap = 64, visited_cap = 384, max_iter = 384;
  float w_mid = 0.4f;
  SymBuffers sb = {};
  bool sb_ready = false;
  ggnn_build_times times = {};
  ggnn_progress_fn progress = nullptr;  // called by ggnn_build_steps after every step
  void* progress_user = nullptr;
};

namespace {

GraphDev device_view(const ggnn_graph* g) {
  GraphDev G = {};
  G.rows = (const uint8_t*)(g->norm ? (const void*)g->norm : g->base);
  G.N = g->N; G.D = g->D; G.K = g->K; G.L = g->L; G.s = g->s; G.g = g->g;
  const int esize = (g->norm || g->dtype == GGNN_F32) ? 4 : 1;
  G.row_bytes = g->D * esize;
  G.nchunks = G.row_bytes / 16;
  G.addr32 = ((uint64_t)g->N * (uint64_t)G.row_bytes < (1ull << 32)) ? 1 : 0;
  for (int l = 0; l < g->L; l++) {
    G.n[l] = g->n[l];
    G.edges[l] = g->edges[l];
    G.to_lower[l] = g->to_lower[l];
    G.to_base[l] = g->to_base[l];
  }
  G.G0 = g->G[0];
  partition_keys(g->N, g->seed, &G);
  return G;
}
int row_dtype(const ggnn_graph* g) { return g->norm ? GGNN_F32 : g->dtype; }

// where the lists of a search live: 1 / 2 = registers with best in one / two registers per lane, 0 = LDS
int register_slots(const SearchParams& sp, bool user_query, const Tuning& t) {
  if (t.cache_mode != 0 || sp.P > kWave) return 0;
  if (sp.B <= kWave) return 1;
  return (user_query && sp.B <= 2 * kWave) ? 2 : 0;
}

int make_search_params(int B, int P, int V, int max_iter, float tau, float dnn, SearchParams* sp, const Tuning& t,
                       bool user_query = false) {
  if (B < 1 || P < 1 || V < 1 || max_iter < 0) return fail(GGNN_ERR_INVALID, "cache capacities must be positive");
  if (max_iter > V) return fail(GGNN_ERR_INVALID, "max_iter (%d) must not exceed visited_cap (%d)", max_iter, V);
  sp->B = B; sp->P = P; sp->max_iter = max_iter;
  sp->H = next_pow2(2 * (max_iter > 0 ? max_iter : 1));
  if (sp->H < 64) sp->H = 64;
  sp->tau = tau; sp->dnn = dnn;
  sp->start = nullptr; sp->n_start = 0; sp->vis = nullptr;
  const int slots = register_slots(*sp, user_query, t);
  const size_t need = slots == 1 ? RegCache::lds_bytes(*sp) : slots == 2 ? RegCache2::lds_bytes(*sp) : LdsCache::lds_bytes(*sp);
  if (need > kMaxLds)
    return fail(GGNN_ERR_LIMIT, "cache of best=%d prioq=%d visited=%d needs %zu bytes of LDS, limit %zu", B, P, V,
                need, kMaxLds);
  return GGNN_OK;
}

hipError_t launch_query_whole(const GraphDev& G, int dtype, int metric, const void* queries, int64_t Q, int k,
                              const SearchParams& sp, int every_layer, int32_t* ids, float* dists, uint32_t* counters,
                              hipStream_t stream, const Tuning& t) {
  const int slots = register_slots(sp, true, t);
  // beyond 384 iterations a power-of-two table would be larger than 1024 slots: size it to the limit
  const bool wide = !G.addr32;  // arrays of 4 GiB and more: the variants with 64-bit row offsets
  if (slots >= 1 && 2 * sp.max_iter + 256 > 1024)
    return (wide ? launch_query_any_wide : launch_query_any)(slots, G, dtype, metric, queries, Q, k, sp, every_layer, ids, dists, counters, stream);
  if (slots == 1) return (wide ? launch_query_reg_wide : launch_query_reg)(G, dtype, metric, queries, Q, k, sp, every_layer, ids, dists, counters, stream);
  if (slots == 2) return (wide ? launch_query_reg2_wide : launch_query_reg2)(G, dtype, metric, queries, Q, k, sp, every_layer, ids, dists, counters, stream);
  return launch_query_lds(G, dtype, metric, queries, Q, k, sp, every_layer, ids, dists, counters, stream);
}

// Workspace of the two-launch path: the lists put aside after the upper layers (state), counters
// (meta), the sort keys, the sorted order and the bins of the counting sort.
struct SplitLayout {
  size_t state_bytes, meta_bytes, q_bytes, total;
  int32_t state_keys, shift, nbins;
};
SplitLayout split_layout(const GraphDev& G, int slots, int64_t Q) {
  SplitLayout lay = {};
  while (((G.n[1] - 1) >> lay.shift) >= kSortBins) lay.shift++;
  lay.nbins = (int32_t)(((G.n[1] - 1) >> lay.shift) + 1);
  lay.state_keys = (slots + 1) * kWave;
  lay.state_bytes = (size_t)Q * lay.state_keys * sizeof(u64);
  lay.meta_bytes = (size_t)Q * 8 * sizeof(int32_t);
  lay.q_bytes = (((size_t)Q * sizeof(int32_t)) + 255) / 256 * 256;
  lay.total = lay.state_bytes + lay.meta_bytes + 2 * lay.q_bytes + ((size_t)lay.nbins + 1) * sizeof(int32_t);
  return lay;
}
// upper layers, counting sort of the queries by the layer-1 point reached, bottom layer; every word of
// the workspace that is read has been written by an earlier step of the same call (the bins are cleared
// by a fill kernel), so the workspace may hold anything on entry
hipError_t launch_query_two(const GraphDev& G, int dtype, int metric, const void* queries, int64_t Q, int k,
                            const SearchParams& sp, int slots, int32_t* ids, float* dists, uint32_t* counters,
                            unsigned char* ws, const SplitLayout& lay, hipStream_t stream) {
  SplitBufs sb = {};
  sb.Q = Q;
  sb.state_keys = lay.state_keys;
  sb.state = (u64*)ws;
  sb.meta = (int32_t*)(ws + lay.state_bytes);
  sb.key = (int32_t*)(ws + lay.state_bytes + lay.meta_bytes);
  int32_t* order = (int32_t*)(ws + lay.state_bytes + lay.meta_bytes + lay.q_bytes);
  int32_t* bins = (int32_t*)(ws + lay.state_bytes + lay.meta_bytes + 2 * lay.q_bytes);
  sb.phase = 1;
  const auto launch_phase = G.addr32 ? launch_query_split : launch_query_split_wide;
  hipError_t e = launch_phase(slots, G, dtype, metric, queries, Q, k, sp, ids, dists, counters, sb, stream);
  if (e == hipSuccess) e = launch_sort_by_key(sb.key, Q, lay.shift, lay.nbins, bins, order, stream);
  if (e == hipSuccess) {
    sb.phase = 2;
    sb.order = order;
    sb.per = (int32_t)((Q + kXcds - 1) / kXcds);
    e = launch_phase(slots, G, dtype, metric, queries, Q, k, sp, ids, dists, counters, sb, stream);
  }
  return e;
}

hipError_t launch_query(const GraphDev& G, int dtype, int metric, const void* queries, int64_t Q, int k,
                        const SearchParams& sp, int every_layer, int32_t* ids, float* dists, uint32_t* counters,
                        hipStream_t stream, const Tuning& t) {
  const int slots = register_slots(sp, true, t);
  // wavefronts the GPU holds at once when the visited table is in LDS (at most 24 per compute unit): a
  // batch that fits gains nothing from a table in global memory, which is slower to probe
  const size_t lds_table = slots == 2 ? RegCache2Any::lds_bytes(sp) : RegCacheAny::lds_bytes(sp);
  const int64_t resident = (int64_t)cu_count() * (int64_t)(kMaxLds / lds_table < 24 ? kMaxLds / lds_table : 24);
  if (slots >= 1 && t.vis_min_iter > 0 && sp.max_iter >= t.vis_min_iter && (Q > resident || t.vis_forced)) {
    // long searches: one visited table per query in global memory, from the stream's memory pool
    const size_t bytes = (size_t)Q * (size_t)RegCacheGV::vis_slots(sp.max_iter) * sizeof(int32_t);
    int32_t* vis = nullptr;
    if (hipMallocAsync((void**)&vis, bytes, stream) == hipSuccess) {
      SearchParams spv = sp;
      spv.vis = vis;
      const hipError_t e = (G.addr32 ? launch_query_gv : launch_query_gv_wide)(slots, G, dtype, metric, queries, Q, k, spv, every_layer, ids, dists, counters, stream);
      const hipError_t f = hipFreeAsync(vis, stream);
      return e != hipSuccess ? e : f;
    }
    (void)hipGetLastError();  // no workspace: the table stays in LDS
  }
  const bool split = every_layer && G.L >= 3 && !sp.start && slots >= 1 && Q >= t.split_min;
  if (!split) return launch_query_whole(G, dtype, metric, queries, Q, k, sp, every_layer, ids, dists, counters, stream, t);
  // workspace from the stream's memory pool
  const SplitLayout lay = split_layout(G, slots, Q);
  unsigned char* ws = nullptr;
  if (hipMallocAsync((void**)&ws, lay.total, stream) != hipSuccess) {
    (void)hipGetLastError();  // no workspace: the one-launch path needs none
    return launch_query_whole(G, dtype, metric, queries, Q, k, sp, every_layer, ids, dists, counters, stream, t);
  }
  const hipError_t e = launch_query_two(G, dtype, metric, queries, Q, k, sp, slots, ids, dists, counters, ws, lay, stream);
  const hipError_t f = hipFreeAsync(ws, stream);
  return e != hipSuccess ? e : f;
}
hipError_t launch_merge(const GraphDev& G, int dtype, int metric, int l_top, int l_m, const SearchParams& sp,
                        int32_t* out_rows, float* dnn1, unsigned long long* work, hipStream_t stream, const Tuning& t) {
  if (register_slots(sp, false, t) != 1) return launch_merge_lds(G, dtype, metric, l_top, l_m, sp, out_rows, dnn1, work, stream);
  return (G.addr32 ? launch_merge_reg : launch_merge_reg_wide)(G, dtype, metric, l_top, l_m, sp, out_rows, dnn1, work, stream);
}
hipError_t launch_sym_search(const GraphDev& G, int dtype, int metric, int layer, int round, float w_mid,
                             const SearchParams& sp, const SymBuffers& sb, unsigned long long* work,
                             hipStream_t stream, const Tuning& t) {
  if (register_slots(sp, false, t) != 1) return launch_sym_search_lds(G, dtype, metric, layer, round, w_mid, sp, sb, work, stream);
  return (G.addr32 ? launch_sym_search_reg : launch_sym_search_reg_wide)(G, dtype, metric, layer, round, w_mid, sp, sb, work, stream);
}

void release_sym_buffers(ggnn_graph* g);
int ensure_sym_buffers(ggnn_graph* g) {
  if (g->sb_ready) return GGNN_OK;
  const int64_t n = g->n[0];
  const int ksym = g->K - g->K / 2;
  SymBuffers& sb = g->sb;
  sb = SymBuffers{};
  const hipError_t e = [&]() -> hipError_t {
    hipError_t r;
#define SYM_ALLOC(field, bytes) \
    if ((r = hipMalloc(&sb.field, (bytes))) != hipSuccess) return r
    SYM_ALLOC(inv, sizeof(int32_t) * n * ksym);
    SYM_ALLOC(ninv, sizeof(int32_t) * n);
    SYM_ALLOC(pref, sizeof(u64) * n * g->K);
    SYM_ALLOC(npref, sizeof(int32_t) * n);
    SYM_ALLOC(ptr, sizeof(int32_t) * n);
    SYM_ALLOC(state, sizeof(int32_t) * n);
    SYM_ALLOC(hold, sizeof(int32_t) * n * ksym);
    SYM_ALLOC(nhold, sizeof(int32_t) * n);
    SYM_ALLOC(head, sizeof(int32_t) * n);
    SYM_ALLOC(next, sizeof(int32_t) * n);
    SYM_ALLOC(pending, sizeof(int32_t));
#undef SYM_ALLOC
    return hipSuccess;
  }();
  if (e != hipSuccess) {
    release_sym_buffers(g);  // what was allocated before the failure is returned
    return fail(e == hipErrorOutOfMemory ? GGNN_ERR_MEMORY : GGNN_ERR_HIP, "buffers of the symmetric linking: %s", hipGetErrorString(e));
  }
  g->sb_ready = true;
  return GGNN_OK;
}

void release_sym_buffers(ggnn_graph* g) {
  SymBuffers& sb = g->sb;
  hipFree(sb.inv); hipFree(sb.ninv); hipFree(sb.pref); hipFree(sb.npref); hipFree(sb.ptr); hipFree(sb.state);
  hipFree(sb.hold); hipFree(sb.nhold); hipFree(sb.head); hipFree(sb.next); hipFree(sb.pending);
  sb = SymBuffers{};
  g->sb_ready = false;
}

struct PhaseTimer {
  hipEvent_t a = nullptr, b = nullptr;
  hipStream_t st;
  explicit PhaseTimer(hipStream_t s) : st(s) {
    hipEventCreate(&a);
    hipEventCreate(&b);
    hipEventRecord(a, st);
  }
  float stop() {
    float ms = 0.0f;
    hipEventRecord(b, st);
    hipEventSynchronize(b);
    hipEventElapsedTime(&ms, a, b);
    return ms;
  }
  ~PhaseTimer() {
    hipEventDestroy(a);
    hipEventDestroy(b);
  }
};

}  // namespace

extern "C" {

const char* ggnn_last_error(void) { return g_err; }

int ggnn_merge_shards(int32_t S, int64_t Q, int32_t k, const int32_t* ids_dev, const float* dists_dev,
                      const int32_t* offsets_dev, int32_t* out_ids_dev, float* out_dists_dev, void* stream,
                      int32_t asynchronous) {
  if (S < 1 || k < 1 || Q < 0) return fail(GGNN_ERR_INVALID, "S, k must be positive and Q not negative");
  if (Q > 0x7FFFFFFFll) return fail(GGNN_ERR_INVALID, "Q too large");
  if (Q == 0) return GGNN_OK;
  if (!ids_dev || !dists_dev || !offsets_dev || !out_ids_dev || !out_dists_dev) return fail(GGNN_ERR_INVALID, "NULL device pointer");
  if ((size_t)S * k * 8 > kMaxLds) return fail(GGNN_ERR_LIMIT, "S * k = %lld keys do not fit one workgroup's LDS", (long long)S * k);
  HIP_TRY(launch_merge_shards(S, Q, k, ids_dev, dists_dev, offsets_dev, out_ids_dev, out_dists_dev, (hipStream_t)stream));
  if (!asynchronous) HIP_TRY(hipStreamSynchronize((hipStream_t)stream));
  return GGNN_OK;
}

int ggnn_gather_probe(const void* rows_dev, int64_t n_rows, int32_t row_bytes, const int32_t* ids_dev, int64_t n_ids,
                      int32_t rows_per_wave, uint32_t* out_dev, void* stream) {
  if (!rows_dev || !ids_dev || !out_dev) return fail(GGNN_ERR_INVALID, "NULL device pointer");
  if (row_bytes < 16 || row_bytes % 16 != 0 || row_bytes > 512) return fail(GGNN_ERR_INVALID, "row_bytes %d not a multiple of 16 in [16, 512]", row_bytes);
  if (n_rows < 1 || n_ids < 1 || rows_per_wave < 1) return fail(GGNN_ERR_INVALID, "sizes must be positive");
  HIP_TRY(launch_gather_probe(rows_dev, row_bytes, ids_dev, n_ids, rows_per_wave, out_dev, (hipStream_t)stream));
  return GGNN_OK;
}

int ggnn_set_cache_mode(int32_t mode) {
  if (mode != 0 && mode != 1) return fail(GGNN_ERR_INVALID, "cache mode %d is neither 0 nor 1", mode);
  g_cache_mode.store(mode);
  return GGNN_OK;
}

int ggnn_set_split_threshold(int64_t min_queries) {
  if (min_queries < 0) return fail(GGNN_ERR_INVALID, "min_queries = %lld is negative", (long long)min_queries);
  g_split_min_queries.store(min_queries == 0 ? kSplitMinQueries : min_queries);
  return GGNN_OK;
}

int ggnn_set_global_visited_threshold(int32_t min_iter) {
  g_vis_global_min_iter.store(min_iter == 0 ? kVisGlobalMinIter : min_iter);  // negative: never
  g_vis_global_forced.store(min_iter > 0);
  return GGNN_OK;
}

void ggnn_free(ggnn_graph* g) {
  if (!g) return;
  for (int l = 0; l < kMaxLevels; l++) {
    hipFree(g->edges[l]); hipFree(g->to_lower[l]); hipFree(g->to_base[l]); hipFree(g->inv_count[l]);
  }
  hipFree(g->edge_tmp); hipFree(g->dnn1); hipFree(g->stats_dev); hipFree(g->stats_partial); hipFree(g->norm); hipFree(g->work_dev);
  release_sym_buffers(g);
  delete g;
}

int ggnn_graph_create(const void* base_dev, int64_t N, int32_t D, int32_t K, int32_t levels, uint64_t seed,
                      const ggnn_build_params* p, ggnn_graph** out) {
  if (!out) return fail(GGNN_ERR_INVALID, "out is NULL");
  *out = nullptr;
  if (!base_dev) return fail(GGNN_ERR_INVALID, "base_dev is NULL");
  ggnn_build_params dflt;
  memset(&dflt, 0, sizeof(dflt));
  if (!p) p = &dflt;
  const int dtype = p->dtype, metric = p->metric;
  if (dtype != GGNN_F32 && dtype != GGNN_U8) return fail(GGNN_ERR_INVALID, "unknown dtype %d", dtype);
  if (metric != GGNN_L2 && metric != GGNN_COSINE) return fail(GGNN_ERR_INVALID, "unknown metric %d", metric);
  if (metric == GGNN_COSINE && dtype != GGNN_F32) return fail(GGNN_ERR_INVALID, "cosine distance needs float32 rows");
  const int s = p->segment_size ? p->segment_size : 32;
  if (s < 2 || s > kWave) return fail(GGNN_ERR_INVALID, "segment_size %d outside [2, 64]", s);
  if (K < 2 || K > kWave) return fail(GGNN_ERR_INVALID, "K = %d outside [2, 64]", K);
  if (levels < 2 || levels > kMaxLevels) return fail(GGNN_ERR_INVALID, "levels = %d outside [2, %d]", levels, kMaxLevels);
  if (N < 2 || N > 0x7FFFFFFFll) return fail(GGNN_ERR_INVALID, "N = %lld outside [2, 2^31)", (long long)N);
  const int esize = dtype == GGNN_F32 ? 4 : 1;
  if (D < 1 || (D * esize) % 16 != 0) return fail(GGNN_ERR_INVALID, "a row of D = %d elements is not a multiple of 16 bytes", D);
  if ((dtype == GGNN_F32 && D > 1024) || (dtype == GGNN_U8 && D > 256))
    return fail(GGNN_ERR_INVALID, "D = %d too large (float32: <= 1024, uint8: <= 256)", D);
  if (((uintptr_t)base_dev) % 16 != 0) return fail(GGNN_ERR_INVALID, "base_dev is not 16-byte aligned");
  ggnn_graph* g = new (std::nothrow) ggnn_graph();
  if (!g) return fail(GGNN_ERR_MEMORY, "host allocation failed");
  g->N = N; g->D = D; g->K = K; g->L = levels; g->s = s; g->dtype = dtype; g->metric = metric; g->seed = seed;
  g->base = base_dev;
  g->stream = (hipStream_t)p->stream;
  g->tau_build = p->tau_build > 0.0f ? p->tau_build : 0.5f;
  g->refinements = p->refinements < 0 ? 0 : (p->refinements == 0 ? 2 : p->refinements);
  g->pq_cap = p->pq_cap > 0 ? p->pq_cap : 64;
  g->visited_cap = p->visited_cap > 0 ? p->visited_cap : 384;
  g->max_iter = p->max_iter > 0 ? p->max_iter : g->visited_cap;
  g->w_mid = p->no_sym_constraint ? 0.0f : 0.4f;
  if (geometry(N, s, levels, &g->g, g->n, g->G) != 0) {
    delete g;
    return fail(GGNN_ERR_INVALID, "N = %lld, s = %d, levels = %d admit no hierarchy", (long long)N, s, levels);
  }
  if ((N + g->G[0] - 1) / g->G[0] > kWave) {
    delete g;
    return fail(GGNN_ERR_INVALID, "bottom segments would hold more than 64 points");
  }
  SearchParams sp;
  int rc = make_search_params(K, g->pq_cap, g->visited_cap, g->max_iter, g->tau_build, 0.0f, &sp, process_tuning());
  if (rc != GGNN_OK) { delete g; return rc; }

#define CREATE_TRY(expr)                                                                   \
  do {                                                                                     \
    hipError_t e_ = (expr);                                                                \
    if (e_ != hipSuccess) {                                                                \
      ggnn_free(g);                                                                        \
      return fail(e_ == hipErrorOutOfMemory ? GGNN_ERR_MEMORY : GGNN_ERR_HIP, "%s: %s", #expr, hipGetErrorString(e_)); \
    }                                                                                      \
  } while (0)
  for (int l = 0; l < levels; l++) {
    const int64_t cnt = g->n[l] * K;
    CREATE_TRY(hipMalloc(&g->edges[l], sizeof(int32_t) * cnt));
    CREATE_TRY(launch_fill_i32(g->edges[l], cnt, -1, g->stream));
    CREATE_TRY(hipMalloc(&g->inv_count[l], sizeof(int32_t) * g->n[l]));
    CREATE_TRY(launch_fill_i32(g->inv_count[l], g->n[l], 0, g->stream));
    if (l >= 1) {
      CREATE_TRY(hipMalloc(&g->to_lower[l], sizeof(int32_t) * g->n[l]));
      CREATE_TRY(hipMalloc(&g->to_base[l], sizeof(int32_t) * g->n[l]));
      CREATE_TRY(launch_fill_i32(g->to_lower[l], g->n[l], 0, g->stream));
      CREATE_TRY(launch_fill_i32(g->to_base[l], g->n[l], 0, g->stream));
    }
  }
  CREATE_TRY(hipMalloc(&g->edge_tmp, sizeof(int32_t) * N * K));
  CREATE_TRY(hipMalloc(&g->dnn1, sizeof(float) * N));
  CREATE_TRY(launch_fill_i32((int32_t*)g->dnn1, N, 0, g->stream));
  CREATE_TRY(hipMalloc(&g->stats_dev, sizeof(float) * 2));
  CREATE_TRY(hipMalloc(&g->stats_partial, sizeof(double) * 2 * 1024));
  CREATE_TRY(hipMalloc(&g->work_dev, sizeof(unsigned long long) * 8 * kWorkSlots));
  CREATE_TRY(launch_fill_i32((int32_t*)g->work_dev, 16 * kWorkSlots, 0, g->stream));
  if (metric == GGNN_COSINE) {
    CREATE_TRY(hipMalloc(&g->norm, sizeof(float) * N * D));
    CREATE_TRY(launch_normalise(base_dev, dtype, N, D, g->norm, g->stream));
  }
  CREATE_TRY(hipStreamSynchronize(g->stream));
#undef CREATE_TRY
  *out = g;
  return GGNN_OK;
}

int ggnn_select(ggnn_graph* g, int32_t l_top) {
  if (!g) return fail(GGNN_ERR_INVALID, "graph is NULL");
  if (l_top < 1 || l_top >= g->L) return fail(GGNN_ERR_INVALID, "l_top = %d outside [1, %d)", l_top, g->L);
  PhaseTimer t(g->stream);
  GraphDev G = device_view(g);
  HIP_TRY(launch_select(G, l_top, g->dnn1, g->to_lower[l_top], g->to_base[l_top], g->stream));
  HIP_TRY(hipStreamSynchronize(g->stream));
  g->times.select_ms += t.stop();
  return GGNN_OK;
}

int ggnn_merge(ggnn_graph* g, int32_t l_top, int32_t l_m) {
  if (!g) return fail(GGNN_ERR_INVALID, "graph is NULL");
  if (l_top < 0 || l_top >= g->L || l_m < 0 || l_m > l_top)
    return fail(GGNN_ERR_INVALID, "merge(%d, %d) outside the hierarchy", l_top, l_m);
  SearchParams sp;
  // during construction the mean first-neighbour distance stands in for the maximum (Eq. 4)
  const Tuning tune = process_tuning();
  int rc = make_search_params(g->K, g->pq_cap, g->visited_cap, g->max_iter, g->tau_build, g->stats[0], &sp, tune);
  if (rc != GGNN_OK) return rc;
  {
    PhaseTimer t(g->stream);
    GraphDev G = device_view(g);
    HIP_TRY(launch_merge(G, row_dtype(g), g->metric, l_top, l_m, sp, g->edge_tmp, g->dnn1, g->work_dev, g->stream, tune));
    // the buffer becomes the layer (inverse links of the layer are thereby discarded)
    HIP_TRY(hipMemcpyAsync(g->edges[l_m], g->edge_tmp, sizeof(int32_t) * g->n[l_m] * g->K, hipMemcpyDeviceToDevice, g->stream));
    HIP_TRY(launch_fill_i32(g->inv_count[l_m], g->n[l_m], 0, g->stream));
    HIP_TRY(hipStreamSynchronize(g->stream));
    g->times.merge_ms += t.stop();
  }
  if (l_m == 0) {
    PhaseTimer t(g->stream);
    HIP_TRY(launch_stats(g->dnn1, g->N, g->stats_partial, g->stats_dev, g->stream));
    HIP_TRY(hipMemcpyAsync(g->stats, g->stats_dev, sizeof(float) * 2, hipMemcpyDeviceToHost, g->stream));
    HIP_TRY(hipStreamSynchronize(g->stream));
    g->times.stats_ms += t.stop();
  }
  return GGNN_OK;
}

int ggnn_sym(ggnn_graph* g, int32_t layer) {
  if (!g) return fail(GGNN_ERR_INVALID, "graph is NULL");
  if (layer < 0 || layer >= g->L) return fail(GGNN_ERR_INVALID, "layer %d outside [0, %d)", layer, g->L);
  int rc = ensure_sym_buffers(g);
  if (rc != GGNN_OK) return rc;
  SearchParams sp;
  const Tuning tune = process_tuning();
  rc = make_search_params(g->K, g->pq_cap, g->visited_cap, g->max_iter, g->tau_build, g->stats[0], &sp, tune);
  if (rc != GGNN_OK) return rc;
  PhaseTimer t(g->stream);
  GraphDev G = device_view(g);
  const SymBuffers& sb = g->sb;
  const int64_t n = g->n[layer];
  const int knn = g->K / 2;
  HIP_TRY(launch_fill_i32(sb.ninv, n, 0, g->stream));
  HIP_TRY(launch_fill_i32(sb.nhold, n, 0, g->stream));
  HIP_TRY(launch_fill_i32(sb.head, n, -1, g->stream));
  for (int round = 0; round < knn; round++) {
    HIP_TRY(launch_sym_search(G, row_dtype(g), g->metric, layer, round, g->w_mid, sp, sb, g->work_dev, g->stream, tune));
    // propose / resolve until a resolve pass turns nobody away.  The host looks at the count of the
    // last of kSymRoundsPerCheck passes only: once a pass has no losers nobody is proposing any more, so
    // the passes after it change nothing and count nothing.
    constexpr int kSymRoundsPerCheck = 4;
    bool first = true;
    for (;;) {
      for (int i = 0; i < kSymRoundsPerCheck; i++) {
        HIP_TRY(launch_fill_i32(sb.pending, 1, 0, g->stream));
        if (first) HIP_TRY(launch_sym_propose_first(G, layer, sb, sp.B, g->stream));
        else HIP_TRY(launch_sym_propose(G, layer, sb, sp.B, g->stream));
        first = false;
        HIP_TRY(launch_sym_resolve(G, layer, sb, sp.B, g->stream));
      }
      int32_t pending = 0;
      HIP_TRY(hipMemcpyAsync(&pending, sb.pending, sizeof(int32_t), hipMemcpyDeviceToHost, g->stream));
      HIP_TRY(hipStreamSynchronize(g->stream));
      if (pending == 0) break;
    }
    HIP_TRY(launch_sym_commit(G, layer, sb, g->stream));
  }
  HIP_TRY(launch_sym_apply(G, layer, sb, g->edges[layer], g->inv_count[layer], g->stream));
  HIP_TRY(hipStreamSynchronize(g->stream));
  g->times.sym_ms += t.stop();
  return GGNN_OK;
}

int ggnn_build_set_progress(ggnn_graph* g, ggnn_progress_fn cb, void* user) {
  if (!g) return fail(GGNN_ERR_INVALID, "graph is NULL");
  g->progress = cb;
  g->progress_user = user;
  return GGNN_OK;
}

int ggnn_build_steps(ggnn_graph* g) {
  if (!g) return fail(GGNN_ERR_INVALID, "graph is NULL");
  g->times = ggnn_build_times{};
  HIP_TRY(launch_fill_i32((int32_t*)g->work_dev, 16 * kWorkSlots, 0, g->stream));
  PhaseTimer total(g->stream);
  const auto t0 = std::chrono::steady_clock::now();
  // one step of the sequence, reported to the progress callback once its work is done
  auto step = [&](const char* name, int l_top, int l_m, int rc) -> int {
    if (rc != GGNN_OK || !g->progress) return rc;
    if (hipStreamSynchronize(g->stream) != hipSuccess) return fail(GGNN_ERR_HIP, "hipStreamSynchronize failed after a construction step");
    g->progress(name, l_top, l_m, std::chrono::duration<double>(std::chrono::steady_clock::now() - t0).count(), g->progress_user);
    return GGNN_OK;
  };
  int rc;
  for (int l_top = 0; l_top < g->L; l_top++) {
    if (l_top > 0 && (rc = step("select", l_top, -1, ggnn_select(g, l_top))) != GGNN_OK) return rc;
    for (int l_m = l_top; l_m >= 0; l_m--) {
      if ((rc = step("merge", l_top, l_m, ggnn_merge(g, l_top, l_m))) != GGNN_OK) return rc;
      if ((rc = step("sym", -1, l_m, ggnn_sym(g, l_m))) != GGNN_OK) return rc;
    }
  }
  for (int r = 0; r < g->refinements; r++) {
    for (int l_m = g->L - 2; l_m >= 0; l_m--) {
      if ((rc = step("merge", g->L - 1, l_m, ggnn_merge(g, g->L - 1, l_m))) != GGNN_OK) return rc;
      if ((rc = step("sym", -1, l_m, ggnn_sym(g, l_m))) != GGNN_OK) return rc;
    }
  }
  g->times.total_ms = total.stop();
  std::vector<unsigned long long> w(8 * kWorkSlots);
  HIP_TRY(hipMemcpy(w.data(), g->work_dev, sizeof(unsigned long long) * w.size(), hipMemcpyDeviceToHost));
  for (int i = 0; i < kWorkSlots; i++) {
    g->times.merge_pops += w[8 * i + 0]; g->times.merge_rows += w[8 * i + 1];
    g->times.sym_pops += w[8 * i + 2]; g->times.sym_rows += w[8 * i + 3];
  }
  release_sym_buffers(g);  // the construction buffers are not needed for queries
  return GGNN_OK;
}

int ggnn_build_ex(const void* base_dev, int64_t N, int32_t D, int32_t K, int32_t levels, uint64_t seed,
                  const ggnn_build_params* p, ggnn_graph** out) {
  int rc = ggnn_graph_create(base_dev, N, D, K, levels, seed, p, out);
  if (rc != GGNN_OK) return rc;
  rc = ggnn_build_steps(*out);
  if (rc != GGNN_OK) {
    ggnn_free(*out);
    *out = nullptr;
    return rc;
  }
  return GGNN_OK;
}

int ggnn_build(const float* base_dev, int64_t N, int32_t D, int32_t K, int32_t levels, uint64_t seed,
               ggnn_graph** out) {
  return ggnn_build_ex(base_dev, N, D, K, levels, seed, nullptr, out);
}

int ggnn_build_get_times(const ggnn_graph* g, ggnn_build_times* out) {
  if (!g || !out) return fail(GGNN_ERR_INVALID, "NULL argument");
  *out = g->times;
  return GGNN_OK;
}

static int query_impl(const ggnn_graph* g, const void* queries_dev, int64_t Q, int32_t k, int32_t beam, float slack,
                      int32_t pq_cap, int32_t visited_cap, int32_t max_iter, int32_t every_layer,
                      const int32_t* start_ids_dev, int32_t n_start, void* stream, int32_t* ids_dev, float* dists_dev,
                      uint32_t* counters_dev, int32_t asynchronous, const Tuning& tune) {
  if (!g) return fail(GGNN_ERR_INVALID, "graph is NULL");
  if (Q < 0 || Q > 0x7FFFFFFFll) return fail(GGNN_ERR_INVALID, "Q = %lld outside [0, 2^31)", (long long)Q);
  if (Q == 0) return GGNN_OK;
  if (!queries_dev || !ids_dev || !dists_dev) return fail(GGNN_ERR_INVALID, "NULL device pointer");
  if (((uintptr_t)queries_dev) % 16 != 0) return fail(GGNN_ERR_INVALID, "queries_dev is not 16-byte aligned");
  if (k < 1) return fail(GGNN_ERR_INVALID, "k = %d must be positive", k);
  if (beam < 0 || !(slack >= 0.0f)) return fail(GGNN_ERR_INVALID, "beam and slack must not be negative");
  const int B = beam > k ? beam : k;
  const int P = pq_cap > 0 ? pq_cap : 64;
  const int V = visited_cap > 0 ? visited_cap : (B >= 100 ? 896 : 384);
  const int it = max_iter > 0 ? max_iter : V;
  SearchParams sp;
  // user queries bound the slack by the maximum first-neighbour distance (Eq. 2, Eq. 3)
  int rc = make_search_params(B, P, V, it, slack, g->stats[1], &sp, tune, true);
  if (rc != GGNN_OK) return rc;
  hipStream_t st = stream ? (hipStream_t)stream : g->stream;
  if (start_ids_dev) {
    if (n_start < 1 || n_start > kWave) return fail(GGNN_ERR_INVALID, "n_start = %d outside [1, 64]", n_start);
    // the kernel trusts the start points: check them here (a small synchronous copy)
    int32_t host[kWave];
    HIP_TRY(hipMemcpy(host, start_ids_dev, sizeof(int32_t) * n_start, hipMemcpyDeviceToHost));
    for (int i = 0; i < n_start; i++) {
      if (host[i] < 0 || host[i] >= g->N) return fail(GGNN_ERR_INVALID, "start point %d = %d outside [0, N)", i, host[i]);
      for (int j = 0; j < i; j++)
        if (host[j] == host[i]) return fail(GGNN_ERR_INVALID, "start point %d is listed twice", host[i]);
    }
    sp.start = start_ids_dev;
    sp.n_start = n_start;
  }
  GraphDev G = device_view(g);
  if (g->metric == GGNN_COSINE && g->dtype != GGNN_F32) return fail(GGNN_ERR_INVALID, "cosine needs float32 queries");
  HIP_TRY(launch_query(G, row_dtype(g), g->metric, queries_dev, Q, k, sp, every_layer ? 1 : 0, ids_dev, dists_dev,
                       counters_dev, st, tune));
  if (!asynchronous) HIP_TRY(hipStreamSynchronize(st));
  return GGNN_OK;
}

int ggnn_query_ex(const ggnn_graph* g, const void* queries_dev, int64_t Q, int32_t k, int32_t beam, float slack,
                  int32_t pq_cap, int32_t visited_cap, int32_t max_iter, int32_t every_layer, void* stream,
                  int32_t* ids_dev, float* dists_dev, uint32_t* counters_dev, int32_t asynchronous) {
  return query_impl(g, queries_dev, Q, k, beam, slack, pq_cap, visited_cap, max_iter, every_layer, nullptr, 0, stream,
                    ids_dev, dists_dev, counters_dev, asynchronous, process_tuning());
}

int ggnn_query_with(const ggnn_graph* g, const void* queries_dev, int64_t Q, int32_t k, int32_t beam, float slack,
                    const ggnn_query_params* p, int32_t* ids_dev, float* dists_dev, uint32_t* counters_dev) {
  ggnn_query_params dflt;
  memset(&dflt, 0, sizeof(dflt));
  if (!p) p = &dflt;
  if (p->cache_mode != 0 && p->cache_mode != 1) return fail(GGNN_ERR_INVALID, "cache_mode %d is neither 0 nor 1", p->cache_mode);
  Tuning tune;
  tune.cache_mode = p->cache_mode;
  tune.split_min = p->split_min_queries == 0 ? kSplitMinQueries : (p->split_min_queries < 0 ? INT64_MAX : p->split_min_queries);
  tune.vis_min_iter = p->global_visited_min_iter == 0 ? kVisGlobalMinIter : p->global_visited_min_iter;
  tune.vis_forced = p->global_visited_min_iter > 0;
  if (p->start_ids_dev == nullptr && p->n_start != 0) return fail(GGNN_ERR_INVALID, "n_start = %d without start_ids_dev", p->n_start);
  return query_impl(g, queries_dev, Q, k, beam, slack, p->pq_cap, p->visited_cap, p->max_iter,
                    p->start_ids_dev ? 0 : p->every_layer, p->start_ids_dev, p->n_start, p->stream, ids_dev, dists_dev,
                    counters_dev, p->asynchronous, tune);
}

int ggnn_query_from(const ggnn_graph* g, const void* queries_dev, int64_t Q, int32_t k, int32_t beam, float slack,
                    int32_t pq_cap, int32_t visited_cap, int32_t max_iter, const int32_t* start_ids_dev, int32_t n_start,
                    void* stream, int32_t* ids_dev, float* dists_dev, uint32_t* counters_dev, int32_t asynchronous) {
  if (!start_ids_dev) return fail(GGNN_ERR_INVALID, "start_ids_dev is NULL");
  return query_impl(g, queries_dev, Q, k, beam, slack, pq_cap, visited_cap, max_iter, 0, start_ids_dev, n_start, stream,
                    ids_dev, dists_dev, counters_dev, asynchronous, process_tuning());
}

int ggnn_query(const ggnn_graph* g, const void* queries_dev, int64_t Q, int32_t k, int32_t beam, float slack,
               int32_t* ids_dev, float* dists_dev) {
  return ggnn_query_ex(g, queries_dev, Q, k, beam, slack, 0, 0, 0, 0, nullptr, ids_dev, dists_dev, nullptr, 0);
}

int ggnn_query_static(const ggnn_graph* g, const void* queries_dev, int64_t Q, int32_t k, int32_t beam, float slack,
                      int32_t pq_cap, int32_t visited_cap, int32_t max_iter, void* stream, int32_t* ids_dev,
                      float* dists_dev, uint32_t* counters_dev, int32_t asynchronous) {
  if (!g) return fail(GGNN_ERR_INVALID, "graph is NULL");
  if (Q < 0 || Q > 0x7FFFFFFFll) return fail(GGNN_ERR_INVALID, "Q = %lld outside [0, 2^31)", (long long)Q);
  if (Q == 0) return GGNN_OK;
  if (!queries_dev || !ids_dev || !dists_dev) return fail(GGNN_ERR_INVALID, "NULL device pointer");
  if (((uintptr_t)queries_dev) % 16 != 0) return fail(GGNN_ERR_INVALID, "queries_dev is not 16-byte aligned");
  if (k < 1) return fail(GGNN_ERR_INVALID, "k = %d must be positive", k);
  if (beam < 0 || !(slack >= 0.0f)) return fail(GGNN_ERR_INVALID, "beam and slack must not be negative");
  if (g->L < 3) return fail(GGNN_ERR_INVALID, "the two-launch search needs at least three levels, the graph has %d", g->L);
  const int B = beam > k ? beam : k;
  const int P = pq_cap > 0 ? pq_cap : 64;
  const int V = visited_cap > 0 ? visited_cap : (B >= 100 ? 896 : 384);
  const int it = max_iter > 0 ? max_iter : V;
  if (P > kWave || B > 2 * kWave)
    return fail(GGNN_ERR_LIMIT, "the two-launch search keeps its lists in registers: prioq <= 64 and best <= 128 (got %d, %d)", P, B);
  SearchParams sp;
  Tuning tune = process_tuning();
  tune.cache_mode = 0;  // the lists live in registers here whatever the process-wide setting
  int rc = make_search_params(B, P, V, it, slack, g->stats[1], &sp, tune, true);
  if (rc != GGNN_OK) return rc;
  const int slots = B <= kWave ? 1 : 2;
  const size_t need_lds = slots == 1 ? RegCache::lds_bytes(sp) : RegCache2::lds_bytes(sp);
  if (need_lds > kMaxLds) return fail(GGNN_ERR_LIMIT, "an iteration limit of %d needs %zu bytes of LDS, limit %zu", it, need_lds, kMaxLds);
  GraphDev G = device_view(g);
  const SplitLayout lay = split_layout(G, slots, Q);
  if (lay.total > kScratchBytes)
    return fail(GGNN_ERR_LIMIT, "%lld queries need a workspace of %zu bytes; the static workspace holds %zu (about %lld queries)",
                (long long)Q, lay.total, kScratchBytes, (long long)(kScratchBytes / (lay.total / (size_t)Q + 1)));
  unsigned char* ws = nullptr;
  rc = scratch_ptr(&ws);
  if (rc != GGNN_OK) return rc;
  hipStream_t st = stream ? (hipStream_t)stream : g->stream;
  HIP_TRY(launch_query_two(G, row_dtype(g), g->metric, queries_dev, Q, k, sp, slots, ids_dev, dists_dev, counters_dev, ws, lay, st));
  if (!asynchronous) HIP_TRY(hipStreamSynchronize(st));
  return GGNN_OK;
}

int ggnn_graph_info(const ggnn_graph* g, ggnn_graph_desc* out) {
  if (!g || !out) return fail(GGNN_ERR_INVALID, "NULL argument");
  memset(out, 0, sizeof(*out));
  out->N = g->N; out->D = g->D; out->K = g->K; out->L = g->L; out->s = g->s; out->g = g->g;
  out->dtype = g->dtype; out->metric = g->metric; out->seed = g->seed;
  int64_t upper = 0;
  for (int l = 0; l < g->L; l++) {
    out->n[l] = g->n[l];
    if (l >= 1) upper += g->n[l];
  }
  out->dnn_mean = g->stats[0];
  out->dnn_max = g->stats[1];
  // appendix "Graph Size": edge lists, two translation tables per upper point, two scalars
  out->graph_bytes = ((g->N + upper) * g->K + 2 * upper + 2) * 4;
  return GGNN_OK;
}

int ggnn_graph_export(const ggnn_graph* g, int32_t layer, int32_t* edges_host, int32_t* to_lower_host,
                      int32_t* to_base_host) {
  if (!g) return fail(GGNN_ERR_INVALID, "graph is NULL");
  if (layer < 0 || layer >= g->L) return fail(GGNN_ERR_INVALID, "layer %d outside [0, %d)", layer, g->L);
  if ((to_lower_host || to_base_host) && layer == 0) return fail(GGNN_ERR_INVALID, "layer 0 has no translation tables");
  HIP_TRY(hipStreamSynchronize(g->stream));
  if (edges_host) HIP_TRY(hipMemcpy(edges_host, g->edges[layer], sizeof(int32_t) * g->n[layer] * g->K, hipMemcpyDeviceToHost));
  if (to_lower_host) HIP_TRY(hipMemcpy(to_lower_host, g->to_lower[layer], sizeof(int32_t) * g->n[layer], hipMemcpyDeviceToHost));
  if (to_base_host) HIP_TRY(hipMemcpy(to_base_host, g->to_base[layer], sizeof(int32_t) * g->n[layer], hipMemcpyDeviceToHost));
  return GGNN_OK;
}

int ggnn_graph_import(ggnn_graph* g, int32_t layer, const int32_t* edges_host, const int32_t* to_lower_host,
                      const int32_t* to_base_host) {
  if (!g) return fail(GGNN_ERR_INVALID, "graph is NULL");
  if (layer < 0 || layer >= g->L) return fail(GGNN_ERR_INVALID, "layer %d outside [0, %d)", layer, g->L);
  if ((to_lower_host || to_base_host) && layer == 0) return fail(GGNN_ERR_INVALID, "layer 0 has no translation tables");
  const int64_t n = g->n[layer];
  const int K = g->K;
  if (edges_host) {
    // the kernels rely on these properties: check them here, on the host
    for (int64_t i = 0; i < n; i++) {
      const int32_t* row = edges_host + i * K;
      bool ended = false;
      for (int a = 0; a < K; a++) {
        if (row[a] == -1) { ended = true; continue; }
        if (ended || row[a] < 0 || row[a] >= n || row[a] == i)
          return fail(GGNN_ERR_INVALID, "layer %d row %lld entry %d is invalid", layer, (long long)i, a);
        for (int b = 0; b < a; b++)
          if (row[b] == row[a]) return fail(GGNN_ERR_INVALID, "layer %d row %lld repeats id %d", layer, (long long)i, row[a]);
      }
    }
  }
  const int64_t n_below = layer >= 1 ? g->n[layer - 1] : 0;
  if (to_lower_host)
    for (int64_t i = 0; i < n; i++)
      if (to_lower_host[i] < 0 || to_lower_host[i] >= n_below) return fail(GGNN_ERR_INVALID, "to_lower[%lld] out of range", (long long)i);
  if (to_base_host)
    for (int64_t i = 0; i < n; i++)
      if (to_base_host[i] < 0 || to_base_host[i] >= g->N) return fail(GGNN_ERR_INVALID, "to_base[%lld] out of range", (long long)i);
  HIP_TRY(hipStreamSynchronize(g->stream));
  if (edges_host) HIP_TRY(hipMemcpy(g->edges[layer], edges_host, sizeof(int32_t) * n * K, hipMemcpyHostToDevice));
  if (to_lower_host) HIP_TRY(hipMemcpy(g->to_lower[layer], to_lower_host, sizeof(int32_t) * n, hipMemcpyHostToDevice));
  if (to_base_host) HIP_TRY(hipMemcpy(g->to_base[layer], to_base_host, sizeof(int32_t) * n, hipMemcpyHostToDevice));
  return GGNN_OK;
}

int ggnn_graph_export_dnn(const ggnn_graph* g, float* dnn1_host, float* mean, float* max) {
  if (!g) return fail(GGNN_ERR_INVALID, "graph is NULL");
  HIP_TRY(hipStreamSynchronize(g->stream));
  if (dnn1_host) HIP_TRY(hipMemcpy(dnn1_host, g->dnn1, sizeof(float) * g->N, hipMemcpyDeviceToHost));
  if (mean) *mean = g->stats[0];
  if (max) *max = g->stats[1];
  return GGNN_OK;
}

int ggnn_graph_import_dnn(ggnn_graph* g, const float* dnn1_host, float mean, float max) {
  if (!g) return fail(GGNN_ERR_INVALID, "graph is NULL");
  if (!(mean >= 0.0f) || !(max >= 0.0f)) return fail(GGNN_ERR_INVALID, "statistics must not be negative");
  HIP_TRY(hipStreamSynchronize(g->stream));
  if (dnn1_host) HIP_TRY(hipMemcpy(g->dnn1, dnn1_host, sizeof(float) * g->N, hipMemcpyHostToDevice));
  g->stats[0] = mean;
  g->stats[1] = max;
  return GGNN_OK;
}

int ggnn_graph_export_inv_count(const ggnn_graph* g, int32_t layer, int32_t* count_host) {
  if (!g || !count_host) return fail(GGNN_ERR_INVALID, "NULL argument");
  if (layer < 0 || layer >= g->L) return fail(GGNN_ERR_INVALID, "layer %d outside [0, %d)", layer, g->L);
  HIP_TRY(hipStreamSynchronize(g->stream));
  HIP_TRY(hipMemcpy(count_host, g->inv_count[layer], sizeof(int32_t) * g->n[layer], hipMemcpyDeviceToHost));
  return GGNN_OK;
}

}  // extern "C"
