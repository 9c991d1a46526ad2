/*
 * ggnn.h -- C ABI of the MI355X (gfx950) implementation of GGNN's hot path:
 * batched best-first search with a slack stopping rule over a hierarchical,
 * fixed-out-degree kNN graph, and the bottom-up graph construction that is driven
 * by the same search (Groh et al., "GGNN: Graph-based GPU Nearest Neighbor Search",
 * arxiv 1912.01059).
 *
 * Conventions
 *  - Every function returns 0 on success or a negative ggnn_status; it never aborts.
 *    ggnn_last_error() returns a thread-local description of the last failure.
 *  - Pointers named *_dev are device (HBM) pointers owned by the caller; pointers named
 *    *_host are host pointers owned by the caller.  The library never frees them.
 *  - Vectors are row-major, D elements per row, rows 16-byte aligned (D*sizeof(element)
 *    must be a multiple of 16).  Ids are int32 (N < 2^31); offsets into the graph's own arrays and into
 *    the vector array are 64-bit (arrays below 4 GiB are served by kernels that use 32-bit byte offsets).
 *  - `base_dev` is BORROWED by the graph and must outlive it (it is not copied, except
 *    that a cosine graph owns a unit-length float32 copy).
 *  - All work is issued on the stream given at creation (or per call for queries); calls
 *    return after the work has completed unless stated otherwise.
 *  - Distances are plain (not squared) Euclidean norms, or 1 - cos for GGNN_COSINE, in
 *    float32.  Every ordered result uses the total order (distance, id).
 *  - float32 sums follow one fixed order, so results are reproducible bit for bit: the
 *    row is cut into 16-byte chunks, chunk c belongs to lane c mod R, a lane accumulates
 *    acc = fma(t, t, acc) over its chunks in ascending order, and the R lanes are combined
 *    by a butterfly (distance R/2, ..., 2, 1).  R = GGNN_ROW_LANES for rows of at most 1024
 *    bytes (for cosine: of the float32 unit-length copy), GGNN_WIDE_ROW_LANES for longer rows.
 *  - Row lengths: a multiple of 16 bytes; float32 D <= 1024, uint8 D <= 256.  The vector array may have
 *    any size the GPU holds (the 12.8 GB of 10^8 x 128 uint8 rows included).
 */
#ifndef GGNN_H
#define GGNN_H
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define GGNN_MAX_LEVELS 8
#define GGNN_STATIC_SCRATCH_BYTES (128u << 20) /* workspace of ggnn_query_static, per GPU */
#define GGNN_ROW_LANES 8
#define GGNN_WIDE_ROW_LANES 64

typedef struct ggnn_graph ggnn_graph; /* opaque, owned by the library */

typedef enum { GGNN_L2 = 0, GGNN_COSINE = 1 } ggnn_metric;
typedef enum { GGNN_F32 = 0, GGNN_U8 = 1 } ggnn_dtype;

typedef enum {
  GGNN_OK = 0,
  GGNN_ERR_INVALID = -1, /* bad argument (null pointer, size out of range, ...) */
  GGNN_ERR_MEMORY = -2,  /* device or host allocation failed                    */
  GGNN_ERR_HIP = -3,     /* a HIP runtime call or kernel launch failed          */
  GGNN_ERR_LIMIT = -4    /* a capacity exceeds what one workgroup's LDS (or the static workspace) holds */
} ggnn_status;

/* Construction parameters (appendix "Choosing Search-Graph Construction Parameters").
 * A zero field selects the default given in brackets. */
typedef struct {
  int32_t metric;         /* ggnn_metric [GGNN_L2]                                     */
  int32_t dtype;          /* ggnn_dtype of base and queries [GGNN_F32]                 */
  int32_t segment_size;   /* s: points per segment and per top layer [32], <= 64.  The paper asks
                             for s > K/2; smaller s is accepted: rows then end in -1 until a merge
                             from a higher layer fills them                             */
  float tau_build;        /* slack factor tau_b of the construction searches [0.5]     */
  int32_t refinements;    /* r refinement passes (Alg. 6) [2]; pass -1 for none        */
  int32_t pq_cap;         /* prioq capacity of the construction searches [64]          */
  int32_t visited_cap;    /* visited capacity of the construction searches [384]       */
  int32_t max_iter;       /* iteration limit per layer [visited_cap]; <= visited_cap   */
  int32_t no_sym_constraint; /* 1 disables the midpoint constraint of Sec. 4.2.1 [0]   */
  void* stream;           /* hipStream_t for all work on this graph [default stream]   */
} ggnn_build_params;

typedef struct {
  int64_t N;                    /* base points                                         */
  int32_t D, K, L, s, g;        /* dims, out-degree, layers, segment size, growth      */
  int32_t dtype, metric;
  int64_t n[GGNN_MAX_LEVELS];   /* points per layer, n[0] = N, n[L-1] = s (Sec. 4.3)   */
  float dnn_mean, dnn_max;      /* mean / max first-neighbour distance (Eq. 3, Eq. 4)  */
  int64_t graph_bytes;          /* edges + translation tables + the two scalars        */
  uint64_t seed;
} ggnn_graph_desc;

/* Per-phase time of a build in milliseconds, measured with HIP events on the graph's
 * stream (cf. the paper's construction-time split, Sec. 5.2.2). */
typedef struct {
  float merge_ms, sym_ms, select_ms, stats_ms, total_ms;
  /* work done by the searches of the build: iterations (adjacency rows read) and base rows
   * gathered, for Merge and for the symmetric-linking queries */
  uint64_t merge_pops, merge_rows, sym_pops, sym_rows;
} ggnn_build_times;

/* ---- construction (Alg. 3: BuildGraph; Alg. 6: RefineGraph) ------------------------ */

/* Builds the whole hierarchy for float32 rows and L2 distance with default parameters.
 * base_dev: N x D float32, device.  K: out-degree (2 <= K <= 64).  levels: L >= 2.
 * seed: drives the bottom-layer partition and the top-layer selection.  *out receives a
 * graph to be released with ggnn_free. */
int ggnn_build(const float* base_dev, int64_t N, int32_t D, int32_t K, int32_t levels, uint64_t seed,
               ggnn_graph** out);

/* Same with explicit parameters (p may be NULL); base_dev has p->dtype elements. */
int ggnn_build_ex(const void* base_dev, int64_t N, int32_t D, int32_t K, int32_t levels, uint64_t seed,
                  const ggnn_build_params* p, ggnn_graph** out);

/* Step-wise construction.  ggnn_graph_create allocates an empty graph (all edges -1, no
 * tables); the steps below are exactly those ggnn_build_ex sequences:
 *   for l_top = 0..L-1: if l_top > 0 select(l_top); for l_m = l_top..0: merge(l_top, l_m); sym(l_m)
 *   then r times: for l_m = L-2..0: merge(L-1, l_m); sym(l_m)
 * ggnn_select (Sec. 4.1): fills layer l_top (l_top >= 1) with s points per segment, taken
 *   equally from the g child segments by weighted reservoir sampling with weight d_nn1.
 * ggnn_merge (Alg. 3 Merge, Alg. 4): replaces the rows of layer l_m by the K nearest
 *   neighbours found by searching from the top segment of layer l_top (exhaustively
 *   inside the own segment when l_top == l_m); on layer 0 also updates d_nn1 and the
 *   two statistics.
 * ggnn_sym (Alg. 5, Sec. 4.2): inserts up to K - K/2 inverse links per row of `layer`. */
int ggnn_graph_create(const void* base_dev, int64_t N, int32_t D, int32_t K, int32_t levels, uint64_t seed,
                      const ggnn_build_params* p, ggnn_graph** out);
int ggnn_select(ggnn_graph* g, int32_t l_top);
int ggnn_merge(ggnn_graph* g, int32_t l_top, int32_t l_m);
int ggnn_sym(ggnn_graph* g, int32_t layer);
int ggnn_build_steps(ggnn_graph* g); /* the sequence above on a created graph; frees the construction buffers
                                       * when it is done (a later ggnn_sym allocates them again) */

/* Progress of a long construction (minutes at 10^8 points).  `cb`, or NULL for none, is called by
 * ggnn_build_steps on the calling thread after every step, once the step's work has completed on
 * the graph's stream (so a construction with a callback waits for the stream after each step):
 * step is "select", "merge" or "sym" (a string that lives as long as the library), l_top / l_m are
 * the layers of the step (-1 where it has none), seconds the wall time since ggnn_build_steps began,
 * user is handed through.  The callback must not call into the library with this graph.  Host
 * pointers; the library keeps them until they are replaced or the graph is freed. */
typedef void (*ggnn_progress_fn)(const char* step, int32_t l_top, int32_t l_m, double seconds, void* user);
int ggnn_build_set_progress(ggnn_graph* g, ggnn_progress_fn cb, void* user);

/* Times of the last ggnn_build* / ggnn_build_steps on this graph. */
int ggnn_build_get_times(const ggnn_graph* g, ggnn_build_times* out);

/* ---- query (Alg. 1, Alg. 2, Eq. 2; Sec. 4.4) --------------------------------------- */

/* Answers Q queries.  queries_dev: Q x D elements of the graph's dtype, device.
 * k results per query; beam: length of the best list the stopping rule looks at (the
 * paper uses max(k, 10); the effective length is max(beam, k)); slack: tau_q of Eq. 2.
 * ids_dev / dists_dev: Q x k, device; row q holds the results ascending by (distance,
 * id), padded with id -1 / distance +inf.  Defaults: prioq 64, visited 384 (896 when
 * beam >= 100), iteration limit = visited capacity, search drops from the top layer
 * straight to the bottom layer (Sec. 4.4).  Runs on the graph's stream. */
int ggnn_query(const ggnn_graph* g, const void* queries_dev, int64_t Q, int32_t k, int32_t beam, float slack,
               int32_t* ids_dev, float* dists_dev);

/* Same with every cache capacity explicit (0 = default as above).
 * max_iter: iteration limit per layer, must be <= visited_cap so that visited never
 * forgets a point.  every_layer: 0 = Sec. 4.4 shortcut, 1 = search every layer on the way
 * down (Alg. 4).  stream: hipStream_t (NULL = the graph's stream).  counters_dev:
 * optional Q x 4 uint32 (device), per query: pops (iterations of Alg. 1); distance evaluations of
 * the method (Alg. 2 Fetch: a point counts again each time it is proposed while unknown to the
 * cache); base rows actually gathered (fewer: re-evaluations of rejected points are skipped); 0.
 * asynchronous != 0 returns right after the launch (no synchronisation).
 * Memory: a call allocates nothing, except that large batches (ggnn_set_split_threshold) and large
 * batches of long searches (ggnn_set_global_visited_threshold) take a workspace from the stream's memory
 * pool (hipMallocAsync / hipFreeAsync on `stream`) for the duration of the call; if the pool cannot
 * provide it, the call proceeds without it. */
int ggnn_query_ex(const ggnn_graph* g, const void* queries_dev, int64_t Q, int32_t k, int32_t beam, float slack,
                  int32_t pq_cap, int32_t visited_cap, int32_t max_iter, int32_t every_layer, void* stream,
                  int32_t* ids_dev, float* dists_dev, uint32_t* counters_dev, int32_t asynchronous);

/* The same search with everything that steers its dispatch passed per call (a zero field selects the
 * default; p may be NULL): nothing process-wide is read, so calls from several threads or streams do not
 * interfere.  The ggnn_set_* calls at the end of this header set the process-wide defaults that ggnn_query,
 * ggnn_query_ex and ggnn_query_from use instead. */
typedef struct {
  int32_t pq_cap, visited_cap, max_iter; /* as ggnn_query_ex                                               */
  int32_t every_layer;                   /* 0: Sec. 4.4 shortcut, 1: every layer (Alg. 4)                  */
  int32_t cache_mode;                    /* 0: best / prioq in registers when they fit, 1: always in LDS   */
  int32_t global_visited_min_iter;       /* as ggnn_set_global_visited_threshold (0 default, < 0 never)    */
  int64_t split_min_queries;             /* as ggnn_set_split_threshold (0 default, < 0 never two launches)*/
  const int32_t* start_ids_dev;          /* as ggnn_query_from, or NULL                                    */
  int32_t n_start;
  int32_t asynchronous;
  void* stream;                          /* hipStream_t, NULL = the graph's stream                         */
} ggnn_query_params;
int ggnn_query_with(const ggnn_graph* g, const void* queries_dev, int64_t Q, int32_t k, int32_t beam, float slack,
                    const ggnn_query_params* p, int32_t* ids_dev, float* dists_dev, uint32_t* counters_dev);

/* For callers that cannot allocate device memory: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  The every-layer search of ggnn_query_ex in its two-launch form
 * (upper layers; counting sort of the queries by the layer-1 point reached; bottom layer, one
 * contiguous part of the sorted order per XCD), with the workspace that ggnn_query_ex takes from the
 * stream's memory pool replaced by a static array of GGNN_STATIC_SCRATCH_BYTES that is part of the
 * library's code object (one copy per GPU, held until the process ends).  The call allocates and frees
 * nothing, issues kernels only (no memset, no copy) and gives the results and counters of
 * ggnn_query_ex(..., every_layer = 1, ...) bit for bit.
 * Limits (GGNN_ERR_LIMIT / GGNN_ERR_INVALID otherwise): the graph has at least three levels; prioq
 * <= 64 and max(beam, k) <= 128 (lists in registers); the workspace Q * (W * 512 + 40) + 512 + 4 *
 * (min(n[1], 65536) + 1) bytes, W = 2 for max(beam, k) <= 64 and 3 beyond, fits the array: about 126 000
 * queries for W = 2 and 84 000 for W = 3.
 * Every call on a GPU uses that GPU's one array, which keeps the last call's contents (nothing in it
 * needs clearing between calls: each call writes what it reads).  Calls that overlap in time on one GPU,
 * from any stream or thread, race on it: serialise them.  The device that holds the graph must be current.
 * Arguments as ggnn_query_ex; stream NULL = the graph's stream. */
int ggnn_query_static(const ggnn_graph* g, const void* queries_dev, int64_t Q, int32_t k, int32_t beam, float slack,
                      int32_t pq_cap, int32_t visited_cap, int32_t max_iter, void* stream, int32_t* ids_dev,
                      float* dists_dev, uint32_t* counters_dev, int32_t asynchronous);

/* Alg. 1 on the bottom layer alone, from start points the caller names instead of the top layer:
 * the search of a flat graph (import its rows as layer 0; the upper layers are not touched), or the
 * start-point comparison of the paper's appendix "Query Starting Points" (centroid, worst point).
 * start_ids_dev: n_start (1..64) distinct base rows, device.  Everything else as ggnn_query_ex. */
int ggnn_query_from(const ggnn_graph* g, const void* queries_dev, int64_t Q, int32_t k, int32_t beam, float slack,
                    int32_t pq_cap, int32_t visited_cap, int32_t max_iter, const int32_t* start_ids_dev, int32_t n_start,
                    void* stream, int32_t* ids_dev, float* dists_dev, uint32_t* counters_dev, int32_t asynchronous);

/* ---- sharding on one GPU (Sec. 4.5) -------------------------------------------------- */

/* Merges the answers S independent shards gave to the same Q queries.  ids_dev / dists_dev:
 * S x Q x k (shard-major), each list ascending and padded with id -1 as ggnn_query writes it;
 * offsets_dev: S int32, the global id of the first base row of each shard.  out_*_dev: Q x k, the
 * k best overall ascending by (distance, global id), padded with -1 / +inf.  S * k * 8 bytes must
 * fit one workgroup's LDS.  stream: hipStream_t; asynchronous != 0 returns after the launch. */
int ggnn_merge_shards(int32_t S, int64_t Q, int32_t k, const int32_t* ids_dev, const float* dists_dev,
                      const int32_t* offsets_dev, int32_t* out_ids_dev, float* out_dists_dev, void* stream,
                      int32_t asynchronous);

/* ---- graph access ------------------------------------------------------------------- */

int ggnn_graph_info(const ggnn_graph* g, ggnn_graph_desc* out);

/* Copies one layer to host arrays (any pointer may be NULL to skip it):
 * edges_host n[layer] x K; to_lower_host / to_base_host n[layer] (layer >= 1 only: index of
 * the point on the layer below, and its base row).  Layer-0 ids are base rows. */
int ggnn_graph_export(const ggnn_graph* g, int32_t layer, int32_t* edges_host, int32_t* to_lower_host,
                      int32_t* to_base_host);
/* Overwrites one layer from host arrays (NULL = leave as is).  Rows must hold distinct
 * ids in [0, n[layer]) followed only by -1 padding, and no self loop; tables must be in
 * range.  Anything else is rejected with GGNN_ERR_INVALID. */
int ggnn_graph_import(ggnn_graph* g, int32_t layer, const int32_t* edges_host, const int32_t* to_lower_host,
                      const int32_t* to_base_host);
/* d_nn1 per base row (N floats, host) and the two statistics derived from it. */
int ggnn_graph_export_dnn(const ggnn_graph* g, float* dnn1_host, float* mean, float* max);
int ggnn_graph_import_dnn(ggnn_graph* g, const float* dnn1_host, float mean, float max);
/* number of inverse links each row of `layer` holds after the last ggnn_sym (host, n[layer]) */
int ggnn_graph_export_inv_count(const ggnn_graph* g, int32_t layer, int32_t* count_host);

/* Where best and prioq live during a search: 0 (default) in registers whenever prioq holds at most
 * 64 entries and best at most 64 (128 for user queries), otherwise in LDS; 1 always in LDS.
 * Results do not depend on it.  Process-wide default (an atomic; every call reads it once at entry);
 * ggnn_query_with takes it per call. */
int ggnn_set_cache_mode(int32_t mode);

/* Batches of at least `min_queries` user queries that search every layer (register cache, three levels or
 * more) are answered in two launches: the upper layers, then the bottom layer with the queries ordered
 * by the layer-1 point each arrived at, one contiguous part of that order per XCD, so that queries of
 * one region share an L2 cache.  Results and counters do not depend on it; the workspace comes from the
 * stream's memory pool (hipMallocAsync) and is returned to it.  Default 12288; 0 restores the default, a
 * value above every batch size turns the two-launch path off.  Process-wide default, as above. */
int ggnn_set_split_threshold(int64_t min_queries);

/* Where user queries keep their visited set.  By default (min_iter = 0) in LDS, except for batches
 * with an iteration limit (max_iter) of 1100 and more that are larger than the number of wavefronts
 * the GPU holds at once with such a table in LDS: those use one table per query in global memory
 * (taken from the stream's memory pool for the duration of the call), which is slower to probe but
 * leaves room for six wavefronts per SIMD.  min_iter > 0: global memory for every batch whose limit
 * is at least min_iter; min_iter < 0: always LDS.  Results and counters do not depend on it (Alg. 2
 * only asks that visited be exact).  Process-wide default, as above.  Returns GGNN_OK. */
int ggnn_set_global_visited_threshold(int32_t min_iter);

/* Measurement aid (not part of the method): gathers rows ids_dev[0..n_ids) (each in [0, n_rows), not
 * checked) of rows_dev (row_bytes per row, multiple of 16, <= 512) with the search kernels' access
 * pattern, rows_per_wave rows per wavefront, and writes one word per lane to out_dev
 * (ceil(n_ids / rows_per_wave) * 64 uint32).  Asynchronous on `stream`.  Timing it gives the rate at
 * which this GPU can serve the random row gathers the search performs. */
int ggnn_gather_probe(const void* rows_dev, int64_t n_rows, int32_t row_bytes, const int32_t* ids_dev, int64_t n_ids,
                      int32_t rows_per_wave, uint32_t* out_dev, void* stream);

void ggnn_free(ggnn_graph* g);
const char* ggnn_last_error(void);

#ifdef __cplusplus
}
#endif
#endif
