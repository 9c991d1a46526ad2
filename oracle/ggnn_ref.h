/*
 * ggnn_ref.h -- CPU oracle for the GGNN hot path (arxiv 1912.01059).
 *
 * TEST INFRASTRUCTURE ONLY.  This is the plain, slow, scalar reference the HIP
 * library is checked against.  It shares no code with the HIP path and nothing in
 * the product path may call it; only tests, the smoke check and the CPU-baseline
 * leg of the benchmark do.
 *
 * What it computes (all host pointers, row-major, caller-owned unless stated):
 *   - exact k nearest neighbours by exhaustive search (Sec. 3.1, Eq. 1);
 *   - the hierarchy geometry (Sec. 4.3; appendix "Graph Size");
 *   - the cache state machine best / prioq / visited with the slack stopping rule
 *     (Alg. 1, Alg. 2, Eq. 2) and the hierarchical query (Alg. 4, Sec. 4.4);
 *   - the bottom-up construction: partition, merge, stats, select, symmetric
 *     linking, refinement (Alg. 3, Alg. 5, Alg. 6, Sec. 4.1-4.3).
 *
 * Order everywhere is the total order on (distance as float32, id).
 */
#ifndef GGNN_REF_H
#define GGNN_REF_H
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum { GGNN_REF_L2 = 0, GGNN_REF_COSINE = 1 };
enum { GGNN_REF_F32 = 0, GGNN_REF_U8 = 1 };
#define GGNN_REF_MAX_LEVELS 8

typedef struct ggnn_ref_graph ggnn_ref_graph;

typedef struct {
  float tau_build;   /* slack factor tau_b used by merge and sym searches      */
  int refinements;   /* r, number of refinement passes (Alg. 6)                */
  int pq_cap;        /* prioq capacity of the construction searches           */
  int visited_cap;   /* visited capacity of the construction searches         */
  int max_iter;      /* iteration limit per layer of the construction searches */
  int sym_constraint;/* 1: midpoint constraint of Sec. 4.2.1, 0: centre on z  */
} ggnn_ref_build_params;

/* Hierarchy geometry (Sec. 4.3, appendix "Graph Size").  Writes the growth factor,
 * the point count n[l] and the segment count G[l] of every layer l (0 = bottom).
 * Returns 0, or -1 if the inputs admit no valid hierarchy. */
int ggnn_ref_geometry(int64_t N, int s, int L, int32_t* g, int64_t* n, int64_t* G);

/* Seeded bijection of [0,N) that defines the bottom-layer partition: position p of
 * the partition order holds base row perm(p).  inv is its inverse. */
int64_t ggnn_ref_perm(uint64_t seed, int64_t N, int64_t p);
int64_t ggnn_ref_perm_inv(uint64_t seed, int64_t N, int64_t row);
/* uniform in (0,1) drawn for base row `row` when layer l_top is selected */
double ggnn_ref_uniform(uint64_t seed, int l_top, int64_t row);

/* Distance between a float32 query and one base row (Eq. 1; cosine: 1 - <q,x> on
 * unit vectors).  `lanes` fixes the float32 summation tree (see ggnn_ref.c). */
float ggnn_ref_distance(const float* q, const void* row, int D, int dtype, int metric, int lanes);

/* Exhaustive search.  queries have the dtype of base.  ids/dists are Q*k, ascending
 * by (distance, id).  For cosine, rows and queries are normalised first. */
int ggnn_ref_bruteforce(const void* base, int64_t N, int D, int dtype, int metric, int lanes,
                        const void* queries, int64_t Q, int k, int32_t* ids, float* dists);

/* Graph object: owns edges and tables; borrows base (must outlive the graph), except
 * that for cosine it owns a normalised float32 copy. */
ggnn_ref_graph* ggnn_ref_graph_create(const void* base, int64_t N, int D, int K, int L, int s,
                                      int dtype, int metric, uint64_t seed, int lanes);
void ggnn_ref_graph_free(ggnn_ref_graph* g);
int32_t  ggnn_ref_graph_g(const ggnn_ref_graph* g);
int64_t  ggnn_ref_graph_n(const ggnn_ref_graph* g, int layer);
int32_t* ggnn_ref_graph_edges(ggnn_ref_graph* g, int layer);     /* n[l]*K               */
int32_t* ggnn_ref_graph_to_lower(ggnn_ref_graph* g, int layer);  /* n[l], layer >= 1     */
int32_t* ggnn_ref_graph_to_base(ggnn_ref_graph* g, int layer);   /* n[l], layer >= 1     */
float*   ggnn_ref_graph_dnn1(ggnn_ref_graph* g);                 /* N                    */
float*   ggnn_ref_graph_stats(ggnn_ref_graph* g);                /* [0]=mean, [1]=max    */
const float* ggnn_ref_graph_normalised(const ggnn_ref_graph* g); /* cosine only, else 0  */

/* Construction steps (Alg. 3, 5, 6).  Each returns 0 or a negative error. */
int ggnn_ref_select(ggnn_ref_graph* g, int l_top);
int ggnn_ref_merge(ggnn_ref_graph* g, int l_top, int l_m, const ggnn_ref_build_params* p);
int ggnn_ref_sym(ggnn_ref_graph* g, int layer, const ggnn_ref_build_params* p);
int ggnn_ref_build(ggnn_ref_graph* g, const ggnn_ref_build_params* p);
/* number of inverse links row `i` of `layer` received in the last sym of that layer */
int32_t* ggnn_ref_graph_inv_count(ggnn_ref_graph* g, int layer);

/* User query: Alg. 1 started on the top segment.  every_layer = 0: drop straight to
 * the bottom layer after the start points (Sec. 4.4); 1: search every layer on the way
 * down (Alg. 4).  B = length of best, P = prioq capacity, V = visited capacity,
 * max_iter = iteration limit per layer.  counters (optional, Q*2 uint32): pops and
 * distance evaluations per query. */
int ggnn_ref_query(const ggnn_ref_graph* g, const void* queries, int64_t Q, int k,
                   int B, float tau, int P, int V, int max_iter, int every_layer,
                   int32_t* ids, float* dists, uint32_t* counters);

/* Sec. 4.5 (sharding): every query is answered on every shard; the S per-shard lists (each Q*k,
 * ascending, padded with id -1) are merged into the k best overall by (distance, global id),
 * global id = offset of the shard + id within the shard.  ids / dists are S*Q*k. */
int ggnn_ref_merge_shards(int S, int64_t Q, int k, const int32_t* ids, const float* dists,
                          const int32_t* offsets, int32_t* out_ids, float* out_dists);

/* Alg. 1 on the bottom layer alone from the given start points (start_ids != NULL), else as
 * ggnn_ref_query. */
int ggnn_ref_query_from(const ggnn_ref_graph* g, const void* queries, int64_t Q, int k,
                        int B, float tau, int P, int V, int max_iter, int every_layer,
                        const int32_t* start_ids, int n_start,
                        int32_t* ids, float* dists, uint32_t* counters);

/* threads the OpenMP loops over queries / points use (timing aid; results do not depend on it) */
int ggnn_ref_num_threads(void);
void ggnn_ref_set_num_threads(int n);

#ifdef __cplusplus
}
#endif
#endif
