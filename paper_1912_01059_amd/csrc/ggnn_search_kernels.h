// Search kernels: user query (Alg. 1 / Alg. 4, Sec. 4.4), construction query (Alg. 3 Merge,
// Alg. 4) and the symmetric-linking query (Alg. 5, Sec. 4.2.1).  One wavefront per query.
// The kernels are templates over the cache implementation (registers or LDS), the element type,
// the row format (element type and lanes per row), the number of 16-byte chunks a lane holds of a
// row, and the metric.
#pragma once
#include "ggnn_launch.h"
#include "ggnn_regcache.h"

namespace ggnn {

#ifndef GGNN_PASSES
#define GGNN_PASSES 2
#endif
constexpr int kPasses = GGNN_PASSES;  // 8 rows per pass: up to 8*kPasses rows in flight per wavefront

// Wavefronts per SIMD the register allocation of query_kernel and merge_kernel aims at: with rows of up
// to 512 bytes six fit (80 registers; the user-query kernel then spills a few registers around
// Transform, once per layer, not inside the search loop), and both are faster for the added residency.
// The sym kernel would spill inside its loop and is left alone.  (Eight per SIMD need 64 registers, one
// gather pass in flight instead of two and a 512-slot table to fit LDS: measured, the 10 000-query batch of
// 512-byte rows takes 0.93 ms instead of 0.73 ms; the smaller table alone costs 9 %.)
template <int DT, int NCH>
struct SearchWavesPerSimd {
  static constexpr int value = (Elem<DT>::lanes == kRowLanes && NCH <= 4) ? 6 : 1;
};

template <int DT, int NCH>
__device__ inline void normalise_query(QueryRegs<DT, NCH>& q) {
  constexpr int E = Elem<DT>::per_chunk;
  float acc = 0.0f;
#pragma unroll
  for (int i = 0; i < NCH * E; i++) acc = __builtin_fmaf(q.v[i], q.v[i], acc);
  acc = row_reduce_t<Elem<DT>::lanes>(acc);
  const float nrm = __builtin_sqrtf(acc);
  if (nrm > 0.0f) {
#pragma unroll
    for (int i = 0; i < NCH * E; i++) q.v[i] = q.v[i] / nrm;
  }
}

// Alg. 1 main loop on one layer.  The popped point is entered into visited while its adjacency
// row is on its way.
template <class C, int DT, int NCH, int METRIC>
__device__ inline void descend(C& c, const GraphDev& G, int layer, const QueryRegs<DT, NCH>& q, int32_t excl_row) {
  const int lane = lane_id();
  const int32_t* __restrict__ E = G.edges[layer];
  int32_t a;
  while ((a = c.pop_head()) >= 0) {
    const int32_t p = (lane < G.K) ? E[(size_t)a * G.K + lane] : -1;
    c.mark_visited(a);
    c.template fetch<DT, NCH, METRIC, kPasses>(G, layer, p, q, excl_row);
  }
}

// PHASE 0: the whole search; 1: the layers above the bottom one, after which the lists are put aside;
// 2: the bottom layer, from the lists put aside, in the order given (see SplitBufs).
template <class C, int DT, int NCH, int METRIC, int PHASE>
__device__ __forceinline__ void query_body(const GraphDev& G, const uint8_t* __restrict__ queries, int k,
                                           const SearchParams& sp, int every_layer, int32_t* __restrict__ ids,
                                           float* __restrict__ dists, uint32_t* __restrict__ counters,
                                           const SplitBufs& sb, int64_t first) {
  extern __shared__ __align__(16) unsigned char lds[];
  const int lane = lane_id();
  int64_t qi = first + blockIdx.x;  // `first`: the launch's first workgroup within the batch (see chunk_blocks)
  if (PHASE == 2) {
    // XCD x takes part x of the sorted order: workgroup b is the (b / 8)-th of XCD b % 8
    const int64_t b = qi;
    const int64_t i = (b % kXcds) * sb.per + b / kXcds;
    if (b / kXcds >= sb.per || i >= sb.Q) return;
    qi = sb.order[i];
  }
  C c;
  c.bind(lds, sp, qi);
  c.init();
  QueryRegs<DT, NCH> q;
  load_query<DT, NCH>(q, queries + (size_t)qi * (size_t)G.row_bytes, G.nchunks);
  if constexpr (METRIC == 1) normalise_query<DT, NCH>(q);

  const int top = G.L - 1;
  if (sp.start) {
    // Alg. 1 on the bottom layer alone, from start points the caller chose (a flat graph, or the
    // start-point comparison of the paper's appendix)
    c.template fetch<DT, NCH, METRIC, kPasses>(G, 0, lane < sp.n_start ? sp.start[lane] : -1, q, -1);
    descend<C, DT, NCH, METRIC>(c, G, 0, q, -1);
  } else {
    // start points: the s points of the top layer (Sec. 3.1, Sec. 4.4), or, in the second of two
    // launches, the lists the first one put aside after the upper layers
    bool resumed = false;
    if constexpr (C::kInRegisters && PHASE == 2) {
      c.load_state(sb.state + (size_t)qi * sb.state_keys, sb.meta + (size_t)qi * 8);
      resumed = true;
    }
    if (!resumed) c.template fetch<DT, NCH, METRIC, kPasses>(G, top, lane < G.s ? lane : -1, q, -1);
    if (every_layer) {
      const int l_first = resumed ? 0 : top - 1, l_last = (PHASE == 1) ? 1 : 0;
      for (int l = l_first; l >= l_last; l--) {
        c.transform(G.to_lower[l + 1]);
        descend<C, DT, NCH, METRIC>(c, G, l, q, -1);
      }
    } else {
      c.transform(G.to_base[top]);
      descend<C, DT, NCH, METRIC>(c, G, 0, q, -1);
    }
  }
  if constexpr (C::kInRegisters && PHASE == 1) {  // first of two launches: the search continues in the second
    if (lane == 0) sb.key[qi] = c.first_id();
    c.save_state(sb.state + (size_t)qi * sb.state_keys, sb.meta + (size_t)qi * 8);
    return;
  }
  c.store_results(k, ids + (size_t)qi * k, dists + (size_t)qi * k);
  if (counters && lane == 0) {
    counters[4 * qi + 0] = c.n_pops();
    counters[4 * qi + 1] = c.n_evals();
    counters[4 * qi + 2] = c.n_gathers();
    counters[4 * qi + 3] = 0;
  }
}

#define GGNN_QUERY_KERNEL(NAME, PHASE)                                                                              \
  template <class C, int DT, int NCH, int METRIC>                                                                   \
  __global__ __launch_bounds__(kWave) __attribute__((amdgpu_waves_per_eu(SearchWavesPerSimd<DT, NCH>::value))) void  \
  NAME(GraphDev G, const uint8_t* __restrict__ queries, int k, SearchParams sp, int every_layer,                    \
       int32_t* __restrict__ ids, float* __restrict__ dists, uint32_t* __restrict__ counters, SplitBufs sb,         \
       int64_t first) {                                                                                             \
    query_body<C, DT, NCH, METRIC, PHASE>(G, queries, k, sp, every_layer, ids, dists, counters, sb, first);         \
  }
GGNN_QUERY_KERNEL(query_kernel, 0)
GGNN_QUERY_KERNEL(query_upper_kernel, 1)
GGNN_QUERY_KERNEL(query_lower_kernel, 2)
#undef GGNN_QUERY_KERNEL

template <class C, int DT, int NCH, int METRIC>
__global__ __launch_bounds__(kWave) __attribute__((amdgpu_waves_per_eu(SearchWavesPerSimd<DT, NCH>::value))) void merge_kernel(GraphDev G, int l_top, int l_m, SearchParams sp,
                                                      int32_t* __restrict__ out_rows, float* __restrict__ dnn1,
                                                      unsigned long long* __restrict__ work, int64_t first) {
  extern __shared__ __align__(16) unsigned char lds[];
  const int lane = lane_id();
  const int64_t z = first + blockIdx.x;
  C c;
  c.bind(lds, sp, z);
  c.init();
  const int32_t zrow = (l_m == 0) ? (int32_t)z : G.to_base[l_m][z];
  QueryRegs<DT, NCH> q;
  load_query<DT, NCH>(q, G.rows + (size_t)zrow * (size_t)G.row_bytes, G.nchunks);

  int64_t seg = (l_m == 0) ? seg0_of_row(G, z) : z / G.s;
  if (l_top == l_m) {
    // Alg. 3: exhaustive search inside the own segment.  Running every member through the
    // cache keeps exactly the K smallest (a rejected point lies beyond the current K-th).
    int32_t p = -1;
    if (l_m == 0) {
      const int64_t lo = seg0_lo(G, seg), hi = seg0_lo(G, seg + 1);
      if (lo + lane < hi) p = (int32_t)perm_fwd(G, lo + lane);
    } else if (lane < G.s) {
      p = (int32_t)(seg * G.s + lane);
    }
    c.template fetch<DT, NCH, METRIC, kPasses>(G, l_m, p, q, zrow);
  } else {
    for (int l = l_m; l < l_top; l++) seg /= G.g;  // top segment of z's sub-graph
    c.template fetch<DT, NCH, METRIC, kPasses>(G, l_top, lane < G.s ? (int32_t)(seg * G.s + lane) : -1, q, zrow);
    for (int l = l_top - 1; l >= l_m; l--) {
      c.transform(G.to_lower[l + 1]);
      descend<C, DT, NCH, METRIC>(c, G, l, q, zrow);
    }
  }
  c.store_row(G.K, out_rows + (size_t)z * G.K);
  if (l_m == 0 && lane == 0) dnn1[z] = (c.count() > 0) ? c.first_d() : 0.0f;
  if (work && lane == 0) {  // totals for the roofline of the construction: pops, rows gathered
    unsigned long long* w = work + (size_t)(blockIdx.x % kWorkSlots) * 8;  // one cache line per slot
    atomicAdd(&w[0], (unsigned long long)c.n_pops());
    atomicAdd(&w[1], (unsigned long long)c.n_gathers());
  }
}

// Alg. 5 for neighbour number `round` of every point z: is there a path from x back to z
// inside the sphere around q_m = z + w (x - z) that touches x (Sec. 4.2.1)?  If not, the
// best list of the search is kept as z's candidates for an inverse link.
template <class C, int DT, int NCH, int METRIC>
__global__ __launch_bounds__(kWave) void sym_search_kernel(GraphDev G, int layer, int round, float w_mid,
                                                           SearchParams sp, SymBuffers sb,
                                                           unsigned long long* __restrict__ work, int64_t first) {
  extern __shared__ __align__(16) unsigned char lds[];
  constexpr int E = Elem<DT>::per_chunk;
  const int lane = lane_id();
  const int64_t z = first + blockIdx.x;
  const int knn = G.K / 2, ksym = G.K - knn;
  const int32_t* __restrict__ Ed = G.edges[layer];
  if (lane == 0) sb.npref[z] = 0;
  const int32_t x = Ed[(size_t)z * G.K + round];
  if (x < 0) return;
  {
    // a direct link back from x makes the search unnecessary
    const int nix = sb.ninv[x];
    const bool hit = (lane < knn && Ed[(size_t)x * G.K + lane] == (int32_t)z) ||
                     (lane < nix && sb.inv[(size_t)x * ksym + lane] == (int32_t)z);
    if (__ballot(hit)) return;
  }
  C c;
  c.bind(lds, sp, z);
  c.init();
  const int32_t zrow = (layer == 0) ? (int32_t)z : G.to_base[layer][z];
  const int32_t xrow = (layer == 0) ? x : G.to_base[layer][x];
  QueryRegs<DT, NCH> q, xq;
  load_query<DT, NCH>(q, G.rows + (size_t)zrow * (size_t)G.row_bytes, G.nchunks);
  load_query<DT, NCH>(xq, G.rows + (size_t)xrow * (size_t)G.row_bytes, G.nchunks);
#pragma unroll
  for (int i = 0; i < NCH * E; i++) {
    const float t = xq.v[i] - q.v[i];
    const float u = w_mid * t;
    q.v[i] = q.v[i] + u;
  }
  {
    // radius: distance from q_m to x, through the same summation order as every distance
    uint4 raw[NCH];
    const int sub = lane & (Elem<DT>::lanes - 1);
#pragma unroll
    for (int ch = 0; ch < NCH; ch++) {
      const int chunk = ch * Elem<DT>::lanes + sub;
      raw[ch] = make_uint4(0, 0, 0, 0);
      if (chunk < G.nchunks) raw[ch] = *(const uint4*)(G.rows + (size_t)xrow * (size_t)G.row_bytes + (size_t)chunk * 16);
    }
    c.set_radius(row_distance<DT, NCH, METRIC>(q, raw));
  }
  c.template fetch<DT, NCH, METRIC, kPasses>(G, layer, lane == 0 ? x : -1, q, -1);
  bool found = false;
  int32_t a;
  while ((a = c.pop()) >= 0) {
    const int nia = sb.ninv[a];
    int32_t p = -1;
    if (lane < knn) p = Ed[(size_t)a * G.K + lane];
    else if (lane < knn + nia) p = sb.inv[(size_t)a * ksym + (lane - knn)];
    if (__ballot(p == (int32_t)z)) { found = true; break; }
    c.template fetch<DT, NCH, METRIC, kPasses>(G, layer, p, q, -1);
  }
  if (!found && c.count() > 0) c.store_prefs(sb.pref + (size_t)z * sp.B, sb.npref + z);
  if (work && lane == 0 && c.n_pops() > 0) {
    unsigned long long* w = work + (size_t)(blockIdx.x % kWorkSlots) * 8;
    atomicAdd(&w[2], (unsigned long long)c.n_pops());
    atomicAdd(&w[3], (unsigned long long)c.n_gathers());
  }
}

// ---- dispatch over element type, chunks per lane and metric ---------------------------
// (kU8Format, defined by the launcher: 3 where the query is a uint8 vector itself, 1 for the sym query)
// (rows of at most 1024 bytes: 8 lanes per row; longer float32 rows: the whole wavefront per row)
#define GGNN_LAUNCH(C, KERNEL, DT, NCH, M, ...) KERNEL<C, DT, NCH, M><<<grid, kWave, lds, stream>>>(__VA_ARGS__)
#define GGNN_DISPATCH(C, KERNEL, ...)                                                       \
  do {                                                                                      \
    const int need = (G.nchunks + kRowLanes - 1) / kRowLanes;                               \
    const int wide = (G.nchunks + kWideRowLanes - 1) / kWideRowLanes;                       \
    if (metric == 1) {                                                                      \
      if (need <= 1) GGNN_LAUNCH(C, KERNEL, 0, 1, 1, __VA_ARGS__);                          \
      else if (need <= 3) GGNN_LAUNCH(C, KERNEL, 0, 3, 1, __VA_ARGS__);                     \
      else if (need <= 4) GGNN_LAUNCH(C, KERNEL, 0, 4, 1, __VA_ARGS__);                     \
      else if (need <= 8) GGNN_LAUNCH(C, KERNEL, 0, 8, 1, __VA_ARGS__);                     \
      else if (wide <= 2) GGNN_LAUNCH(C, KERNEL, 2, 2, 1, __VA_ARGS__);                     \
      else if (wide <= 4) GGNN_LAUNCH(C, KERNEL, 2, 4, 1, __VA_ARGS__);                     \
      else return hipErrorInvalidValue;                                                     \
    } else if (dtype == 0) {                                                                \
      if (need <= 1) GGNN_LAUNCH(C, KERNEL, 0, 1, 0, __VA_ARGS__);                          \
      else if (need <= 3) GGNN_LAUNCH(C, KERNEL, 0, 3, 0, __VA_ARGS__);                     \
      else if (need <= 4) GGNN_LAUNCH(C, KERNEL, 0, 4, 0, __VA_ARGS__);                     \
      else if (need <= 8) GGNN_LAUNCH(C, KERNEL, 0, 8, 0, __VA_ARGS__);                     \
      else if (wide <= 2) GGNN_LAUNCH(C, KERNEL, 2, 2, 0, __VA_ARGS__);                     \
      else if (wide <= 4) GGNN_LAUNCH(C, KERNEL, 2, 4, 0, __VA_ARGS__);                     \
      else return hipErrorInvalidValue;                                                     \
    } else {                                                                                \
      if (need <= 1) GGNN_LAUNCH(C, KERNEL, kU8Format, 1, 0, __VA_ARGS__);                  \
      else if (need <= 2) GGNN_LAUNCH(C, KERNEL, kU8Format, 2, 0, __VA_ARGS__);             \
      else return hipErrorInvalidValue;                                                     \
    }                                                                                       \
  } while (0)

template <class C>
hipError_t launch_query_t(const GraphDev& G, int dtype, int metric, const void* queries, int64_t Q, int k,
                          const SearchParams& sp, int every_layer, int32_t* ids, float* dists, uint32_t* counters,
                          hipStream_t stream) {
  if (Q <= 0) return hipSuccess;
  const size_t lds = C::lds_bytes(sp);
  constexpr int kU8Format = 3;
  const SplitBufs sb = {};
  for (int64_t first = 0; first < Q; first += kMaxBlocksPerLaunch) {
    const dim3 grid(chunk_blocks(Q, first));
    GGNN_DISPATCH(C, query_kernel, G, (const uint8_t*)queries, k, sp, every_layer, ids, dists, counters, sb, first);
  }
  return hipGetLastError();
}
// one of the two launches of a large batch (sb.phase 1 or 2; register cache only)
template <class C>
hipError_t launch_query_split_t(const GraphDev& G, int dtype, int metric, const void* queries, int64_t Q, int k,
                                const SearchParams& sp, int32_t* ids, float* dists, uint32_t* counters,
                                const SplitBufs& sb, hipStream_t stream) {
  if (Q <= 0) return hipSuccess;
  const int64_t blocks = sb.phase == 2 ? (int64_t)kXcds * sb.per : Q;
  const size_t lds = C::lds_bytes(sp);
  constexpr int kU8Format = 3;
  const int every_layer = 1;
  for (int64_t first = 0; first < blocks; first += kMaxBlocksPerLaunch) {
    const dim3 grid(chunk_blocks(blocks, first));
    if (sb.phase == 1) {
      GGNN_DISPATCH(C, query_upper_kernel, G, (const uint8_t*)queries, k, sp, every_layer, ids, dists, counters, sb, first);
    } else {
      GGNN_DISPATCH(C, query_lower_kernel, G, (const uint8_t*)queries, k, sp, every_layer, ids, dists, counters, sb, first);
    }
  }
  return hipGetLastError();
}
template <class C>
hipError_t launch_merge_t(const GraphDev& G, int dtype, int metric, int l_top, int l_m, const SearchParams& sp,
                          int32_t* out_rows, float* dnn1, unsigned long long* work, hipStream_t stream) {
  const size_t lds = C::lds_bytes(sp);
  constexpr int kU8Format = 3;
  for (int64_t first = 0; first < G.n[l_m]; first += kMaxBlocksPerLaunch) {
    const dim3 grid(chunk_blocks(G.n[l_m], first));
    GGNN_DISPATCH(C, merge_kernel, G, l_top, l_m, sp, out_rows, dnn1, work, first);
  }
  return hipGetLastError();
}
template <class C>
hipError_t launch_sym_search_t(const GraphDev& G, int dtype, int metric, int layer, int round, float w_mid,
                               const SearchParams& sp, const SymBuffers& sb, unsigned long long* work,
                               hipStream_t stream) {
  const size_t lds = C::lds_bytes(sp);
  constexpr int kU8Format = 1;
  for (int64_t first = 0; first < G.n[layer]; first += kMaxBlocksPerLaunch) {
    const dim3 grid(chunk_blocks(G.n[layer], first));
    GGNN_DISPATCH(C, sym_search_kernel, G, layer, round, w_mid, sp, sb, work, first);
  }
  return hipGetLastError();
}

}  // namespace ggnn
