// Device-side building blocks of the GGNN search on gfx950: one 64-lane wavefront per
// query, the cache of Sec. 3.1.1 (best / prioq as sorted arrays of packed keys, visited as
// an exact hash set) in LDS, distances as coalesced 16-byte gathers with 8 lanes per row.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ggnn {

typedef unsigned long long u64;

constexpr int kWave = 64;
constexpr int kRowLanes = 8;            // lanes that share one row of at most 1024 bytes (GGNN_ROW_LANES)
constexpr int kRowsPerPass = kWave / kRowLanes;
constexpr int kWideRowLanes = 64;       // longer rows take the whole wavefront (GGNN_WIDE_ROW_LANES)
constexpr int kMaxLevels = 8;

// What a kernel needs to know about the graph (passed by value).
struct GraphDev {
  const uint8_t* rows;   // base vectors (or the unit-length copy for cosine)
  int64_t N;
  int32_t D, K, L, s, g;
  int32_t row_bytes, nchunks;  // bytes per row, 16-byte chunks per row
  int32_t addr32;              // 1: the vector array is smaller than 4 GiB (host side: which kernel variant to launch)
  int64_t n[kMaxLevels];
  const int32_t* edges[kMaxLevels];
  const int32_t* to_lower[kMaxLevels];
  const int32_t* to_base[kMaxLevels];
  int64_t G0;                  // bottom segments
  uint32_t fkey[4];            // round keys of the partition permutation
  int32_t fbits;               // half width of the Feistel network
  uint64_t seed;
};

// Cache capacities and the constants of the stopping rule (Eq. 2).
struct SearchParams {
  int32_t B, P, H;     // best length, prioq capacity, hash slots (power of two >= 2*max_iter)
  int32_t max_iter;
  float tau, dnn;
  const int32_t* start;  // user queries only: explicit start points on the bottom layer, or null
  int32_t n_start;
  int32_t* vis;          // user queries only: per-query visited tables in global memory, or null
};

// A large batch of user queries is answered in two launches: the upper layers first, then the bottom
// layer with the queries ordered by the layer-1 point they arrived at, one contiguous part of that
// order per XCD (workgroups go to the XCDs in turn), so that queries of one region share an L2.
struct SplitBufs {
  int32_t phase;         // 0: whole search in one launch, 1: upper layers, 2: bottom layer
  int32_t per;           // phase 2: queries per XCD part
  int64_t Q;
  u64* state;            // Q x state_keys keys: best, then prioq, as the wavefront holds them
  int32_t state_keys;
  int32_t* meta;         // Q x 8: nb, np, pops, evals, gathers
  int32_t* key;          // Q: layer-1 id of the best point so far (phase 1 writes)
  const int32_t* order;  // Q: query numbers in sorted order (phase 2 reads)
};
constexpr int kXcds = 8;

// ---- packed keys: (float32 distance, int32 id) ordered as one unsigned 64-bit integer.
// Distances are >= +0, so their bit patterns order like the values; +inf sorts last.
__device__ __forceinline__ u64 make_key(float d, int32_t id) {
  return ((u64)__float_as_uint(d) << 32) | (uint32_t)id;
}
__device__ __forceinline__ float key_d(u64 k) { return __uint_as_float((uint32_t)(k >> 32)); }
__device__ __forceinline__ int32_t key_id(u64 k) { return (int32_t)(uint32_t)k; }

// One wavefront per workgroup: the barrier only orders LDS traffic between lanes.
__device__ __forceinline__ void wave_sync() { __syncthreads(); }

__device__ __forceinline__ int lane_id() { return threadIdx.x; }

// ---- partition permutation (bottom-layer segments): 4-round Feistel network with cycle walking
// (host-callable as well: tests/host_index_sweep.cpp walks every index expression of the bottom layer
// at full size on the CPU, under the address and undefined-behaviour sanitizers)
__host__ __device__ __forceinline__ uint32_t mix32(uint32_t h) {
  h ^= h >> 16; h *= 0x85EBCA6Bu;
  h ^= h >> 13; h *= 0xC2B2AE35u;
  h ^= h >> 16;
  return h;
}
__host__ __device__ __forceinline__ uint64_t mix64(uint64_t x) {
  x ^= x >> 30; x *= 0xBF58476D1CE4E5B9ull;
  x ^= x >> 27; x *= 0x94D049BB133111EBull;
  x ^= x >> 31;
  return x;
}
__host__ __device__ inline int64_t perm_fwd(const GraphDev& G, int64_t p) {
  const uint32_t mask = (uint32_t)((1ull << G.fbits) - 1);
  uint64_t x = (uint64_t)p;
  do {
    uint32_t Lh = (uint32_t)(x >> G.fbits) & mask, Rh = (uint32_t)x & mask;
#pragma unroll
    for (int r = 0; r < 4; r++) {
      uint32_t t = Lh ^ (mix32(Rh ^ G.fkey[r]) & mask);
      Lh = Rh; Rh = t;
    }
    x = ((uint64_t)Lh << G.fbits) | Rh;
  } while ((int64_t)x >= G.N);
  return (int64_t)x;
}
__host__ __device__ inline int64_t perm_inv(const GraphDev& G, int64_t row) {
  const uint32_t mask = (uint32_t)((1ull << G.fbits) - 1);
  uint64_t x = (uint64_t)row;
  do {
    uint32_t Lh = (uint32_t)(x >> G.fbits) & mask, Rh = (uint32_t)x & mask;
#pragma unroll
    for (int r = 3; r >= 0; r--) {
      uint32_t t = Rh ^ (mix32(Lh ^ G.fkey[r]) & mask);
      Rh = Lh; Lh = t;
    }
    x = ((uint64_t)Lh << G.fbits) | Rh;
  } while ((int64_t)x >= G.N);
  return (int64_t)x;
}
__host__ __device__ __forceinline__ int64_t seg0_lo(const GraphDev& G, int64_t j) { return (j * G.N) / G.G0; }
__host__ __device__ __forceinline__ int64_t seg0_of_row(const GraphDev& G, int64_t row) {
  return ((perm_inv(G, row) + 1) * G.G0 - 1) / G.N;
}

// ---- the cache ------------------------------------------------------------------------
struct Cache {
  u64* best; u64* pq; u64* tmp;   // LDS
  int32_t* hash;                  // LDS, H slots, -1 = empty
  int32_t* surv_id; int32_t* surv_row; float* surv_d;  // LDS, 64 each
  int32_t B, P, hmask;
  int32_t nb, np, iter, max_iter;
  float tau, dnn, radius;
  float d_first, d_kth;           // best[0].d and best[B-1].d (+inf while best is not full)
  uint32_t pops, evals;
};

__host__ __device__ inline size_t cache_lds_bytes(int B, int P, int H) {
  return (size_t)(B + P + (B + P)) * 8 + (size_t)H * 4 + 3 * 64 * 4;
}

__device__ inline void cache_bind(Cache& c, unsigned char* lds, const SearchParams& sp) {
  c.B = sp.B; c.P = sp.P; c.hmask = sp.H - 1;
  c.best = (u64*)lds;
  c.pq = c.best + sp.B;
  c.tmp = c.pq + sp.P;
  c.hash = (int32_t*)(c.tmp + sp.B + sp.P);
  c.surv_id = c.hash + sp.H;
  c.surv_row = c.surv_id + 64;
  c.surv_d = (float*)(c.surv_row + 64);
  c.max_iter = sp.max_iter; c.tau = sp.tau; c.dnn = sp.dnn;
}

__device__ inline void hash_clear(Cache& c) {
  for (int i = lane_id(); i <= c.hmask; i += kWave) c.hash[i] = -1;
  wave_sync();
}
__device__ __forceinline__ uint32_t hash_slot(const Cache& c, int32_t id) {
  return (mix32((uint32_t)id)) & (uint32_t)c.hmask;
}
__device__ inline bool hash_has(const Cache& c, int32_t id) {
  uint32_t h = hash_slot(c, id);
  int32_t v;
  while ((v = c.hash[h]) != -1) {
    if (v == id) return true;
    h = (h + 1) & (uint32_t)c.hmask;
  }
  return false;
}
// uniform call: every lane passes the same id
__device__ inline void hash_insert(Cache& c, int32_t id) {
  if (lane_id() == 0) {
    uint32_t h = hash_slot(c, id);
    while (c.hash[h] != -1) h = (h + 1) & (uint32_t)c.hmask;
    c.hash[h] = id;
  }
  wave_sync();
}

// Alg. 2 Init
__device__ inline void cache_init(Cache& c) {
  c.nb = c.np = 0; c.iter = 0; c.pops = c.evals = 0;
  c.radius = INFINITY; c.d_first = INFINITY; c.d_kth = INFINITY;
  hash_clear(c);
}

// Eq. 2: d_best_k + tau * min(d_best_1, d_nn1); +inf while best is empty
__device__ __forceinline__ float cache_thr(const Cache& c) {
  if (c.nb == 0) return INFINITY;
  float xi = c.tau * fminf(c.d_first, c.dnn);
  return c.d_kth + xi;
}
__device__ __forceinline__ bool cache_crit(const Cache& c, float d) { return d <= cache_thr(c) && d <= c.radius; }

// sorted insertion of one key into a[0..n) with capacity cap; uniform call
__device__ inline void list_insert(u64* a, int32_t& n, int32_t cap, u64 key) {
  const int lane = lane_id();
  int pos = 0;
  for (int i0 = 0; i0 < n; i0 += kWave) {
    int idx = i0 + lane;
    bool lt = idx < n && a[idx] < key;
    pos += __popcll(__ballot(lt));
  }
  if (pos >= cap) return;
  int hi = n < cap - 1 ? n : cap - 1;  // entries [pos, hi) move one slot up
  if (hi > pos) {
    for (int b0 = (hi - 1) & ~(kWave - 1); b0 >= (pos & ~(kWave - 1)); b0 -= kWave) {
      int idx = b0 + lane;
      bool mv = idx >= pos && idx < hi;
      u64 e = mv ? a[idx] : 0;
      wave_sync();
      if (mv) a[idx + 1] = e;
      wave_sync();
    }
  }
  if (lane == 0) a[pos] = key;
  if (n < cap) n++;
  wave_sync();
}

// Alg. 2 Push
__device__ inline void cache_push(Cache& c, int32_t id, float d) {
  u64 key = make_key(d, id);
  list_insert(c.best, c.nb, c.B, key);
  list_insert(c.pq, c.np, c.P, key);
  c.d_first = key_d(c.best[0]);
  c.d_kth = (c.nb < c.B) ? INFINITY : key_d(c.best[c.B - 1]);
}

// Alg. 2 Pop; returns -1 when the search on this layer ends
__device__ inline int32_t cache_pop(Cache& c) {
  if (c.np == 0 || c.iter >= c.max_iter) return -1;
  u64 head = c.pq[0];
  if (!cache_crit(c, key_d(head))) return -1;
  const int lane = lane_id();
  for (int i0 = 0; i0 < c.np - 1; i0 += kWave) {
    int idx = i0 + lane;
    bool mv = idx < c.np - 1;
    u64 e = mv ? c.pq[idx + 1] : 0;
    wave_sync();
    if (mv) c.pq[idx] = e;
    wave_sync();
  }
  c.np--;
  int32_t id = key_id(head);
  hash_insert(c, id);
  c.iter++;
  c.pops++;
  return id;
}

// rank sort of n distinct keys: dst[rank] = key for rank < cap
__device__ inline void rank_sort(const u64* src, int n, u64* dst, int cap) {
  for (int i = lane_id(); i < n; i += kWave) {
    u64 key = src[i];
    int r = 0;
    for (int j = 0; j < n; j++) r += src[j] < key;
    if (r < cap) dst[r] = key;
  }
  wave_sync();
}

// Alg. 4 Transform: ids -> ids of the same points on the next layer to search; visited is
// emptied and prioq re-seeded with best and the left-over prioq entries.
__device__ inline void cache_transform(Cache& c, const int32_t* __restrict__ table) {
  const int lane = lane_id();
  for (int i = lane; i < c.nb; i += kWave) {
    u64 k = c.best[i];
    c.best[i] = (k & 0xFFFFFFFF00000000ull) | (uint32_t)table[key_id(k)];
  }
  for (int i = lane; i < c.np; i += kWave) {
    u64 k = c.pq[i];
    c.pq[i] = (k & 0xFFFFFFFF00000000ull) | (uint32_t)table[key_id(k)];
  }
  wave_sync();
  rank_sort(c.best, c.nb, c.tmp, c.nb);
  for (int i = lane; i < c.nb; i += kWave) c.best[i] = c.tmp[i];
  wave_sync();
  int m = c.nb;
  for (int i0 = 0; i0 < c.np; i0 += kWave) {
    int idx = i0 + lane;
    bool keep = idx < c.np;
    u64 k = keep ? c.pq[idx] : 0;
    if (keep) {
      for (int j = 0; j < c.nb; j++) keep = keep && key_id(c.best[j]) != key_id(k);
    }
    u64 mask = __ballot(keep);
    if (keep) c.tmp[m + __popcll(mask & ((1ull << lane) - 1))] = k;
    m += __popcll(mask);
  }
  wave_sync();
  // tmp[0..m) holds distinct ids; the P smallest become the new prioq
  u64* scratch = c.pq;
  rank_sort(c.tmp, m, scratch, c.P);
  c.np = m < c.P ? m : c.P;
  c.iter = 0;
  if (c.nb > 0) {
    c.d_first = key_d(c.best[0]);
    c.d_kth = (c.nb < c.B) ? INFINITY : key_d(c.best[c.B - 1]);
  }
  hash_clear(c);
}

// ---- distances ------------------------------------------------------------------------
// Row formats: 0 = float32 (4 per 16-byte chunk), 8 lanes per row; 1 = uint8 (16 per chunk), 8 lanes
// per row; 2 = float32, the whole wavefront per row (rows longer than 1024 bytes); 3 = uint8 with an
// integer query (below).
template <int DT> struct Elem;
template <> struct Elem<0> { static constexpr int per_chunk = 4, lanes = kRowLanes; };
template <> struct Elem<1> { static constexpr int per_chunk = 16, lanes = kRowLanes; };
template <> struct Elem<2> { static constexpr int per_chunk = 4, lanes = kWideRowLanes; };
// 3 = uint8 rows against a uint8 query (user queries and Merge; the sym query is a real-valued point
// and takes format 1): sum (q-x)^2 = sum q^2 + sum x^2 - 2 sum q x in exact integer arithmetic with
// 4-way byte dot products.  The sum is below 2^24, so it is the float32 sum of format 1 bit for bit.
template <> struct Elem<3> { static constexpr int per_chunk = 16, lanes = kRowLanes; };
// rows a wavefront takes per gather instruction, and gather instructions issued before the first use
template <int DT, int PASSES> struct RowSched {
  static constexpr int rows_per_pass = kWave / Elem<DT>::lanes;
  static constexpr int passes = (Elem<DT>::lanes == kWave) ? 3 * PASSES : PASSES;
};

template <int DT>
__device__ __forceinline__ void chunk_to_float(const uint4& v, float* out) {
  if (DT != 1) {
    out[0] = __uint_as_float(v.x); out[1] = __uint_as_float(v.y);
    out[2] = __uint_as_float(v.z); out[3] = __uint_as_float(v.w);
  } else {
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int i = 0; i < 4; i++) {
      out[4 * i + 0] = (float)(w[i] & 0xFF);
      out[4 * i + 1] = (float)((w[i] >> 8) & 0xFF);
      out[4 * i + 2] = (float)((w[i] >> 16) & 0xFF);
      out[4 * i + 3] = (float)(w[i] >> 24);
    }
  }
}

// butterfly over the 8 lanes that share a row: lane l adds the value of lane l^4, then l^2, then
// l^1.  Done with DPP moves (no LDS traffic): the l^4 exchange is a shift by four lanes within a
// row of 16, to the right for the upper half of each group and to the left for the lower half
// (bank masks 0xA / 0x5); the other two are quad permutations.
template <int CTRL, int BANK_MASK>
__device__ __forceinline__ float dpp_move(float old, float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(old), __float_as_int(v), CTRL, 0xf, BANK_MASK, false));
}
__device__ __forceinline__ float row_reduce(float acc) {
  float t = dpp_move<0x114, 0xA>(0.0f, acc);  // row_shr:4 -> lanes 4..7 and 12..15 of each row
  t = dpp_move<0x104, 0x5>(t, acc);           // row_shl:4 -> lanes 0..3 and 8..11
  acc = acc + t;
  acc = acc + dpp_move<0x4E, 0xF>(0.0f, acc);  // quad_perm [2,3,0,1]
  acc = acc + dpp_move<0xB1, 0xF>(0.0f, acc);  // quad_perm [1,0,3,2]
  return acc;
}
// the same butterfly over LANES lanes (8 or 64): distances 32, 16, 8 go through the LDS crossbar
// (ds_bpermute, no LDS memory), the last three are the DPP steps above
template <int LANES>
__device__ __forceinline__ float row_reduce_t(float acc) {
  if (LANES == kWideRowLanes) {
    acc = acc + __shfl_xor(acc, 32, kWave);
    acc = acc + __shfl_xor(acc, 16, kWave);
    acc = acc + __shfl_xor(acc, 8, kWave);
  }
  return row_reduce(acc);
}

// The query vector: lane (sub = lane mod row lanes) keeps the elements of chunks sub, sub + lanes, ...
template <int DT, int NCH>
struct QueryRegs {
  float v[NCH * Elem<DT>::per_chunk];
};
template <int NCH>
struct QueryRegs<3, NCH> {
  uint32_t w[NCH * 4];  // the query's bytes, four to a word
  uint32_t qq;          // sum of the squares of this lane's query elements
};

template <int DT, int NCH>
__device__ inline void load_query(QueryRegs<DT, NCH>& q, const uint8_t* row, int nchunks) {
  constexpr int RL = Elem<DT>::lanes;
  const int sub = lane_id() & (RL - 1);
  if constexpr (DT == 3) q.qq = 0;
#pragma unroll
  for (int c = 0; c < NCH; c++) {
    int chunk = c * RL + sub;
    uint4 raw = make_uint4(0, 0, 0, 0);
    if (chunk < nchunks) raw = *(const uint4*)(row + (size_t)chunk * 16);
    if constexpr (DT == 3) {
      const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
      for (int i = 0; i < 4; i++) {
        q.w[c * 4 + i] = w[i];
        q.qq = __builtin_amdgcn_udot4(w[i], w[i], q.qq, false);
      }
    } else {
      chunk_to_float<DT>(raw, &q.v[c * Elem<DT>::per_chunk]);  // chunks past the row read as zeros
    }
  }
}

// one row against the query: METRIC 0: sum (q-x)^2, 1: sum q*x, in the fixed order
template <int DT, int NCH, int METRIC>
__device__ __forceinline__ float row_sum(const QueryRegs<DT, NCH>& q, const uint4 (&raw)[NCH]) {
  if constexpr (DT == 3) {
    static_assert(METRIC == 0, "integer rows have no cosine distance");
    uint32_t xx = q.qq, qx = 0;
#pragma unroll
    for (int c = 0; c < NCH; c++) {
      const uint32_t w[4] = {raw[c].x, raw[c].y, raw[c].z, raw[c].w};
#pragma unroll
      for (int i = 0; i < 4; i++) {
        xx = __builtin_amdgcn_udot4(w[i], w[i], xx, false);
        qx = __builtin_amdgcn_udot4(q.w[c * 4 + i], w[i], qx, false);
      }
    }
    return row_reduce((float)(xx - 2u * qx));  // per lane at most 32 * 255^2: exact in float32, as is the total
  } else {
    constexpr int E = Elem<DT>::per_chunk;
    float acc = 0.0f;
#pragma unroll
    for (int c = 0; c < NCH; c++) {
      float x[E];
      chunk_to_float<DT>(raw[c], x);
#pragma unroll
      for (int e = 0; e < E; e++) {
        if (METRIC == 0) {
          float t = q.v[c * E + e] - x[e];
          acc = __builtin_fmaf(t, t, acc);
        } else {
          acc = __builtin_fmaf(q.v[c * E + e], x[e], acc);
        }
      }
    }
    return row_reduce_t<Elem<DT>::lanes>(acc);
  }
}
// from the sum to the distance: METRIC 0: sqrt(sum), 1: max(0, 1 - sum)
template <int METRIC>
__device__ __forceinline__ float finish_distance(float sum) {
  if (METRIC == 0) return __builtin_sqrtf(sum);
  return fmaxf(0.0f, 1.0f - sum);
}
template <int DT, int NCH, int METRIC>
__device__ __forceinline__ float row_distance(const QueryRegs<DT, NCH>& q, const uint4 (&raw)[NCH]) {
  return finish_distance<METRIC>(row_sum<DT, NCH, METRIC>(q, raw));
}

// One batch of survivors (rows b0 .. of surv_row): requests the rows (8 lanes x 16 bytes per row, or
// the whole wavefront per long row), every load issued before the first use, then leaves the sum of
// every row in surv_sum.  A pass takes kWave / lanes rows.  Lanes without a row read row 0 (their sums
// are never stored), so nothing is spent on clearing registers or masking loads; the arithmetic of a
// pass without rows is skipped.  A32: every byte offset into the array fits 32 bits, and the address is
// the uniform base plus a 32-bit lane offset plus a constant per chunk; otherwise (arrays of 4 GiB and
// more, served by kernel variants of their own so that the common case keeps its register budget) the
// lane offset is formed in 64 bits.  FULL: every lane owns NCH chunks of the row (no ragged tail).
__host__ __device__ __forceinline__ uint64_t row_offset(uint32_t row, uint32_t row_bytes, uint32_t sub) {
  return (uint64_t)row * row_bytes + (uint64_t)sub * 16u;
}
template <int DT, int NCH, int METRIC, int NP, bool FULL, bool A32>
__device__ __forceinline__ void gather_sum_t(const GraphDev& G, const QueryRegs<DT, NCH>& q, const int32_t* surv_row,
                                             float* surv_sum, int b0, int ns) {
  constexpr int RL = Elem<DT>::lanes, RPP = kWave / RL;
  const int lane = lane_id(), sub = lane & (RL - 1), grp = lane / RL;
  uint4 raw[NP][NCH];
#pragma unroll
  for (int ps = 0; ps < NP; ps++) {
    const int r = b0 + ps * RPP + grp;
    const uint32_t row = (r < ns) ? (uint32_t)surv_row[r] : 0u;
    const uint8_t* ptr;
    if (A32) ptr = G.rows + (uint32_t)row_offset(row, (uint32_t)G.row_bytes, (uint32_t)sub);
    else ptr = G.rows + row_offset(row, (uint32_t)G.row_bytes, (uint32_t)sub);
#pragma unroll
    for (int ch = 0; ch < NCH; ch++) {
      if (FULL) {
        raw[ps][ch] = *(const uint4*)(ptr + ch * RL * 16);
      } else {
        raw[ps][ch] = make_uint4(0, 0, 0, 0);  // chunks past the row read as zeros
        if (ch * RL + sub < G.nchunks) raw[ps][ch] = *(const uint4*)(ptr + ch * RL * 16);
      }
    }
  }
#pragma unroll
  for (int ps = 0; ps < NP; ps++) {
    if (b0 + ps * RPP < ns) {  // uniform
      const int r = b0 + ps * RPP + grp;
      const float sum = row_sum<DT, NCH, METRIC>(q, raw[ps]);
      if (r < ns && sub == 0) surv_sum[r] = sum;
    }
  }
}
template <int DT, int NCH, int METRIC, int NP, bool A32>
__device__ __forceinline__ void gather_sum(const GraphDev& G, const QueryRegs<DT, NCH>& q, const int32_t* surv_row,
                                           float* surv_sum, int b0, int ns) {
  const bool full = G.nchunks == NCH * Elem<DT>::lanes;
  if (full) gather_sum_t<DT, NCH, METRIC, NP, true, A32>(G, q, surv_row, surv_sum, b0, ns);
  else gather_sum_t<DT, NCH, METRIC, NP, false, A32>(G, q, surv_row, surv_sum, b0, ns);
}

// Alg. 2 Fetch.  Lane j holds proposal p (or -1).  Known points are dropped against the
// cache as it stands; the survivors' rows are gathered (8 lanes per row, every load of a
// batch issued before the first use), and the survivors are then pushed in list order.
template <int DT, int NCH, int METRIC, int PASSES>
__device__ inline void cache_fetch(Cache& c, const GraphDev& G, int layer, int32_t p,
                                   const QueryRegs<DT, NCH>& q, int32_t excl_row) {
  const int lane = lane_id();
  bool alive = p >= 0;
  int32_t row = -1;
  if (alive) {
    row = (layer == 0) ? p : G.to_base[layer][p];
    alive = row != excl_row;
  }
  if (alive) alive = !hash_has(c, p);
  for (int i = 0; i < c.nb; i++) alive = alive && key_id(c.best[i]) != p;
  for (int i = 0; i < c.np; i++) alive = alive && key_id(c.pq[i]) != p;
  const u64 mask = __ballot(alive);
  const int ns = __popcll(mask);
  if (ns == 0) return;
  if (alive) {
    int r = __popcll(mask & ((1ull << lane) - 1));
    c.surv_id[r] = p;
    c.surv_row[r] = row;
  }
  wave_sync();
  constexpr int RL = Elem<DT>::lanes, RPP = RowSched<DT, PASSES>::rows_per_pass, NP = RowSched<DT, PASSES>::passes;
  const int sub = lane & (RL - 1), grp = lane / RL;
  for (int b0 = 0; b0 < ns; b0 += RPP * NP) {
    uint4 raw[NP][NCH];
#pragma unroll
    for (int ps = 0; ps < NP; ps++) {
      int r = b0 + ps * RPP + grp;
      bool act = r < ns;
      const uint8_t* ptr = G.rows + (size_t)(act ? c.surv_row[r] : 0) * (size_t)G.row_bytes;
#pragma unroll
      for (int ch = 0; ch < NCH; ch++) {
        int chunk = ch * RL + sub;
        raw[ps][ch] = make_uint4(0, 0, 0, 0);
        if (act && chunk < G.nchunks) raw[ps][ch] = *(const uint4*)(ptr + (size_t)chunk * 16);
      }
    }
#pragma unroll
    for (int ps = 0; ps < NP; ps++) {
      int r = b0 + ps * RPP + grp;
      float d = row_distance<DT, NCH, METRIC>(q, raw[ps]);
      if (r < ns && sub == 0) c.surv_d[r] = d;
    }
  }
  wave_sync();
  c.evals += ns;
  for (int i = 0; i < ns; i++) {
    float d = c.surv_d[i];
    if (cache_crit(c, d)) cache_push(c, c.surv_id[i], d);
  }
}

// Alg. 1 main loop on one layer
template <int DT, int NCH, int METRIC, int PASSES>
__device__ inline void cache_descend(Cache& c, const GraphDev& G, int layer, const QueryRegs<DT, NCH>& q,
                                     int32_t excl_row) {
  const int lane = lane_id();
  const int32_t* __restrict__ E = G.edges[layer];
  int32_t a;
  while ((a = cache_pop(c)) >= 0) {
    int32_t p = (lane < G.K) ? E[(size_t)a * G.K + lane] : -1;
    cache_fetch<DT, NCH, METRIC, PASSES>(c, G, layer, p, q, excl_row);
  }
}

// The LDS-resident cache behind the interface the kernels use (any capacities that fit in LDS).
struct LdsCache {
  static constexpr bool kInRegisters = false;
  Cache c;
  __host__ __device__ static size_t lds_bytes(const SearchParams& sp) { return cache_lds_bytes(sp.B, sp.P, sp.H); }
  __device__ void bind(unsigned char* lds, const SearchParams& sp, int64_t) { cache_bind(c, lds, sp); }
  __device__ void init() { cache_init(c); }
  __device__ void set_radius(float r) { c.radius = r; }
  template <int DT, int NCH, int METRIC, int PASSES>
  __device__ void fetch(const GraphDev& G, int layer, int32_t p, const QueryRegs<DT, NCH>& q, int32_t excl_row) {
    cache_fetch<DT, NCH, METRIC, PASSES>(c, G, layer, p, q, excl_row);
  }
  __device__ int32_t pop() { return cache_pop(c); }
  __device__ int32_t pop_head() { return cache_pop(c); }
  __device__ void mark_visited(int32_t) {}
  __device__ int32_t next_head() const { return c.np > 0 ? key_id(c.pq[0]) : -1; }
  __device__ void transform(const int32_t* __restrict__ table) { cache_transform(c, table); }
  __device__ int32_t count() const { return c.nb; }
  __device__ float first_d() const { return c.d_first; }
  __device__ uint32_t n_pops() const { return c.pops; }
  __device__ uint32_t n_evals() const { return c.evals; }
  __device__ uint32_t n_gathers() const { return c.evals; }
  __device__ void store_results(int k, int32_t* __restrict__ ids, float* __restrict__ dists) const {
    for (int j = lane_id(); j < k; j += kWave) {
      const u64 key = (j < c.nb) ? c.best[j] : make_key(INFINITY, -1);
      ids[j] = key_id(key);
      dists[j] = key_d(key);
    }
  }
  __device__ void store_row(int K, int32_t* __restrict__ out) const {
    const int lane = lane_id();
    if (lane < K) out[lane] = (lane < c.nb) ? key_id(c.best[lane]) : -1;
  }
  __device__ void store_prefs(u64* __restrict__ pref, int32_t* __restrict__ npref) const {
    for (int i = lane_id(); i < c.nb; i += kWave) pref[i] = c.best[i];
    if (lane_id() == 0) *npref = c.nb;
  }
};

}  // namespace ggnn
