// The cache of Sec. 3.1.1 for a prioq of at most 64 and a best list of at most 64 * NB entries:
// both lists live in registers, entry i in lane i mod 64 of register i / 64 (packed (distance, id)
// keys, empty = all ones), so that a sorted
// insertion is one compare, one whole-wave shift (DPP) and a select, and a pop is a shift the
// other way.  visited is an exact hash set in LDS; the same table also remembers points that
// were evaluated and rejected: the threshold of Eq. 2 never grows during a search on one layer,
// so a point rejected once is rejected whenever it is proposed again, and skipping it changes no
// result (rejected entries may be left out when the table fills up; visited entries never are).
// Whether a proposal already sits in best or prioq is decided exactly by comparing it with the
// entry every lane holds; a bit map in LDS (one bit per hash bucket, set when an id of that bucket
// enters a list, rebuilt from the lists every few iterations and when the layer changes) first rules
// out the many proposals that cannot be listed.
#pragma once
#include "ggnn_device.h"

namespace ggnn {

constexpr u64 kEmptyKey = ~0ull;

// whole-wave shift by one lane (GFX9 DPP wave_shr:1 / wave_shl:1); the vacated lane gets `fill`, and so
// does every enabled lane whose source lane is disabled (a DPP move leaves such a lane at its old value,
// which is `fill` here): the sorted insertions below rely on that
__device__ __forceinline__ u64 wave_shift_up(u64 v, u64 fill) {
  int lo = __builtin_amdgcn_update_dpp((int)(uint32_t)fill, (int)(uint32_t)v, 0x138, 0xf, 0xf, false);
  int hi = __builtin_amdgcn_update_dpp((int)(uint32_t)(fill >> 32), (int)(uint32_t)(v >> 32), 0x138, 0xf, 0xf, false);
  return ((u64)(uint32_t)hi << 32) | (uint32_t)lo;
}
__device__ __forceinline__ u64 wave_shift_down(u64 v, u64 fill) {
  int lo = __builtin_amdgcn_update_dpp((int)(uint32_t)fill, (int)(uint32_t)v, 0x130, 0xf, 0xf, false);
  int hi = __builtin_amdgcn_update_dpp((int)(uint32_t)(fill >> 32), (int)(uint32_t)(v >> 32), 0x130, 0xf, 0xf, false);
  return ((u64)(uint32_t)hi << 32) | (uint32_t)lo;
}
// value of `v` in lane `src` (any lane index per lane; ds_bpermute: the LDS crossbar, no LDS memory)
__device__ __forceinline__ u64 lane_gather_u64(u64 v, int src) {
  const uint32_t lo = (uint32_t)__builtin_amdgcn_ds_bpermute(src << 2, (int)(uint32_t)v);
  const uint32_t hi = (uint32_t)__builtin_amdgcn_ds_bpermute(src << 2, (int)(uint32_t)(v >> 32));
  return ((u64)hi << 32) | lo;
}
__device__ __forceinline__ u64 read_lane_u64(u64 v, int lane) {
  uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)v, lane);
  uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(v >> 32), lane);
  return ((u64)hi << 32) | lo;
}

// GV: the visited ids live in a table in global memory (one per query, handed in through
// SearchParams::vis) instead of LDS, which then holds the rejected ids only: for searches of a thousand
// iterations and more the LDS table is what limits the wavefronts a compute unit holds.
// ANY: the LDS table may have any multiple of 64 slots (searches of a few hundred to a thousand
// iterations, where the step to the next power of two would cost a wavefront per SIMD).
// A64: the vector array holds 4 GiB or more, rows are addressed with 64-bit offsets.
template <int NB, bool GV = false, bool ANY = false, bool A64 = false>
struct RegCacheT {
  static constexpr bool kInRegisters = true;
  static constexpr int kBestSlots = NB;
  u64 best[NB], pq;             // entry i: best[i / 64] of lane i % 64; kEmptyKey beyond the fill level
  int32_t B, P, nb, np;
  int32_t iter, max_iter;
  float tau, dnn, radius, d1, dk, thr_now;
  u64 last_best;                 // key of best[B-1]
  int32_t* hash; int32_t hmask, hshift;  // LDS: visited ids (unless GV), and rejected ids with the top bit set
  int32_t* vis; int32_t vmask, vshift;   // GV: visited ids in global memory
  uint32_t* listed_bits;         // LDS: kListedBuckets bits
  int32_t nrej, rej_cap;
  u64* stage;                    // LDS: 4 x 64 keys for Transform
  int32_t* surv_id; int32_t* surv_row; float* surv_d;  // LDS, 64 each
  uint32_t pops, evals, gathers;

  static constexpr int kListedBuckets = 8192;
  // From this many keys per fetch on, prioq takes them all at once; fewer are inserted one by one.  (The
  // construction searches insert about 13 keys per fetch, user queries 2 - 3: with the threshold at 3 the
  // fixed cost of the joint insertion made user queries 2 - 10 % slower; at 8 the constructions are 1 - 5 %
  // faster than with per-key counting and user queries unchanged; at 16, or with one-by-one insertion
  // only, the constructions are 3 % and 8 % slower.)
  static constexpr int kMultiInsertFrom = 8;
  // Hash slots (a power of two).  Up to 384 iterations: 1024 slots (4 KB, which six wavefronts per SIMD
  // can afford), filled to three eighths (or by the visited ids plus 128 rejected ids, if that is more):
  // probing a fuller table costs more than the rejected ids it remembers save, an emptier one gathers
  // too many rows again (measured: 1/4, 3/8, 1/2, 3/4).  Beyond, LDS decides how many wavefronts a
  // compute unit holds, and the table may fill to three quarters.
  __host__ __device__ static int hash_slots(int max_iter) {
    int h = 1024;
    if (GV || 2 * max_iter + 256 <= h) return h;
    if (ANY) return (2 * max_iter + 256 + 63) / 64 * 64;
    while (3 * h < 4 * (max_iter + 128)) h <<= 1;
    return h;
  }
  // visited ids plus rejected ids the table may hold
  __host__ __device__ static int hash_fill(int max_iter) {
    const int h = hash_slots(max_iter);
    if (GV) return h / 2;
    if (2 * max_iter + 256 <= h) return (h * 3 / 8 > max_iter + 128) ? h * 3 / 8 : max_iter + 128;
    if (ANY) return h / 2;
    return h / 4 * 3;
  }
  // GV: slots of the visited table in global memory (a power of two, filled to at most one half)
  __host__ __device__ static int vis_slots(int max_iter) {
    int h = 64;
    while (h < 2 * max_iter) h <<= 1;
    return h;
  }
  // the staging area of Transform ((2 NB + 2) x 64 keys) shares its memory with the hash table,
  // which Transform empties anyway
  __host__ __device__ static size_t hash_bytes(const SearchParams& sp) {
    const size_t h = (size_t)hash_slots(sp.max_iter) * 4;
    const size_t st = (size_t)(2 * NB + 2) * 64 * 8;
    return h > st ? h : st;
  }
  __host__ __device__ static size_t lds_bytes(const SearchParams& sp) {
    return hash_bytes(sp) + 3 * 64 * 4 + kListedBuckets / 8;
  }

  __device__ void bind(unsigned char* lds, const SearchParams& sp, int64_t query) {
    B = sp.B; P = sp.P; max_iter = sp.max_iter; tau = sp.tau; dnn = sp.dnn;
    if (GV) {
      const int VS = vis_slots(sp.max_iter);
      vis = sp.vis + (size_t)query * (size_t)VS;
      vmask = VS - 1;
      vshift = 32 - (31 - __builtin_clz((unsigned)VS));
    }
    const int H = hash_slots(sp.max_iter);
    stage = (u64*)lds;
    hash = (int32_t*)lds;
    hmask = H - 1;
    hshift = 32 - (31 - __builtin_clz((unsigned)H));
    surv_id = (int32_t*)(lds + hash_bytes(sp));
    surv_row = surv_id + 64;
    surv_d = (float*)(surv_row + 64);
    listed_bits = (uint32_t*)(surv_d + 64);
    rej_cap = GV ? hash_fill(sp.max_iter) : hash_fill(sp.max_iter) - sp.max_iter;
  }
  // ---- which ids may be in best or prioq: one bit per bucket (a zero bit rules a proposal out)
  // one multiplicative hash serves both tables: its top bits index the visited / rejected table,
  // bits 6.. the bit map
  __device__ __forceinline__ static uint32_t hash_of(int32_t id) { return (uint32_t)id * 0x9E3779B1u; }
  __device__ __forceinline__ static uint32_t listed_bucket(int32_t id) {
    return (hash_of(id) >> 6) & (uint32_t)(kListedBuckets - 1);
  }
  __device__ __forceinline__ uint32_t slot_of(int32_t id) const {
    if constexpr (ANY) return __umul24(hash_of(id) >> 16, (uint32_t)hmask + 1u) >> 16;  // top 16 bits x slots
    else return hash_of(id) >> hshift;
  }
  __device__ __forceinline__ uint32_t next_slot(uint32_t h) const {
    if constexpr (ANY) return h == (uint32_t)hmask ? 0u : h + 1;
    else return (h + 1) & (uint32_t)hmask;
  }
  __device__ void listed_clear() {
    for (int i = lane_id(); i < kListedBuckets / 32; i += kWave) listed_bits[i] = 0;
    wave_sync();
  }
  __device__ __forceinline__ bool maybe_listed(int32_t id) const {
    const uint32_t h = listed_bucket(id);
    return (listed_bits[h >> 5] >> (h & 31)) & 1u;
  }
  // The global table is written and read by this wavefront only: relaxed accesses of work-group scope,
  // and a work-group fence between a write and the reads that must see it.
  __device__ __forceinline__ static int32_t vis_load(const int32_t* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
  }
  __device__ __forceinline__ static void vis_store(int32_t* p, int32_t v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
  }
  __device__ __forceinline__ static void vis_fence() { __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "workgroup"); }
  __device__ void clear_hash() {
    for (int i = lane_id(); i <= hmask; i += kWave) hash[i] = -1;
    nrej = 0;
    if (GV) {
      for (int i = lane_id(); i <= vmask; i += kWave) vis_store(&vis[i], -1);
      vis_fence();
    }
    wave_sync();
  }
  // Alg. 2 Init
  __device__ void init() {
#pragma unroll
    for (int e = 0; e < NB; e++) best[e] = kEmptyKey;
    pq = kEmptyKey;
    nb = np = 0; iter = 0; pops = evals = gathers = 0;
    radius = INFINITY; d1 = dk = thr_now = INFINITY; last_best = kEmptyKey;
    listed_clear();
    clear_hash();
  }
  __device__ void set_radius(float r) { radius = r; }

  // 0: unknown, 1: visited, 2: evaluated before and rejected
  __device__ int probe(int32_t id) const {
    if constexpr (GV) {
      // the first probe of the global table is under way while the LDS table (rejected ids) is searched
      uint32_t gh = hash_of(id) >> vshift;
      int32_t gv = vis_load(&vis[gh]);
      int kind = 0;
      uint32_t h = slot_of(id);
      int32_t v;
      while ((v = hash[h]) != -1) {
        if ((v & 0x7FFFFFFF) == id) { kind = 2; break; }
        h = next_slot(h);
      }
      while (gv != -1) {
        if (gv == id) return 1;
        gh = (gh + 1) & (uint32_t)vmask;
        gv = vis_load(&vis[gh]);
      }
      return kind;
    } else {
      uint32_t h = slot_of(id);
      int32_t v;
      while ((v = hash[h]) != -1) {
        if ((v & 0x7FFFFFFF) == id) return (v < 0) ? 2 : 1;
        h = next_slot(h);
      }
      return 0;
    }
  }
  __device__ void insert_visited(int32_t id) {  // uniform call
    if (GV) {
      if (lane_id() == 0) {
        uint32_t h = hash_of(id) >> vshift;
        while (vis_load(&vis[h]) != -1) h = (h + 1) & (uint32_t)vmask;
        vis_store(&vis[h], id);
      }
      return;  // the fence before the next probes orders this write before them
    }
    if (lane_id() == 0) {
      uint32_t h = slot_of(id);
      while (hash[h] != -1) h = next_slot(h);
      hash[h] = id;
    }
    wave_sync();
  }
  __device__ void insert_rejected(bool mine, int32_t id) {
    const int cnt = __popcll(__ballot(mine));
    if (cnt == 0 || nrej + cnt > rej_cap) return;
    nrej += cnt;
    if (mine) {
      uint32_t h = slot_of(id);
      while (atomicCAS(&hash[h], -1, (int32_t)((uint32_t)id | 0x80000000u)) != -1) h = next_slot(h);
    }
    wave_sync();
  }

  __device__ float first_d() const { return d1; }
  __device__ int32_t count() const { return nb; }
  __device__ uint32_t n_pops() const { return pops; }
  __device__ uint32_t n_evals() const { return evals; }
  __device__ uint32_t n_gathers() const { return gathers; }
  // Eq. 2; d1 / dk are best[0].d and best[B-1].d (+inf while best is not full)
  __device__ float thr() const { return thr_now; }
  __device__ void refresh_bounds() {
    d1 = __uint_as_float((uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(best[0] >> 32), 0));
#pragma unroll
    for (int e = 0; e < NB; e++)
      if (((B - 1) >> 6) == e) last_best = read_lane_u64(best[e], (B - 1) & 63);  // all ones while best is not full
    dk = (nb < B) ? INFINITY : key_d(last_best);
    const float xi = tau * fminf(d1, dnn);
    thr_now = (nb == 0) ? INFINITY : dk + xi;
  }

  // sorted insertion into a register list; entries beyond `cap` fall off
  __device__ static void list_insert(u64& L, int32_t& n, int32_t cap, u64 key) {
    const int lane = lane_id();
    const bool lt = L < key;
    const int pos = __popcll(__ballot(lt));
    // The entries not below the key move up one lane, with only those lanes enabled: the first of
    // them finds its source lane disabled and takes the shift's fill value, the key itself.
    if (!lt) L = wave_shift_up(L, key);
    if (cap < kWave && lane >= cap) L = kEmptyKey;
    if (pos < cap && n < cap) n++;
  }
  // the same for best, which may span several registers: what leaves lane 63 of one register
  // enters lane 0 of the next
  __device__ void best_insert(u64 key) {
    const int lane = lane_id();
    bool lt[NB];
    int pos = 0;
#pragma unroll
    for (int e = 0; e < NB; e++) {
      lt[e] = best[e] < key;
      pos += __popcll(__ballot(lt[e]));
    }
    if (pos >= B) return;
    if (NB == 1) {  // as list_insert: only the entries not below the key are enabled for the shift
      if (!lt[0]) best[0] = wave_shift_up(best[0], key);
      if (lane >= B) best[0] = kEmptyKey;
      if (nb < B) nb++;
      return;
    }
    u64 carry = key;
#pragma unroll
    for (int e = 0; e < NB; e++) {
      const u64 leaving = (e + 1 < NB) ? read_lane_u64(best[e], 63) : 0;
      const u64 up = wave_shift_up(best[e], carry);
      const int gi = e * kWave + lane;
      best[e] = lt[e] ? best[e] : (gi == pos ? key : up);
      if (gi >= B) best[e] = kEmptyKey;
      carry = leaving;
    }
    if (nb < B) nb++;
  }
  // Alg. 2 Pop, first half: take the head off prioq (or -1 when the search on this layer ends).
  // The caller completes the pop with mark_visited(id) once the adjacency load is under way.
  __device__ int32_t pop_head() {
    if (np == 0 || iter >= max_iter) return -1;
    const u64 head = read_lane_u64(pq, 0);
    const float d = key_d(head);
    if (!(d <= thr() && d <= radius)) return -1;
    pq = wave_shift_down(pq, kEmptyKey);
    np--;
    iter++;
    pops++;
    return key_id(head);
  }
  __device__ void mark_visited(int32_t id) {
    insert_visited(id);
    if ((iter & (kRelistEvery - 1)) == 0) relist();
  }
  // The bit map only ever gains bits while a layer is searched, and most ids that enter prioq fall off
  // its end again: every kRelistEvery iterations it is rebuilt from the two lists as they stand, so that
  // a set bit keeps meaning "probably listed" (few exact membership tests) in long searches too.
  static constexpr int kRelistEvery = 4;
  __device__ void relist() {
    listed_clear();
    mark_lists();
    wave_sync();
  }
  __device__ __forceinline__ void mark_lists() {
    const int lane = lane_id();
#pragma unroll
    for (int e = 0; e < NB; e++) {
      if (e * kWave + lane < nb) {
        const uint32_t h = listed_bucket(key_id(best[e]));
        atomicOr(&listed_bits[h >> 5], 1u << (h & 31));
      }
    }
    if (lane < np) {
      const uint32_t h = listed_bucket(key_id(pq));
      atomicOr(&listed_bits[h >> 5], 1u << (h & 31));
    }
  }
  __device__ int32_t next_head() const { return np > 0 ? key_id(read_lane_u64(pq, 0)) : -1; }
  __device__ int32_t pop() {
    const int32_t id = pop_head();
    if (id >= 0) mark_visited(id);
    return id;
  }

  // Alg. 4 Transform (see the LDS variant in ggnn_device.h for the reading); staged through LDS
  __device__ void transform(const int32_t* __restrict__ table) {
    const int lane = lane_id();
    u64* sb = stage; u64* sp = stage + NB * 64; u64* out = stage + (NB + 1) * 64;
#pragma unroll
    for (int e = 0; e < NB; e++) {
      const int gi = e * kWave + lane;
      if (gi < nb) best[e] = (best[e] & 0xFFFFFFFF00000000ull) | (uint32_t)table[key_id(best[e])];
      sb[gi] = best[e];
    }
    if (lane < np) pq = (pq & 0xFFFFFFFF00000000ull) | (uint32_t)table[key_id(pq)];
    wave_sync();
    // best: same distances, ties re-ordered by the new ids
#pragma unroll
    for (int e = 0; e < NB; e++) {
      if (e * kWave + lane < nb) {
        int r = 0;
        for (int j = 0; j < nb; j++) r += sb[j] < best[e];
        out[r] = best[e];
      }
    }
    wave_sync();
#pragma unroll
    for (int e = 0; e < NB; e++) best[e] = (e * kWave + lane < nb) ? out[e * kWave + lane] : kEmptyKey;
    wave_sync();
#pragma unroll
    for (int e = 0; e < NB; e++) sb[e * kWave + lane] = best[e];
    // prioq entries that are also in best are dropped from the union
    bool dup = false;
    if (lane < np)
      for (int j = 0; j < nb; j++) dup = dup || key_id(out[j]) == key_id(pq);
    sp[lane] = (lane < np && !dup) ? pq : kEmptyKey;
    wave_sync();
    const int m = nb + __popcll(__ballot(lane < np && !dup));
    // rank of every entry in the union; the P smallest form the new prioq
    int rb[NB], rp = 0;
#pragma unroll
    for (int e = 0; e < NB; e++) {
      rb[e] = e * kWave + lane;
      for (int j = 0; j < np; j++) rb[e] += sp[j] < best[e];
    }
    const u64 mine = sp[lane];
    for (int j = 0; j < nb; j++) rp += sb[j] < mine;
    for (int j = 0; j < np; j++) rp += sp[j] < mine;
    wave_sync();
#pragma unroll
    for (int e = 0; e < NB; e++)
      if (e * kWave + lane < nb && rb[e] < kWave) out[rb[e]] = best[e];
    if (mine != kEmptyKey && rp < kWave) out[rp] = mine;
    wave_sync();
    np = m < P ? m : P;
    pq = (lane < np) ? out[lane] : kEmptyKey;
    iter = 0;
    if (nb > 0) refresh_bounds();
    listed_clear();
    mark_lists();
    clear_hash();
  }

  // Alg. 2 Fetch
  template <int DT, int NCH, int METRIC, int PASSES>
  __device__ void fetch(const GraphDev& G, int layer, int32_t p, const QueryRegs<DT, NCH>& q, int32_t excl_row) {
    const int lane = lane_id();
    bool alive = p >= 0;
    int32_t row = -1;
    if (alive) {
      row = (layer == 0) ? p : G.to_base[layer][p];
      alive = row != excl_row;
    }
    const bool bit = maybe_listed(p);  // read alongside the first probe, not after the last (any p indexes the map)
    bool seen_rejected = false;
    if constexpr (GV) vis_fence();  // the popped id's entry is in the table (the adjacency row was awaited anyway)
    if (alive) {
      const int kind = probe(p);
      alive = kind == 0;
      seen_rejected = kind == 2;
    }
    // membership in best / prioq: only proposals whose bucket bit is set can be listed;
    // each of those is broadcast and compared with the entry every lane holds
    u64 cand = __ballot(alive && bit);
    u64 known = 0;
    while (cand) {
      const int j = __builtin_ctzll(cand);
      cand &= cand - 1;
      const int32_t pid = __builtin_amdgcn_readlane(p, j);
      bool hit = key_id(pq) == pid;
#pragma unroll
      for (int e = 0; e < NB; e++) hit = hit || key_id(best[e]) == pid;
      if (__ballot(hit)) known |= 1ull << j;
    }
    alive = alive && !((known >> lane) & 1);
    const u64 mask = __ballot(alive);
    const int ns = __popcll(mask);
    // a point rejected before would be evaluated and rejected again: counted, not gathered
    evals += ns + __popcll(__ballot(seen_rejected));
    if (ns == 0) return;
    gathers += ns;
    if (alive) {
      const int r = __popcll(mask & ((1ull << lane) - 1));
      surv_id[r] = p;
      surv_row[r] = row;
    }
    wave_sync();
    // rows of one chunk per lane (128 bytes) cost four registers each: a third pass is in flight
    constexpr int RPP = RowSched<DT, PASSES>::rows_per_pass;
    constexpr int NP = (Elem<DT>::lanes == kRowLanes && NCH == 1) ? RowSched<DT, PASSES>::passes + 1 : RowSched<DT, PASSES>::passes;
    for (int b0 = 0; b0 < ns; b0 += RPP * NP) gather_sum<DT, NCH, METRIC, NP, !A64>(G, q, surv_row, surv_d, b0, ns);
    wave_sync();
    // Alg. 2 Push, for the survivors in list order with the threshold re-evaluated after every push.
    // The threshold only shrinks, and only when a key enters best: the candidates that may enter
    // best are taken one by one, in order, and every lane notes the threshold in force when its own
    // candidate is reached; all others are decided at once against that threshold.
    const bool mine = lane < ns;
    const float d = mine ? finish_distance<METRIC>(surv_d[lane]) : INFINITY;  // one sqrt for the whole fetch
    const int32_t id = mine ? surv_id[lane] : -1;
    const u64 key = make_key(d, id);
    const bool in = mine && d <= thr() && d <= radius;
    const u64 last_best0 = (nb < B) ? kEmptyKey : last_best;
    float mythr = thr();
    u64 first = __ballot(in && key < last_best0);
    while (first) {
      const int r = __builtin_ctzll(first);
      first &= first - 1;
      const u64 kr = read_lane_u64(key, r);
      if (key_d(kr) <= thr() && (nb < B || kr < last_best)) {
        best_insert(kr);
        refresh_bounds();
        mythr = (lane > r) ? thr() : mythr;
      }
    }
    const bool ok = in && d <= mythr;  // accepted
    // prioq: a key beyond the last entry of a full prioq would fall off at once
    const u64 pq_last = (np < P) ? kEmptyKey : read_lane_u64(pq, P - 1);
    const bool goes_in = ok && key < pq_last;
    u64 ins = __ballot(goes_in);
    const int m = __popcll(ins);
    if (m < kMultiInsertFrom) {
      while (ins) {
        const int r = __builtin_ctzll(ins);
        ins &= ins - 1;
        list_insert(pq, np, P, read_lane_u64(key, r));
      }
    } else {
      // Several keys at once: every prioq entry counts the new keys below it (it moves up by that
      // many places), every new key counts the entries and the other new keys below it; both
      // then go to their places through LDS (the survivor arrays are free by now).  The result is
      // that of inserting one by one: the P smallest of the union, in order.
      // The survivor lanes are read in turn, eight per trip (a key that is not inserted reads as the
      // empty key, which is below nothing), so that a key costs two lane reads, two compares and two
      // adds and no scalar bookkeeping; the number of prioq entries below a new key is found by a
      // binary search over the lanes of the sorted prioq.
      const u64 kin = goes_in ? key : kEmptyKey;
      int up = 0, rank = 0;
      for (int t0 = 0; t0 < ns; t0 += 8) {
#pragma unroll
        for (int t = 0; t < 8; t++) {
          const u64 kr = read_lane_u64(kin, t0 + t);
          up += (kr < pq) ? 1 : 0;
          rank += (kr < key) ? 1 : 0;
        }
      }
      int below = 0;
#pragma unroll
      for (int step = kWave / 2; step >= 1; step >>= 1) {
        const u64 e = lane_gather_u64(pq, below + step - 1);
        below += (e < kin) ? step : 0;
      }
      rank += below;
      u64* out = (u64*)surv_id;  // 64 keys: surv_id and surv_row
      if (lane < np && lane + up < P) out[lane + up] = pq;
      if (goes_in && rank < P) out[rank] = key;
      wave_sync();
      np = (np + m < P) ? np + m : P;
      pq = (lane < np) ? out[lane] : kEmptyKey;
      wave_sync();
    }
    if (ok && (key < pq_last || key < last_best0)) {  // whatever entered a list is marked in the bit map
      const uint32_t h = listed_bucket(id);
      atomicOr(&listed_bits[h >> 5], 1u << (h & 31));
    }
    insert_rejected(mine && !ok, id);
  }

  // the lists and counters of a search that continues in another launch
  __device__ __forceinline__ void save_state(u64* __restrict__ st, int32_t* __restrict__ meta) const {
    const int lane = lane_id();
#pragma unroll
    for (int e = 0; e < NB; e++) st[e * kWave + lane] = best[e];
    st[NB * kWave + lane] = pq;
    if (lane == 0) {
      meta[0] = nb; meta[1] = np; meta[2] = (int32_t)pops; meta[3] = (int32_t)evals; meta[4] = (int32_t)gathers;
    }
  }
  __device__ __forceinline__ void load_state(const u64* __restrict__ st, const int32_t* __restrict__ meta) {  // after init()
    const int lane = lane_id();
#pragma unroll
    for (int e = 0; e < NB; e++) best[e] = st[e * kWave + lane];
    pq = st[NB * kWave + lane];
    nb = meta[0]; np = meta[1]; pops = (uint32_t)meta[2]; evals = (uint32_t)meta[3]; gathers = (uint32_t)meta[4];
  }
  __device__ int32_t first_id() const { return nb > 0 ? key_id(read_lane_u64(best[0], 0)) : 0; }

  // results
  __device__ void store_results(int k, int32_t* __restrict__ ids, float* __restrict__ dists) const {
    const int lane = lane_id();
#pragma unroll
    for (int e = 0; e < NB; e++) {
      const int j = e * kWave + lane;
      if (j < k) {
        ids[j] = (j < nb) ? key_id(best[e]) : -1;
        dists[j] = (j < nb) ? key_d(best[e]) : INFINITY;
      }
    }
    for (int j = NB * kWave + lane; j < k; j += kWave) {  // best cannot hold that many
      ids[j] = -1;
      dists[j] = INFINITY;
    }
  }
  __device__ void store_row(int K, int32_t* __restrict__ out) const {
    const int lane = lane_id();
    if (lane < K) out[lane] = (lane < nb) ? key_id(best[0]) : -1;  // K <= 64
  }
  __device__ void store_prefs(u64* __restrict__ pref, int32_t* __restrict__ npref) const {
    const int lane = lane_id();
#pragma unroll
    for (int e = 0; e < NB; e++)
      if (e * kWave + lane < nb) pref[e * kWave + lane] = best[e];
    if (lane == 0) *npref = nb;
  }
};

using RegCache = RegCacheT<1>;   // best of at most 64 entries
using RegCache2 = RegCacheT<2>;  // best of at most 128 entries
using RegCacheGV = RegCacheT<1, true>;   // the same with the visited ids in global memory (user queries)
using RegCache2GV = RegCacheT<2, true>;
using RegCacheAny = RegCacheT<1, false, true>;  // LDS table of any multiple of 64 slots (user queries)
using RegCache2Any = RegCacheT<2, false, true>;

}  // namespace ggnn
