/*
 * ggnn_ref.c -- CPU oracle for the GGNN hot path (arxiv 1912.01059).
 *
 * TEST INFRASTRUCTURE ONLY: plain scalar C, written from the paper, independent of
 * the HIP library (no shared code, headers, tables or helpers).  See ggnn_ref.h.
 *
 * Readings of the paper fixed here (each is also stated where it is used):
 *  - distances are plain Euclidean norms, not squared (Eq. 1, Eq. 2);
 *  - every ordered structure uses the total order (distance, id);
 *  - float32 sums follow one fixed tree so that a parallel implementation can
 *    reproduce them bit for bit: the row is cut into 16-byte chunks, chunk c goes to
 *    accumulator c mod `lanes`, every accumulator runs acc = fma(t, t, acc) over its
 *    chunks in ascending order, and the accumulators are then combined by a
 *    butterfly (distance lanes/2, ..., 2, 1).
 */
#include "ggnn_ref.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define MAXL GGNN_REF_MAX_LEVELS

struct ggnn_ref_graph {
  int64_t N;
  int D, K, L, s, g;
  int dtype, metric, lanes;
  uint64_t seed;
  int64_t n[MAXL], G[MAXL];
  int32_t* edges[MAXL];
  int32_t* to_lower[MAXL];
  int32_t* to_base[MAXL];
  int32_t* inv_count[MAXL];
  float* dnn1;
  float stats[2]; /* mean, max of dnn1 (Sec. 4.1, Eq. 3 and Eq. 4) */
  const void* base;
  float* norm; /* cosine: owned unit-length copy of base */
};

typedef struct {
  float d;
  int32_t id;
} ent;

static int ent_less(ent a, ent b) { return a.d < b.d || (a.d == b.d && a.id < b.id); }

int ggnn_ref_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

void ggnn_ref_set_num_threads(int n) {
#ifdef _OPENMP
  if (n >= 1) omp_set_num_threads(n);
#else
  (void)n;
#endif
}

/* ------------------------------------------------------------------ hashing */

static uint64_t mix64(uint64_t x) {
  x ^= x >> 30; x *= 0xBF58476D1CE4E5B9ull;
  x ^= x >> 27; x *= 0x94D049BB133111EBull;
  x ^= x >> 31;
  return x;
}
static uint32_t mix32(uint32_t h) {
  h ^= h >> 16; h *= 0x85EBCA6Bu;
  h ^= h >> 13; h *= 0xC2B2AE35u;
  h ^= h >> 16;
  return h;
}

/* Bottom-layer partition (Sec. 4.1 "logically partition the entire dataset into
 * small batches"; Fig. 1 calls it random): a seeded bijection of [0,N) made of a
 * 4-round balanced Feistel network on 2h bits, 4^h >= N, iterated until the value
 * falls below N (cycle walking). */
static int feistel_half_bits(int64_t N) {
  int h = 1;
  while ((((int64_t)1) << (2 * h)) < N) h++;
  return h;
}
static uint32_t feistel_key(uint64_t seed, int r) {
  return (uint32_t)mix64(seed + 0x9E3779B97F4A7C15ull * (uint64_t)(r + 1));
}
int64_t ggnn_ref_perm(uint64_t seed, int64_t N, int64_t p) {
  int h = feistel_half_bits(N);
  uint32_t mask = (uint32_t)((((uint64_t)1) << h) - 1);
  uint64_t x = (uint64_t)p;
  do {
    uint32_t Lh = (uint32_t)(x >> h) & mask, Rh = (uint32_t)x & mask;
    for (int r = 0; r < 4; r++) {
      uint32_t f = mix32(Rh ^ feistel_key(seed, r)) & mask;
      uint32_t t = Lh ^ f;
      Lh = Rh;
      Rh = t;
    }
    x = ((uint64_t)Lh << h) | Rh;
  } while ((int64_t)x >= N);
  return (int64_t)x;
}
int64_t ggnn_ref_perm_inv(uint64_t seed, int64_t N, int64_t row) {
  int h = feistel_half_bits(N);
  uint32_t mask = (uint32_t)((((uint64_t)1) << h) - 1);
  uint64_t x = (uint64_t)row;
  do {
    uint32_t Lh = (uint32_t)(x >> h) & mask, Rh = (uint32_t)x & mask;
    for (int r = 3; r >= 0; r--) {
      uint32_t f = mix32(Lh ^ feistel_key(seed, r)) & mask;
      uint32_t t = Rh ^ f;
      Rh = Lh;
      Lh = t;
    }
    x = ((uint64_t)Lh << h) | Rh;
  } while ((int64_t)x >= N);
  return (int64_t)x;
}

double ggnn_ref_uniform(uint64_t seed, int l_top, int64_t row) {
  uint64_t x = mix64(seed ^ mix64(((uint64_t)l_top << 56) + (uint64_t)row + 0x632BE59BD9B4E019ull));
  return ((double)(x >> 12) + 0.5) * (1.0 / 4503599627370496.0); /* 2^-52 */
}

/* ----------------------------------------------------------------- geometry */

static int64_t ipow(int64_t b, int e) {
  int64_t r = 1;
  for (int i = 0; i < e; i++) r *= b;
  return r;
}

/* Sec. 4.3 and appendix "Graph Size": g ~ (N/s)^(1/(L-1)), rounded up or down such
 * that the bottom segment size s0 = N / g^(L-1) is closest to s; upper layer l holds
 * s * g^(L-1-l) points in g^(L-1-l) segments of s points. */
int ggnn_ref_geometry(int64_t N, int s, int L, int32_t* g_out, int64_t* n, int64_t* G) {
  if (N < 2 || s < 2 || L < 2 || L > MAXL) return -1;
  double gs = pow((double)N / (double)s, 1.0 / (double)(L - 1));
  int64_t cand[2];
  cand[0] = (int64_t)floor(gs);
  cand[1] = (int64_t)ceil(gs);
  int64_t best_g = -1;
  double best_err = 0.0;
  for (int i = 0; i < 2; i++) {
    int64_t c = cand[i] < 1 ? 1 : cand[i];
    double err = fabs((double)N / (double)ipow(c, L - 1) - (double)s);
    if (best_g < 0 || err < best_err) { /* on a tie the smaller factor stays */
      best_g = c;
      best_err = err;
    }
  }
  if (best_g < 1) return -1;
  int64_t g = best_g;
  for (int l = 0; l < L; l++) {
    G[l] = ipow(g, L - 1 - l);
    n[l] = (l == 0) ? N : (int64_t)s * G[l];
  }
  if (G[0] > N) return -1;
  /* every child must be able to supply its share of a parent segment */
  int64_t s0_min = N / G[0];
  int64_t share_max = ((int64_t)s + g - 1) / g;
  if (s0_min < share_max || s0_min < 2) return -1;
  if (L > 2 && n[1] > N) return -1;
  *g_out = (int32_t)g;
  return 0;
}

static int64_t seg0_lo(const ggnn_ref_graph* g, int64_t j) { return (j * g->N) / g->G[0]; }
static int64_t seg0_of_pos(const ggnn_ref_graph* g, int64_t pos) {
  return ((pos + 1) * g->G[0] - 1) / g->N;
}
/* segment index of point id of layer l */
static int64_t seg_of(const ggnn_ref_graph* g, int l, int64_t id) {
  if (l == 0) return seg0_of_pos(g, ggnn_ref_perm_inv(g->seed, g->N, id));
  return id / g->s;
}
static int64_t base_of(const ggnn_ref_graph* g, int l, int32_t id) {
  return l == 0 ? (int64_t)id : (int64_t)g->to_base[l][id];
}

/* ----------------------------------------------------------------- distance */

static int row_dtype(const ggnn_ref_graph* g) { return g->norm ? GGNN_REF_F32 : g->dtype; }
static const void* row_ptr(const ggnn_ref_graph* g, int64_t row) {
  if (g->norm) return g->norm + row * g->D;
  if (g->dtype == GGNN_REF_U8) return (const uint8_t*)g->base + row * g->D;
  return (const float*)g->base + row * g->D;
}

/* The fixed float32 summation tree described at the top of this file.
 * mode 0: sum of (q-x)^2, mode 1: sum of q*x. */
static float tree_sum(const float* q, const void* row, int D, int dtype, int lanes, int mode) {
  float part[64];
  int per_chunk = (dtype == GGNN_REF_U8) ? 16 : 4;
  int nchunks = (D + per_chunk - 1) / per_chunk;
  for (int l = 0; l < lanes; l++) part[l] = 0.0f;
  for (int c = 0; c < nchunks; c++) {
    int l = c % lanes;
    for (int e = 0; e < per_chunk; e++) {
      int j = c * per_chunk + e;
      if (j >= D) break;
      float x = (dtype == GGNN_REF_U8) ? (float)((const uint8_t*)row)[j] : ((const float*)row)[j];
      if (mode == 0) {
        float t = q[j] - x;
        part[l] = fmaf(t, t, part[l]);
      } else {
        part[l] = fmaf(q[j], x, part[l]);
      }
    }
  }
  for (int step = lanes / 2; step >= 1; step /= 2) {
    float nxt[64];
    for (int l = 0; l < lanes; l++) nxt[l] = part[l] + part[l ^ step];
    for (int l = 0; l < lanes; l++) part[l] = nxt[l];
  }
  return part[0];
}

float ggnn_ref_distance(const float* q, const void* row, int D, int dtype, int metric, int lanes) {
  if (metric == GGNN_REF_COSINE) {
    float dot = tree_sum(q, row, D, dtype, lanes, 1);
    return fmaxf(0.0f, 1.0f - dot);
  }
  return sqrtf(tree_sum(q, row, D, dtype, lanes, 0));
}

/* unit-length copy: x / sqrt(sum x^2), the sum taken over the same tree */
static void normalise(const float* x, int D, int lanes, float* out) {
  float nrm = sqrtf(tree_sum(x, x, D, GGNN_REF_F32, lanes, 1));
  for (int j = 0; j < D; j++) out[j] = (nrm > 0.0f) ? x[j] / nrm : x[j];
}

static void to_float_row(const void* src, int64_t idx, int D, int dtype, float* out) {
  if (dtype == GGNN_REF_U8) {
    const uint8_t* p = (const uint8_t*)src + idx * D;
    for (int j = 0; j < D; j++) out[j] = (float)p[j];
  } else {
    memcpy(out, (const float*)src + idx * D, sizeof(float) * (size_t)D);
  }
}

/* -------------------------------------------------------------- brute force */

/* Sec. 3.1: the k rows with the smallest distance to q, ascending by (d, id). */
int ggnn_ref_bruteforce(const void* base, int64_t N, int D, int dtype, int metric, int lanes,
                        const void* queries, int64_t Q, int k, int32_t* ids, float* dists) {
  if (k < 1 || N < 1 || D < 1) return -1;
  float* nb = NULL;
  const void* rows = base;
  int rdt = dtype;
  if (metric == GGNN_REF_COSINE) {
    nb = (float*)malloc(sizeof(float) * (size_t)N * D);
    if (!nb) return -2;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < N; i++) {
      float tmp[4096];
      to_float_row(base, i, D, dtype, tmp);
      normalise(tmp, D, lanes, nb + i * D);
    }
    rows = nb;
    rdt = GGNN_REF_F32;
  }
  size_t rb = (size_t)D * (rdt == GGNN_REF_U8 ? 1 : 4);
#pragma omp parallel for schedule(dynamic, 1)
  for (int64_t qi = 0; qi < Q; qi++) {
    float q[4096], qn[4096];
    to_float_row(queries, qi, D, dtype, q);
    if (metric == GGNN_REF_COSINE) {
      normalise(q, D, lanes, qn);
      memcpy(q, qn, sizeof(float) * (size_t)D);
    }
    ent* top = (ent*)malloc(sizeof(ent) * (size_t)k);
    int cnt = 0;
    for (int64_t i = 0; i < N; i++) {
      ent e;
      e.d = ggnn_ref_distance(q, (const char*)rows + (size_t)i * rb, D, rdt, metric, lanes);
      e.id = (int32_t)i;
      if (cnt == k && !ent_less(e, top[k - 1])) continue;
      int pos = (cnt < k) ? cnt : k - 1;
      while (pos > 0 && ent_less(e, top[pos - 1])) {
        top[pos] = top[pos - 1];
        pos--;
      }
      top[pos] = e;
      if (cnt < k) cnt++;
    }
    for (int j = 0; j < k; j++) {
      ids[qi * k + j] = (j < cnt) ? top[j].id : -1;
      dists[qi * k + j] = (j < cnt) ? top[j].d : INFINITY;
    }
    free(top);
  }
  free(nb);
  return 0;
}

/* -------------------------------------------------------------------- graph */

ggnn_ref_graph* ggnn_ref_graph_create(const void* base, int64_t N, int D, int K, int L, int s,
                                      int dtype, int metric, uint64_t seed, int lanes) {
  if (!base || D < 1 || D > 4096 || K < 2 || lanes < 1 || lanes > 64 || (lanes & (lanes - 1))) return NULL;
  ggnn_ref_graph* g = (ggnn_ref_graph*)calloc(1, sizeof(*g));
  if (!g) return NULL;
  g->N = N; g->D = D; g->K = K; g->L = L; g->s = s;
  g->dtype = dtype; g->metric = metric; g->lanes = lanes; g->seed = seed; g->base = base;
  int32_t gf;
  if (ggnn_ref_geometry(N, s, L, &gf, g->n, g->G) != 0) { free(g); return NULL; }
  g->g = gf;
  for (int l = 0; l < L; l++) {
    size_t cnt = (size_t)g->n[l] * (size_t)K;
    g->edges[l] = (int32_t*)malloc(sizeof(int32_t) * cnt);
    for (size_t i = 0; i < cnt; i++) g->edges[l][i] = -1;
    g->inv_count[l] = (int32_t*)calloc((size_t)g->n[l], sizeof(int32_t));
    if (l >= 1) {
      g->to_lower[l] = (int32_t*)malloc(sizeof(int32_t) * (size_t)g->n[l]);
      g->to_base[l] = (int32_t*)malloc(sizeof(int32_t) * (size_t)g->n[l]);
      for (int64_t i = 0; i < g->n[l]; i++) g->to_lower[l][i] = g->to_base[l][i] = -1;
    }
  }
  g->dnn1 = (float*)calloc((size_t)N, sizeof(float));
  g->stats[0] = g->stats[1] = 0.0f;
  if (metric == GGNN_REF_COSINE) {
    g->norm = (float*)malloc(sizeof(float) * (size_t)N * D);
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < N; i++) {
      float tmp[4096];
      to_float_row(base, i, D, dtype, tmp);
      normalise(tmp, D, lanes, g->norm + i * D);
    }
  }
  return g;
}

void ggnn_ref_graph_free(ggnn_ref_graph* g) {
  if (!g) return;
  for (int l = 0; l < g->L; l++) {
    free(g->edges[l]); free(g->to_lower[l]); free(g->to_base[l]); free(g->inv_count[l]);
  }
  free(g->dnn1); free(g->norm); free(g);
}
int32_t ggnn_ref_graph_g(const ggnn_ref_graph* g) { return g->g; }
int64_t ggnn_ref_graph_n(const ggnn_ref_graph* g, int l) { return (l >= 0 && l < g->L) ? g->n[l] : -1; }
int32_t* ggnn_ref_graph_edges(ggnn_ref_graph* g, int l) { return (l >= 0 && l < g->L) ? g->edges[l] : NULL; }
int32_t* ggnn_ref_graph_to_lower(ggnn_ref_graph* g, int l) { return (l >= 1 && l < g->L) ? g->to_lower[l] : NULL; }
int32_t* ggnn_ref_graph_to_base(ggnn_ref_graph* g, int l) { return (l >= 1 && l < g->L) ? g->to_base[l] : NULL; }
int32_t* ggnn_ref_graph_inv_count(ggnn_ref_graph* g, int l) { return (l >= 0 && l < g->L) ? g->inv_count[l] : NULL; }
float* ggnn_ref_graph_dnn1(ggnn_ref_graph* g) { return g->dnn1; }
float* ggnn_ref_graph_stats(ggnn_ref_graph* g) { return g->stats; }
const float* ggnn_ref_graph_normalised(const ggnn_ref_graph* g) { return g->norm; }

/* -------------------------------------------------------------------- cache */

/* The multi-purpose cache of Sec. 3.1.1 / Alg. 2 as a scalar state machine. */
typedef struct {
  const ggnn_ref_graph* g;
  const float* q;      /* query vector (float32; unit length for cosine) */
  int B, P, V, max_iter;
  float tau, dnn, radius;
  ent* best; int nb;   /* sorted, capacity B  */
  ent* pq; int np;     /* sorted, capacity P, holds not-yet-popped candidates */
  int32_t* vis; int nv, vhead; /* FIFO ring of popped ids, capacity V */
  int iter;
  int64_t excl_base;   /* base row never admitted (the query's own row), or -1 */
  uint32_t pops, evals;
} cache_t;

static int cache_alloc(cache_t* c, int B, int P, int V) {
  c->best = (ent*)malloc(sizeof(ent) * (size_t)(B > 0 ? B : 1));
  c->pq = (ent*)malloc(sizeof(ent) * (size_t)(P > 0 ? P : 1));
  c->vis = (int32_t*)malloc(sizeof(int32_t) * (size_t)(V > 0 ? V : 1));
  c->B = B; c->P = P; c->V = V;
  return (c->best && c->pq && c->vis) ? 0 : -1;
}
static void cache_release(cache_t* c) { free(c->best); free(c->pq); free(c->vis); }

/* Alg. 2 Init */
static void cache_init(cache_t* c, const ggnn_ref_graph* g, const float* q, float tau, float dnn,
                       int max_iter, int64_t excl_base) {
  c->g = g; c->q = q; c->tau = tau; c->dnn = dnn; c->radius = INFINITY;
  c->max_iter = max_iter; c->excl_base = excl_base;
  c->nb = c->np = c->nv = c->vhead = 0; c->iter = 0; c->pops = c->evals = 0;
}

/* Eq. 2: d_best_k + xi, xi = tau * min(d_best_1, d_nn1).  While best is not full the
 * k-th best distance is +inf, so everything is admitted. */
static float cache_thr(const cache_t* c) {
  if (c->nb == 0) return INFINITY;
  float dk = (c->nb < c->B) ? INFINITY : c->best[c->B - 1].d;
  float xi = c->tau * fminf(c->best[0].d, c->dnn);
  return dk + xi;
}
/* Alg. 2 Criteria (plus the search-radius bound of Sec. 4.2.1 when one is set) */
static int cache_crit(const cache_t* c, float d) { return d <= cache_thr(c) && d <= c->radius; }

static int list_has(const ent* a, int n, int32_t id) {
  for (int i = 0; i < n; i++) if (a[i].id == id) return 1;
  return 0;
}
static int cache_known(const cache_t* c, int32_t id) {
  if (list_has(c->best, c->nb, id) || list_has(c->pq, c->np, id)) return 1;
  for (int i = 0; i < c->nv; i++) if (c->vis[i] == id) return 1;
  return 0;
}

static void sorted_insert(ent* a, int* n, int cap, ent e) {
  if (cap <= 0) return;
  if (*n == cap && !ent_less(e, a[cap - 1])) return;
  int pos = (*n < cap) ? *n : cap - 1;
  while (pos > 0 && ent_less(e, a[pos - 1])) { a[pos] = a[pos - 1]; pos--; }
  a[pos] = e;
  if (*n < cap) (*n)++;
}
/* Alg. 2 Push: one sorted insertion into best and into prioq; an entry that falls
 * off the end of either list is lost. */
static void cache_push(cache_t* c, int32_t id, float d) {
  ent e; e.d = d; e.id = id;
  sorted_insert(c->best, &c->nb, c->B, e);
  sorted_insert(c->pq, &c->np, c->P, e);
}

/* Alg. 2 Fetch.  Known points are removed from the proposals against the cache as it
 * stands before the fetch; the survivors are then taken in list order, the criterion
 * being re-evaluated after every push. */
static void cache_fetch(cache_t* c, int layer, const int32_t* list, int n) {
  int32_t surv[1024];
  int ns = 0;
  for (int i = 0; i < n; i++) {
    int32_t p = list[i];
    if (p < 0) continue;
    if (c->excl_base >= 0 && base_of(c->g, layer, p) == c->excl_base) continue;
    if (cache_known(c, p)) continue;
    surv[ns++] = p;
  }
  for (int i = 0; i < ns; i++) {
    int32_t p = surv[i];
    float d = ggnn_ref_distance(c->q, row_ptr(c->g, base_of(c->g, layer, p)), c->g->D,
                                row_dtype(c->g), c->g->metric, c->g->lanes);
    c->evals++;
    if (cache_crit(c, d)) cache_push(c, p, d);
  }
}

/* Alg. 2 Pop: head of prioq, or -1 when the head fails the criterion, the queue is
 * empty or the iteration limit is reached.  The popped id enters visited. */
static int32_t cache_pop(cache_t* c) {
  if (c->np == 0) return -1;
  if (!cache_crit(c, c->pq[0].d)) return -1;
  if (c->iter >= c->max_iter) return -1;
  int32_t id = c->pq[0].id;
  for (int i = 1; i < c->np; i++) c->pq[i - 1] = c->pq[i];
  c->np--;
  if (c->V > 0) {
    c->vis[c->vhead] = id;
    c->vhead = (c->vhead + 1) % c->V;
    if (c->nv < c->V) c->nv++;
  }
  c->iter++;
  c->pops++;
  return id;
}

/* Alg. 4 Transform: ids become the ids of the same points one layer further down (or
 * on the bottom layer), distances are kept, every point may be visited again: visited
 * is emptied and prioq is re-seeded with best and the left-over prioq entries. */
static void cache_transform(cache_t* c, const int32_t* table) {
  for (int i = 0; i < c->nb; i++) c->best[i].id = table[c->best[i].id];
  for (int i = 0; i < c->np; i++) c->pq[i].id = table[c->pq[i].id];
  /* best keeps its order by distance but equal distances may need re-ordering by id */
  for (int i = 1; i < c->nb; i++) {
    ent e = c->best[i]; int j = i;
    while (j > 0 && ent_less(e, c->best[j - 1])) { c->best[j] = c->best[j - 1]; j--; }
    c->best[j] = e;
  }
  ent* all = (ent*)malloc(sizeof(ent) * (size_t)(c->nb + c->np + 1));
  int na = 0;
  for (int i = 0; i < c->nb; i++) all[na++] = c->best[i];
  for (int i = 0; i < c->np; i++) if (!list_has(c->best, c->nb, c->pq[i].id)) all[na++] = c->pq[i];
  for (int i = 1; i < na; i++) {
    ent e = all[i]; int j = i;
    while (j > 0 && ent_less(e, all[j - 1])) { all[j] = all[j - 1]; j--; }
    all[j] = e;
  }
  c->np = (na < c->P) ? na : c->P;
  for (int i = 0; i < c->np; i++) c->pq[i] = all[i];
  free(all);
  c->nv = c->vhead = 0;
  c->iter = 0;
}

/* Alg. 1 main loop on one layer */
static void cache_descend(cache_t* c, int layer) {
  const ggnn_ref_graph* g = c->g;
  int32_t a;
  while ((a = cache_pop(c)) >= 0) cache_fetch(c, layer, g->edges[layer] + (int64_t)a * g->K, g->K);
}

/* -------------------------------------------------------------------- query */

int ggnn_ref_query(const ggnn_ref_graph* g, const void* queries, int64_t Q, int k,
                   int B, float tau, int P, int V, int max_iter, int every_layer,
                   int32_t* ids, float* dists, uint32_t* counters) {
  return ggnn_ref_query_from(g, queries, Q, k, B, tau, P, V, max_iter, every_layer, NULL, 0, ids, dists, counters);
}

/* The same with explicit start points: when `start` is given, Alg. 1 runs on the bottom layer alone
 * from those points (a flat graph; appendix "Query Starting Points"). */
int ggnn_ref_query_from(const ggnn_ref_graph* g, const void* queries, int64_t Q, int k,
                        int B, float tau, int P, int V, int max_iter, int every_layer,
                        const int32_t* start_ids, int n_start,
                        int32_t* ids, float* dists, uint32_t* counters) {
  if (!g || !queries || k < 1 || B < k || P < 1 || V < 1 || max_iter < 0) return -1;
  int top = g->L - 1;
  int err = 0;
#pragma omp parallel for schedule(dynamic, 16)
  for (int64_t qi = 0; qi < Q; qi++) {
    float q[4096], qn[4096];
    to_float_row(queries, qi, g->D, g->dtype, q);
    if (g->metric == GGNN_REF_COSINE) { normalise(q, g->D, g->lanes, qn); memcpy(q, qn, sizeof(float) * (size_t)g->D); }
    cache_t c;
    if (cache_alloc(&c, B, P, V) != 0) { err = 1; continue; }
    /* user queries use the maximum first-neighbour distance in the slack (Eq. 2, Eq. 3) */
    cache_init(&c, g, q, tau, g->stats[1], max_iter, -1);
    /* start points: the s points of the top layer (Sec. 3.1, Sec. 4.4) */
    int32_t start[1024];
    int ns = (int)g->n[top];
    for (int i = 0; i < ns; i++) start[i] = i;
    if (start_ids) {
      cache_fetch(&c, 0, start_ids, n_start);
      cache_descend(&c, 0);
    } else {
    cache_fetch(&c, top, start, ns);
    if (every_layer) {
      /* Alg. 4: search every layer below the top one in turn */
      for (int l = top - 1; l >= 0; l--) {
        cache_transform(&c, g->to_lower[l + 1]);
        cache_descend(&c, l);
      }
    } else {
      /* Sec. 4.4: continue directly on the bottom layer */
      cache_transform(&c, g->to_base[top]);
      cache_descend(&c, 0);
    }
    }
    for (int j = 0; j < k; j++) {
      ids[qi * k + j] = (j < c.nb) ? c.best[j].id : -1;
      dists[qi * k + j] = (j < c.nb) ? c.best[j].d : INFINITY;
    }
    if (counters) { counters[2 * qi] = c.pops; counters[2 * qi + 1] = c.evals; }
    cache_release(&c);
  }
  return err ? -2 : 0;
}

/* -------------------------------------------------------------------- build */

/* members of segment `seg` of layer l, as layer-l ids */
static int seg_members(const ggnn_ref_graph* g, int l, int64_t seg, int32_t* out) {
  int cnt = 0;
  if (l == 0) {
    int64_t lo = seg0_lo(g, seg), hi = seg0_lo(g, seg + 1);
    for (int64_t p = lo; p < hi; p++) out[cnt++] = (int32_t)ggnn_ref_perm(g->seed, g->N, p);
  } else {
    for (int i = 0; i < g->s; i++) out[cnt++] = (int32_t)(seg * g->s + i);
  }
  return cnt;
}

/* Sec. 4.1 Select: every child sub-graph supplies an equal share of the s points of
 * its parent's new top segment (child j of a parent gives floor((j+1)s/g)-floor(js/g)
 * points), drawn by weighted reservoir sampling with weight d_nn1: the points with
 * the largest key log(u)/w win (Efraimidis-Spirakis; same order as u^(1/w)). */
int ggnn_ref_select(ggnn_ref_graph* g, int l_top) {
  if (l_top < 1 || l_top >= g->L) return -1;
  int lc = l_top - 1;
  int64_t nseg = g->G[l_top];
#pragma omp parallel for schedule(dynamic, 64)
  for (int64_t t = 0; t < nseg; t++) {
    int32_t mem[1024];
    double key[1024];
    int out = 0;
    for (int j = 0; j < g->g; j++) {
      int share = (int)(((int64_t)(j + 1) * g->s) / g->g - ((int64_t)j * g->s) / g->g);
      int cnt = seg_members(g, lc, t * g->g + j, mem);
      for (int i = 0; i < cnt; i++) {
        int64_t row = base_of(g, lc, mem[i]);
        double w = (double)g->dnn1[row];
        double u = ggnn_ref_uniform(g->seed, l_top, row);
        key[i] = (w > 0.0) ? log(u) / w : -INFINITY;
      }
      for (int r = 0; r < share; r++) {
        /* r-th largest key, ties towards the smaller id */
        int bi = -1;
        for (int i = 0; i < cnt; i++) {
          if (mem[i] < 0) continue;
          if (bi < 0 || key[i] > key[bi] || (key[i] == key[bi] && mem[i] < mem[bi])) bi = i;
        }
        int64_t o = t * g->s + out++;
        g->to_lower[l_top][o] = mem[bi];
        g->to_base[l_top][o] = (int32_t)base_of(g, lc, mem[bi]);
        mem[bi] = -1;
      }
    }
  }
  return 0;
}

/* Sec. 4.1 Stats: mean and maximum over the bottom layer of the distance to the first
 * neighbour (Eq. 3, Eq. 4). */
static void stats_update(ggnn_ref_graph* g) {
  double sum = 0.0;
  float mx = 0.0f;
  for (int64_t i = 0; i < g->N; i++) {
    sum += (double)g->dnn1[i];
    if (g->dnn1[i] > mx) mx = g->dnn1[i];
  }
  g->stats[0] = (float)(sum / (double)g->N);
  g->stats[1] = mx;
}

/* Alg. 3 Merge / Alg. 4 Query: the K nearest neighbours of every point of layer l_m,
 * found by brute force inside its own segment when l_top == l_m, else by the
 * hierarchical query started on the top segment of its sub-graph. */
int ggnn_ref_merge(ggnn_ref_graph* g, int l_top, int l_m, const ggnn_ref_build_params* p) {
  if (l_top < 0 || l_top >= g->L || l_m < 0 || l_m > l_top) return -1;
  int K = g->K;
  int64_t n = g->n[l_m];
  int32_t* buf = (int32_t*)malloc(sizeof(int32_t) * (size_t)n * K);
  if (!buf) return -2;
  int err = 0;
#pragma omp parallel for schedule(dynamic, 64)
  for (int64_t z = 0; z < n; z++) {
    float q[4096];
    int64_t zb = base_of(g, l_m, (int32_t)z);
    if (g->norm) memcpy(q, g->norm + zb * g->D, sizeof(float) * (size_t)g->D);
    else to_float_row(g->base, zb, g->D, g->dtype, q);
    ent res[1024];
    int nres = 0;
    if (l_top == l_m) {
      int32_t mem[1024];
      int cnt = seg_members(g, l_m, seg_of(g, l_m, z), mem);
      for (int i = 0; i < cnt; i++) {
        if (base_of(g, l_m, mem[i]) == zb) continue;
        ent e;
        e.id = mem[i];
        e.d = ggnn_ref_distance(q, row_ptr(g, base_of(g, l_m, mem[i])), g->D, row_dtype(g), g->metric, g->lanes);
        sorted_insert(res, &nres, K, e);
      }
    } else {
      cache_t c;
      if (cache_alloc(&c, K, p->pq_cap, p->visited_cap) != 0) { err = 1; continue; }
      /* during construction the mean first-neighbour distance replaces the maximum (Eq. 4) */
      cache_init(&c, g, q, p->tau_build, g->stats[0], p->max_iter, zb);
      int64_t seg = seg_of(g, l_m, z);
      for (int l = l_m; l < l_top; l++) seg /= g->g; /* top segment of z's sub-graph */
      int32_t start[1024];
      int ns = seg_members(g, l_top, seg, start);
      cache_fetch(&c, l_top, start, ns);
      for (int l = l_top - 1; l >= l_m; l--) {
        cache_transform(&c, g->to_lower[l + 1]);
        cache_descend(&c, l);
      }
      nres = c.nb < K ? c.nb : K;
      for (int i = 0; i < nres; i++) res[i] = c.best[i];
      cache_release(&c);
    }
    for (int i = 0; i < K; i++) buf[z * K + i] = (i < nres) ? res[i].id : -1;
    if (l_m == 0) g->dnn1[z] = (nres > 0) ? res[0].d : 0.0f;
  }
  if (err) { free(buf); return -2; }
  memcpy(g->edges[l_m], buf, sizeof(int32_t) * (size_t)n * K);
  free(buf);
  memset(g->inv_count[l_m], 0, sizeof(int32_t) * (size_t)n);
  if (l_m == 0) stats_update(g);
  return 0;
}

/* ---------------------------------------------------------------------- sym */

typedef struct {
  int32_t z;
  int npref, ptr;
  ent* pref; /* best list of the failed search: candidates in order of preference */
} sym_req;

static int row_has(const int32_t* row, int n, int32_t id) {
  for (int i = 0; i < n; i++) if (row[i] == id) return 1;
  return 0;
}

/* Alg. 5 / Sec. 4.2.  The paper runs all points in parallel and lets atomics decide
 * who gets a free inverse-link slot; the outcome then depends on timing.  This
 * reference fixes one schedule: in round i every point z handles its i-th neighbour
 * x_i against the inverse lists as they stood at the start of the round; the links
 * requested in a round are then granted by priority (smaller distance, then smaller
 * z), a request that loses its slot moving on to its next candidate, until nothing
 * changes (deferred acceptance -- the result does not depend on processing order). */
int ggnn_ref_sym(ggnn_ref_graph* g, int layer, const ggnn_ref_build_params* p) {
  if (layer < 0 || layer >= g->L) return -1;
  int K = g->K, knn = K / 2, ksym = K - knn;
  int64_t n = g->n[layer];
  const int32_t* E = g->edges[layer];
  int32_t* inv = (int32_t*)malloc(sizeof(int32_t) * (size_t)n * ksym);
  int32_t* ninv = (int32_t*)calloc((size_t)n, sizeof(int32_t));
  sym_req* req = (sym_req*)calloc((size_t)n, sizeof(sym_req));
  if (!inv || !ninv || !req) return -2;

  for (int round = 0; round < knn; round++) {
    /* searches of this round (independent of each other) */
#pragma omp parallel for schedule(dynamic, 64)
    for (int64_t z = 0; z < n; z++) {
      req[z].npref = 0; req[z].ptr = 0; req[z].z = (int32_t)z;
      int32_t x = E[z * K + round];
      if (x < 0) continue;
      /* a direct link back from x makes the search unnecessary */
      if (row_has(E + (int64_t)x * K, knn, (int32_t)z) || row_has(inv + (int64_t)x * ksym, ninv[x], (int32_t)z)) continue;
      float zv[4096], xv[4096], q[4096];
      int64_t zb = base_of(g, layer, (int32_t)z), xb = base_of(g, layer, x);
      if (g->norm) { memcpy(zv, g->norm + zb * g->D, sizeof(float) * (size_t)g->D); memcpy(xv, g->norm + xb * g->D, sizeof(float) * (size_t)g->D); }
      else { to_float_row(g->base, zb, g->D, g->dtype, zv); to_float_row(g->base, xb, g->D, g->dtype, xv); }
      /* Sec. 4.2.1: the search is centred on q_m = z + 0.4 (x - z) and bounded by the
       * distance from q_m to x; without the constraint it is centred on z */
      float w = p->sym_constraint ? 0.4f : 0.0f;
      for (int j = 0; j < g->D; j++) { float t = xv[j] - zv[j]; float u = w * t; q[j] = zv[j] + u; }
      cache_t c;
      cache_alloc(&c, K, p->pq_cap, p->visited_cap);
      cache_init(&c, g, q, p->tau_build, g->stats[0], p->max_iter, -1);
      c.radius = ggnn_ref_distance(q, row_ptr(g, xb), g->D, row_dtype(g), g->metric, g->lanes);
      cache_fetch(&c, layer, &x, 1);
      int found = 0;
      int32_t a;
      while (!found && (a = cache_pop(&c)) >= 0) {
        int32_t prop[1024];
        int np = 0;
        for (int i = 0; i < knn; i++) prop[np++] = E[(int64_t)a * K + i];
        for (int i = 0; i < ninv[a]; i++) prop[np++] = inv[(int64_t)a * ksym + i];
        if (row_has(prop, np, (int32_t)z)) { found = 1; break; }
        cache_fetch(&c, layer, prop, np);
      }
      if (!found && c.nb > 0) {
        req[z].pref = (ent*)malloc(sizeof(ent) * (size_t)c.nb);
        memcpy(req[z].pref, c.best, sizeof(ent) * (size_t)c.nb);
        req[z].npref = c.nb;
      }
      cache_release(&c);
    }
    /* grant the requested links */
    /* one spare slot per row: a newcomer is stored before the worst holder is evicted */
    const int hs = ksym + 1;
    int32_t* hold = (int32_t*)malloc(sizeof(int32_t) * (size_t)n * hs); /* request index = z */
    int32_t* nhold = (int32_t*)calloc((size_t)n, sizeof(int32_t));
    int64_t* queue = (int64_t*)malloc(sizeof(int64_t) * (size_t)(n + 1));
    int64_t qh = 0, qt = 0, qcap = n + 1;
    for (int64_t z = 0; z < n; z++) if (req[z].npref > 0) { queue[qt] = z; qt = (qt + 1) % qcap; }
    while (qh != qt) {
      int64_t r = queue[qh]; qh = (qh + 1) % qcap;
      sym_req* R = &req[r];
      while (R->ptr < R->npref) {
        int32_t cand = R->pref[R->ptr].id;
        int cap = ksym - ninv[cand];
        if (cap > 0 && cand != R->z && !row_has(E + (int64_t)cand * K, knn, R->z) &&
            !row_has(inv + (int64_t)cand * ksym, ninv[cand], R->z)) break;
        R->ptr++;
      }
      if (R->ptr >= R->npref) continue; /* no candidate with free capacity: link dropped */
      int32_t cand = R->pref[R->ptr].id;
      int cap = ksym - ninv[cand];
      int32_t* H = hold + (int64_t)cand * hs;
      H[nhold[cand]++] = (int32_t)r;
      if (nhold[cand] > cap) {
        /* evict the holder with the largest (distance to its own midpoint, z) */
        int wi = 0;
        for (int i = 1; i < nhold[cand]; i++) {
          sym_req* A = &req[H[i]]; sym_req* Wr = &req[H[wi]];
          ent ea = A->pref[A->ptr], ew = Wr->pref[Wr->ptr];
          ea.id = A->z; ew.id = Wr->z;
          if (ent_less(ew, ea)) wi = i;
        }
        int32_t loser = H[wi];
        H[wi] = H[--nhold[cand]];
        req[loser].ptr++;
        queue[qt] = loser; qt = (qt + 1) % qcap;
      }
    }
    for (int64_t c2 = 0; c2 < n; c2++) {
      int32_t* H = hold + c2 * hs;
      /* append the granted links in ascending (distance, z) */
      for (int i = 1; i < nhold[c2]; i++) {
        int32_t h = H[i]; int j = i;
        while (j > 0) {
          sym_req* A = &req[h]; sym_req* Bq = &req[H[j - 1]];
          ent ea = A->pref[A->ptr], eb = Bq->pref[Bq->ptr];
          ea.id = A->z; eb.id = Bq->z;
          if (!ent_less(ea, eb)) break;
          H[j] = H[j - 1]; j--;
        }
        H[j] = h;
      }
      for (int i = 0; i < nhold[c2]; i++) inv[c2 * ksym + ninv[c2]++] = req[H[i]].z;
    }
    free(hold); free(nhold); free(queue);
    for (int64_t z = 0; z < n; z++) { free(req[z].pref); req[z].pref = NULL; req[z].npref = 0; }
  }

  /* Sec. 4.2: a row keeps at least k_nn true neighbours; its inverse links replace the
   * farthest ones.  A link that repeats a kept neighbour is dropped, which keeps one
   * more neighbour (repeated until stable). */
  int32_t* E2 = g->edges[layer];
  for (int64_t c2 = 0; c2 < n; c2++) {
    int32_t* row = E2 + c2 * K;
    int valid = 0;
    while (valid < K && row[valid] >= 0) valid++;
    int32_t links[1024];
    int nl = ninv[c2], keep;
    for (;;) {
      keep = (valid < K - nl) ? valid : K - nl;
      int m = 0;
      for (int i = 0; i < ninv[c2]; i++) if (!row_has(row, keep, inv[c2 * ksym + i])) links[m++] = inv[c2 * ksym + i];
      if (m == nl) break;
      nl = m;
    }
    int o = keep;
    for (int i = 0; i < nl; i++) row[o++] = links[i];
    for (; o < K; o++) row[o] = -1;
    g->inv_count[layer][c2] = nl;
  }
  free(inv); free(ninv); free(req);
  return 0;
}

/* Alg. 3 (bottom-up, top-down construction) followed by r passes of Alg. 6. */
int ggnn_ref_build(ggnn_ref_graph* g, const ggnn_ref_build_params* p) {
  int rc;
  for (int l_top = 0; l_top < g->L; l_top++) {
    if (l_top > 0 && (rc = ggnn_ref_select(g, l_top)) != 0) return rc;
    for (int l_m = l_top; l_m >= 0; l_m--) {
      if ((rc = ggnn_ref_merge(g, l_top, l_m, p)) != 0) return rc;
      if ((rc = ggnn_ref_sym(g, l_m, p)) != 0) return rc;
    }
  }
  for (int r = 0; r < p->refinements; r++) {
    for (int l_m = g->L - 2; l_m >= 0; l_m--) {
      if ((rc = ggnn_ref_merge(g, g->L - 1, l_m, p)) != 0) return rc;
      if ((rc = ggnn_ref_sym(g, l_m, p)) != 0) return rc;
    }
  }
  return 0;
}

/* ------------------------------------------------------------------- shards */

/* Sec. 4.5: merge of the per-shard answers (plain definition: pool all, sort, take k). */
int ggnn_ref_merge_shards(int S, int64_t Q, int k, const int32_t* ids, const float* dists,
                          const int32_t* offsets, int32_t* out_ids, float* out_dists) {
  if (S < 1 || k < 1 || Q < 0) return -1;
  for (int64_t q = 0; q < Q; q++) {
    ent* top = (ent*)malloc(sizeof(ent) * (size_t)k);
    int cnt = 0;
    for (int s = 0; s < S; s++) {
      for (int j = 0; j < k; j++) {
        int32_t id = ids[((int64_t)s * Q + q) * k + j];
        if (id < 0) continue;
        ent e;
        e.id = id + offsets[s];
        e.d = dists[((int64_t)s * Q + q) * k + j];
        sorted_insert(top, &cnt, k, e);
      }
    }
    for (int j = 0; j < k; j++) {
      out_ids[q * k + j] = (j < cnt) ? top[j].id : -1;
      out_dists[q * k + j] = (j < cnt) ? top[j].d : INFINITY;
    }
    free(top);
  }
  return 0;
}
