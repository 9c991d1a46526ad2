// Host-side geometry of the hierarchy (Sec. 4.3, appendix "Graph Size") and the keys of the partition
// permutation: what ggnn_graph_create derives from (N, s, L, seed) before anything touches the GPU.
#pragma once
#include <math.h>
#include <stdint.h>

#include "ggnn_device.h"

namespace ggnn {

inline int64_t ipow(int64_t b, int e) {
  int64_t r = 1;
  for (int i = 0; i < e; i++) r *= b;
  return r;
}

// growth factor g = floor or ceiling of (N/s)^(1/(L-1)), whichever brings the bottom segment size
// N / g^(L-1) closest to s (tie: the smaller); layer l holds s * g^(L-1-l) points in g^(L-1-l)
// segments, layer 0 the N base points.  Returns -1 if no valid hierarchy exists.
inline int geometry(int64_t N, int s, int L, int* g_out, int64_t* n, int64_t* G) {
  const double root = pow((double)N / (double)s, 1.0 / (double)(L - 1));
  int64_t cand[2] = {(int64_t)floor(root), (int64_t)ceil(root)};
  int64_t g = -1;
  double err = 0.0;
  for (int i = 0; i < 2; i++) {
    int64_t c = cand[i] < 1 ? 1 : cand[i];
    double e = fabs((double)N / (double)ipow(c, L - 1) - (double)s);
    if (g < 0 || e < err) { g = c; err = e; }
  }
  for (int l = 0; l < L; l++) {
    G[l] = ipow(g, L - 1 - l);
    n[l] = (l == 0) ? N : (int64_t)s * G[l];
  }
  if (G[0] > N) return -1;
  const int64_t s0_min = N / G[0];
  const int64_t share_max = ((int64_t)s + g - 1) / g;
  if (s0_min < share_max || s0_min < 2) return -1;
  if (L > 2 && n[1] > N) return -1;
  *g_out = (int)g;
  return 0;
}

// half width and round keys of the Feistel network over [0, 4^h), 4^h >= N
inline void partition_keys(int64_t N, uint64_t seed, GraphDev* G) {
  int h = 1;
  while ((((int64_t)1) << (2 * h)) < N) h++;
  G->fbits = h;
  for (int r = 0; r < 4; r++) G->fkey[r] = (uint32_t)mix64(seed + 0x9E3779B97F4A7C15ull * (uint64_t)(r + 1));
  G->seed = seed;
}

}  // namespace ggnn
