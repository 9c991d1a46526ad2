// Host-side sweep of every index and address expression the bottom layer of a construction uses
// (partition permutation and its inverse, segment bounds, segment of a row, row offsets of the gather,
// indices of the result rows, and the way a launch of n workgroups is cut into chunks), at the sizes
// given on the command line -- by default the 10^8 x 128-byte workload.  Compiled for the host only,
// with the address and undefined-behaviour sanitizers (see tests/test_host_indexing.py); every value is
// also checked against the size of the array it indexes.  Prints "ok" and exits 0, or says what failed.
#include <stdio.h>
#include <stdlib.h>

#include <vector>

#include "ggnn_geometry.h"
#include "ggnn_launch.h"

using namespace ggnn;

#define CHECK(cond, ...)                  \
  do {                                    \
    if (!(cond)) {                        \
      fprintf(stderr, "FAILED: " #cond ": " __VA_ARGS__); \
      fprintf(stderr, "\n");              \
      return 1;                           \
    }                                     \
  } while (0)

int main(int argc, char** argv) {
  const int64_t N = argc > 1 ? atoll(argv[1]) : 100000000ll;
  const int row_bytes = argc > 2 ? atoi(argv[2]) : 128;
  const int K = argc > 3 ? atoi(argv[3]) : 24;
  const int L = argc > 4 ? atoi(argv[4]) : 4;
  const int s = argc > 5 ? atoi(argv[5]) : 32;
  const int64_t stride = argc > 6 ? atoll(argv[6]) : 1;  // positions visited: every stride-th
  GraphDev G = {};
  int64_t G_seg[kMaxLevels];
  int g = 0;
  CHECK(geometry(N, s, L, &g, G.n, G_seg) == 0, "no hierarchy for N=%lld", (long long)N);
  G.N = N; G.K = K; G.L = L; G.s = s; G.g = g; G.G0 = G_seg[0];
  G.row_bytes = row_bytes; G.nchunks = row_bytes / 16;
  partition_keys(N, 42, &G);
  const uint64_t array_bytes = (uint64_t)N * (uint64_t)row_bytes;
  const uint64_t edge_words = (uint64_t)N * (uint64_t)K;
  printf("N=%lld g=%d G0=%lld array=%llu bytes, edges=%llu words\n", (long long)N, g, (long long)G.G0,
         (unsigned long long)array_bytes, (unsigned long long)edge_words);

  // segments: contiguous, cover [0, N), at most one wavefront of points each
  int64_t covered = 0;
  for (int64_t j = 0; j < G.G0; j++) {
    const int64_t lo = seg0_lo(G, j), hi = seg0_lo(G, j + 1);
    CHECK(lo == covered && hi > lo && hi - lo <= kWave, "segment %lld = [%lld, %lld)", (long long)j, (long long)lo, (long long)hi);
    covered = hi;
  }
  CHECK(covered == N, "segments cover %lld positions", (long long)covered);

  // permutation: a bijection of [0, N) with perm_inv as its inverse; the segment a row is assigned to
  // is the one that holds its position
  std::vector<bool> hit(stride == 1 ? (size_t)N : 0);
  for (int64_t p = 0; p < N; p += stride) {
    const int64_t row = perm_fwd(G, p);
    CHECK(row >= 0 && row < N, "perm_fwd(%lld) = %lld", (long long)p, (long long)row);
    if (stride == 1) {
      CHECK(!hit[(size_t)row], "row %lld is the image of two positions", (long long)row);
      hit[(size_t)row] = true;
    }
    CHECK(perm_inv(G, row) == p, "perm_inv(perm_fwd(%lld))", (long long)p);
    const int64_t seg = seg0_of_row(G, row);
    CHECK(seg >= 0 && seg < G.G0 && seg0_lo(G, seg) <= p && p < seg0_lo(G, seg + 1), "row %lld -> segment %lld", (long long)row, (long long)seg);
    // the gather reads 16 bytes per lane at row_offset(row, row_bytes, lane) + 128 * chunk, chunk < nchunks / 8
    const int last_sub = (G.nchunks - 1) % kRowLanes, last_ch = (G.nchunks - 1) / kRowLanes;
    const uint64_t off = row_offset((uint32_t)row, (uint32_t)row_bytes, (uint32_t)last_sub) + (uint64_t)last_ch * kRowLanes * 16;
    CHECK(off + 16 <= array_bytes, "row %lld: byte offset %llu", (long long)row, (unsigned long long)off);
    // result rows and first-neighbour distances are indexed by the row itself
    CHECK((uint64_t)row * (uint64_t)K + (uint64_t)K <= edge_words, "result row %lld", (long long)row);
  }
  // whether 32-bit offsets suffice is decided by the array size
  const bool addr32 = array_bytes < (1ull << 32);
  if (!addr32) {
    const uint64_t far = row_offset((uint32_t)(N - 1), (uint32_t)row_bytes, 0);
    CHECK((uint64_t)(uint32_t)far != far, "the last row's offset should not fit 32 bits");
  }

  // launches: one workgroup per point, in chunks; every chunk's work-item count fits the 32 bits a
  // dispatch counts them in, and the chunks cover [0, N) exactly once
  int64_t launched = 0;
  for (int64_t first = 0; first < N; first += kMaxBlocksPerLaunch) {
    const uint64_t blocks = chunk_blocks(N, first);
    CHECK(blocks >= 1 && blocks * (uint64_t)kWave <= 0xFFFFFFFFull, "chunk at %lld has %llu workgroups", (long long)first, (unsigned long long)blocks);
    CHECK(first % kXcds == 0, "chunk start %lld breaks the workgroup -> XCD order", (long long)first);
    launched += (int64_t)blocks;
  }
  CHECK(launched == N, "chunks launch %lld workgroups", (long long)launched);
  // (a single launch of N workgroups of 64 work-items would need this many work-items in one dimension)
  printf("one launch would need %llu work-items per dimension (limit %llu): %s\n", (unsigned long long)N * kWave,
         0xFFFFFFFFull, (uint64_t)N * kWave > 0xFFFFFFFFull ? "does not fit" : "fits");
  printf("ok\n");
  return 0;
}
