// Construction kernels other than the searches: top-layer selection (Sec. 4.1), the two
// first-neighbour statistics (Eq. 3, Eq. 4), granting and applying inverse links (Alg. 5).
#include "ggnn_launch.h"

namespace ggnn {

__global__ void fill_i32_kernel(int32_t* p, int64_t n, int32_t v) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) p[i] = v;
}
hipError_t launch_fill_i32(int32_t* p, int64_t n, int32_t v, hipStream_t stream) {
  if (n <= 0) return hipSuccess;
  int64_t blocks = (n + 255) / 256;
  if (blocks > 65536) blocks = 65536;
  fill_i32_kernel<<<(unsigned)blocks, 256, 0, stream>>>(p, n, v);
  return hipGetLastError();
}

// Counting sort of the query numbers by key >> shift: histogram, exclusive scan (one workgroup),
// scatter.  Used to order a large batch by the layer-1 point each query arrived at.
__global__ void sort_hist_kernel(const int32_t* __restrict__ key, int64_t Q, int shift, int32_t* __restrict__ bins) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < Q) atomicAdd(&bins[key[i] >> shift], 1);
}
__global__ __launch_bounds__(1024) void sort_scan_kernel(int32_t* __restrict__ bins, int nbins) {
  __shared__ int32_t part[1024];
  const int t = threadIdx.x;
  const int per = (nbins + 1023) / 1024;
  const int lo = t * per, hi = (lo + per < nbins) ? lo + per : nbins;
  int32_t sum = 0;
  for (int i = lo; i < hi; i++) sum += bins[i];
  part[t] = sum;
  __syncthreads();
  for (int d = 1; d < 1024; d <<= 1) {  // inclusive scan of the partial sums
    const int32_t v = (t >= d) ? part[t - d] : 0;
    __syncthreads();
    part[t] += v;
    __syncthreads();
  }
  int32_t run = part[t] - sum;  // exclusive prefix of this thread's bins
  for (int i = lo; i < hi; i++) {
    const int32_t c = bins[i];
    bins[i] = run;
    run += c;
  }
}
__global__ void sort_scatter_kernel(const int32_t* __restrict__ key, int64_t Q, int shift, int32_t* __restrict__ bins,
                                    int32_t* __restrict__ order) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < Q) order[atomicAdd(&bins[key[i] >> shift], 1)] = (int32_t)i;
}
hipError_t launch_sort_by_key(const int32_t* key, int64_t Q, int shift, int nbins, int32_t* bins, int32_t* order,
                              hipStream_t stream) {
  hipError_t e = launch_fill_i32(bins, nbins + 1, 0, stream);
  if (e != hipSuccess) return e;
  const unsigned blocks = (unsigned)((Q + 255) / 256);
  sort_hist_kernel<<<blocks, 256, 0, stream>>>(key, Q, shift, bins);
  sort_scan_kernel<<<1, 1024, 0, stream>>>(bins, nbins);
  sort_scatter_kernel<<<blocks, 256, 0, stream>>>(key, Q, shift, bins, order);
  return hipGetLastError();
}

// unit-length float32 copy of the base rows (cosine): x / sqrt(sum x^2), the sum taken in
// the fixed order of every distance; RL lanes per row (8, or 64 for rows longer than 1024 bytes)
template <int RL>
__global__ __launch_bounds__(kWave) void normalise_kernel(const uint8_t* __restrict__ base, int dtype, int64_t N,
                                                          int D, float* __restrict__ out, int64_t first) {
  const int lane = threadIdx.x, sub = lane & (RL - 1), grp = lane / RL;
  const int64_t row = (first + blockIdx.x) * (kWave / RL) + grp;
  const bool act = row < N;
  const int per = (dtype == 1) ? 16 : 4;
  const int nchunks = (D + per - 1) / per;
  float acc = 0.0f;
  if (act) {
    for (int chunk = sub; chunk < nchunks; chunk += RL) {
      for (int e = 0; e < per; e++) {
        int j = chunk * per + e;
        if (j >= D) break;
        float x = (dtype == 1) ? (float)base[(size_t)row * D + j] : ((const float*)base)[(size_t)row * D + j];
        acc = __builtin_fmaf(x, x, acc);
      }
    }
  }
  acc = row_reduce_t<RL>(acc);
  const float nrm = __builtin_sqrtf(acc);
  if (act) {
    for (int chunk = sub; chunk < nchunks; chunk += RL) {
      for (int e = 0; e < per; e++) {
        int j = chunk * per + e;
        if (j >= D) break;
        float x = (dtype == 1) ? (float)base[(size_t)row * D + j] : ((const float*)base)[(size_t)row * D + j];
        out[(size_t)row * D + j] = (nrm > 0.0f) ? x / nrm : x;
      }
    }
  }
}
hipError_t launch_normalise(const void* base, int dtype, int64_t N, int D, float* out, hipStream_t stream) {
  // the unit-length copy is float32: its row length decides how many lanes share a row
  const bool wide = (size_t)D * 4 > (size_t)kRowLanes * 8 * 16;
  const int64_t blocks = wide ? N : (N + kRowsPerPass - 1) / kRowsPerPass;
  for (int64_t first = 0; first < blocks; first += kMaxBlocksPerLaunch) {
    const unsigned nb = chunk_blocks(blocks, first);
    if (wide) normalise_kernel<kWideRowLanes><<<nb, kWave, 0, stream>>>((const uint8_t*)base, dtype, N, D, out, first);
    else normalise_kernel<kRowLanes><<<nb, kWave, 0, stream>>>((const uint8_t*)base, dtype, N, D, out, first);
  }
  return hipGetLastError();
}

// Sec. 4.1 Select: one wavefront per child segment.  Child j of a parent supplies
// floor((j+1)s/g) - floor(js/g) of the parent's s points: the members with the largest
// Efraimidis-Spirakis key log(u)/w, w = d_nn1, ties towards the smaller id.
__device__ inline double select_uniform(uint64_t seed, int l_top, int64_t row) {
  uint64_t x = mix64(seed ^ mix64(((uint64_t)l_top << 56) + (uint64_t)row + 0x632BE59BD9B4E019ull));
  return ((double)(x >> 12) + 0.5) * (1.0 / 4503599627370496.0);
}
__global__ __launch_bounds__(kWave) void select_kernel(GraphDev G, int l_top, const float* __restrict__ dnn1,
                                                       int32_t* __restrict__ to_lower, int32_t* __restrict__ to_base,
                                                       int64_t first) {
  __shared__ double key[kWave];
  __shared__ int32_t mem[kWave];
  const int lane = threadIdx.x;
  const int lc = l_top - 1;
  const int64_t child = first + blockIdx.x;
  const int64_t t = child / G.g;
  const int j = (int)(child % G.g);
  const int share = (int)(((int64_t)(j + 1) * G.s) / G.g - ((int64_t)j * G.s) / G.g);
  if (share == 0) return;
  const int offset = (int)(((int64_t)j * G.s) / G.g);
  int cnt;
  int32_t m = -1;
  if (lc == 0) {
    int64_t lo = seg0_lo(G, child), hi = seg0_lo(G, child + 1);
    cnt = (int)(hi - lo);
    if (lane < cnt) m = (int32_t)perm_fwd(G, lo + lane);
  } else {
    cnt = G.s;
    if (lane < cnt) m = (int32_t)(child * G.s + lane);
  }
  int32_t row = -1;
  double kv = 0.0;
  if (lane < cnt) {
    row = (lc == 0) ? m : G.to_base[lc][m];
    double w = (double)dnn1[row];
    kv = (w > 0.0) ? log(select_uniform(G.seed, l_top, row)) / w : -INFINITY;
  }
  key[lane] = kv;
  mem[lane] = m;
  __syncthreads();
  if (lane < cnt) {
    int rank = 0;
    for (int i = 0; i < cnt; i++) rank += (key[i] > kv) || (key[i] == kv && mem[i] < m);
    if (rank < share) {
      to_lower[t * G.s + offset + rank] = m;
      to_base[t * G.s + offset + rank] = row;
    }
  }
}
hipError_t launch_select(const GraphDev& G, int l_top, const float* dnn1, int32_t* to_lower, int32_t* to_base,
                         hipStream_t stream) {
  const int64_t children = G.n[l_top] / G.s * G.g;
  for (int64_t first = 0; first < children; first += kMaxBlocksPerLaunch)
    select_kernel<<<chunk_blocks(children, first), kWave, 0, stream>>>(G, l_top, dnn1, to_lower, to_base, first);
  return hipGetLastError();
}

// Sec. 4.1 Stats: mean and maximum of d_nn1 over the bottom layer.  Two fixed-shape stages
// (float64 partial sums per block, then one block), so the result is reproducible.
constexpr int kStatBlocks = 1024;
__global__ __launch_bounds__(256) void stats_stage1(const float* __restrict__ x, int64_t n, double* __restrict__ partial) {
  __shared__ double ssum[256];
  __shared__ double smax[256];
  const int64_t per = (n + kStatBlocks - 1) / kStatBlocks;
  const int64_t lo = (int64_t)blockIdx.x * per;
  const int64_t hi = lo + per < n ? lo + per : n;
  double s = 0.0, m = 0.0;
  for (int64_t i = lo + threadIdx.x; i < hi; i += 256) {
    double v = (double)x[i];
    s += v;
    m = v > m ? v : m;
  }
  ssum[threadIdx.x] = s;
  smax[threadIdx.x] = m;
  __syncthreads();
  for (int w = 128; w >= 1; w >>= 1) {
    if ((int)threadIdx.x < w) {
      ssum[threadIdx.x] += ssum[threadIdx.x + w];
      smax[threadIdx.x] = smax[threadIdx.x] > smax[threadIdx.x + w] ? smax[threadIdx.x] : smax[threadIdx.x + w];
    }
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    partial[blockIdx.x] = ssum[0];
    partial[kStatBlocks + blockIdx.x] = smax[0];
  }
}
__global__ __launch_bounds__(kStatBlocks) void stats_stage2(const double* __restrict__ partial, int64_t n, float* __restrict__ out) {
  __shared__ double ssum[kStatBlocks];
  __shared__ double smax[kStatBlocks];
  ssum[threadIdx.x] = partial[threadIdx.x];
  smax[threadIdx.x] = partial[kStatBlocks + threadIdx.x];
  __syncthreads();
  for (int w = kStatBlocks / 2; w >= 1; w >>= 1) {
    if ((int)threadIdx.x < w) {
      ssum[threadIdx.x] += ssum[threadIdx.x + w];
      smax[threadIdx.x] = smax[threadIdx.x] > smax[threadIdx.x + w] ? smax[threadIdx.x] : smax[threadIdx.x + w];
    }
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    out[0] = (float)(ssum[0] / (double)n);
    out[1] = (float)smax[0];
  }
}
hipError_t launch_stats(const float* x, int64_t n, double* partial, float* out, hipStream_t stream) {
  stats_stage1<<<kStatBlocks, 256, 0, stream>>>(x, n, partial);
  stats_stage2<<<1, kStatBlocks, 0, stream>>>(partial, n, out);
  return hipGetLastError();
}

// ---- granting inverse links (Alg. 5, last loop) -----------------------------------------
// The paper lets atomics decide which request gets a free slot of a row.  Here the slots of
// a row go to the requests with the smallest (distance, z); a request that loses moves on to
// its next candidate.  Repeating propose / resolve until no request is left proposing gives
// the same links whatever the order in which the hardware runs the threads.

__device__ inline bool row_has(const int32_t* row, int n, int32_t id) {
  for (int i = 0; i < n; i++)
    if (row[i] == id) return true;
  return false;
}

__global__ void sym_propose_kernel(GraphDev G, int layer, SymBuffers sb, int B, int first) {
  const int64_t z = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (z >= G.n[layer]) return;
  const int knn = G.K / 2, ksym = G.K - knn;
  if (first) {
    sb.ptr[z] = 0;
    sb.state[z] = sb.npref[z] > 0 ? 1 : 0;
  }
  if (sb.state[z] != 1) return;
  const int np = sb.npref[z];
  int ptr = sb.ptr[z];
  const int32_t* __restrict__ Ed = G.edges[layer];
  int32_t cand = -1;
  for (; ptr < np; ptr++) {
    cand = key_id(sb.pref[(size_t)z * B + ptr]);
    const int ni = sb.ninv[cand];
    if (ksym - ni > 0 && cand != (int32_t)z && !row_has(Ed + (size_t)cand * G.K, knn, (int32_t)z) &&
        !row_has(sb.inv + (size_t)cand * ksym, ni, (int32_t)z))
      break;
  }
  sb.ptr[z] = ptr;
  if (ptr >= np) {
    sb.state[z] = 0;  // no candidate with a free slot: the link is dropped
    return;
  }
  sb.next[z] = atomicExch(&sb.head[cand], (int32_t)z);
}

__device__ inline u64 request_key(const SymBuffers& sb, int B, int32_t r) {
  u64 k = sb.pref[(size_t)r * B + sb.ptr[r]];
  return (k & 0xFFFFFFFF00000000ull) | (uint32_t)r;  // (distance to the request's midpoint, z)
}

__global__ void sym_resolve_kernel(GraphDev G, int layer, SymBuffers sb, int B) {
  const int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (p >= G.n[layer]) return;
  int32_t r = sb.head[p];
  if (r < 0) return;
  sb.head[p] = -1;
  const int knn = G.K / 2, ksym = G.K - knn;
  const int cap = ksym - sb.ninv[p];
  int32_t* H = sb.hold + (size_t)p * ksym;  // kept ascending by request_key
  int nh = sb.nhold[p];
  int losers = 0;
  while (r >= 0) {
    const int32_t nxt = sb.next[r];
    const u64 kr = request_key(sb, B, r);
    int32_t out = -1;
    if (nh < cap) {
      int pos = nh++;
      while (pos > 0 && request_key(sb, B, H[pos - 1]) > kr) { H[pos] = H[pos - 1]; pos--; }
      H[pos] = r;
      sb.state[r] = 2;
    } else if (request_key(sb, B, H[nh - 1]) > kr) {
      out = H[nh - 1];
      int pos = nh - 1;
      while (pos > 0 && request_key(sb, B, H[pos - 1]) > kr) { H[pos] = H[pos - 1]; pos--; }
      H[pos] = r;
      sb.state[r] = 2;
    } else {
      out = r;
    }
    if (out >= 0) {
      sb.state[out] = 1;
      sb.ptr[out] = sb.ptr[out] + 1;
      losers++;
    }
    r = nxt;
  }
  sb.nhold[p] = nh;
  if (losers) atomicAdd(sb.pending, losers);
}

__global__ void sym_commit_kernel(GraphDev G, int layer, SymBuffers sb) {
  const int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (p >= G.n[layer]) return;
  const int knn = G.K / 2, ksym = G.K - knn;
  const int nh = sb.nhold[p];
  int ni = sb.ninv[p];
  for (int i = 0; i < nh; i++) sb.inv[(size_t)p * ksym + ni++] = sb.hold[(size_t)p * ksym + i];
  sb.ninv[p] = ni;
  sb.nhold[p] = 0;
}

// Sec. 4.2: a row keeps at least k_nn true neighbours, its inverse links replace the
// farthest ones; a link that repeats a kept neighbour is dropped (until stable).
__global__ void sym_apply_kernel(GraphDev G, int layer, SymBuffers sb, int32_t* __restrict__ edges,
                                 int32_t* __restrict__ inv_count) {
  const int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (p >= G.n[layer]) return;
  const int K = G.K, knn = K / 2, ksym = K - knn;
  int32_t* row = edges + (size_t)p * K;
  const int32_t* links = sb.inv + (size_t)p * ksym;
  const int ni = sb.ninv[p];
  int valid = 0;
  while (valid < K && row[valid] >= 0) valid++;
  int nl = ni, keep;
  for (;;) {
    keep = valid < K - nl ? valid : K - nl;
    int m = 0;
    for (int i = 0; i < ni; i++) m += !row_has(row, keep, links[i]);
    if (m == nl) break;
    nl = m;
  }
  int o = keep;
  for (int i = 0; i < ni; i++)
    if (!row_has(row, keep, links[i])) row[o++] = links[i];
  for (; o < K; o++) row[o] = -1;
  inv_count[p] = nl;
}

// Measurement aid: reads rows ids[0..n) of `rows` with the access pattern of the search kernels
// (8 lanes x 16 bytes per row, 8 rows per wave instruction, 24 rows in flight per wavefront) and
// folds them into one word per wavefront, so that only the gather itself is timed.
__global__ __launch_bounds__(kWave) void gather_probe_kernel(const uint8_t* __restrict__ rows, int row_bytes,
                                                             const int32_t* __restrict__ ids, int64_t n,
                                                             int rows_per_wave, uint32_t* __restrict__ out,
                                                             int64_t first_block) {
  const int lane = threadIdx.x, sub = lane & (kRowLanes - 1), grp = lane / kRowLanes;
  const int nchunks = row_bytes / 16;
  const int64_t block = first_block + blockIdx.x;
  const int64_t first = block * rows_per_wave;
  uint32_t acc = 0;
  for (int r0 = 0; r0 < rows_per_wave; r0 += 3 * kRowsPerPass) {
    uint4 v[3][4];
#pragma unroll
    for (int ps = 0; ps < 3; ps++) {
      const int64_t i = first + r0 + ps * kRowsPerPass + grp;
      const bool act = (r0 + ps * kRowsPerPass + grp) < rows_per_wave && i < n;
      const uint8_t* ptr = rows + (size_t)(act ? ids[i] : 0) * (size_t)row_bytes;
#pragma unroll
      for (int ch = 0; ch < 4; ch++) {
        const int chunk = ch * kRowLanes + sub;
        v[ps][ch] = make_uint4(0, 0, 0, 0);
        if (act && chunk < nchunks) v[ps][ch] = *(const uint4*)(ptr + (size_t)chunk * 16);
      }
    }
#pragma unroll
    for (int ps = 0; ps < 3; ps++)
#pragma unroll
      for (int ch = 0; ch < 4; ch++) acc ^= v[ps][ch].x ^ v[ps][ch].y ^ v[ps][ch].z ^ v[ps][ch].w;
  }
  out[(size_t)block * kWave + lane] = acc;
}
hipError_t launch_gather_probe(const void* rows, int row_bytes, const int32_t* ids, int64_t n, int rows_per_wave,
                               uint32_t* out, hipStream_t stream) {
  const int64_t waves = (n + rows_per_wave - 1) / rows_per_wave;
  for (int64_t first = 0; first < waves; first += kMaxBlocksPerLaunch)
    gather_probe_kernel<<<chunk_blocks(waves, first), kWave, 0, stream>>>((const uint8_t*)rows, row_bytes, ids, n,
                                                                         rows_per_wave, out, first);
  return hipGetLastError();
}

// Sec. 4.5 (sharding): the S per-shard answers of one query (each k entries, ascending, padded
// with id -1) are merged into the k best overall by (distance, global id).  One wavefront per
// query: the S*k keys go to LDS, every valid key counts the smaller ones, and a key of rank r < k
// is result r (the keys are distinct because global ids are).
__global__ __launch_bounds__(kWave) void merge_shards_kernel(int S, int64_t Q, int k, const int32_t* __restrict__ ids,
                                                             const float* __restrict__ dists,
                                                             const int32_t* __restrict__ offsets,
                                                             int32_t* __restrict__ out_ids, float* __restrict__ out_dists,
                                                             int64_t first) {
  extern __shared__ __align__(16) unsigned char lds[];
  u64* keys = (u64*)lds;
  const int lane = threadIdx.x;
  const int64_t q = first + blockIdx.x;
  const int n = S * k;
  for (int i = lane; i < n; i += kWave) {
    const int s = i / k, j = i - s * k;
    const int32_t id = ids[((size_t)s * Q + q) * k + j];
    keys[i] = (id < 0) ? ~0ull : make_key(dists[((size_t)s * Q + q) * k + j], id + offsets[s]);
  }
  for (int j = lane; j < k; j += kWave) {
    out_ids[(size_t)q * k + j] = -1;
    out_dists[(size_t)q * k + j] = INFINITY;
  }
  __syncthreads();
  for (int i = lane; i < n; i += kWave) {
    const u64 key = keys[i];
    if (key == ~0ull) continue;
    int r = 0;
    for (int j = 0; j < n; j++) r += keys[j] < key;
    if (r < k) {
      out_ids[(size_t)q * k + r] = key_id(key);
      out_dists[(size_t)q * k + r] = key_d(key);
    }
  }
}
hipError_t launch_merge_shards(int S, int64_t Q, int k, const int32_t* ids, const float* dists, const int32_t* offsets,
                               int32_t* out_ids, float* out_dists, hipStream_t stream) {
  if (Q <= 0) return hipSuccess;
  for (int64_t first = 0; first < Q; first += kMaxBlocksPerLaunch)
    merge_shards_kernel<<<chunk_blocks(Q, first), kWave, (size_t)S * k * 8, stream>>>(S, Q, k, ids, dists, offsets, out_ids,
                                                                                      out_dists, first);
  return hipGetLastError();
}

static inline unsigned blocks_for(int64_t n) { return (unsigned)((n + 255) / 256); }

hipError_t launch_sym_propose(const GraphDev& G, int layer, const SymBuffers& sb, int B, hipStream_t stream);
hipError_t launch_sym_propose_impl(const GraphDev& G, int layer, const SymBuffers& sb, int B, int first, hipStream_t stream) {
  sym_propose_kernel<<<blocks_for(G.n[layer]), 256, 0, stream>>>(G, layer, sb, B, first);
  return hipGetLastError();
}
hipError_t launch_sym_propose(const GraphDev& G, int layer, const SymBuffers& sb, int B, hipStream_t stream) {
  return launch_sym_propose_impl(G, layer, sb, B, 0, stream);
}
hipError_t launch_sym_propose_first(const GraphDev& G, int layer, const SymBuffers& sb, int B, hipStream_t stream) {
  return launch_sym_propose_impl(G, layer, sb, B, 1, stream);
}
hipError_t launch_sym_resolve(const GraphDev& G, int layer, const SymBuffers& sb, int B, hipStream_t stream) {
  sym_resolve_kernel<<<blocks_for(G.n[layer]), 256, 0, stream>>>(G, layer, sb, B);
  return hipGetLastError();
}
hipError_t launch_sym_commit(const GraphDev& G, int layer, const SymBuffers& sb, hipStream_t stream) {
  sym_commit_kernel<<<blocks_for(G.n[layer]), 256, 0, stream>>>(G, layer, sb);
  return hipGetLastError();
}
hipError_t launch_sym_apply(const GraphDev& G, int layer, const SymBuffers& sb, int32_t* edges, int32_t* inv_count,
                            hipStream_t stream) {
  sym_apply_kernel<<<blocks_for(G.n[layer]), 256, 0, stream>>>(G, layer, sb, edges, inv_count);
  return hipGetLastError();
}

}  // namespace ggnn
