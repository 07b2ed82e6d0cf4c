// Grouping of nodes by element: a stable counting sort of z plus the tile table.
//
// Algorithm 2 of arXiv 2504.10700 reads the weights W[z_i,...] per atom.  Grouping the
// atoms of one element lets a wave keep that element's weights in registers and turns
// the dW reduction into a per-element segmented sum in a fixed order.
//
// Three small launches: (1) every wave counts the elements of its contiguous slice of
// z, (2) one workgroup scans the count matrix and writes the tile table, (3) every wave
// scatters its slice to its final positions.  The sort is stable (positions inside an
// element follow node order), so `perm` and everything derived from it is reproducible.
#include "sc_internal.h"

namespace sc {
namespace {

constexpr int kGroupThreads = kGroupWavesPerWG * kLanes;

__global__ __launch_bounds__(kGroupThreads) void group_count_kernel(const int32_t* __restrict__ z, int n, int Z,
                                                                    int nodes_per_wave,
                                                                    int32_t* __restrict__ counts) {
  extern __shared__ int32_t lds[];  // [kGroupWavesPerWG][Z]
  const int wave = threadIdx.x / kLanes, lane = threadIdx.x % kLanes;
  const int gw = blockIdx.x * kGroupWavesPerWG + wave;
  int32_t* mine = lds + wave * Z;
  for (int e = lane; e < Z; e += kLanes) mine[e] = 0;
  __syncthreads();
  const long long lo = static_cast<long long>(gw) * nodes_per_wave;
  const long long hi = (lo + nodes_per_wave < n) ? lo + nodes_per_wave : n;
  for (long long i = lo + lane; i < hi; i += kLanes) {
    const int e = z[i];
    if (e >= 0 && e < Z) atomicAdd(&mine[e], 1);
  }
  __syncthreads();
  for (int e = lane; e < Z; e += kLanes) counts[static_cast<size_t>(gw) * Z + e] = mine[e];
}

// Exclusive scan of v[0..n) (n <= 4*256) held in LDS, in place, by a 256-thread block.
// Returns the total to every thread.  scratch: 256 ints of LDS.
__device__ int block_exclusive_scan(int32_t* v, int n, int32_t* scratch) {
  const int t = threadIdx.x;
  const int per = (n + 255) / 256;
  const int b = t * per;
  int local = 0;
  for (int i = 0; i < per; ++i)
    if (b + i < n) local += v[b + i];
  scratch[t] = local;
  __syncthreads();
  for (int d = 1; d < 256; d <<= 1) {
    const int add = (t >= d) ? scratch[t - d] : 0;
    __syncthreads();
    scratch[t] += add;
    __syncthreads();
  }
  const int total = scratch[255];
  int run = scratch[t] - local;
  __syncthreads();
  for (int i = 0; i < per; ++i)
    if (b + i < n) {
      const int c = v[b + i];
      v[b + i] = run;
      run += c;
    }
  __syncthreads();
  return total;
}

__global__ __launch_bounds__(256) void group_scan_kernel(int Z, int group_waves, int tile_nodes, int max_tiles,
                                                         int32_t* __restrict__ counts,
                                                         int32_t* __restrict__ seg_off,
                                                         int32_t* __restrict__ tile_off,
                                                         int32_t* __restrict__ ntiles_out,
                                                         TileDesc* __restrict__ tiles) {
  __shared__ int32_t total[SC_MAX_ELEMENTS];
  __shared__ int32_t seg[SC_MAX_ELEMENTS + 1];
  __shared__ int32_t til[SC_MAX_ELEMENTS + 1];
  __shared__ int32_t scratch[256];
  const int t = threadIdx.x;
  // column-wise exclusive prefix over the waves: counts[w][e] <- nodes of e in waves < w
  for (int e = t; e < Z; e += 256) {
    int run = 0;
    for (int w = 0; w < group_waves; ++w) {
      const size_t idx = static_cast<size_t>(w) * Z + e;
      const int c = counts[idx];
      counts[idx] = run;
      run += c;
    }
    total[e] = run;
    seg[e] = run;
    til[e] = (run + tile_nodes - 1) / tile_nodes;
  }
  __syncthreads();
  const int n_valid = block_exclusive_scan(seg, Z, scratch);
  const int n_tiles = block_exclusive_scan(til, Z, scratch);
  if (t == 0) {
    seg[Z] = n_valid;
    til[Z] = n_tiles;
    *ntiles_out = (n_tiles < max_tiles) ? n_tiles : max_tiles;
  }
  __syncthreads();
  for (int e = t; e <= Z; e += 256) {
    seg_off[e] = seg[e];
    tile_off[e] = til[e];
  }
  // tile table: element e owns tiles [til[e], til[e+1]); its nodes are split evenly
  for (int i = t; i < n_tiles && i < max_tiles; i += 256) {
    int lo = 0, hi = Z;  // last e with til[e] <= i
    while (hi - lo > 1) {
      const int mid = (lo + hi) >> 1;
      if (til[mid] <= i) lo = mid; else hi = mid;
    }
    // skip empty elements that share the same offset
    const int e = lo;
    const int nt = til[e + 1] - til[e];
    const int j = i - til[e];
    const long long c = total[e];
    const int s0 = static_cast<int>(c * j / nt), s1 = static_cast<int>(c * (j + 1) / nt);
    tiles[i] = TileDesc{e, seg[e] + s0, s1 - s0, 0};
  }
}

__global__ __launch_bounds__(kGroupThreads) void group_scatter_kernel(const int32_t* __restrict__ z, int n, int Z,
                                                                      int nodes_per_wave,
                                                                      const int32_t* __restrict__ counts,
                                                                      const int32_t* __restrict__ seg_off,
                                                                      int32_t* __restrict__ perm) {
  extern __shared__ int32_t lds[];  // [kGroupWavesPerWG][Z] running cursors
  const int wave = threadIdx.x / kLanes, lane = threadIdx.x % kLanes;
  const int gw = blockIdx.x * kGroupWavesPerWG + wave;
  int32_t* cursor = lds + wave * Z;
  for (int e = lane; e < Z; e += kLanes) cursor[e] = seg_off[e] + counts[static_cast<size_t>(gw) * Z + e];
  __syncthreads();
  const long long lo = static_cast<long long>(gw) * nodes_per_wave;
  const long long hi = (lo + nodes_per_wave < n) ? lo + nodes_per_wave : n;
  const unsigned long long lt_mask = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
  for (long long c0 = lo; c0 < hi; c0 += kLanes) {  // wave-uniform trip count
    const long long i = c0 + lane;
    int e = -1;
    if (i < hi) e = z[i];
    const bool valid = (e >= 0 && e < Z);
    // rank of every lane among the lanes of the same element, in lane (= node) order
    unsigned long long todo = __ballot(valid);
    int rank = 0, leader = 0, group = 0;
    while (todo) {
      const int ld = __ffsll(static_cast<long long>(todo)) - 1;
      const int el = __shfl(e, ld);
      const unsigned long long same = __ballot(valid && e == el);
      if (valid && e == el) {
        rank = __popcll(same & lt_mask);
        leader = ld;
        group = __popcll(same);
      }
      todo &= ~same;
    }
    int base = 0;
    if (valid && lane == leader) base = atomicAdd(&cursor[e], group);
    base = __shfl(base, leader);
    if (valid) perm[base + rank] = static_cast<int32_t>(i);
  }
}

}  // namespace

hipError_t launch_grouping(const sc_plan* plan, int64_t n, const int32_t* z, const Workspace& ws,
                           const LaunchShape& shape, hipStream_t stream) {
  const int Z = plan->cfg.num_elements;
  const int wgs = shape.group_waves / kGroupWavesPerWG;
  const size_t lds = static_cast<size_t>(kGroupWavesPerWG) * Z * sizeof(int32_t);
  hipLaunchKernelGGL(group_count_kernel, dim3(wgs), dim3(kGroupThreads), lds, stream, z, static_cast<int>(n), Z,
                     shape.nodes_per_group_wave, ws.counts);
  hipLaunchKernelGGL(group_scan_kernel, dim3(1), dim3(256), 0, stream, Z, shape.group_waves, shape.tile_nodes,
                     shape.max_tiles, ws.counts, ws.seg_off, ws.tile_off, ws.ntiles, ws.tiles);
  hipLaunchKernelGGL(group_scatter_kernel, dim3(wgs), dim3(kGroupThreads), lds, stream, z, static_cast<int>(n), Z,
                     shape.nodes_per_group_wave, ws.counts, ws.seg_off, ws.perm);
  return hipGetLastError();
}

}  // namespace sc
