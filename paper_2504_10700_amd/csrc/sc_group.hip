// Grouping of nodes by element: a stable counting sort of z plus the tile table.
//
// Algorithm 2 of arXiv 2504.10700 reads the weights W[z_i,...] per atom.  Grouping the
// atoms of one element lets a wave keep that element's weights in registers and turns
// the dW reduction into a per-element segmented sum in a fixed order.
//
// Every wave owns a contiguous slice of z.  (1) it counts the elements of its slice,
// (2) the count matrix [element][wave] is scanned along the waves and over the elements
// and the tile table is written, (3) every wave scatters its slice to its final
// positions.  The sort is stable (positions inside an element follow node order), so
// `perm` and everything derived from it is reproducible.  Small batches run the three
// phases in ONE single-workgroup launch with the count matrix in LDS; large batches use
// three launches with the matrix in the workspace.
#include "sc_internal.h"

namespace sc {
namespace {

constexpr int kGroupThreads = kGroupWavesPerWG * kLanes;
constexpr int kFusedWaves = 16;
constexpr int kFusedThreads = kFusedWaves * kLanes;
constexpr int kBatch = 8;          // 64-node chunks whose z loads are issued together (multi-launch kernels)
constexpr int kFusedChunks = 16;   // 64-node chunks per wave of the single-launch kernel
constexpr int kFusedMaxNodes = kFusedWaves * kFusedChunks * kLanes;

// Stable scatter of one 64-node chunk: lane holds element e (valid or not); cursor[e *
// cursor_stride] is this wave's next free position of element e (LDS).  The lanes that
// hold the same element are found bit by bit (one ballot per bit of the element index),
// which costs the same whatever the number of distinct elements in the chunk.
__device__ __forceinline__ void scatter_chunk(int e, bool valid, int node, int lane, int z_bits, int32_t* cursor,
                                              int cursor_stride, int32_t* __restrict__ perm) {
  const unsigned long long lt_mask = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
  unsigned long long same = __ballot(valid);
  for (int b = 0; b < z_bits; ++b) {
    const bool bit = (e >> b) & 1;
    const unsigned long long m = __ballot(bit);
    same &= bit ? m : ~m;
  }
  // `same` = valid lanes holding this lane's element (meaningless on invalid lanes)
  const int rank = __popcll(same & lt_mask);
  const int group = __popcll(same);
  const int leader = valid ? __ffsll(static_cast<long long>(same)) - 1 : lane;
  int base = 0;
  if (valid && lane == leader) base = atomicAdd(&cursor[e * cursor_stride], group);
  base = __shfl(base, leader);
  if (valid) perm[base + rank] = node;
}

// Exclusive scan of v[0..n) (LDS, n <= 64 * 16) in place by ONE wave; returns the total to
// every lane of that wave.
__device__ int wave_exclusive_scan(int32_t* v, int n, int lane) {
  constexpr int kMaxPer = SC_MAX_ELEMENTS / kLanes;
  const int per = (n + kLanes - 1) / kLanes;
  int c[kMaxPer], local = 0;
#pragma unroll
  for (int k = 0; k < kMaxPer; ++k) {
    const int i = lane * per + k;
    c[k] = (k < per && i < n) ? v[i] : 0;
    local += c[k];
  }
  int incl = local;
#pragma unroll
  for (int d = 1; d < kLanes; d <<= 1) {
    const int up = __shfl_up(incl, d);
    if (lane >= d) incl += up;
  }
  int run = incl - local;
#pragma unroll
  for (int k = 0; k < kMaxPer; ++k) {
    const int i = lane * per + k;
    if (k < per && i < n) v[i] = run;
    run += c[k];
  }
  return __shfl(incl, kLanes - 1);
}

// Given total[e] (nodes per element, LDS) writes seg/til (LDS, Z+1 entries), the global
// copies and the tile table.  All threads of the block call it.
__device__ void offsets_and_tiles(int Z, int tile_nodes, int max_tiles, const int32_t* total, int32_t* seg,
                                  int32_t* til, int32_t* __restrict__ seg_off, int32_t* __restrict__ tile_off,
                                  int32_t* __restrict__ ntiles_out, TileDesc* __restrict__ tiles) {
  const int t = threadIdx.x, nt = blockDim.x;
  for (int e = t; e < Z; e += nt) {
    seg[e] = total[e];
    til[e] = (total[e] + tile_nodes - 1) / tile_nodes;
  }
  __syncthreads();
  if (t < kLanes) {  // wave 0
    const int n_valid = wave_exclusive_scan(seg, Z, t);
    const int n_tiles = wave_exclusive_scan(til, Z, t);
    if (t == 0) {
      seg[Z] = n_valid;
      til[Z] = n_tiles;
      *ntiles_out = (n_tiles < max_tiles) ? n_tiles : max_tiles;
    }
  }
  __syncthreads();
  const int n_tiles = til[Z];
  for (int e = t; e <= Z; e += nt) {
    seg_off[e] = seg[e];
    tile_off[e] = til[e];
  }
  // tile table: element e owns tiles [til[e], til[e+1]); its nodes are split evenly
  // (the first `rem` tiles take one node more)
  for (int i = t; i < n_tiles && i < max_tiles; i += nt) {
    int lo = 0, hi = Z;  // last e with til[e] <= i (empty elements share an offset with the next one)
    while (hi - lo > 1) {
      const int mid = (lo + hi) >> 1;
      if (til[mid] <= i) lo = mid; else hi = mid;
    }
    const int e = lo;
    const int nt_e = til[e + 1] - til[e];
    const int j = i - til[e];
    const int base = total[e] / nt_e, rem = total[e] % nt_e;
    const int s0 = j * base + (j < rem ? j : rem);
    tiles[i] = TileDesc{e, seg[e] + s0, base + (j < rem ? 1 : 0), 0};
  }
  // unused descriptors say "empty": the main kernels need no separate tile count
  for (int i = n_tiles + t; i < max_tiles; i += nt) tiles[i] = TileDesc{0, 0, 0, 0};
}

// ---------------------------------------------------------------- one launch (small batches)
__global__ __launch_bounds__(kFusedThreads) void group_fused_kernel(const int32_t* __restrict__ z, int n, int Z,
                                                                    int tile_nodes, int max_tiles,
                                                                    int32_t* __restrict__ seg_off,
                                                                    int32_t* __restrict__ tile_off,
                                                                    int32_t* __restrict__ ntiles_out,
                                                                    TileDesc* __restrict__ tiles,
                                                                    int32_t* __restrict__ perm) {
  extern __shared__ int32_t lds[];
  int32_t* counts = lds;                        // [Z][kFusedWaves]
  int32_t* total = counts + Z * kFusedWaves;    // [Z]
  int32_t* seg = total + Z;                     // [Z+1]
  int32_t* til = seg + Z + 1;                   // [Z+1]
  const int wave = threadIdx.x / kLanes, lane = threadIdx.x % kLanes;
  for (int i = threadIdx.x; i < Z * kFusedWaves; i += kFusedThreads) counts[i] = 0;
  __syncthreads();
  // every wave keeps its slice of z in registers (at most kFusedChunks 64-node chunks)
  const int per_wave = ((n + kFusedWaves - 1) / kFusedWaves + kLanes - 1) / kLanes * kLanes;
  const int lo = wave * per_wave;
  const int hi = (lo + per_wave < n) ? lo + per_wave : n;
  int zs[kFusedChunks];
#pragma unroll
  for (int c = 0; c < kFusedChunks; ++c) {
    const int i = lo + c * kLanes + lane;
    zs[c] = (i < hi) ? z[i] : -1;
  }
#pragma unroll
  for (int c = 0; c < kFusedChunks; ++c)
    if (zs[c] >= 0 && zs[c] < Z) atomicAdd(&counts[zs[c] * kFusedWaves + wave], 1);
  __syncthreads();
  for (int e = threadIdx.x; e < Z; e += kFusedThreads) {
    int run = 0;
    for (int w = 0; w < kFusedWaves; ++w) {
      const int c = counts[e * kFusedWaves + w];
      counts[e * kFusedWaves + w] = run;
      run += c;
    }
    total[e] = run;
  }
  __syncthreads();
  offsets_and_tiles(Z, tile_nodes, max_tiles, total, seg, til, seg_off, tile_off, ntiles_out, tiles);
  __syncthreads();
  for (int i = threadIdx.x; i < Z * kFusedWaves; i += kFusedThreads) counts[i] += seg[i / kFusedWaves];
  __syncthreads();
  const int z_bits = 32 - __builtin_clz(Z);  // bits needed for 0..Z-1 (one spare when Z is a power of two)
#pragma unroll
  for (int c = 0; c < kFusedChunks; ++c) {
    if (lo + c * kLanes >= hi) break;  // wave-uniform
    const int e = zs[c];
    scatter_chunk(e, e >= 0 && e < Z, lo + c * kLanes + lane, lane, z_bits, counts + wave, kFusedWaves, perm);
  }
}

// ---------------------------------------------------------------- three launches (large batches)
__global__ __launch_bounds__(kGroupThreads) void group_count_kernel(const int32_t* __restrict__ z, int n, int Z,
                                                                    int W, int nodes_per_wave,
                                                                    int32_t* __restrict__ counts) {
  extern __shared__ int32_t lds[];  // [kGroupWavesPerWG][Z]
  const int wave = threadIdx.x / kLanes, lane = threadIdx.x % kLanes;
  const int gw = blockIdx.x * kGroupWavesPerWG + wave;
  int32_t* mine = lds + wave * Z;
  for (int e = lane; e < Z; e += kLanes) mine[e] = 0;
  __syncthreads();
  const long long lo = static_cast<long long>(gw) * nodes_per_wave;
  const long long hi = (lo + nodes_per_wave < n) ? lo + nodes_per_wave : n;
  for (long long c0 = lo; c0 < hi; c0 += kBatch * kLanes) {  // kBatch independent loads in flight
    int zs[kBatch];
#pragma unroll
    for (int c = 0; c < kBatch; ++c) {
      const long long i = c0 + c * kLanes + lane;
      zs[c] = (i < hi) ? z[i] : -1;
    }
#pragma unroll
    for (int c = 0; c < kBatch; ++c)
      if (zs[c] >= 0 && zs[c] < Z) atomicAdd(&mine[zs[c]], 1);
  }
  __syncthreads();
  for (int e = lane; e < Z; e += kLanes) counts[static_cast<size_t>(e) * W + gw] = mine[e];
}

// counts is [Z][W]; a wave scans one row at a time (W <= kMaxGroupWaves = 4 per lane).
__global__ __launch_bounds__(kFusedThreads) void group_scan_kernel(int Z, int W, int tile_nodes, int max_tiles,
                                                                   int32_t* __restrict__ counts,
                                                                   int32_t* __restrict__ seg_off,
                                                                   int32_t* __restrict__ tile_off,
                                                                   int32_t* __restrict__ ntiles_out,
                                                                   TileDesc* __restrict__ tiles) {
  __shared__ int32_t total[SC_MAX_ELEMENTS];
  __shared__ int32_t seg[SC_MAX_ELEMENTS + 1];
  __shared__ int32_t til[SC_MAX_ELEMENTS + 1];
  const int wave = threadIdx.x / kLanes, lane = threadIdx.x % kLanes;
  constexpr int kPer = kMaxGroupWaves / kLanes;
  constexpr int kRows = 4;  // rows whose loads are issued together
  for (int e0 = wave; e0 < Z; e0 += kFusedWaves * kRows) {
    int c[kRows][kPer];
#pragma unroll
    for (int r = 0; r < kRows; ++r) {
      const int e = e0 + r * kFusedWaves;
#pragma unroll
      for (int k = 0; k < kPer; ++k) {
        const int w = lane * kPer + k;
        c[r][k] = (e < Z && w < W) ? counts[static_cast<size_t>(e) * W + w] : 0;
      }
    }
#pragma unroll
    for (int r = 0; r < kRows; ++r) {
      const int e = e0 + r * kFusedWaves;
      if (e >= Z) break;  // wave-uniform
      int local = 0;
#pragma unroll
      for (int k = 0; k < kPer; ++k) local += c[r][k];
      int incl = local;  // inclusive scan over the lanes
#pragma unroll
      for (int d = 1; d < kLanes; d <<= 1) {
        const int up = __shfl_up(incl, d);
        if (lane >= d) incl += up;
      }
      int run = incl - local;
#pragma unroll
      for (int k = 0; k < kPer; ++k) {
        const int w = lane * kPer + k;
        if (w < W) counts[static_cast<size_t>(e) * W + w] = run;
        run += c[r][k];
      }
      if (lane == kLanes - 1) total[e] = incl;
    }
  }
  __syncthreads();
  offsets_and_tiles(Z, tile_nodes, max_tiles, total, seg, til, seg_off, tile_off, ntiles_out, tiles);
}

__global__ __launch_bounds__(kGroupThreads) void group_scatter_kernel(const int32_t* __restrict__ z, int n, int Z,
                                                                      int W, int nodes_per_wave,
                                                                      const int32_t* __restrict__ counts,
                                                                      const int32_t* __restrict__ seg_off,
                                                                      int32_t* __restrict__ perm) {
  extern __shared__ int32_t lds[];  // [kGroupWavesPerWG][Z] running cursors
  const int wave = threadIdx.x / kLanes, lane = threadIdx.x % kLanes;
  const int gw = blockIdx.x * kGroupWavesPerWG + wave;
  int32_t* cursor = lds + wave * Z;
  for (int e = lane; e < Z; e += kLanes) cursor[e] = seg_off[e] + counts[static_cast<size_t>(e) * W + gw];
  __syncthreads();
  const long long lo = static_cast<long long>(gw) * nodes_per_wave;
  const long long hi = (lo + nodes_per_wave < n) ? lo + nodes_per_wave : n;
  const int z_bits = 32 - __builtin_clz(Z);
  for (long long c0 = lo; c0 < hi; c0 += kBatch * kLanes) {  // wave-uniform trip count
    int zs[kBatch];
#pragma unroll
    for (int c = 0; c < kBatch; ++c) {
      const long long i = c0 + c * kLanes + lane;
      zs[c] = (i < hi) ? z[i] : -1;
    }
#pragma unroll
    for (int c = 0; c < kBatch; ++c) {
      if (c0 + c * kLanes >= hi) break;  // wave-uniform
      const int e = zs[c];
      scatter_chunk(e, e >= 0 && e < Z, static_cast<int>(c0 + c * kLanes + lane), lane, z_bits, cursor, 1, perm);
    }
  }
}

}  // namespace

hipError_t launch_grouping(const sc_plan* plan, int64_t n, const int32_t* z, const Workspace& ws,
                           const LaunchShape& shape, hipStream_t stream) {
  const int Z = plan->cfg.num_elements;
  if (shape.group_waves == 0) {  // single launch
    const size_t lds = sizeof(int32_t) * (static_cast<size_t>(Z) * kFusedWaves + 3 * Z + 2);
    hipLaunchKernelGGL(group_fused_kernel, dim3(1), dim3(kFusedThreads), lds, stream, z, static_cast<int>(n), Z,
                       shape.tile_nodes, shape.max_tiles, ws.seg_off, ws.tile_off, ws.ntiles, ws.tiles, ws.perm);
    return hipGetLastError();
  }
  const int W = shape.group_waves;
  const int wgs = W / kGroupWavesPerWG;
  const size_t lds = static_cast<size_t>(kGroupWavesPerWG) * Z * sizeof(int32_t);
  hipLaunchKernelGGL(group_count_kernel, dim3(wgs), dim3(kGroupThreads), lds, stream, z, static_cast<int>(n), Z, W,
                     shape.nodes_per_group_wave, ws.counts);
  hipLaunchKernelGGL(group_scan_kernel, dim3(1), dim3(kFusedThreads), 0, stream, Z, W, shape.tile_nodes,
                     shape.max_tiles, ws.counts, ws.seg_off, ws.tile_off, ws.ntiles, ws.tiles);
  hipLaunchKernelGGL(group_scatter_kernel, dim3(wgs), dim3(kGroupThreads), lds, stream, z, static_cast<int>(n), Z, W,
                     shape.nodes_per_group_wave, ws.counts, ws.seg_off, ws.perm);
  return hipGetLastError();
}

}  // namespace sc
