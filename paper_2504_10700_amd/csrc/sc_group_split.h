// Grouping of nodes by element as ROLES of larger launches (device code, included by the
// kernels that host it).
//
// The same stable counting sort as sc_group.hip, cut in two so that no launch of its own is
// needed and no single workgroup sits on the critical path:
//   count role    (hosted by the launch that prepares the folded weights) every wave counts the
//                 elements of its contiguous slice of z and writes one row of the count
//                 matrix counts[wave][element];
//   window role   (same launch, only for a forward pass) one workgroup per window of 1024 nodes
//                 orders the window's nodes by element: the order in which the forward kernel,
//                 which needs no grouping for its results, visits them so that it meets long
//                 runs of one element;
//   scatter role  (hosted by the forward launch, whose own work does not need the grouping)
//                 every workgroup sums the matrix columns on its own - the totals per element
//                 and the counts of all earlier waves - scans the totals over the elements and
//                 scatters its four slices to their final positions in perm;
//   table role    one workgroup of the same launch writes the element offsets and the tile
//                 descriptors.
// The result (perm, seg_off, tile_off, tiles, ntiles) is bit for bit what launch_grouping
// writes: the stable sort has one answer.
#pragma once
#include "sc_internal.h"

namespace sc {

constexpr int kSplitThreads = kGroupWavesPerWG * kLanes;   // 256, the block size of the hosting kernels

struct SplitGroupArgs {
  const int32_t* z;
  int n, Z;
  int W;               // waves of the counting sort = rows of counts (a multiple of kGroupWavesPerWG)
  int nodes_per_wave;
  int tile_nodes, max_tiles;
  int32_t* counts;     // [W][Z]
  int32_t* seg_off;    // [Z+1]
  int32_t* tile_off;   // [Z+1]
  int32_t* ntiles;     // [1]
  TileDesc* tiles;     // [max_tiles]
  int32_t* perm;       // [n]
  // window order for the forward kernel (both null: not wanted): position j holds a node and its
  // element index (Z for an index outside [0, Z)); every window of kWindowNodes positions holds
  // the nodes of the same range of the batch, stably ordered by element, invalid ones last
  int32_t* wnode;      // [n]
  int32_t* wkey;       // [n]
};

// dynamic LDS (bytes) a hosting kernel must provide for the count, scatter and table roles
inline size_t split_group_lds_bytes(int Z) { return sizeof(int32_t) * (static_cast<size_t>(kGroupWavesPerWG + 1) * Z + 4 + 256); }

// Stable scatter of one 64-node chunk: lane holds element e (valid or not); cursor[e] is this
// wave's next free position of element e (LDS).  The lanes that hold the same element are found
// bit by bit (one ballot per bit of the element index), which costs the same whatever the
// number of distinct elements in the chunk.
__device__ __forceinline__ void split_scatter_chunk(int e, bool valid, int node, int lane, int z_bits, int32_t* cursor,
                                                    int32_t* __restrict__ perm) {
  const unsigned long long lt_mask = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
  unsigned long long same = __ballot(valid);
  for (int b = 0; b < z_bits; ++b) {
    const bool bit = (e >> b) & 1;
    const unsigned long long m = __ballot(bit);
    same &= bit ? m : ~m;
  }
  const int rank = __popcll(same & lt_mask);
  const int group = __popcll(same);
  const int leader = valid ? __ffsll(static_cast<long long>(same)) - 1 : lane;
  int base = 0;
  if (valid && lane == leader) base = atomicAdd(&cursor[e], group);
  base = __shfl(base, leader);
  if (valid) perm[base + rank] = node;
}

// Exclusive scan of v[0..n) (LDS, n <= 1024) in place by ONE wave; returns the total.  Lane l owns
// the `per` consecutive entries from l * per; they are read twice (sum, then running sums) so that
// the loops run `per` times (two for 89 elements), not the sixteen of the largest n.
__device__ __forceinline__ int split_wave_scan(int32_t* v, int n, int lane) {
  const int per = (n + kLanes - 1) / kLanes;   // uniform
  const int first = lane * per;
  int local = 0;
  for (int k = 0; k < per; ++k) local += (first + k < n) ? v[first + k] : 0;
  int incl = local;
#pragma unroll
  for (int d = 1; d < kLanes; d <<= 1) {
    const int up = __shfl_up(incl, d);
    if (lane >= d) incl += up;
  }
  int run = incl - local;
  for (int k = 0; k < per; ++k) {
    if (first + k < n) {
      const int c = v[first + k];
      v[first + k] = run;
      run += c;
    }
  }
  return __shfl(incl, kLanes - 1);
}

// Workgroup `wg` (of W / 4) counts the slices of its four waves.  lds: 4 * Z ints.
__device__ __forceinline__ void split_count_role(const SplitGroupArgs& g, int wg, int32_t* lds) {
  constexpr int kBatch = 8;
  const int wave = threadIdx.x / kLanes, lane = threadIdx.x % kLanes;
  const int gw = wg * kGroupWavesPerWG + wave;
  int32_t* mine = lds + wave * g.Z;
  for (int e = lane; e < g.Z; e += kLanes) mine[e] = 0;
  __syncthreads();
  const long long lo = static_cast<long long>(gw) * g.nodes_per_wave;
  const long long hi = (lo + g.nodes_per_wave < g.n) ? lo + g.nodes_per_wave : g.n;
  for (long long c0 = lo; c0 < hi; c0 += kBatch * kLanes) {
    int zs[kBatch];
#pragma unroll
    for (int c = 0; c < kBatch; ++c) {
      const long long i = c0 + c * kLanes + lane;
      zs[c] = (i < hi) ? g.z[i] : -1;
    }
#pragma unroll
    for (int c = 0; c < kBatch; ++c)
      if (zs[c] >= 0 && zs[c] < g.Z) atomicAdd(&mine[zs[c]], 1);
  }
  __syncthreads();
  for (int e = lane; e < g.Z; e += kLanes) g.counts[static_cast<size_t>(gw) * g.Z + e] = mine[e];
}

// Window order for the forward kernel: workgroup `win` orders the nodes [win * kWindowNodes, ...) of
// the batch by element (stable; nodes with an index outside [0, Z) last) and writes, for every
// position of the window, the node and its element index.  A counting sort inside the workgroup:
// every wave counts its 256 nodes (kept in registers), the counts are summed over the waves and
// scanned over the elements, every wave places its nodes.  lds: split_window_lds_bytes(Z).
constexpr int kWindowChunks = 4;                                              // 64-node chunks per wave
constexpr int kWindowNodes = kGroupWavesPerWG * kWindowChunks * kLanes;       // 1024
inline size_t split_window_lds_bytes(int Z) { return sizeof(int32_t) * (static_cast<size_t>(2 * kGroupWavesPerWG + 1) * Z + 2 * kGroupWavesPerWG); }

__device__ __forceinline__ void split_window_role(const SplitGroupArgs& g, int win, int32_t* lds) {
  const int wave = threadIdx.x / kLanes, lane = threadIdx.x % kLanes;
  int32_t* mine = lds + wave * g.Z;                                   // [4][Z] counts per wave
  int32_t* invalid = lds + kGroupWavesPerWG * g.Z;                    // [4] nodes with an index outside [0, Z), per wave
  int32_t* cursor_invalid = invalid + kGroupWavesPerWG;               // [4]
  int32_t* seg = cursor_invalid + kGroupWavesPerWG;                   // [Z] totals of the window, then their scan
  int32_t* cursor = seg + g.Z;                                        // [4][Z]
  const long long base = static_cast<long long>(win) * kWindowNodes;
  const long long lo = base + static_cast<long long>(wave) * kWindowChunks * kLanes;
  const long long hi = (lo + kWindowChunks * kLanes < g.n) ? lo + kWindowChunks * kLanes : g.n;
  int zs[kWindowChunks];
#pragma unroll
  for (int c = 0; c < kWindowChunks; ++c) {
    const long long i = lo + c * kLanes + lane;
    zs[c] = (i < hi) ? g.z[i] : -1;
  }
  for (int e = lane; e < g.Z; e += kLanes) mine[e] = 0;
  if (threadIdx.x < kGroupWavesPerWG) invalid[threadIdx.x] = 0;
  __syncthreads();
#pragma unroll
  for (int c = 0; c < kWindowChunks; ++c) {
    if (zs[c] >= 0 && zs[c] < g.Z) atomicAdd(&mine[zs[c]], 1);
    else if (lo + c * kLanes + lane < hi) atomicAdd(&invalid[wave], 1);
  }
  __syncthreads();
  for (int e = threadIdx.x; e < g.Z; e += kSplitThreads) {
    int run = 0;
#pragma unroll
    for (int v = 0; v < kGroupWavesPerWG; ++v) {
      cursor[v * g.Z + e] = run;      // nodes of e in the earlier waves
      run += lds[v * g.Z + e];
    }
    seg[e] = run;
  }
  __syncthreads();
  int n_valid = 0;
  if (wave == 0) n_valid = split_wave_scan(seg, g.Z, lane);
  if (threadIdx.x == 0) {
    int run = n_valid;                 // the invalid nodes follow the valid ones
#pragma unroll
    for (int v = 0; v < kGroupWavesPerWG; ++v) {
      cursor_invalid[v] = run;
      run += invalid[v];
    }
  }
  __syncthreads();
  int32_t* my_cursor = cursor + wave * g.Z;
  for (int e = lane; e < g.Z; e += kLanes) my_cursor[e] += seg[e];
  __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
  __builtin_amdgcn_wave_barrier();
  // the four chunks step by step side by side (ballots, then the four cursor updates, then the four
  // broadcasts), so that the LDS latencies overlap; the updates of one cursor stay in chunk order
  const int z_bits = 32 - __builtin_clz(g.Z);
  const unsigned long long lt_mask = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
  bool in_range[kWindowChunks], valid[kWindowChunks];
  unsigned long long same[kWindowChunks], bad[kWindowChunks];
  int leader[kWindowChunks], base_pos[kWindowChunks], bad_pos[kWindowChunks];
#pragma unroll
  for (int c = 0; c < kWindowChunks; ++c) {
    in_range[c] = lo + c * kLanes + lane < hi;
    valid[c] = in_range[c] && zs[c] >= 0 && zs[c] < g.Z;
    same[c] = __ballot(valid[c]);
    for (int b = 0; b < z_bits; ++b) {
      const bool bit = (zs[c] >> b) & 1;
      const unsigned long long m = __ballot(bit);
      same[c] &= bit ? m : ~m;
    }
    bad[c] = __ballot(in_range[c] && !valid[c]);
    leader[c] = valid[c] ? __ffsll(static_cast<long long>(same[c])) - 1 : lane;
  }
#pragma unroll
  for (int c = 0; c < kWindowChunks; ++c) {
    base_pos[c] = 0;
    if (valid[c] && lane == leader[c]) base_pos[c] = atomicAdd(&my_cursor[zs[c]], __popcll(same[c]));
    bad_pos[c] = 0;
    if (bad[c] != 0ull && lane == __ffsll(static_cast<long long>(bad[c])) - 1)
      bad_pos[c] = atomicAdd(&cursor_invalid[wave], __popcll(bad[c]));
  }
#pragma unroll
  for (int c = 0; c < kWindowChunks; ++c) {
    base_pos[c] = __shfl(base_pos[c], leader[c]);
    if (bad[c] != 0ull) bad_pos[c] = __shfl(bad_pos[c], __ffsll(static_cast<long long>(bad[c])) - 1);   // uniform
  }
#pragma unroll
  for (int c = 0; c < kWindowChunks; ++c) {
    if (!in_range[c]) continue;
    const int pos = valid[c] ? base_pos[c] + __popcll(same[c] & lt_mask) : bad_pos[c] + __popcll(bad[c] & lt_mask);
    g.wnode[base + pos] = static_cast<int32_t>(lo + c * kLanes + lane);
    g.wkey[base + pos] = valid[c] ? zs[c] : g.Z;
  }
}

// Column sums of the count matrix for element e: the total and, for the four waves w0..w0+3,
// the number of nodes of e in all earlier waves.  Loads in batches of 32 independent ones.
__device__ __forceinline__ int split_column(const SplitGroupArgs& g, int e, int w0, int (&before)[kGroupWavesPerWG]) {
  constexpr int kLoads = 32;
  int run = 0;
#pragma unroll
  for (int v = 0; v < kGroupWavesPerWG; ++v) before[v] = 0;
  for (int w = 0; w < g.W; w += kLoads) {
    int c[kLoads];
#pragma unroll
    for (int k = 0; k < kLoads; ++k) c[k] = (w + k < g.W) ? g.counts[static_cast<size_t>(w + k) * g.Z + e] : 0;
#pragma unroll
    for (int k = 0; k < kLoads; ++k) {
#pragma unroll
      for (int v = 0; v < kGroupWavesPerWG; ++v)
        if (w + k == w0 + v) before[v] = run;
      run += c[k];
    }
  }
  return run;
}

// Workgroup `wg` scatters the slices of its four waves.  lds: 5 * Z ints.
__device__ __forceinline__ void split_scatter_role(const SplitGroupArgs& g, int wg, int32_t* lds) {
  constexpr int kBatch = 8;
  const int wave = threadIdx.x / kLanes, lane = threadIdx.x % kLanes;
  const int w0 = wg * kGroupWavesPerWG;
  int32_t* cursor = lds;                            // [4][Z]
  int32_t* seg = lds + kGroupWavesPerWG * g.Z;      // [Z] totals, then their exclusive scan
  for (int e = threadIdx.x; e < g.Z; e += kSplitThreads) {
    int before[kGroupWavesPerWG];
    seg[e] = split_column(g, e, w0, before);
#pragma unroll
    for (int v = 0; v < kGroupWavesPerWG; ++v) cursor[v * g.Z + e] = before[v];
  }
  __syncthreads();
  if (wave == 0) split_wave_scan(seg, g.Z, lane);
  __syncthreads();
  for (int e = threadIdx.x; e < g.Z; e += kSplitThreads) {
#pragma unroll
    for (int v = 0; v < kGroupWavesPerWG; ++v) cursor[v * g.Z + e] += seg[e];
  }
  __syncthreads();
  int32_t* mine = cursor + wave * g.Z;
  const int gw = w0 + wave;
  const long long lo = static_cast<long long>(gw) * g.nodes_per_wave;
  const long long hi = (lo + g.nodes_per_wave < g.n) ? lo + g.nodes_per_wave : g.n;
  const int z_bits = 32 - __builtin_clz(g.Z);
  for (long long c0 = lo; c0 < hi; c0 += kBatch * kLanes) {   // wave-uniform trip count
    int zs[kBatch];
#pragma unroll
    for (int c = 0; c < kBatch; ++c) {
      const long long i = c0 + c * kLanes + lane;
      zs[c] = (i < hi) ? g.z[i] : -1;
    }
#pragma unroll
    for (int c = 0; c < kBatch; ++c) {
      if (c0 + c * kLanes >= hi) break;  // wave-uniform
      const int e = zs[c];
      split_scatter_chunk(e, e >= 0 && e < g.Z, static_cast<int>(c0 + c * kLanes + lane), lane, z_bits, mine, g.perm);
    }
  }
}

// One workgroup: element offsets, tile offsets, tile count and tile descriptors.
//
// Tiles: the grouped sequence (positions 0..n_valid of perm) is cut every g.tile_nodes positions
// and at every change of element; a tile is one piece.  Whole pieces take one workgroup of a main
// kernel for the same time, and the pieces next to element boundaries are shorter, so the
// descriptors are stored LARGEST FIRST: workgroups are dispatched in index order, the short
// pieces come last and fill the slots the first finishers leave (largest-first list scheduling;
// with equal tiles - every element split evenly - the last round of workgroups ran with most of
// the chip idle: 2.2 rounds cost three).  The per-tile dW rows stay in (element, position) order
// through TileDesc::id, which is what the second stage of the dW reduction walks.
// lds: split_group_lds_bytes(Z).
constexpr int kTileSizeBins = 256;   // tiles of 255 nodes and more share a bin

__device__ __forceinline__ TileDesc split_tile(const SplitGroupArgs& g, const int32_t* total, const int32_t* seg,
                                               const int32_t* til, int i) {
  int lo = 0, hi = g.Z;  // last e with til[e] <= i (empty elements share an offset with the next one)
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (til[mid] <= i) lo = mid; else hi = mid;
  }
  const int e = lo;
  const int r = seg[e] / g.tile_nodes + (i - til[e]);             // the cut this piece lies in
  const long long cut0 = static_cast<long long>(r) * g.tile_nodes, cut1 = cut0 + g.tile_nodes;
  const int end_e = seg[e] + total[e];
  const int start = cut0 > seg[e] ? static_cast<int>(cut0) : seg[e];
  const int end = cut1 < end_e ? static_cast<int>(cut1) : end_e;
  return TileDesc{e, start, end - start, i};
}

__device__ __forceinline__ void split_table_role(const SplitGroupArgs& g, int32_t* lds) {
  int32_t* total = lds;            // [Z]
  int32_t* seg = total + g.Z;      // [Z+1]
  int32_t* til = seg + g.Z + 1;    // [Z+1]
  int32_t* bins = til + g.Z + 1;   // [kTileSizeBins] tiles per size, largest size first; then their offsets
  const int t = threadIdx.x;
  for (int e = t; e < g.Z; e += kSplitThreads) {
    int before[kGroupWavesPerWG];
    total[e] = split_column(g, e, -kGroupWavesPerWG, before);
    seg[e] = total[e];
  }
  for (int b = t; b < kTileSizeBins; b += kSplitThreads) bins[b] = 0;
  __syncthreads();
  if (t < kLanes) {  // wave 0
    const int n_valid = split_wave_scan(seg, g.Z, t);
    if (t == 0) seg[g.Z] = n_valid;
  }
  __syncthreads();
  for (int e = t; e < g.Z; e += kSplitThreads)   // cuts that element e's positions touch
    til[e] = total[e] > 0 ? (seg[e] + total[e] - 1) / g.tile_nodes - seg[e] / g.tile_nodes + 1 : 0;
  __syncthreads();
  if (t < kLanes) {
    const int n_tiles = split_wave_scan(til, g.Z, t);
    if (t == 0) {
      til[g.Z] = n_tiles;
      *g.ntiles = (n_tiles < g.max_tiles) ? n_tiles : g.max_tiles;
    }
  }
  __syncthreads();
  const int n_tiles = til[g.Z] < g.max_tiles ? til[g.Z] : g.max_tiles;
  for (int e = t; e <= g.Z; e += kSplitThreads) {
    g.seg_off[e] = seg[e];
    g.tile_off[e] = til[e];
  }
  // largest first: count the tiles per size, scan, place
  auto bin_of = [](int count) { return kTileSizeBins - 1 - (count < kTileSizeBins - 1 ? count : kTileSizeBins - 1); };
  for (int i = t; i < n_tiles; i += kSplitThreads) atomicAdd(&bins[bin_of(split_tile(g, total, seg, til, i).count)], 1);
  __syncthreads();
  if (t < kLanes) split_wave_scan(bins, kTileSizeBins, t);
  __syncthreads();
  for (int i = t; i < n_tiles; i += kSplitThreads) {
    const TileDesc d = split_tile(g, total, seg, til, i);
    g.tiles[atomicAdd(&bins[bin_of(d.count)], 1)] = d;
  }
  // unused descriptors say "empty": the main kernels need no separate tile count
  for (int i = n_tiles + t; i < g.max_tiles; i += kSplitThreads) g.tiles[i] = TileDesc{0, 0, 0, 0};
}

}  // namespace sc
