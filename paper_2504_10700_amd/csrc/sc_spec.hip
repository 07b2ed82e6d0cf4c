// Specialised kernels: hand-written memory / scheduling skeleton around generated
// straight-line arithmetic (csrc/generated/*.inc, written by codegen/generate.py).
//
// Mapping (Algorithm 2 of arXiv 2504.10700 is independent per atom and channel):
//   lane      = channel (64 consecutive channels per wave: the A row of a node is read as
//               64 B per lane, a wave covers 4 KB of contiguous HBM; B/dB rows are 16 B per lane)
//   forward   workgroup = 4 waves = a tile of consecutive nodes of the batch x one 64-channel
//               block; a wave visits its share of the nodes grouped by element and reads the
//               folded weights of a run once
//   backward, second-order pass
//             workgroup = 4 waves = one tile of the grouping (nodes of ONE element) x one
//               64-channel block, the element's folded weights in registers; its waves add their
//               dW' rows through LDS, so one partial row set leaves per tile; the grid is
//               remapped so that each XCD (own L2) gets a contiguous range of tiles
// Per node the next node's rows are requested before the current one is evaluated
// (two register sets, ping-pong), so HBM latency hides behind ~300-800 VALU operations.
// kCM instances of the forward and backward kernels serve the component-major layout
// ([node][component][channel], SC_COMPONENT_MAJOR): same mapping and arithmetic, rows accessed
// through Cols instead of Row.
//
// One step (forward + backward of one batch) is four launches:
//   1 prepare   the weights of every (element, channel) folded into the internal basis once,
//               wf[element][channel block][kS][64]; other workgroups of the same launch count the
//               elements of z (first half of the grouping) and, for larger batches, order every
//               window of 1024 nodes by element (the order of the forward's visits)
//   2 forward   nodes in batch order, inside a window by element (no grouping needed: every node
//               reads the folded weights of its element from wf, which stays in L2, once per run
//               of an element): consecutive workgroups stream the same stretch of memory.  Other
//               workgroups of the same launch finish the grouping (scatter + tile table), which
//               only the backward needs
//   3 backward  nodes grouped by element (tiles), weights of the tile's element in registers,
//               dW' summed per tile without atomics
//   4 finalize  per (element, channel block): sum of the per-tile dW' rows in a fixed order
//               (fp64) and the map to the external paths
#include <type_traits>

#include "sc_group_split.h"
#include "sc_spec.h"

namespace sc {
namespace {

__device__ __forceinline__ float sc_fma(float x, float y, float z) { return __builtin_fmaf(x, y, z); }
__device__ __forceinline__ double sc_fma(double x, double y, double z) { return __builtin_fma(x, y, z); }

#include "generated/sc_gen_l3n3_0e1o.inc"
#include "generated/sc_gen_l3n3_0e1o2e.inc"
#include "generated/sc_gen_l3n3_0e1o2e3o.inc"
#include "generated/sc_gen_l1n2_0e.inc"
#include "generated/sc_gen_l3n3_0e.inc"

constexpr int kSpecWaves = 4;
constexpr int kSpecThreads = kSpecWaves * kLanes;
constexpr int kXcds = 8;

__device__ __forceinline__ int wave_of_thread() { return __builtin_amdgcn_readfirstlane(threadIdx.x / kLanes); }

// Row of N elements of T at p (p is aligned to the row size if that is a multiple of 16 B,
// else only to sizeof(T)): 16-byte accesses plus a scalar tail.
template <typename T, int N>
struct Row {
  static constexpr int V = 16 / sizeof(T);
  static constexpr int kAlign = (N * sizeof(T)) % 16 == 0 ? 16 : sizeof(T);
  typedef T Vec __attribute__((ext_vector_type(V), aligned(kAlign)));

  static __device__ __forceinline__ void load(const T* __restrict__ p, T (&v)[N]) {
#pragma unroll
    for (int i = 0; i + V <= N; i += V) {
      const Vec x = *reinterpret_cast<const Vec*>(p + i);
#pragma unroll
      for (int k = 0; k < V; ++k) v[i + k] = x[k];
    }
#pragma unroll
    for (int i = N / V * V; i < N; ++i) v[i] = p[i];
  }
  static __device__ __forceinline__ void store(T* __restrict__ p, const T (&v)[N]) {
#pragma unroll
    for (int i = 0; i + V <= N; i += V) {
      Vec x;
#pragma unroll
      for (int k = 0; k < V; ++k) x[k] = v[i + k];
      // A row of one 16-byte piece makes the wave's store one contiguous KB: streamed past the
      // cache (measured faster).  Longer rows are written by several instructions that each touch
      // a part of every line: left to the L2 to merge (streaming them measured slower).
      if constexpr (N * sizeof(T) == 16) __builtin_nontemporal_store(x, reinterpret_cast<Vec*>(p + i));
      else *reinterpret_cast<Vec*>(p + i) = x;
    }
#pragma unroll
    for (int i = N / V * V; i < N; ++i) p[i] = v[i];
  }
};

// Store of a wave's rows (N elements per lane, lane rows N elements apart = one contiguous
// block of 64*N elements) as fully coalesced instructions: each lane's row goes through an
// LDS block of the same layout and comes back transposed, so that store instruction k
// writes the k-th contiguous 1 KB of the block instead of 64 scattered 16-byte pieces
// (four times fewer, four times larger write requests to L2; measured -10% on the whole
// backward kernel; the same trick on the loads of A gained nothing).  stage: 64*N elements
// of LDS owned by this wave; block: where lane 0's row goes (16-byte aligned); live_lanes: the
// lanes whose rows exist (fewer than 64 in the last channel block of a channel count that is not
// a multiple of 64).
// kStream: non-temporal stores (the rows are not read again soon and each instruction writes
// whole lines).  Measured on one box, library against library: forward 28.4 -> 27.0 us at 10k
// nodes (neutral at 200k), second-order kernel 78.7 -> 77.5 us; a wash for the backward's dA
// at 10k nodes and 1% slower at 200k, so the backward leaves it off.
template <typename T, int N, bool kStream = true>
__device__ __forceinline__ void store_rows_coalesced(T* __restrict__ block, T* stage, int lane, const T (&v)[N],
                                                     int live_lanes = kLanes) {
  constexpr int V = 16 / sizeof(T);
  typedef T Vec __attribute__((ext_vector_type(V)));
  __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");  // earlier reads of the stage are done
  __builtin_amdgcn_wave_barrier();
  if constexpr (N % V == 0) {
#pragma unroll
    for (int j = 0; j < N / V; ++j) {
      Vec x;
#pragma unroll
      for (int k = 0; k < V; ++k) x[k] = v[j * V + k];
      *reinterpret_cast<Vec*>(stage + lane * N + j * V) = x;
    }
  } else {  // rows that are not a whole number of 16-byte pieces (e.g. 9 components)
#pragma unroll
    for (int j = 0; j < N; ++j) stage[lane * N + j] = v[j];
  }
  __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");  // other lanes' pieces are visible
  __builtin_amdgcn_wave_barrier();
  // 16-byte pieces of the block: 64*N/V of them, fewer if the last channel block is not full
  // (live_lanes * N is a multiple of V: channel counts are multiples of four)
  constexpr int kPieces = kLanes * N / V;
  const int pieces = live_lanes * N / V;
#pragma unroll
  for (int q0 = 0; q0 < kPieces; q0 += kLanes) {
    const int q = q0 + lane;
    if ((live_lanes == kLanes && q0 + kLanes <= kPieces) || q < pieces) {   // the first test is a constant for full blocks
      const Vec x = *reinterpret_cast<const Vec*>(stage + q * V);
      if constexpr (kStream) __builtin_nontemporal_store(x, reinterpret_cast<Vec*>(block + q * V));
      else *reinterpret_cast<Vec*>(block + q * V) = x;
    }
  }
}

// Storage type of the per-node rows (A, B, dB, dA, H, ...) when it differs from the arithmetic
// type T: bfloat16 bits (SC_BF16: rows in bfloat16, arithmetic, weights and dW in fp32).
typedef __bf16 bf16_bits;

__device__ __forceinline__ float bf16_to_f32(bf16_bits b) { return static_cast<float>(b); }
// round to nearest, ties to even (the chip's own conversion instruction, two values at a time)
__device__ __forceinline__ bf16_bits f32_to_bf16(float f) { return static_cast<bf16_bits>(f); }

// Rows of N elements stored as TS, handled as T.  TS == T is Row<T, N> itself.
template <typename T, typename TS, int N>
struct RowIO {
  typedef TS Vec8 __attribute__((ext_vector_type(N * sizeof(TS) == 8 ? N : 2), aligned(8)));   // an 8-byte row in one access
  static __device__ __forceinline__ void load(const TS* __restrict__ p, T (&v)[N]) {
    TS raw[N];
    if constexpr (N * sizeof(TS) == 8) {
      const Vec8 x = *reinterpret_cast<const Vec8*>(p);
#pragma unroll
      for (int i = 0; i < N; ++i) raw[i] = x[i];
    } else {
      Row<TS, N>::load(p, raw);
    }
#pragma unroll
    for (int i = 0; i < N; ++i) v[i] = bf16_to_f32(raw[i]);
  }
  static __device__ __forceinline__ void store(TS* __restrict__ p, const T (&v)[N]) {
    TS raw[N];
#pragma unroll
    for (int i = 0; i < N; ++i) raw[i] = f32_to_bf16(v[i]);
    if constexpr (N * sizeof(TS) == 8) {
      Vec8 x;
#pragma unroll
      for (int i = 0; i < N; ++i) x[i] = raw[i];
      *reinterpret_cast<Vec8*>(p) = x;
    } else {
      Row<TS, N>::store(p, raw);
    }
  }
};
template <typename T, int N>
struct RowIO<T, T, N> : Row<T, N> {};

// Component-major rows (SC_COMPONENT_MAJOR: tensors laid out [node][component][channel]): the N
// components of one (node, channel) lie K elements apart, and a wave's access to one component
// covers 64 consecutive channels - coalesced as it is, loads and stores alike, so nothing passes
// through LDS.  p points at component 0 of the lane's channel.
template <typename T, int N>
struct Cols {
  static __device__ __forceinline__ void load(const T* __restrict__ p, int K, T (&v)[N]) {
#pragma unroll
    for (int i = 0; i < N; ++i) v[i] = p[static_cast<size_t>(i) * K];
  }
  template <bool kStream>
  static __device__ __forceinline__ void store(T* __restrict__ p, int K, const T (&v)[N]) {
#pragma unroll
    for (int i = 0; i < N; ++i) {
      if constexpr (kStream) __builtin_nontemporal_store(v[i], p + static_cast<size_t>(i) * K);
      else p[static_cast<size_t>(i) * K] = v[i];
    }
  }
};

// store_rows_coalesced for rows stored as TS; `stage` is this wave's LDS block of 64*N elements of T
// (large enough for TS, which is never wider).
template <typename T, typename TS, int N, bool kStream>
struct RowsOut {
  static __device__ __forceinline__ void store(TS* __restrict__ block, T* stage, int lane, const T (&v)[N], int live_lanes) {
    TS raw[N];
#pragma unroll
    for (int i = 0; i < N; ++i) raw[i] = f32_to_bf16(v[i]);
    store_rows_coalesced<TS, N, kStream>(block, reinterpret_cast<TS*>(stage), lane, raw, live_lanes);
  }
};
template <typename T, int N, bool kStream>
struct RowsOut<T, T, N, kStream> {
  static __device__ __forceinline__ void store(T* __restrict__ block, T* stage, int lane, const T (&v)[N], int live_lanes) {
    store_rows_coalesced<T, N, kStream>(block, stage, lane, v, live_lanes);
  }
};
#define store_rows_as RowsOutCall
template <typename T, typename TS, int N, bool kStream = true>
__device__ __forceinline__ void RowsOutCall(TS* __restrict__ block, T* stage, int lane, const T (&v)[N],
                                            int live_lanes = kLanes) {
  RowsOut<T, TS, N, kStream>::store(block, stage, lane, v, live_lanes);
}

// blockIdx -> logical work item such that the blocks an XCD receives (round-robin by
// blockIdx) form one contiguous range.  gridDim.x is a multiple of kXcds.
__device__ __forceinline__ int xcd_contiguous_block() {
  const int per = gridDim.x / kXcds;
  return (blockIdx.x % kXcds) * per + blockIdx.x / kXcds;
}

// Folded weights: wf[element][channel block][kS][64 channels]: every internal row of an
// (element, channel block) is 256 contiguous bytes (fp32), so a wave reads it with one fully
// coalesced instruction.  (Rows per lane - [element][channel][kS] read as 16-byte pieces - make
// every load instruction touch 64 cache lines; with the weights read per node that bound the
// natural-order forward by the tag rate of the vector cache: 614 us instead of 440 at 200k nodes.)
template <typename T, typename G>
__device__ __forceinline__ void load_folded(const T* __restrict__ wf, int z, int chblocks, int cb, int lane,
                                            T (&w)[G::kS]) {
  const T* src = wf + (static_cast<size_t>(z) * chblocks + cb) * G::kS * kLanes + lane;
#pragma unroll
  for (int s = 0; s < G::kS; ++s) w[s] = src[s * kLanes];
}

// Launch 1.  Workgroups [0, window_wgs): window role (order of the forward pass); the next
// count_wgs: count role of the grouping.  The others: one wave per (element, 64 channels) folds
// W[element, :, channel] into wf.
template <typename T, typename G>
__global__ __launch_bounds__(kSpecThreads) void spec_prepare_kernel(SplitGroupArgs ga, int count_wgs, int window_wgs, int K,
                                                                    int chblocks, int n_pairs,
                                                                    const T* __restrict__ W, T* __restrict__ wf) {
  extern __shared__ unsigned char lds_raw[];
  if (static_cast<int>(blockIdx.x) < window_wgs) {   // the longest role first
    split_window_role(ga, blockIdx.x, reinterpret_cast<int32_t*>(lds_raw));
    return;
  }
  if (static_cast<int>(blockIdx.x) < window_wgs + count_wgs) {
    split_count_role(ga, blockIdx.x - window_wgs, reinterpret_cast<int32_t*>(lds_raw));
    return;
  }
  const int lane = threadIdx.x & (kLanes - 1);
  const int pair = (static_cast<int>(blockIdx.x) - window_wgs - count_wgs) * kSpecWaves + wave_of_thread();
  if (pair >= n_pairs) return;
  const int z = pair / chblocks, cb = pair % chblocks;
  const int live = K - cb * kLanes < kLanes ? K - cb * kLanes : kLanes;
  const int ch = cb * kLanes + (lane < live ? lane : live - 1);   // dead lanes repeat the last channel
  T w[G::kS], wz[G::kP];
  // all kP rows are requested before the first is used (one memory latency, not one per few rows)
  const T* src = W + static_cast<size_t>(z) * G::kP * K + ch;
#pragma unroll
  for (int p = 0; p < G::kP; ++p) wz[p] = src[static_cast<size_t>(p) * K];
  asm volatile("" ::: "memory");
  G::fold(wz, 1, w);
  T* dst = wf + static_cast<size_t>(pair) * G::kS * kLanes + lane;   // pair = element * chblocks + channel block
#pragma unroll
  for (int s = 0; s < G::kS; ++s) dst[s * kLanes] = w[s];
}

// The grouping alone (a backward pass that cannot reuse a forward's grouping): scatter and table roles.
__global__ __launch_bounds__(kSpecThreads) void spec_scatter_kernel(SplitGroupArgs ga, int scatter_wgs) {
  extern __shared__ unsigned char lds_raw[];
  if (static_cast<int>(blockIdx.x) < scatter_wgs) split_scatter_role(ga, blockIdx.x, reinterpret_cast<int32_t*>(lds_raw));
  else split_table_role(ga, reinterpret_cast<int32_t*>(lds_raw));
}

// Launch 2.  Workgroups [0, scatter_wgs): scatter role; the next `table` (0 or 1): table role;
// the others: forward of `tile` consecutive nodes x one 64-channel block, a
// contiguous quarter of the nodes per wave.  A node whose element index is outside [0, Z) is
// skipped (its row of B is left untouched), as the grouped kernels do.
template <typename T, typename G, typename TS = T, bool kCM = false>
__global__ __launch_bounds__(kSpecThreads) void spec_forward_kernel(SplitGroupArgs ga, int scatter_wgs, int table, int K,
                                                                    int chblocks, int n, int Z, int tile,
                                                                    const TS* __restrict__ A,
                                                                    const int32_t* __restrict__ z,
                                                                    const T* __restrict__ wf, TS* __restrict__ B) {
  extern __shared__ unsigned char lds_raw[];
  int block = blockIdx.x;
  if (block < scatter_wgs) {
    split_scatter_role(ga, block, reinterpret_cast<int32_t*>(lds_raw));
    return;
  }
  if (block < scatter_wgs + table) {
    split_table_role(ga, reinterpret_cast<int32_t*>(lds_raw));
    return;
  }
  block -= scatter_wgs + table;
  const int lane = threadIdx.x & (kLanes - 1);
  const int wave = wave_of_thread();
  T* stage = reinterpret_cast<T*>(lds_raw) + wave * kLanes * G::kNLM;  // [64][kNLM] per wave (if used)
  constexpr bool kStageB = G::kNLM * sizeof(TS) != 16;  // 16-byte rows are coalesced as they are
  const int t = block / chblocks, cb = block % chblocks;
  const int s0 = t * tile;
  const int in_tile = (n - s0 < tile) ? n - s0 : tile;
  const int j0 = s0 + in_tile * wave / kSpecWaves, j1 = s0 + in_tile * (wave + 1) / kSpecWaves;
  if (j0 >= j1) return;
  const int live = K - cb * kLanes < kLanes ? K - cb * kLanes : kLanes;   // channels of this block
  const int ch = cb * kLanes + (lane < live ? lane : live - 1);           // dead lanes repeat the last channel
  // This wave's nodes (at most 64: one per lane) are visited grouped by element - a stable sort of
  // their element indices inside the wave - so that a run of nodes of one element reads the
  // folded weights once (they are re-read per node otherwise: 61 of 432 us at 200k nodes).  The
  // indices are read at once, which also takes them off the per-node chain of dependent loads.
  // Nodes with an element index outside [0, Z) sort last and are skipped.  (A third row buffer, i.e.
  // the rows of node p+2 requested while node p is evaluated, measured the same at 10k nodes and 3%
  // slower at 200k.)
  // With the window order of the prepare launch (ga.wnode) the wave's positions hold nodes of a
  // 1024-node window that are ordered by element already, so the runs are long: 0.2 instead of 0.8
  // reads of the weights per node with 89 elements of skewed frequency, which is what the forward
  // gains from a batch ordered by element (427 -> 385 us at 200k nodes; the weights are L2 hits, but
  // 2.4 GB of them per launch next to 1.6 GB of A).  The sort inside the wave stays: it moves nodes
  // with an invalid index to the end and joins runs across a window boundary.
  const int cnt = j1 - j0;
  int key = Z, mine = j0 + lane;   // the lane's node and its element index
  if (lane < cnt) {
    int e;
    if (ga.wnode) {   // positions follow the window order written by the count role (uniform)
      mine = ga.wnode[j0 + lane];
      mine = mine < 0 ? 0 : (mine >= n ? n - 1 : mine);
      e = ga.wkey[j0 + lane];
    } else {
      e = z[j0 + lane];
    }
    key = (e >= 0 && e < Z) ? e : Z;
  }
  int rank = lane;   // lanes past the last node keep their own slot
  if (lane < cnt) rank = 0;
  for (int k = 0; k < cnt; ++k) {   // uniform trip count
    const int zk = __builtin_amdgcn_readlane(key, k);
    if (lane < cnt && (zk < key || (zk == key && k < lane))) ++rank;
  }
  const int order = __builtin_amdgcn_ds_permute(rank << 2, lane);   // order[p] = lane of the node visited p-th
  auto visit = [&](int p, int& node, int& e) {
    const int idx = __builtin_amdgcn_readlane(order, p);
    e = __builtin_amdgcn_readlane(key, idx);
    node = __builtin_amdgcn_readlane(mine, idx);
  };
  // Rows: two register sets in turn (the next node's row is requested before the current node is
  // evaluated).  Weights: ONE register set, reloaded from the folded table (L2) right before a node of
  // another element is evaluated - a second set for prefetching them costs 29-68 registers and with
  // them a wave per SIMD, which hides that latency better than the prefetch does.
  T a0[G::kNlm], a1[G::kNlm], w[G::kS], b[G::kNLM];
  static_assert(!kCM || std::is_same<T, TS>::value, "component-major rows are stored in the arithmetic type");
  auto load_a = [&](int node, T (&a)[G::kNlm]) {
    if constexpr (kCM) Cols<TS, G::kNlm>::load(A + static_cast<size_t>(node) * G::kNlm * K + ch, K, a);
    else RowIO<T, TS, G::kNlm>::load(A + (static_cast<size_t>(node) * K + ch) * G::kNlm, a);
  };
  auto store_b = [&](int node) {
    if constexpr (kCM) {
      if (lane < live) Cols<TS, G::kNLM>::template store<true>(B + static_cast<size_t>(node) * G::kNLM * K + ch, K, b);
    } else if constexpr (kStageB) {
      store_rows_as<T, TS, G::kNLM>(B + (static_cast<size_t>(node) * K + cb * kLanes) * G::kNLM, stage, lane, b, live);
    } else if (lane < live) {
      RowIO<T, TS, G::kNLM>::store(B + (static_cast<size_t>(node) * K + ch) * G::kNLM, b);
    }
  };
  // The loop takes two nodes per trip and every load in it is issued without a condition of its
  // own, in a fixed order: the weights of a new element first, then the rows of the next node, then
  // the arithmetic of the current node, which waits for its own operands only.  (A request under
  // a condition makes the compiler wait for ALL outstanding loads at the join, the request just
  // issued included, before the arithmetic it is meant to overlap; the scheduling barrier keeps the
  // compiler from moving the request down into that arithmetic to save registers.)  The last trip
  // of an even share requests its last node's rows once more; an odd share ends with a single node.
  const int valid = __builtin_popcountll(__ballot(key < Z));   // they come first in the visiting order
  if (valid == 0) return;   // no valid node in this wave's share
  int n0, e0, n1, e1, e_w = -1;
  visit(0, n0, e0);
  load_a(n0, a0);
  int p = 0;
  for (; p + 1 < valid; p += 2) {
    if (e0 != e_w) {
      load_folded<T, G>(wf, e0, chblocks, cb, lane, w);
      e_w = e0;
    }
    visit(p + 1, n1, e1);
    load_a(n1, a1);
    __builtin_amdgcn_sched_barrier(0);
    G::forward(a0, w, b);
    store_b(n0);
    if (e1 != e_w) {
      load_folded<T, G>(wf, e1, chblocks, cb, lane, w);
      e_w = e1;
    }
    visit(p + 2 < valid ? p + 2 : valid - 1, n0, e0);
    load_a(n0, a0);
    __builtin_amdgcn_sched_barrier(0);
    G::forward(a1, w, b);
    store_b(n1);
  }
  if (p < valid) {
    if (e0 != e_w) load_folded<T, G>(wf, e0, chblocks, cb, lane, w);
    G::forward(a0, w, b);
    store_b(n0);
  }
}

// kOcc = waves per SIMD the kernel is held to (0: the compiler's choice, which every launch uses now).
// The fp32 kernel of the small basis needs 171 registers if left alone, three over the limit for
// three waves per SIMD; held to 168 (two values go to scratch) it ran three workgroups per CU
// instead of two, which paid while small batches were cut into many equal tiles (51.1 -> 49.3 us
// at 10k nodes).  With tiles processed largest first and about one and a half whole tiles per CU
// the third workgroup is rarely resident, and the unconstrained kernel is faster (step 82.8 -> 80.8
// us at 10k nodes, same box).
// kStreamDA: the dA rows are streamed past the cache (non-temporal stores), for batches up to
// 40 000 nodes: the kernel itself gains 2 us at 10k nodes and the launches after it another 3 us,
// whereas at 200k nodes the backward loses 2% with them and the next forward gains as much.
// kFull: the channel count is a multiple of 64, no lane is ever idle.  The fp32 kernel of the
// 49-row basis sits at the limit for two waves per SIMD: 250 registers without the idle-lane
// handling, 295 (one wave per SIMD, 736 instead of 496 us at 50k nodes / 256 channels) with it.
template <typename T, typename G, int kOcc = 0, bool kStreamDA = false, bool kFull = false, typename TS = T, bool kCM = false>
__global__ __launch_bounds__(kSpecThreads) __attribute__((amdgpu_waves_per_eu(kOcc == 0 ? 1 : kOcc, 8)))
void spec_backward_kernel(int K, int chblocks, int n_blocks,
                                                                     const TS* __restrict__ A,
                                                                     const T* __restrict__ wf,
                                                                     const TS* __restrict__ dB, TS* __restrict__ dA,
                                                                     T* __restrict__ partial,
                                                                     const TileDesc* __restrict__ tiles,
                                                                     const int32_t* __restrict__ perm) {
  extern __shared__ unsigned char lds_raw[];
  T* red = reinterpret_cast<T*>(lds_raw);  // [kSpecWaves][kS][64]
  T* stage = red + kSpecWaves * G::kS * kLanes + wave_of_thread() * kLanes * G::kNlm;  // [64][kNlm] per wave
  const int lane = threadIdx.x & (kLanes - 1);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kLanes);
  const int logical = blockIdx.x;   // descriptors are stored largest tile first: dispatch order is the schedule
  if (logical >= n_blocks) return;  // uniform per workgroup
  const int tile = logical / chblocks, cb = logical % chblocks;
  const TileDesc td = tiles[tile];
  if (td.count == 0) return;        // unused descriptor; uniform per workgroup
  const int j0 = td.start + td.count * wave / kSpecWaves;
  const int j1 = td.start + td.count * (wave + 1) / kSpecWaves;
  const int live = kFull ? kLanes : (K - cb * kLanes < kLanes ? K - cb * kLanes : kLanes);   // channels of this block
  const int ch = cb * kLanes + (lane < live ? lane : live - 1);           // dead lanes repeat the last channel
  T dw[G::kS];
#pragma unroll
  for (int s = 0; s < G::kS; ++s) dw[s] = T(0);
  if (j0 < j1) {
    T w[G::kS];
    load_folded<T, G>(wf, td.z, chblocks, cb, lane, w);
    T a0[G::kNlm], a1[G::kNlm], g0[G::kNLM], g1[G::kNLM], da[G::kNlm];
    static_assert(!kCM || std::is_same<T, TS>::value, "component-major rows are stored in the arithmetic type");
    auto load_rows = [&](size_t node, T (&a)[G::kNlm], T (&g)[G::kNLM]) {
      if constexpr (kCM) {
        Cols<TS, G::kNlm>::load(A + node * G::kNlm * K + ch, K, a);
        Cols<TS, G::kNLM>::load(dB + node * G::kNLM * K + ch, K, g);
      } else {
        RowIO<T, TS, G::kNlm>::load(A + (node * K + ch) * G::kNlm, a);
        RowIO<T, TS, G::kNLM>::load(dB + (node * K + ch) * G::kNLM, g);
      }
    };
    auto store_da = [&](size_t node) {
      if constexpr (kCM) {
        if (kFull || lane < live) Cols<TS, G::kNlm>::template store<kStreamDA>(dA + node * G::kNlm * K + ch, K, da);
      } else {
        store_rows_as<T, TS, G::kNlm, kStreamDA>(dA + (node * K + cb * kLanes) * G::kNlm, stage, lane, da, live);
      }
    };
    size_t node0 = perm ? perm[j0] : j0, node1 = 0;   // no permutation: the batch is already grouped
    load_rows(node0, a0, g0);
    for (int j = j0; j < j1; j += 2) {
      if (j + 1 < j1) {
        node1 = perm ? perm[j + 1] : j + 1;
        load_rows(node1, a1, g1);
      }
      G::backward(a0, w, g0, da, dw);
      store_da(node0);
      if (j + 1 < j1) {
        if (j + 2 < j1) {
          node0 = perm ? perm[j + 2] : j + 2;
          load_rows(node0, a0, g0);
        }
        G::backward(a1, w, g1, da, dw);
        store_da(node1);
      }
    }
  }
  // sum the waves' dW' rows in wave order and write the tile's partial rows
#pragma unroll
  for (int s = 0; s < G::kS; ++s) red[(wave * G::kS + s) * kLanes + lane] = dw[s];
  __syncthreads();
  T* out = partial + (static_cast<size_t>(td.id) * chblocks + cb) * G::kS * kLanes;   // rows in (element, position) order
  for (int i = threadIdx.x; i < G::kS * kLanes; i += kSpecThreads) {
    T acc = red[i];
#pragma unroll
    for (int v = 1; v < kSpecWaves; ++v) acc += red[v * G::kS * kLanes + i];
    out[i] = acc;
  }
}

// Second-order pass: the backward skeleton with one more input row (H) and one more output
// row (ddB) per node; its dW2' rows leave through the same per-tile partial rows.
//
// The generated program keeps about 290 values live.  Two kernels:
//  * spec_double_backward_kernel keeps everything in registers (256 VGPRs + AGPRs, one wave
//    per SIMD);
//  * spec_double_backward_lds_kernel keeps the folded weights w' and the dW2' accumulators
//    (2 x kS values per lane) in LDS columns - w' is re-read and the accumulators are updated
//    once per node - which brings it under 256 registers without scratch, so that two waves
//    share a SIMD (measured on MI355X, fp32, 0e+1o: 80 us instead of 106 us at 10k nodes,
//    1.24 ms instead of 1.45 ms at 200k).  It is used where it fits (kUseLdsState): for the
//    larger basis or fp64 it would spill.  Small changes to its text move the register
//    allocation across the spill threshold: check the compiler's resource report
//    (-Rpass-analysis=kernel-resource-usage) after touching it.
// Rows of one node in the second-order kernels, in either layout (see Cols).
template <typename T, typename TS, typename G, bool kCM>
struct NodeRows2 {
  static __device__ __forceinline__ void load(const TS* __restrict__ A, const TS* __restrict__ H, const TS* __restrict__ dB,
                                              size_t node, int K, int ch, T (&a)[G::kNlm], T (&h)[G::kNlm], T (&g)[G::kNLM]) {
    if constexpr (kCM) {
      Cols<TS, G::kNlm>::load(A + node * G::kNlm * K + ch, K, a);
      Cols<TS, G::kNlm>::load(H + node * G::kNlm * K + ch, K, h);
      Cols<TS, G::kNLM>::load(dB + node * G::kNLM * K + ch, K, g);
    } else {
      RowIO<T, TS, G::kNlm>::load(A + (node * K + ch) * G::kNlm, a);
      RowIO<T, TS, G::kNlm>::load(H + (node * K + ch) * G::kNlm, h);
      RowIO<T, TS, G::kNLM>::load(dB + (node * K + ch) * G::kNLM, g);
    }
  }
  template <bool kFull>
  static __device__ __forceinline__ void store(TS* __restrict__ dA2, TS* __restrict__ ddB, size_t node, int K, int cb, int ch,
                                               T* stage, int lane, int live, const T (&da)[G::kNlm], const T (&ddb)[G::kNLM]) {
    if constexpr (kCM) {
      if (kFull || lane < live) {
        Cols<TS, G::kNlm>::template store<true>(dA2 + node * G::kNlm * K + ch, K, da);
        Cols<TS, G::kNLM>::template store<true>(ddB + node * G::kNLM * K + ch, K, ddb);
      }
    } else {
      constexpr bool kStageB = G::kNLM * sizeof(TS) != 16;
      store_rows_as<T, TS, G::kNlm>(dA2 + (node * K + cb * kLanes) * G::kNlm, stage, lane, da, live);
      if constexpr (kStageB) store_rows_as<T, TS, G::kNLM>(ddB + (node * K + cb * kLanes) * G::kNLM, stage, lane, ddb, live);
      else if (kFull || lane < live) RowIO<T, TS, G::kNLM>::store(ddB + (node * K + ch) * G::kNLM, ddb);
    }
  }
};

template <typename T, typename G, bool kFull, typename TS = T, bool kCM = false>
__global__ __launch_bounds__(kSpecThreads) void spec_double_backward_kernel(
    int K, int chblocks, int n_blocks, const TS* __restrict__ A, const T* __restrict__ W, const TS* __restrict__ dB,
    const TS* __restrict__ H, TS* __restrict__ ddB, TS* __restrict__ dA2, T* __restrict__ partial,
    const TileDesc* __restrict__ tiles, const int32_t* __restrict__ perm) {
  extern __shared__ unsigned char lds_raw[];
  T* red = reinterpret_cast<T*>(lds_raw);  // [kSpecWaves][kS][64]
  T* stage = red + kSpecWaves * G::kS * kLanes + wave_of_thread() * kLanes * G::kNlm;  // [64][kNlm] per wave
  static_assert(!kCM || std::is_same<T, TS>::value, "component-major rows are stored in the arithmetic type");
  const int lane = threadIdx.x & (kLanes - 1);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kLanes);
  const int logical = blockIdx.x;   // descriptors are stored largest tile first: dispatch order is the schedule
  if (logical >= n_blocks) return;  // uniform per workgroup
  const int tile = logical / chblocks, cb = logical % chblocks;
  const TileDesc td = tiles[tile];
  if (td.count == 0) return;        // unused descriptor; uniform per workgroup
  const int j0 = td.start + td.count * wave / kSpecWaves;
  const int j1 = td.start + td.count * (wave + 1) / kSpecWaves;
  const int live = kFull ? kLanes : (K - cb * kLanes < kLanes ? K - cb * kLanes : kLanes);   // channels of this block
  const int ch = cb * kLanes + (lane < live ? lane : live - 1);           // dead lanes repeat the last channel
  T dw[G::kS];
#pragma unroll
  for (int s = 0; s < G::kS; ++s) dw[s] = T(0);
  if (j0 < j1) {
    T w[G::kS];
    G::fold(W + static_cast<size_t>(td.z) * G::kP * K + ch, K, w);
    // one register set of inputs: the next node's rows are requested right after the
    // arithmetic of the current one has consumed them, ahead of its stores
    T a[G::kNlm], h[G::kNlm], g[G::kNLM], da[G::kNlm], ddb[G::kNLM];
    size_t node = perm ? perm[j0] : j0;   // no permutation: the batch is already grouped
    NodeRows2<T, TS, G, kCM>::load(A, H, dB, node, K, ch, a, h, g);
    for (int j = j0; j < j1; ++j) {
      G::double_backward(a, w, g, h, ddb, da, dw);
      const size_t cur = node;
      if (j + 1 < j1) {
        node = perm ? perm[j + 1] : j + 1;
        NodeRows2<T, TS, G, kCM>::load(A, H, dB, node, K, ch, a, h, g);
      }
      NodeRows2<T, TS, G, kCM>::template store<kFull>(dA2, ddB, cur, K, cb, ch, stage, lane, live, da, ddb);
    }
  }
#pragma unroll
  for (int s = 0; s < G::kS; ++s) red[(wave * G::kS + s) * kLanes + lane] = dw[s];
  __syncthreads();
  T* out = partial + (static_cast<size_t>(td.id) * chblocks + cb) * G::kS * kLanes;   // rows in (element, position) order
  for (int i = threadIdx.x; i < G::kS * kLanes; i += kSpecThreads) {
    T acc = red[i];
#pragma unroll
    for (int v = 1; v < kSpecWaves; ++v) acc += red[v * G::kS * kLanes + i];
    out[i] = acc;
  }
}

// See above.  LDS: w' [kSpecWaves][kS][64] | sums [kSpecWaves][kS][64] | stage [kSpecWaves][64][kNlm].
template <typename T, typename G, bool kFull, typename TS = T, bool kCM = false>
__global__ __launch_bounds__(kSpecThreads) __attribute__((amdgpu_waves_per_eu(2, 2))) void spec_double_backward_lds_kernel(
    int K, int chblocks, int n_blocks, const TS* __restrict__ A, const T* __restrict__ W, const TS* __restrict__ dB,
    const TS* __restrict__ H, TS* __restrict__ ddB, TS* __restrict__ dA2, T* __restrict__ partial,
    const TileDesc* __restrict__ tiles, const int32_t* __restrict__ perm) {
  extern __shared__ unsigned char lds_raw[];
  T* red = reinterpret_cast<T*>(lds_raw);  // [kSpecWaves][kS][64]: every wave's w' columns
  T* acc_all = red + kSpecWaves * G::kS * kLanes;                         // [kSpecWaves][kS][64] dW2' sums
  T* stage = acc_all + kSpecWaves * G::kS * kLanes + wave_of_thread() * kLanes * G::kNlm;  // [64][kNlm] per wave
  static_assert(!kCM || std::is_same<T, TS>::value, "component-major rows are stored in the arithmetic type");
  const int lane = threadIdx.x & (kLanes - 1);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kLanes);
  const int logical = blockIdx.x;   // descriptors are stored largest tile first: dispatch order is the schedule
  if (logical >= n_blocks) return;  // uniform per workgroup
  const int tile = logical / chblocks, cb = logical % chblocks;
  const TileDesc td = tiles[tile];
  if (td.count == 0) return;        // unused descriptor; uniform per workgroup
  const int j0 = td.start + td.count * wave / kSpecWaves;
  const int j1 = td.start + td.count * (wave + 1) / kSpecWaves;
  const int live = kFull ? kLanes : (K - cb * kLanes < kLanes ? K - cb * kLanes : kLanes);   // channels of this block
  const int ch = kFull ? cb * kLanes + lane : cb * kLanes + (lane < live ? lane : live - 1);   // dead lanes repeat the last channel
  T* dwl = acc_all + wave * G::kS * kLanes + lane;
#pragma unroll
  for (int s = 0; s < G::kS; ++s) dwl[s * kLanes] = T(0);
  if (j0 < j1) {
    T* wl = red + wave * G::kS * kLanes + lane;   // this wave's slice of red holds w' until the end
    {
      T w0[G::kS];
      G::fold(W + static_cast<size_t>(td.z) * G::kP * K + ch, K, w0);
#pragma unroll
      for (int s = 0; s < G::kS; ++s) wl[s * kLanes] = w0[s];
    }
    // one register set of inputs: the next node's rows are requested right after the
    // arithmetic of the current one has consumed them, ahead of its stores
    T a[G::kNlm], h[G::kNlm], g[G::kNLM], da[G::kNlm], ddb[G::kNLM];
    size_t node = perm ? perm[j0] : j0;   // no permutation: the batch is already grouped
    NodeRows2<T, TS, G, kCM>::load(A, H, dB, node, K, ch, a, h, g);
    for (int j = j0; j < j1; ++j) {
      T w[G::kS];
      asm volatile("" ::: "memory");  // keep the reads of w' inside the loop (registers are short)
#pragma unroll
      for (int s = 0; s < G::kS; ++s) w[s] = wl[s * kLanes];
      T dw[G::kS];
#pragma unroll
      for (int s = 0; s < G::kS; ++s) dw[s] = T(0);
      G::double_backward(a, w, g, h, ddb, da, dw);
#pragma unroll
      for (int s = 0; s < G::kS; ++s) dwl[s * kLanes] += dw[s];
      const size_t cur = node;
      if (j + 1 < j1) {
        node = perm ? perm[j + 1] : j + 1;
        NodeRows2<T, TS, G, kCM>::load(A, H, dB, node, K, ch, a, h, g);
      }
      NodeRows2<T, TS, G, kCM>::template store<kFull>(dA2, ddB, cur, K, cb, ch, stage, lane, live, da, ddb);
    }
  }
  __syncthreads();
  T* out = partial + (static_cast<size_t>(td.id) * chblocks + cb) * G::kS * kLanes;   // rows in (element, position) order
  for (int i = threadIdx.x; i < G::kS * kLanes; i += kSpecThreads) {
    T acc = acc_all[i];
#pragma unroll
    for (int v = 1; v < kSpecWaves; ++v) acc += acc_all[v * G::kS * kLanes + i];
    out[i] = acc;
  }
}

template <typename T, typename G>
constexpr bool kUseLdsState = sizeof(T) == 4 && G::kS <= 32;

// Second stage of the dW reduction and the map to the external paths, one launch.  The fold
// matrix F (dW[p] = sum_s F[s,p] r[s]) falls into small independent blocks of one to three
// internal rows s and the external paths p that depend on them (generated descriptors), so one
// wave per (element, channel block, block of F) can do both steps without waiting for anyone:
// it adds the block's rows over the element's tiles in tile order, in fp64, with the rows of up
// to 32 tiles requested together (16 for two-row blocks), and writes the block's external paths.  Elements without nodes
// own no tiles and get zeros.  Every sum has a fixed order: results are bitwise reproducible.
// What was measured on the way here (10k / 200k nodes): a sum kernel followed by an unfold kernel
// 11.2 / 15.6 us; one workgroup per (element, channel block) for all rows 13.5 / 31 us (the twelve
// workgroups of the six frequent elements own 60% of the bytes); four waves per block, a quarter
// of the tiles each, combined through LDS 13 / 14.4 us (four times the waves, most of them idle
// for the rare elements).  A device-scope "last workgroup finishes the job" scheme inside the
// backward kernel was far slower than a launch: its fences flush the per-XCD L2s on this chip.
template <typename T, int R, int kMaxR>
__device__ __forceinline__ void finalize_sum(const T* __restrict__ src, size_t tstride, int t0, int t1,
                                             const int (&row)[kMaxR], double (&acc)[kMaxR]) {
  constexpr int kRegs = R * static_cast<int>(sizeof(T) / 4);   // registers per tile in flight
  constexpr int U = kRegs <= 1 ? 32 : kRegs <= 2 ? 16 : 8;   // (more in flight measured slower: fewer resident waves)
  // batches of U tiles; past the last tile it is read again and dropped
  for (int t = t0; t < t1; t += U) {
    T v[U][R];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const T* at = src + (t + u < t1 ? t + u : t1 - 1) * tstride;
#pragma unroll
      for (int r = 0; r < R; ++r) v[u][r] = at[row[r] * kLanes];
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const bool in = t + u < t1;
#pragma unroll
      for (int r = 0; r < R; ++r) acc[r] += in ? static_cast<double>(v[u][r]) : 0.0;
    }
  }
}

template <typename T, typename G>
__global__ __launch_bounds__(kLanes) void spec_finalize_kernel(int K, int chblocks, int max_tiles,
                                                               const T* __restrict__ partial,
                                                               const int32_t* __restrict__ tile_off,
                                                               T* __restrict__ dW) {
  constexpr int S = G::kS, R = G::kMaxBlockRows;
  const int lane = threadIdx.x;
  const int blk = blockIdx.x % G::kNumBlocks;
  const int cb = (blockIdx.x / G::kNumBlocks) % chblocks;
  const int e = blockIdx.x / (G::kNumBlocks * chblocks);
  const typename G::Block d = G::kBlocks[blk];   // the whole descriptor at once: one scalar-load latency
  int t0 = tile_off[e], t1 = tile_off[e + 1];
  if (t1 > max_tiles) t1 = max_tiles;
  const size_t tstride = static_cast<size_t>(chblocks) * S * kLanes;
  const T* src = partial + static_cast<size_t>(cb) * S * kLanes + lane;
  double sum[R];
#pragma unroll
  for (int r = 0; r < R; ++r) sum[r] = 0.0;
  if (d.n_rows == 1) finalize_sum<T, 1, R>(src, tstride, t0, t1, d.row, sum);
  else if (R >= 2 && d.n_rows == 2) finalize_sum<T, (R >= 2 ? 2 : 1), R>(src, tstride, t0, t1, d.row, sum);
  else finalize_sum<T, R, R>(src, tstride, t0, t1, d.row, sum);
  if (cb * kLanes + lane >= K) return;   // lanes past the last channel
  T* out = dW + static_cast<size_t>(e) * G::kP * K + cb * kLanes + lane;
#pragma unroll
  for (int i = 0; i < G::kMaxBlockPaths; ++i) {
    if (i < d.n_paths) {   // uniform
      double v = 0.0;
#pragma unroll
      for (int r = 0; r < R; ++r)
        if (d.coef[i][r] != 0.0) v += d.coef[i][r] * sum[r];   // uniform; rows in ascending order
      out[static_cast<size_t>(d.path[i]) * K] = static_cast<T>(v);
    }
  }
}

template <typename G>
bool matches(const sc_plan* plan) {
  const sc_config& c = plan->cfg;
  if (c.l_max != G::kLmax || c.nu_max != G::kNuMax || c.num_out != G::kNumOut) return false;
  for (int o = 0; o < G::kNumOut; ++o)
    if (c.out_l[o] != G::kOutL[o] || c.out_parity[o] != G::kOutParity[o]) return false;
  // the grouped kernels keep kS + kNlm columns per wave in LDS: 160 KB per compute unit at most
  // (the four-irrep kernel in fp64 would need 171 KB: the table-driven kernels serve that plan)
  const size_t lds = (c.dtype == SC_F64 ? 8 : 4) * static_cast<size_t>(kSpecWaves) * (G::kS + G::kNlm) * kLanes;
  if (lds > 160 * 1024) return false;
  // channel counts that are not a multiple of 64 leave lanes of the last channel block idle; a multiple
  // of four (eight for bfloat16 rows) keeps every row block 16-byte aligned
  return c.num_channels % (c.dtype == SC_BF16 ? 8 : 4) == 0 && static_cast<int>(plan->table.paths.size()) == G::kP;
}

SplitGroupArgs group_args(const sc_plan* plan, int64_t n, const int32_t* z, const Workspace& ws,
                          const LaunchShape& shape, bool window_order = false) {
  SplitGroupArgs g{};
  g.z = z;
  g.n = static_cast<int>(n);
  g.Z = plan->cfg.num_elements;
  g.W = shape.split_waves;
  g.nodes_per_wave = shape.split_nodes_per_wave;
  g.tile_nodes = shape.tile_nodes;
  g.max_tiles = shape.max_tiles;
  g.counts = ws.counts;
  g.seg_off = ws.seg_off;
  g.tile_off = ws.tile_off;
  g.ntiles = ws.ntiles;
  g.tiles = ws.tiles;
  g.perm = ws.perm;
  g.wnode = window_order ? ws.wnode : nullptr;
  g.wkey = window_order ? ws.wkey : nullptr;
  return g;
}

template <typename K>
hipError_t raise_lds_limit(K kernel, size_t lds) {
  if (lds <= 64 * 1024) return hipSuccess;  // above the default dynamic LDS limit: raise it for this kernel
  return hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                             static_cast<int>(lds));
}

template <typename T, typename G>
hipError_t prepare_launch(const sc_plan* plan, int64_t n, const int32_t* z, const void* W, const Workspace& ws,
                          const LaunchShape& shape, bool count, bool fold, bool window_order, hipStream_t stream) {
  const int count_wgs = count ? shape.split_waves / kGroupWavesPerWG : 0;
  const bool window = window_order && ws.wnode && ws.wkey;
  const int window_wgs = window ? static_cast<int>((n + kWindowNodes - 1) / kWindowNodes) : 0;
  const int n_pairs = fold ? plan->cfg.num_elements * shape.chblocks : 0;
  const int grid = window_wgs + count_wgs + (n_pairs + kSpecWaves - 1) / kSpecWaves;
  if (grid == 0) return hipSuccess;
  const size_t lds = window ? split_window_lds_bytes(plan->cfg.num_elements)
                            : count ? split_group_lds_bytes(plan->cfg.num_elements) : 0;
  hipLaunchKernelGGL((spec_prepare_kernel<T, G>), dim3(grid), dim3(kSpecThreads), lds, stream,
                     group_args(plan, n, z, ws, shape, window), count_wgs, window_wgs, plan->cfg.num_channels, shape.chblocks, n_pairs,
                     static_cast<const T*>(W), static_cast<T*>(ws.wfold));
  return hipGetLastError();
}

// Nodes per workgroup of the natural-order forward.  All workgroups do the same work, so the
// kernel takes (rounds of resident workgroups) x (nodes per wave): the tile is the multiple of
// four nodes in 8..32 (8..64 for the larger bases) that minimises that product for this batch on this chip (10k nodes, 128
// channels, four workgroups per CU: 20 nodes = one round of five nodes per wave instead of two
// rounds of four with 16); among sizes within 2% of the best the largest up to `most` wins, since
// longer shares per wave meet more runs of one element (measured best at 200k nodes before the
// window order: 24..32 nodes with the 29-row basis, 48 with the 49-row basis, whose weights cost
// more to re-read).  From eight rounds on the rounds no longer tell (workgroups are replaced as
// they end) and, with the window order making the runs long whatever the share, the small bases
// do best with five nodes per wave: 200k nodes, 29-row basis, forward 373 us with 20 nodes per
// workgroup against 376 (16), 381 (24), 387 (28), 391 (32); the 49-row basis shows no preference
// between 20 and 48 (268 us at 50k nodes, 256 channels) and keeps the rule above.
inline int forward_tile_nodes(int64_t n, int chblocks, int64_t resident_wgs, int most) {
  auto cost = [&](int t) {
    const int64_t wgs = (n + t - 1) / t * chblocks;
    return static_cast<double>((wgs + resident_wgs - 1) / resident_wgs) * (t / kSpecWaves);
  };
  if (most <= 32 && (n + 19) / 20 * chblocks >= 8 * resident_wgs) return 20;
  double best = cost(8);
  for (int t = 12; t <= most; t += 4) best = cost(t) < best ? cost(t) : best;
  int pick = 8;
  for (int t = 8; t <= most; t += 4)
    if (cost(t) <= best * 1.02) pick = t;
  return pick;
}

template <typename T, typename G, typename TS, bool kCM = false>
hipError_t fwd_launch(const sc_plan* plan, int64_t n, const void* A, const int32_t* z, void* B, const Workspace& ws,
                      const LaunchShape& shape, int group, bool window_order, hipStream_t stream) {
  // group: 0 no grouping roles, 1 scatter + table, 2 table only (the batch is already grouped)
  const bool scatter = group == 1;
  const int table = group != 0;
  const int scatter_wgs = scatter ? shape.split_waves / kGroupWavesPerWG : 0;
  size_t lds = (G::kNLM * sizeof(TS) != 16) ? sizeof(T) * kSpecWaves * G::kNLM * kLanes : 0;
  if (table && split_group_lds_bytes(plan->cfg.num_elements) > lds) lds = split_group_lds_bytes(plan->cfg.num_elements);
  static const int wgs_per_cu = [] {   // resident workgroups per compute unit of this instance
    int nb = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, spec_forward_kernel<T, G, TS, kCM>, kSpecThreads, 0) != hipSuccess || nb < 1)
      nb = 1;
    return nb;
  }();
  const int tile = shape.fwd_tile_nodes > 0 ? shape.fwd_tile_nodes
                                            : forward_tile_nodes(n, shape.chblocks, static_cast<int64_t>(wgs_per_cu) * plan->num_cus,
                                                                 G::kS > 32 ? 64 : 32);
  const int tiles = static_cast<int>((n + tile - 1) / tile);
  const int grid = scatter_wgs + table + tiles * shape.chblocks;
  hipLaunchKernelGGL((spec_forward_kernel<T, G, TS, kCM>), dim3(grid), dim3(kSpecThreads), lds, stream,
                     group_args(plan, n, z, ws, shape, window_order), scatter_wgs, table, plan->cfg.num_channels, shape.chblocks,
                     static_cast<int>(n), plan->cfg.num_elements, tile, static_cast<const TS*>(A), z,
                     static_cast<const T*>(ws.wfold), static_cast<TS*>(B));
  return hipGetLastError();
}

template <typename T, typename G, typename TS, bool kCM = false>
hipError_t bwd_launch(const sc_plan* plan, int64_t n, const void* A, const void* dB, void* dA,
                      const Workspace& ws, const LaunchShape& shape, hipStream_t stream) {   // ws.perm may be null
  const int n_blocks = shape.max_tiles * shape.chblocks;
  const int grid = (n_blocks + kXcds - 1) / kXcds * kXcds;
  const size_t lds = sizeof(T) * kSpecWaves * (G::kS + G::kNlm) * kLanes;
  const bool full = plan->cfg.num_channels % kLanes == 0;
  auto kernel = full ? &spec_backward_kernel<T, G, 0, false, true, TS, kCM> : &spec_backward_kernel<T, G, 0, false, false, TS, kCM>;
  if constexpr (sizeof(T) == 4) {
    // small batches: dA streamed past the cache (see the kernel)
    if (n <= 40000 && full) kernel = &spec_backward_kernel<T, G, 0, true, true, TS, kCM>;
  }
  const hipError_t e = raise_lds_limit(kernel, lds);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(kernel, dim3(grid), dim3(kSpecThreads), lds, stream, plan->cfg.num_channels, shape.chblocks,
                     n_blocks, static_cast<const TS*>(A), static_cast<const T*>(ws.wfold), static_cast<const TS*>(dB),
                     static_cast<TS*>(dA), static_cast<T*>(ws.partial), ws.tiles, ws.perm);
  return hipGetLastError();
}

template <typename T, typename G, typename TS, bool kCM = false>
hipError_t dbl_launch(const sc_plan* plan, const void* A, const void* W, const void* dB, const void* H, void* ddB,
                      void* dA2, const Workspace& ws, const LaunchShape& shape, hipStream_t stream) {
  const int n_blocks = shape.max_tiles * shape.chblocks;
  const int grid = (n_blocks + kXcds - 1) / kXcds * kXcds;
  constexpr bool kLds = kUseLdsState<T, G>;
  const size_t lds = sizeof(T) * kSpecWaves * ((kLds ? 2 : 1) * G::kS + G::kNlm) * kLanes;
  const bool full = plan->cfg.num_channels % kLanes == 0;   // no idle lanes: an instance without their handling
  auto kernel = full ? &spec_double_backward_kernel<T, G, true, TS, kCM> : &spec_double_backward_kernel<T, G, false, TS, kCM>;
  if constexpr (kLds) kernel = full ? &spec_double_backward_lds_kernel<T, G, true, TS, kCM> : &spec_double_backward_lds_kernel<T, G, false, TS, kCM>;
  const hipError_t e = raise_lds_limit(kernel, lds);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(kernel, dim3(grid), dim3(kSpecThreads), lds, stream, plan->cfg.num_channels, shape.chblocks,
                     n_blocks, static_cast<const TS*>(A), static_cast<const T*>(W), static_cast<const TS*>(dB),
                     static_cast<const TS*>(H), static_cast<TS*>(ddB), static_cast<TS*>(dA2),
                     static_cast<T*>(ws.partial), ws.tiles, ws.perm);
  return hipGetLastError();
}

template <typename T, typename G>
hipError_t finalize_launch(const sc_plan* plan, void* dW, const Workspace& ws, const LaunchShape& shape,
                           hipStream_t stream) {
  const int Z = plan->cfg.num_elements;
  hipLaunchKernelGGL((spec_finalize_kernel<T, G>), dim3(Z * shape.chblocks * G::kNumBlocks), dim3(kLanes), 0, stream,
                     plan->cfg.num_channels, shape.chblocks, shape.max_tiles, static_cast<const T*>(ws.partial),
                     ws.tile_off, static_cast<T*>(dW));
  return hipGetLastError();
}

// Calls fn.template operator()<T, G, TS>() for the plan's dtype (T arithmetic and weights, TS
// storage of the per-node rows) and generated kernel.
template <typename G, typename F>
hipError_t dispatch_dtype(const sc_plan* plan, F&& fn) {
  switch (plan->cfg.dtype) {
    case SC_F64: return fn.template operator()<double, G, double>();
    case SC_BF16: return fn.template operator()<float, G, bf16_bits>();
    default: return fn.template operator()<float, G, float>();
  }
}

template <typename F>
hipError_t dispatch(const sc_plan* plan, F&& fn) {
  switch (plan->specialised) {
    case 1: return dispatch_dtype<Gen_l3n3_0e1o>(plan, fn);
    case 2: return dispatch_dtype<Gen_l3n3_0e1o2e>(plan, fn);
    case 3: return dispatch_dtype<Gen_l3n3_0e1o2e3o>(plan, fn);
    case 4: return dispatch_dtype<Gen_l1n2_0e>(plan, fn);
    case 5: return dispatch_dtype<Gen_l3n3_0e>(plan, fn);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace

int spec_lookup(const sc_plan* plan) {
  if (matches<Gen_l3n3_0e1o>(plan)) return 1;
  if (matches<Gen_l3n3_0e1o2e>(plan)) return 2;
  if (matches<Gen_l3n3_0e1o2e3o>(plan)) return 3;
  if (matches<Gen_l1n2_0e>(plan)) return 4;
  if (matches<Gen_l3n3_0e>(plan)) return 5;
  return 0;
}

int spec_basis_size(int id) {
  return id == 1 ? Gen_l3n3_0e1o::kS : id == 2 ? Gen_l3n3_0e1o2e::kS : id == 3 ? Gen_l3n3_0e1o2e3o::kS : id == 4 ? Gen_l1n2_0e::kS : id == 5 ? Gen_l3n3_0e::kS : 0;
}

template <typename G>
void op_counts(int32_t ops[3], int32_t flops[3]) {
  for (int i = 0; i < 3; ++i) {
    ops[i] = G::kOps[i];
    flops[i] = G::kFlops[i];
  }
}

void spec_op_counts(int id, int32_t ops[3], int32_t flops[3]) {
  for (int i = 0; i < 3; ++i) ops[i] = flops[i] = 0;
  if (id == 1) op_counts<Gen_l3n3_0e1o>(ops, flops);
  if (id == 2) op_counts<Gen_l3n3_0e1o2e>(ops, flops);
  if (id == 3) op_counts<Gen_l3n3_0e1o2e3o>(ops, flops);
  if (id == 4) op_counts<Gen_l1n2_0e>(ops, flops);
  if (id == 5) op_counts<Gen_l3n3_0e>(ops, flops);
}

int spec_waves_per_tile() { return kSpecWaves; }

size_t spec_folded_bytes(const sc_plan* plan) {
  const size_t chblocks = (plan->cfg.num_channels + kLanes - 1) / kLanes;   // whole 64-channel rows
  return static_cast<size_t>(plan->cfg.num_elements) * chblocks * kLanes * spec_basis_size(plan->specialised) *
         (plan->cfg.dtype == SC_F64 ? 8 : 4);   // weights: fp32 also for bfloat16 rows
}

struct PrepareFn {
  const sc_plan* plan; int64_t n; const int32_t* z; const void* W; const Workspace& ws; const LaunchShape& shape;
  bool count, fold, window_order; hipStream_t stream;
  template <typename T, typename G, typename TS> hipError_t operator()() const { return prepare_launch<T, G>(plan, n, z, W, ws, shape, count, fold, window_order, stream); }
};
struct ForwardFn {
  const sc_plan* plan; int64_t n; const void* A; const int32_t* z; void* B; const Workspace& ws; const LaunchShape& shape;
  int group; bool window_order, component_major; hipStream_t stream;
  template <typename T, typename G, typename TS> hipError_t operator()() const {
    if constexpr (std::is_same<T, TS>::value) {
      if (component_major) return fwd_launch<T, G, TS, true>(plan, n, A, z, B, ws, shape, group, window_order, stream);
    } else if (component_major) {
      return hipErrorInvalidValue;   // refused by the caller: rows stored in another type have no such kernel
    }
    return fwd_launch<T, G, TS>(plan, n, A, z, B, ws, shape, group, window_order, stream);
  }
};
struct BackwardFn {
  const sc_plan* plan; int64_t n; const void* A; const void* dB; void* dA; const Workspace& ws; const LaunchShape& shape;
  bool component_major; hipStream_t stream;
  template <typename T, typename G, typename TS> hipError_t operator()() const {
    if constexpr (std::is_same<T, TS>::value) {
      if (component_major) return bwd_launch<T, G, TS, true>(plan, n, A, dB, dA, ws, shape, stream);
    } else if (component_major) {
      return hipErrorInvalidValue;
    }
    return bwd_launch<T, G, TS>(plan, n, A, dB, dA, ws, shape, stream);
  }
};
struct DoubleBackwardFn {
  const sc_plan* plan; const void* A; const void* W; const void* dB; const void* H; void* ddB; void* dA2; const Workspace& ws;
  const LaunchShape& shape; bool component_major; hipStream_t stream;
  template <typename T, typename G, typename TS> hipError_t operator()() const {
    if constexpr (std::is_same<T, TS>::value) {
      if (component_major) return dbl_launch<T, G, TS, true>(plan, A, W, dB, H, ddB, dA2, ws, shape, stream);
    } else if (component_major) {
      return hipErrorInvalidValue;
    }
    return dbl_launch<T, G, TS>(plan, A, W, dB, H, ddB, dA2, ws, shape, stream);
  }
};
struct FinalizeFn {
  const sc_plan* plan; void* dW; const Workspace& ws; const LaunchShape& shape; hipStream_t stream;
  template <typename T, typename G, typename TS> hipError_t operator()() const { return finalize_launch<T, G>(plan, dW, ws, shape, stream); }
};

hipError_t launch_spec_prepare(const sc_plan* plan, int64_t n, const int32_t* z, const void* W, const Workspace& ws,
                               const LaunchShape& shape, bool count, bool fold, bool window_order, hipStream_t stream) {
  return dispatch(plan, PrepareFn{plan, n, z, W, ws, shape, count, fold, window_order, stream});
}

hipError_t launch_spec_scatter(const sc_plan* plan, int64_t n, const int32_t* z, const Workspace& ws,
                               const LaunchShape& shape, bool table_only, hipStream_t stream) {
  const int scatter_wgs = table_only ? 0 : shape.split_waves / kGroupWavesPerWG;
  hipLaunchKernelGGL(spec_scatter_kernel, dim3(scatter_wgs + 1), dim3(kSpecThreads),
                     split_group_lds_bytes(plan->cfg.num_elements), stream, group_args(plan, n, z, ws, shape), scatter_wgs);
  return hipGetLastError();
}

hipError_t launch_spec_forward(const sc_plan* plan, int64_t n, const void* A, const int32_t* z, void* B,
                               const Workspace& ws, const LaunchShape& shape, int group, bool window_order,
                               bool component_major, hipStream_t stream) {
  return dispatch(plan, ForwardFn{plan, n, A, z, B, ws, shape, group, window_order && ws.wnode && ws.wkey, component_major, stream});
}

hipError_t launch_spec_backward(const sc_plan* plan, int64_t n, const void* A, const void* dB, void* dA,
                                const Workspace& ws, const LaunchShape& shape, bool component_major,
                                hipStream_t stream) {
  return dispatch(plan, BackwardFn{plan, n, A, dB, dA, ws, shape, component_major, stream});
}

hipError_t launch_spec_double_backward(const sc_plan* plan, int64_t, const void* A, const void* W, const void* dB,
                                       const void* H, void* ddB, void* dA2, const Workspace& ws,
                                       const LaunchShape& shape, bool component_major, hipStream_t stream) {
  return dispatch(plan, DoubleBackwardFn{plan, A, W, dB, H, ddB, dA2, ws, shape, component_major, stream});
}

hipError_t launch_spec_finalize(const sc_plan* plan, void* dW, const Workspace& ws, const LaunchShape& shape,
                                hipStream_t stream) {
  return dispatch(plan, FinalizeFn{plan, dW, ws, shape, stream});
}

}  // namespace sc
