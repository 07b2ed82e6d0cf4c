// Specialised kernels: hand-written memory / scheduling skeleton around generated
// straight-line arithmetic (csrc/generated/*.inc, written by codegen/generate.py).
//
// Mapping (Algorithm 2 of arXiv 2504.10700 is independent per atom and channel):
//   lane      = channel (64 consecutive channels per wave: the A row of a node is read as
//               64 B per lane, a wave covers 4 KB of contiguous HBM; B/dB rows are 16 B per lane)
//   wave      = a run of nodes of ONE element (weights folded once into registers)
//   workgroup = 4 waves = one tile of the grouping pass x one 64-channel block; its waves
//               add their dW' rows through LDS, so one partial row set leaves per tile
//   grid      = tiles x channel blocks, remapped so that each XCD (own L2) gets a contiguous
//               range of tiles: neighbouring tiles share the element's weights
// Per node the next node's rows are requested before the current one is evaluated
// (two register sets, ping-pong), so HBM latency hides behind ~300-800 VALU operations.
#include "sc_spec.h"

namespace sc {
namespace {

__device__ __forceinline__ float sc_fma(float x, float y, float z) { return __builtin_fmaf(x, y, z); }
__device__ __forceinline__ double sc_fma(double x, double y, double z) { return __builtin_fma(x, y, z); }

#include "generated/sc_gen_l3n3_0e1o.inc"
#include "generated/sc_gen_l3n3_0e1o2e.inc"

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
// of LDS owned by this wave; block: where lane 0's row goes (16-byte aligned).
// kStream: non-temporal stores (the rows are not read again soon and each instruction writes
// whole lines).  Measured on one box, library against library: forward 28.4 -> 27.0 us at 10k
// nodes (neutral at 200k), second-order kernel 78.7 -> 77.5 us; a wash for the backward's dA
// at 10k nodes and 1% slower at 200k, so the backward leaves it off.
template <typename T, int N, bool kStream = true>
__device__ __forceinline__ void store_rows_coalesced(T* __restrict__ block, T* stage, int lane, const T (&v)[N]) {
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
  constexpr int kPieces = kLanes * N / V;  // 16-byte pieces of the block (64*N is a multiple of V)
#pragma unroll
  for (int q0 = 0; q0 < kPieces; q0 += kLanes) {
    const int q = q0 + lane;
    if (q0 + kLanes <= kPieces || q < kPieces) {
      const Vec x = *reinterpret_cast<const Vec*>(stage + q * V);
      if constexpr (kStream) __builtin_nontemporal_store(x, reinterpret_cast<Vec*>(block + q * V));
      else *reinterpret_cast<Vec*>(block + q * V) = x;
    }
  }
}

// blockIdx -> logical work item such that the blocks an XCD receives (round-robin by
// blockIdx) form one contiguous range.  gridDim.x is a multiple of kXcds.
__device__ __forceinline__ int xcd_contiguous_block() {
  const int per = gridDim.x / kXcds;
  return (blockIdx.x % kXcds) * per + blockIdx.x / kXcds;
}

template <typename T, typename G>
__global__ __launch_bounds__(kSpecThreads) void spec_forward_kernel(int K, int chblocks, int n_blocks,
                                                                    const T* __restrict__ A,
                                                                    const T* __restrict__ W, T* __restrict__ B,
                                                                    const TileDesc* __restrict__ tiles,
                                                                    const int32_t* __restrict__ perm) {
  extern __shared__ unsigned char lds_raw[];
  const int lane = threadIdx.x & (kLanes - 1);
  const int wave = wave_of_thread();
  T* stage = reinterpret_cast<T*>(lds_raw) + wave * kLanes * G::kNLM;  // [64][kNLM] per wave (if used)
  constexpr bool kStageB = G::kNLM * sizeof(T) != 16;  // 16-byte rows are coalesced as they are
  const int logical = xcd_contiguous_block();
  if (logical >= n_blocks) return;
  const int tile = logical / chblocks, cb = logical % chblocks;
  const TileDesc td = tiles[tile];
  const int j0 = td.start + td.count * wave / kSpecWaves;
  const int j1 = td.start + td.count * (wave + 1) / kSpecWaves;
  if (j0 >= j1) return;  // also covers the unused descriptors (count 0)
  const int ch = cb * kLanes + lane;
  T w[G::kS];
  G::fold(W + static_cast<size_t>(td.z) * G::kP * K + ch, K, w);

  T a0[G::kNlm], a1[G::kNlm], b[G::kNLM];
  size_t node0 = perm[j0], node1 = 0;
  Row<T, G::kNlm>::load(A + (node0 * K + ch) * G::kNlm, a0);
  for (int j = j0; j < j1; j += 2) {
    if (j + 1 < j1) {
      node1 = perm[j + 1];
      Row<T, G::kNlm>::load(A + (node1 * K + ch) * G::kNlm, a1);
    }
    G::forward(a0, w, b);
    if constexpr (kStageB) store_rows_coalesced<T, G::kNLM>(B + (node0 * K + cb * kLanes) * G::kNLM, stage, lane, b);
    else Row<T, G::kNLM>::store(B + (node0 * K + ch) * G::kNLM, b);
    if (j + 1 < j1) {
      if (j + 2 < j1) {
        node0 = perm[j + 2];
        Row<T, G::kNlm>::load(A + (node0 * K + ch) * G::kNlm, a0);
      }
      G::forward(a1, w, b);
      if constexpr (kStageB) store_rows_coalesced<T, G::kNLM>(B + (node1 * K + cb * kLanes) * G::kNLM, stage, lane, b);
      else Row<T, G::kNLM>::store(B + (node1 * K + ch) * G::kNLM, b);
    }
  }
}

// kOcc = waves per SIMD the kernel is held to (0: the compiler's choice).  The fp32 kernel of the
// small basis needs 171 registers if left alone, three over the limit for three waves per SIMD;
// held to 168 (two values go to scratch) it runs three workgroups per CU instead of two.  On a
// small batch a workgroup's life is a chain of latencies (fold, first rows, a handful of nodes,
// the dW sum) and the third workgroup pays: 51.1 -> 49.3 us at 10k nodes, 138.7 -> 136.6 at
// 30k, measured on one box; from 60k nodes on the unconstrained kernel is 1% faster.
template <typename T, typename G, int kOcc = 0>
__global__ __launch_bounds__(kSpecThreads) __attribute__((amdgpu_waves_per_eu(kOcc == 0 ? 1 : kOcc, 8)))
void spec_backward_kernel(int K, int chblocks, int n_blocks,
                                                                     const T* __restrict__ A,
                                                                     const T* __restrict__ W,
                                                                     const T* __restrict__ dB, T* __restrict__ dA,
                                                                     T* __restrict__ partial,
                                                                     const TileDesc* __restrict__ tiles,
                                                                     const int32_t* __restrict__ perm) {
  extern __shared__ unsigned char lds_raw[];
  T* red = reinterpret_cast<T*>(lds_raw);  // [kSpecWaves][kS][64]
  T* stage = red + kSpecWaves * G::kS * kLanes + wave_of_thread() * kLanes * G::kNlm;  // [64][kNlm] per wave
  const int lane = threadIdx.x & (kLanes - 1);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kLanes);
  const int logical = xcd_contiguous_block();
  if (logical >= n_blocks) return;  // uniform per workgroup
  const int tile = logical / chblocks, cb = logical % chblocks;
  const TileDesc td = tiles[tile];
  if (td.count == 0) return;        // unused descriptor; uniform per workgroup
  const int j0 = td.start + td.count * wave / kSpecWaves;
  const int j1 = td.start + td.count * (wave + 1) / kSpecWaves;
  const int ch = cb * kLanes + lane;
  T dw[G::kS];
#pragma unroll
  for (int s = 0; s < G::kS; ++s) dw[s] = T(0);
  if (j0 < j1) {
    T w[G::kS];
    G::fold(W + static_cast<size_t>(td.z) * G::kP * K + ch, K, w);
    T a0[G::kNlm], a1[G::kNlm], g0[G::kNLM], g1[G::kNLM], da[G::kNlm];
    size_t node0 = perm[j0], node1 = 0;
    Row<T, G::kNlm>::load(A + (node0 * K + ch) * G::kNlm, a0);
    Row<T, G::kNLM>::load(dB + (node0 * K + ch) * G::kNLM, g0);
    for (int j = j0; j < j1; j += 2) {
      if (j + 1 < j1) {
        node1 = perm[j + 1];
        Row<T, G::kNlm>::load(A + (node1 * K + ch) * G::kNlm, a1);
        Row<T, G::kNLM>::load(dB + (node1 * K + ch) * G::kNLM, g1);
      }
      G::backward(a0, w, g0, da, dw);
      store_rows_coalesced<T, G::kNlm, false>(dA + (node0 * K + cb * kLanes) * G::kNlm, stage, lane, da);
      if (j + 1 < j1) {
        if (j + 2 < j1) {
          node0 = perm[j + 2];
          Row<T, G::kNlm>::load(A + (node0 * K + ch) * G::kNlm, a0);
          Row<T, G::kNLM>::load(dB + (node0 * K + ch) * G::kNLM, g0);
        }
        G::backward(a1, w, g1, da, dw);
        store_rows_coalesced<T, G::kNlm, false>(dA + (node1 * K + cb * kLanes) * G::kNlm, stage, lane, da);
      }
    }
  }
  // sum the waves' dW' rows in wave order and write the tile's partial rows
#pragma unroll
  for (int s = 0; s < G::kS; ++s) red[(wave * G::kS + s) * kLanes + lane] = dw[s];
  __syncthreads();
  T* out = partial + (static_cast<size_t>(tile) * chblocks + cb) * G::kS * kLanes;
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
template <typename T, typename G>
__global__ __launch_bounds__(kSpecThreads) void spec_double_backward_kernel(
    int K, int chblocks, int n_blocks, const T* __restrict__ A, const T* __restrict__ W, const T* __restrict__ dB,
    const T* __restrict__ H, T* __restrict__ ddB, T* __restrict__ dA2, T* __restrict__ partial,
    const TileDesc* __restrict__ tiles, const int32_t* __restrict__ perm) {
  extern __shared__ unsigned char lds_raw[];
  T* red = reinterpret_cast<T*>(lds_raw);  // [kSpecWaves][kS][64]
  T* stage = red + kSpecWaves * G::kS * kLanes + wave_of_thread() * kLanes * G::kNlm;  // [64][kNlm] per wave
  constexpr bool kStageB = G::kNLM * sizeof(T) != 16;
  const int lane = threadIdx.x & (kLanes - 1);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kLanes);
  const int logical = xcd_contiguous_block();
  if (logical >= n_blocks) return;  // uniform per workgroup
  const int tile = logical / chblocks, cb = logical % chblocks;
  const TileDesc td = tiles[tile];
  if (td.count == 0) return;        // unused descriptor; uniform per workgroup
  const int j0 = td.start + td.count * wave / kSpecWaves;
  const int j1 = td.start + td.count * (wave + 1) / kSpecWaves;
  const int ch = cb * kLanes + lane;
  T dw[G::kS];
#pragma unroll
  for (int s = 0; s < G::kS; ++s) dw[s] = T(0);
  if (j0 < j1) {
    T w[G::kS];
    G::fold(W + static_cast<size_t>(td.z) * G::kP * K + ch, K, w);
    // one register set of inputs: the next node's rows are requested right after the
    // arithmetic of the current one has consumed them, ahead of its stores
    T a[G::kNlm], h[G::kNlm], g[G::kNLM], da[G::kNlm], ddb[G::kNLM];
    size_t node = perm[j0];
    Row<T, G::kNlm>::load(A + (node * K + ch) * G::kNlm, a);
    Row<T, G::kNlm>::load(H + (node * K + ch) * G::kNlm, h);
    Row<T, G::kNLM>::load(dB + (node * K + ch) * G::kNLM, g);
    for (int j = j0; j < j1; ++j) {
      G::double_backward(a, w, g, h, ddb, da, dw);
      const size_t cur = node;
      if (j + 1 < j1) {
        node = perm[j + 1];
        Row<T, G::kNlm>::load(A + (node * K + ch) * G::kNlm, a);
        Row<T, G::kNlm>::load(H + (node * K + ch) * G::kNlm, h);
        Row<T, G::kNLM>::load(dB + (node * K + ch) * G::kNLM, g);
      }
      store_rows_coalesced<T, G::kNlm>(dA2 + (cur * K + cb * kLanes) * G::kNlm, stage, lane, da);
      if constexpr (kStageB) store_rows_coalesced<T, G::kNLM>(ddB + (cur * K + cb * kLanes) * G::kNLM, stage, lane, ddb);
      else Row<T, G::kNLM>::store(ddB + (cur * K + ch) * G::kNLM, ddb);
    }
  }
#pragma unroll
  for (int s = 0; s < G::kS; ++s) red[(wave * G::kS + s) * kLanes + lane] = dw[s];
  __syncthreads();
  T* out = partial + (static_cast<size_t>(tile) * chblocks + cb) * G::kS * kLanes;
  for (int i = threadIdx.x; i < G::kS * kLanes; i += kSpecThreads) {
    T acc = red[i];
#pragma unroll
    for (int v = 1; v < kSpecWaves; ++v) acc += red[v * G::kS * kLanes + i];
    out[i] = acc;
  }
}

// See above.  LDS: w' [kSpecWaves][kS][64] | sums [kSpecWaves][kS][64] | stage [kSpecWaves][64][kNlm].
template <typename T, typename G>
__global__ __launch_bounds__(kSpecThreads) __attribute__((amdgpu_waves_per_eu(2, 2))) void spec_double_backward_lds_kernel(
    int K, int chblocks, int n_blocks, const T* __restrict__ A, const T* __restrict__ W, const T* __restrict__ dB,
    const T* __restrict__ H, T* __restrict__ ddB, T* __restrict__ dA2, T* __restrict__ partial,
    const TileDesc* __restrict__ tiles, const int32_t* __restrict__ perm) {
  extern __shared__ unsigned char lds_raw[];
  T* red = reinterpret_cast<T*>(lds_raw);  // [kSpecWaves][kS][64]: every wave's w' columns
  T* acc_all = red + kSpecWaves * G::kS * kLanes;                         // [kSpecWaves][kS][64] dW2' sums
  T* stage = acc_all + kSpecWaves * G::kS * kLanes + wave_of_thread() * kLanes * G::kNlm;  // [64][kNlm] per wave
  constexpr bool kStageB = G::kNLM * sizeof(T) != 16;
  const int lane = threadIdx.x & (kLanes - 1);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kLanes);
  const int logical = xcd_contiguous_block();
  if (logical >= n_blocks) return;  // uniform per workgroup
  const int tile = logical / chblocks, cb = logical % chblocks;
  const TileDesc td = tiles[tile];
  if (td.count == 0) return;        // unused descriptor; uniform per workgroup
  const int j0 = td.start + td.count * wave / kSpecWaves;
  const int j1 = td.start + td.count * (wave + 1) / kSpecWaves;
  const int ch = cb * kLanes + lane;
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
    size_t node = perm[j0];
    Row<T, G::kNlm>::load(A + (node * K + ch) * G::kNlm, a);
    Row<T, G::kNlm>::load(H + (node * K + ch) * G::kNlm, h);
    Row<T, G::kNLM>::load(dB + (node * K + ch) * G::kNLM, g);
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
        node = perm[j + 1];
        Row<T, G::kNlm>::load(A + (node * K + ch) * G::kNlm, a);
        Row<T, G::kNlm>::load(H + (node * K + ch) * G::kNlm, h);
        Row<T, G::kNLM>::load(dB + (node * K + ch) * G::kNLM, g);
      }
      store_rows_coalesced<T, G::kNlm>(dA2 + (cur * K + cb * kLanes) * G::kNlm, stage, lane, da);
      if constexpr (kStageB) store_rows_coalesced<T, G::kNLM>(ddB + (cur * K + cb * kLanes) * G::kNLM, stage, lane, ddb);
      else Row<T, G::kNLM>::store(ddB + (cur * K + ch) * G::kNLM, ddb);
    }
  }
  __syncthreads();
  T* out = partial + (static_cast<size_t>(tile) * chblocks + cb) * G::kS * kLanes;
  for (int i = threadIdx.x; i < G::kS * kLanes; i += kSpecThreads) {
    T acc = acc_all[i];
#pragma unroll
    for (int v = 1; v < kSpecWaves; ++v) acc += acc_all[v * G::kS * kLanes + i];
    out[i] = acc;
  }
}

template <typename T, typename G>
constexpr bool kUseLdsState = sizeof(T) == 4 && G::kS <= 32;

// Second stage of the dW reduction, two small launches (device-scope fences, which a
// single-launch "last wave finishes the job" scheme needs, flush the per-XCD L2s and cost
// far more than a launch on this chip).
// (1) One workgroup of four waves per (element, channel block, internal row): each wave sums
//     the row over a contiguous quarter of the element's tiles in tile order (sixteen
//     independent loads in flight), the four sums are added in wave order into
//     reduced[e][cb][s][lane] in fp64.  Elements without nodes own no tiles and get zeros.
// (2) One wave per (element, channel block): maps the S reduced rows to the P external
//     paths with the generated unfold.
// Every sum has a fixed order: results are bitwise reproducible.
constexpr int kReduceWaves = 4;

template <typename T, typename G>
__global__ __launch_bounds__(kReduceWaves * kLanes) void spec_reduce_kernel(int chblocks, int max_tiles,
                                                                            const T* __restrict__ partial,
                                                                            const int32_t* __restrict__ tile_off,
                                                                            double* __restrict__ reduced) {
  constexpr int S = G::kS;
  __shared__ double part[kReduceWaves][kLanes];
  const int lane = threadIdx.x % kLanes, wave = threadIdx.x / kLanes;
  const int s = blockIdx.x % S;
  const int cb = (blockIdx.x / S) % chblocks;
  const int e = blockIdx.x / (S * chblocks);
  int t0 = tile_off[e], t1 = tile_off[e + 1];
  if (t1 > max_tiles) t1 = max_tiles;
  // the element's tiles are cut into kReduceWaves contiguous ranges, one per wave
  const int nt = t1 - t0;
  const int w0 = t0 + nt * wave / kReduceWaves, w1 = t0 + nt * (wave + 1) / kReduceWaves;
  const size_t tstride = static_cast<size_t>(chblocks) * S * kLanes;
  const T* src = partial + (static_cast<size_t>(cb) * S + s) * kLanes + lane;
  constexpr int U = 16;
  double a[U];
#pragma unroll
  for (int k = 0; k < U; ++k) a[k] = 0.0;
  int t = w0;
  for (; t + U <= w1; t += U) {
    T v[U];
#pragma unroll
    for (int k = 0; k < U; ++k) v[k] = src[(t + k) * tstride];
#pragma unroll
    for (int k = 0; k < U; ++k) a[k] += static_cast<double>(v[k]);
  }
  for (; t < w1; ++t) a[0] += static_cast<double>(src[t * tstride]);
#pragma unroll
  for (int w = U / 2; w >= 1; w /= 2)
#pragma unroll
    for (int k = 0; k < w; ++k) a[k] += a[k + w];
  part[wave][lane] = a[0];
  __syncthreads();
  if (wave == 0) {
    double sum = part[0][lane];
#pragma unroll
    for (int w = 1; w < kReduceWaves; ++w) sum += part[w][lane];
    reduced[((static_cast<size_t>(e) * chblocks + cb) * S + s) * kLanes + lane] = sum;
  }
}

template <typename T, typename G>
__global__ __launch_bounds__(kLanes) void spec_unfold_kernel(int K, int chblocks,
                                                             const double* __restrict__ reduced,
                                                             T* __restrict__ dW) {
  constexpr int S = G::kS;
  const int lane = threadIdx.x;
  const int cb = blockIdx.x % chblocks;
  const int e = blockIdx.x / chblocks;
  const double* mine = reduced + (static_cast<size_t>(e) * chblocks + cb) * S * kLanes;
  double r[S];
#pragma unroll
  for (int q = 0; q < S; ++q) r[q] = mine[q * kLanes + lane];
  G::unfold(r, dW + static_cast<size_t>(e) * G::kP * K + cb * kLanes + lane, K);
}

template <typename G>
bool matches(const sc_plan* plan) {
  const sc_config& c = plan->cfg;
  if (c.l_max != G::kLmax || c.nu_max != G::kNuMax || c.num_out != G::kNumOut) return false;
  for (int o = 0; o < G::kNumOut; ++o)
    if (c.out_l[o] != G::kOutL[o] || c.out_parity[o] != G::kOutParity[o]) return false;
  return c.num_channels % kLanes == 0 && static_cast<int>(plan->table.paths.size()) == G::kP;
}

template <typename T, typename G>
hipError_t fwd_launch(const sc_plan* plan, const void* A, const void* W, void* B, const Workspace& ws,
                      const LaunchShape& shape, hipStream_t stream) {
  const int n_blocks = shape.max_tiles * shape.chblocks;
  const int grid = (n_blocks + kXcds - 1) / kXcds * kXcds;
  const size_t lds = (G::kNLM * sizeof(T) != 16) ? sizeof(T) * kSpecWaves * G::kNLM * kLanes : 0;
  hipLaunchKernelGGL((spec_forward_kernel<T, G>), dim3(grid), dim3(kSpecThreads), lds, stream,
                     plan->cfg.num_channels, shape.chblocks, n_blocks, static_cast<const T*>(A),
                     static_cast<const T*>(W), static_cast<T*>(B), ws.tiles, ws.perm);
  return hipGetLastError();
}

template <typename T, typename G>
hipError_t bwd_launch(const sc_plan* plan, int64_t n, const void* A, const void* W, const void* dB, void* dA,
                      const Workspace& ws, const LaunchShape& shape, hipStream_t stream) {
  const int n_blocks = shape.max_tiles * shape.chblocks;
  const int grid = (n_blocks + kXcds - 1) / kXcds * kXcds;
  const size_t lds = sizeof(T) * kSpecWaves * (G::kS + G::kNlm) * kLanes;
  auto kernel = &spec_backward_kernel<T, G, 0>;
  if constexpr (sizeof(T) == 4 && G::kS <= 32) {
    if (n <= 40000) kernel = &spec_backward_kernel<T, G, 3>;   // small batches: three waves per SIMD (see the kernel)
  }
  if (lds > 64 * 1024) {  // above the default dynamic LDS limit: raise it for this kernel
    const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds));
    if (e != hipSuccess) return e;
  }
  hipLaunchKernelGGL(kernel, dim3(grid), dim3(kSpecThreads), lds, stream, plan->cfg.num_channels, shape.chblocks,
                     n_blocks, static_cast<const T*>(A), static_cast<const T*>(W), static_cast<const T*>(dB),
                     static_cast<T*>(dA), static_cast<T*>(ws.partial), ws.tiles, ws.perm);
  return hipGetLastError();
}

template <typename T, typename G>
hipError_t dbl_launch(const sc_plan* plan, const void* A, const void* W, const void* dB, const void* H, void* ddB,
                      void* dA2, const Workspace& ws, const LaunchShape& shape, hipStream_t stream) {
  const int n_blocks = shape.max_tiles * shape.chblocks;
  const int grid = (n_blocks + kXcds - 1) / kXcds * kXcds;
  constexpr bool kLds = kUseLdsState<T, G>;
  const size_t lds = sizeof(T) * kSpecWaves * ((kLds ? 2 : 1) * G::kS + G::kNlm) * kLanes;
  auto kernel = &spec_double_backward_kernel<T, G>;
  if constexpr (kLds) kernel = &spec_double_backward_lds_kernel<T, G>;
  if (lds > 64 * 1024) {  // above the default dynamic LDS limit: raise it for this kernel
    const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds));
    if (e != hipSuccess) return e;
  }
  hipLaunchKernelGGL(kernel, dim3(grid), dim3(kSpecThreads), lds, stream, plan->cfg.num_channels, shape.chblocks,
                     n_blocks, static_cast<const T*>(A), static_cast<const T*>(W), static_cast<const T*>(dB),
                     static_cast<const T*>(H), static_cast<T*>(ddB), static_cast<T*>(dA2),
                     static_cast<T*>(ws.partial), ws.tiles, ws.perm);
  return hipGetLastError();
}

template <typename T, typename G>
hipError_t finalize_launch(const sc_plan* plan, void* dW, const Workspace& ws, const LaunchShape& shape,
                           hipStream_t stream) {
  const int Z = plan->cfg.num_elements;
  hipLaunchKernelGGL((spec_reduce_kernel<T, G>), dim3(Z * shape.chblocks * G::kS), dim3(kReduceWaves * kLanes), 0, stream,
                     shape.chblocks, shape.max_tiles, static_cast<const T*>(ws.partial), ws.tile_off, ws.reduced);
  hipLaunchKernelGGL((spec_unfold_kernel<T, G>), dim3(Z * shape.chblocks), dim3(kLanes), 0, stream,
                     plan->cfg.num_channels, shape.chblocks, ws.reduced, static_cast<T*>(dW));
  return hipGetLastError();
}

}  // namespace

int spec_lookup(const sc_plan* plan) {
  if (matches<Gen_l3n3_0e1o>(plan)) return 1;
  if (matches<Gen_l3n3_0e1o2e>(plan)) return 2;
  return 0;
}

int spec_basis_size(int id) { return id == 1 ? Gen_l3n3_0e1o::kS : id == 2 ? Gen_l3n3_0e1o2e::kS : 0; }

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
}

int spec_waves_per_tile() { return kSpecWaves; }

hipError_t launch_spec_forward(const sc_plan* plan, int64_t, const void* A, const void* W, void* B,
                               const Workspace& ws, const LaunchShape& shape, hipStream_t stream) {
  const bool f64 = plan->cfg.dtype == SC_F64;
  if (plan->specialised == 1)
    return f64 ? fwd_launch<double, Gen_l3n3_0e1o>(plan, A, W, B, ws, shape, stream)
               : fwd_launch<float, Gen_l3n3_0e1o>(plan, A, W, B, ws, shape, stream);
  if (plan->specialised == 2)
    return f64 ? fwd_launch<double, Gen_l3n3_0e1o2e>(plan, A, W, B, ws, shape, stream)
               : fwd_launch<float, Gen_l3n3_0e1o2e>(plan, A, W, B, ws, shape, stream);
  return hipErrorInvalidValue;
}

hipError_t launch_spec_backward(const sc_plan* plan, int64_t n, const void* A, const void* W, const void* dB,
                                void* dA, const Workspace& ws, const LaunchShape& shape, hipStream_t stream) {
  const bool f64 = plan->cfg.dtype == SC_F64;
  if (plan->specialised == 1)
    return f64 ? bwd_launch<double, Gen_l3n3_0e1o>(plan, n, A, W, dB, dA, ws, shape, stream)
               : bwd_launch<float, Gen_l3n3_0e1o>(plan, n, A, W, dB, dA, ws, shape, stream);
  if (plan->specialised == 2)
    return f64 ? bwd_launch<double, Gen_l3n3_0e1o2e>(plan, n, A, W, dB, dA, ws, shape, stream)
               : bwd_launch<float, Gen_l3n3_0e1o2e>(plan, n, A, W, dB, dA, ws, shape, stream);
  return hipErrorInvalidValue;
}

hipError_t launch_spec_double_backward(const sc_plan* plan, int64_t, const void* A, const void* W, const void* dB,
                                       const void* H, void* ddB, void* dA2, const Workspace& ws,
                                       const LaunchShape& shape, hipStream_t stream) {
  const bool f64 = plan->cfg.dtype == SC_F64;
  if (plan->specialised == 1)
    return f64 ? dbl_launch<double, Gen_l3n3_0e1o>(plan, A, W, dB, H, ddB, dA2, ws, shape, stream)
               : dbl_launch<float, Gen_l3n3_0e1o>(plan, A, W, dB, H, ddB, dA2, ws, shape, stream);
  if (plan->specialised == 2)
    return f64 ? dbl_launch<double, Gen_l3n3_0e1o2e>(plan, A, W, dB, H, ddB, dA2, ws, shape, stream)
               : dbl_launch<float, Gen_l3n3_0e1o2e>(plan, A, W, dB, H, ddB, dA2, ws, shape, stream);
  return hipErrorInvalidValue;
}

hipError_t launch_spec_finalize(const sc_plan* plan, void* dW, const Workspace& ws, const LaunchShape& shape,
                                hipStream_t stream) {
  const bool f64 = plan->cfg.dtype == SC_F64;
  if (plan->specialised == 1)
    return f64 ? finalize_launch<double, Gen_l3n3_0e1o>(plan, dW, ws, shape, stream)
               : finalize_launch<float, Gen_l3n3_0e1o>(plan, dW, ws, shape, stream);
  if (plan->specialised == 2)
    return f64 ? finalize_launch<double, Gen_l3n3_0e1o2e>(plan, dW, ws, shape, stream)
               : finalize_launch<float, Gen_l3n3_0e1o2e>(plan, dW, ws, shape, stream);
  return hipErrorInvalidValue;
}

}  // namespace sc
