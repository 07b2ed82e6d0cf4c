// Specialised kernels of the channelwise tensor product: hand-written memory / scheduling
// skeleton around generated straight-line arithmetic (csrc/generated/tp_gen_*.inc, written by
// codegen/generate_tp.py).
//
// Mapping (Algorithm 1 of arXiv 2504.10700 is independent per edge and channel; the pooling
// sums the edges of a receiver):
//   lane      = channel (64 consecutive channels per wave): a path's weights R[e][p][:] are one
//               contiguous 256 B row per wave, the sender's features h[j][k][:] 16 B per lane
//   wave      = forward: one (receiving atom, 64-channel block); it walks the edges the atom
//               receives and keeps the atom's sum in registers.  Backward: one (sending atom,
//               64-channel block); it walks the edges the atom sends, keeps the atom's h row and
//               its dh sum in registers and gathers the receivers' dA rows; per edge it writes dR
//               and the channel block's partial of dY.  Either way: no atomics, a fixed summation
//               order, one store per atom.  The second-order pass walks by receiver (ddA in
//               registers) and writes every edge's share of d2h, which a small kernel sums per sender.
//   Y[e][:]   is the same for all lanes: it is read with scalar loads and enters the
//               arithmetic as scalar operands
// The next edge's rows are requested before the current edge is evaluated (two register sets
// in turn); the sender index of the edge after next is read one step further ahead so that
// no row load waits for an index.
#include "tp_internal.h"

namespace tp {
namespace {

using sc::kLanes;

__device__ __forceinline__ float sc_fma(float x, float y, float z) { return __builtin_fmaf(x, y, z); }
__device__ __forceinline__ double sc_fma(double x, double y, double z) { return __builtin_fma(x, y, z); }

#include "generated/tp_gen_y3h0o3.inc"
#include "generated/tp_gen_y3h1o3.inc"

constexpr int kWaves = 4;
constexpr int kThreads = kWaves * kLanes;
constexpr int kStageStride = kLanes + 1;  // LDS row stride of the dY transpose (odd: two-way conflicts at most)

// N consecutive elements at p (aligned to 16 B if the row size is a multiple of 16 B).
template <typename T, int N>
__device__ __forceinline__ void load_row(const T* __restrict__ p, T (&v)[N]) {
  constexpr int V = 16 / sizeof(T);
  if constexpr ((N * sizeof(T)) % 16 == 0) {
    typedef T Vec __attribute__((ext_vector_type(V)));
#pragma unroll
    for (int i = 0; i < N; i += V) {
      const Vec x = *reinterpret_cast<const Vec*>(p + i);
#pragma unroll
      for (int k = 0; k < V; ++k) v[i + k] = x[k];
    }
  } else {
#pragma unroll
    for (int i = 0; i < N; ++i) v[i] = p[i];
  }
}

template <typename T, int N>
__device__ __forceinline__ void store_row(T* __restrict__ p, const T (&v)[N]) {
  constexpr int V = 16 / sizeof(T);
  if constexpr ((N * sizeof(T)) % 16 == 0) {
    typedef T Vec __attribute__((ext_vector_type(V)));
#pragma unroll
    for (int i = 0; i < N; i += V) {
      Vec x;
#pragma unroll
      for (int k = 0; k < V; ++k) x[k] = v[i + k];
      // A row of one 16-byte piece makes the wave's store one contiguous KB: streamed past the
      // cache (measured faster).  Longer rows are written by several instructions that each touch
      // a part of every line: left to the L2 to merge (streaming them measured slower).
      if constexpr (N * sizeof(T) == 16) __builtin_nontemporal_store(x, reinterpret_cast<Vec*>(p + i));
      else *reinterpret_cast<Vec*>(p + i) = x;
    }
  } else {
#pragma unroll
    for (int i = 0; i < N; ++i) p[i] = v[i];
  }
}

// R[e][p][ch] for all paths of edge e.
template <typename T, int P>
__device__ __forceinline__ void load_weights(const T* __restrict__ R, int e, int K, int ch, T (&r)[P]) {
  const T* base = R + static_cast<size_t>(e) * P * K + ch;
#pragma unroll
  for (int p = 0; p < P; ++p) r[p] = base[static_cast<size_t>(p) * K];
}

// Y[e][:], identical for all lanes (e is wave-uniform): scalar loads.
template <typename T, int N>
__device__ __forceinline__ void load_uniform(const T* __restrict__ Y, int e, T (&y)[N]) {
  const T* base = Y + static_cast<size_t>(e) * N;
#pragma unroll
  for (int a = 0; a < N; ++a) y[a] = base[a];
}

__device__ __forceinline__ int uniform(int v) { return __builtin_amdgcn_readfirstlane(v); }

// blockIdx -> logical block such that the blocks an XCD receives (round-robin by blockIdx) form
// one contiguous range of atoms: the atoms of one structure, which share their senders' rows of
// h, then meet in one XCD's L2.  gridDim.x is a multiple of kXcds.
constexpr int kXcds = 8;
__device__ __forceinline__ int64_t xcd_contiguous_block() {
  const int64_t per = gridDim.x / kXcds;
  return (blockIdx.x % kXcds) * per + blockIdx.x / kXcds;
}

// Sum of dy[a] over the 64 lanes in a fixed order, written to out[a] (a < N): lane 4a+q adds the
// sixteen lanes 16q..16q+15 of component a from an LDS transpose (stage: N * kStageStride
// elements owned by this wave), then the four quarters are combined with two exchanges.
template <typename T, int N>
__device__ __forceinline__ void lane_sum_store(T* stage, int lane, const T (&dy)[N], T* __restrict__ out) {
  static_assert(N <= 16, "one lane quartet per component");
  __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");  // the previous edge's reads of the stage are done
  __builtin_amdgcn_wave_barrier();
#pragma unroll
  for (int a = 0; a < N; ++a) stage[a * kStageStride + lane] = dy[a];
  __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
  __builtin_amdgcn_wave_barrier();
  const int a = lane >> 2, q = lane & 3;
  T s = T(0);
  if (a < N) {
#pragma unroll
    for (int i = 0; i < 16; ++i) s += stage[a * kStageStride + q * 16 + i];
  }
  s += __shfl_xor(s, 1);
  s += __shfl_xor(s, 2);
  if (q == 0 && a < N) out[a] = s;
}

// Store of a wave's rows (N elements per lane, lane rows N elements apart = one contiguous block
// of 64*N elements) as whole lines: every lane's row goes through an LDS block of the same
// layout and comes back so that store instruction k writes the k-th contiguous KB of the block
// instead of 64 pieces of 16 bytes (partial lines, N*sizeof(T)/16 times the write requests);
// streamed past the cache.  stage: 64*N elements of LDS owned by this wave; block: where lane
// 0's row goes (16-byte aligned).  N*sizeof(T) is a multiple of 16.
template <typename T, int N>
__device__ __forceinline__ void store_rows_coalesced(T* __restrict__ block, T* stage, int lane, const T (&v)[N]) {
  constexpr int V = 16 / sizeof(T);
  static_assert(N % V == 0, "rows are whole 16-byte pieces");
  typedef T Vec __attribute__((ext_vector_type(V)));
  __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");  // earlier reads of the stage are done
  __builtin_amdgcn_wave_barrier();
#pragma unroll
  for (int j = 0; j < N / V; ++j) {
    Vec x;
#pragma unroll
    for (int k = 0; k < V; ++k) x[k] = v[j * V + k];
    *reinterpret_cast<Vec*>(stage + lane * N + j * V) = x;
  }
  __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");  // the other lanes' pieces are visible
  __builtin_amdgcn_wave_barrier();
#pragma unroll
  for (int q0 = 0; q0 < kLanes * N / V; q0 += kLanes) {
    const int q = q0 + lane;
    const Vec x = *reinterpret_cast<const Vec*>(stage + q * V);
    __builtin_nontemporal_store(x, reinterpret_cast<Vec*>(block + q * V));
  }
}

template <typename T, typename G>
__global__ __launch_bounds__(kThreads) void forward_kernel(int K, int chblocks, int64_t n_units,
                                                           const T* __restrict__ Y, const T* __restrict__ h,
                                                           const T* __restrict__ R,
                                                           const EdgeList el, T* __restrict__ A) {
  __shared__ __attribute__((aligned(16))) T out_stage[kWaves][kLanes * G::kNout];
  const int lane = threadIdx.x & (kLanes - 1);
  const int wave = uniform(threadIdx.x / kLanes);
  const int64_t unit = xcd_contiguous_block() * kWaves + wave;
  if (unit >= n_units) return;
  const size_t node = unit / chblocks;
  const int cb = static_cast<int>(unit % chblocks);
  const int ch = cb * kLanes + lane;
  const int e0 = uniform(el.first(node)), e1 = uniform(el.first(node + 1));
  T acc[G::kNout];
#pragma unroll
  for (int c = 0; c < G::kNout; ++c) acc[c] = T(0);
  if (e0 < e1) {
    T r0[G::kP], r1[G::kP], h0[G::kNh], h1[G::kNh], y[G::kNY];
    load_weights<T, G::kP>(R, e0, K, ch, r0);
    load_row<T, G::kNh>(h + (el.snd(e0) * K + ch) * G::kNh, h0);
    int jn = (e0 + 1 < e1) ? el.raw(e0 + 1) : 0;  // sender of the next edge, read one step ahead
    for (int e = e0; e < e1; e += 2) {
      int jn2 = 0;
      if (e + 1 < e1) {
        load_weights<T, G::kP>(R, e + 1, K, ch, r1);
        load_row<T, G::kNh>(h + (el.node(jn) * K + ch) * G::kNh, h1);
        if (e + 2 < e1) jn2 = el.raw(e + 2);
      }
      load_uniform<T, G::kNY>(Y, e, y);
      G::forward(y, h0, r0, acc);
      if (e + 1 < e1) {
        if (e + 2 < e1) {
          load_weights<T, G::kP>(R, e + 2, K, ch, r0);
          load_row<T, G::kNh>(h + (el.node(jn2) * K + ch) * G::kNh, h0);
          if (e + 3 < e1) jn = el.raw(e + 3);
        }
        load_uniform<T, G::kNY>(Y, e + 1, y);
        G::forward(y, h1, r1, acc);
      }
    }
  }
  store_rows_coalesced<T, G::kNout>(A + (node * K + cb * kLanes) * G::kNout, out_stage[wave], lane, acc);
}

// receiver[e] for every edge, from the receivers' offsets: one thread per receiving atom.
__global__ __launch_bounds__(256) void edge_receiver_kernel(int64_t n_out_nodes, const EdgeList el,
                                                            int32_t* __restrict__ receiver) {
  const int64_t node = blockIdx.x * static_cast<int64_t>(blockDim.x) + threadIdx.x;
  if (node >= n_out_nodes) return;
  const int e0 = el.first(node), e1 = el.first(node + 1);
  for (int e = e0; e < e1; ++e) receiver[e] = static_cast<int32_t>(node);
}

// The backward walks the edges grouped by SENDER: one wave = one (sending atom, 64-channel block).
// It keeps the atom's h row and its dh sum in registers, walks the edges the atom sends
// (send_edge order: the order of the sum) and gathers per edge the dA row of the receiver (rows of
// one structure, met in the XCD's L2) next to the edge's own R rows; dR and the channel block's
// partial of dY leave per edge, dh leaves once per atom: no per-edge shares
// of dh go to memory and come back.  Atoms that send nothing get a zero row.  Every index is
// clamped where it is used.
template <typename T, typename G>
__global__ __launch_bounds__(kThreads) void backward_by_sender_kernel(
    int K, int chblocks, int64_t n_units, int64_t n_out_nodes, int n_edges, const T* __restrict__ Y,
    const T* __restrict__ h, const T* __restrict__ R, const int32_t* __restrict__ send_ptr,
    const int32_t* __restrict__ send_edge, const int32_t* __restrict__ receiver, const T* __restrict__ dA,
    T* __restrict__ dR, T* __restrict__ dY_partial, T* __restrict__ dh) {
  __shared__ T stage_all[kWaves][G::kNY * kStageStride];
  const int lane = threadIdx.x & (kLanes - 1);
  const int wave = uniform(threadIdx.x / kLanes);
  T* stage = stage_all[wave];
  const int64_t unit = xcd_contiguous_block() * kWaves + wave;
  if (unit >= n_units) return;
  const size_t node = unit / chblocks;
  const int cb = static_cast<int>(unit % chblocks);
  const int ch = cb * kLanes + lane;
  auto pos = [&](int v) { return v < 0 ? 0 : (v > n_edges ? n_edges : v); };
  auto edge = [&](int q) {
    const int e = send_edge[q];
    return e < 0 ? 0 : (e >= n_edges ? n_edges - 1 : e);
  };
  auto atom = [&](int r) { return static_cast<size_t>(r < 0 ? 0 : (r >= n_out_nodes ? n_out_nodes - 1 : r)); };
  const int q0 = uniform(pos(send_ptr[node])), q1 = uniform(pos(send_ptr[node + 1]));
  T acc[G::kNh];
#pragma unroll
  for (int c = 0; c < G::kNh; ++c) acc[c] = T(0);
  if (q0 < q1) {
    T hh[G::kNh];
    load_row<T, G::kNh>(h + (node * K + ch) * G::kNh, hh);
    T r0[G::kP], r1[G::kP], g0[G::kNout], g1[G::kNout];
    int ea = uniform(edge(q0)), eb = 0;
    load_weights<T, G::kP>(R, ea, K, ch, r0);
    load_row<T, G::kNout>(dA + (atom(uniform(receiver[ea])) * K + ch) * G::kNout, g0);
    // edge id and receiver of the edge after the current one, read one step ahead of its rows
    int en = (q0 + 1 < q1) ? uniform(edge(q0 + 1)) : 0;
    int rn = uniform(receiver[en]);

    // One edge: arithmetic, dR row stores, dY summed over the 64 lanes in a fixed order, dh added up.
    auto finish_edge = [&](int e, const T (&r)[G::kP], const T (&g)[G::kNout]) {
      T y[G::kNY], dr[G::kP], dy[G::kNY], dhe[G::kNh];
      load_uniform<T, G::kNY>(Y, e, y);
      G::backward(y, hh, r, g, dr, dy, dhe);
      T* out = dR + static_cast<size_t>(e) * G::kP * K + ch;
#pragma unroll
      for (int p = 0; p < G::kP; ++p) __builtin_nontemporal_store(dr[p], out + static_cast<size_t>(p) * K);
#pragma unroll
      for (int c = 0; c < G::kNh; ++c) acc[c] += dhe[c];
      lane_sum_store<T, G::kNY>(stage, lane, dy, dY_partial + (static_cast<size_t>(cb) * n_edges + e) * G::kNY);
    };

    for (int q = q0; q < q1; q += 2) {
      if (q + 1 < q1) {
        eb = en;
        load_weights<T, G::kP>(R, eb, K, ch, r1);
        load_row<T, G::kNout>(dA + (atom(rn) * K + ch) * G::kNout, g1);
        if (q + 2 < q1) {
          en = uniform(edge(q + 2));
          rn = uniform(receiver[en]);
        }
      }
      finish_edge(ea, r0, g0);
      if (q + 1 < q1) {
        if (q + 2 < q1) {
          ea = en;
          load_weights<T, G::kP>(R, ea, K, ch, r0);
          load_row<T, G::kNout>(dA + (atom(rn) * K + ch) * G::kNout, g0);
          if (q + 3 < q1) {
            en = uniform(edge(q + 3));
            rn = uniform(receiver[en]);
          }
        }
        finish_edge(eb, r1, g1);
      }
    }
  }
  store_row<T, G::kNh>(dh + (node * K + ch) * G::kNh, acc);
}

// Second-order pass: the backward's walk with the cotangents HR (per edge and path), Hh (at the
// sender) and HY (wave-uniform) as additional inputs; ddA of the receiver is summed in registers
// and stored once, d2R / d2Y partial / d2h share leave per edge like dR / dY / dh.
template <typename T, typename G>
__global__ __launch_bounds__(kThreads) void double_backward_kernel(
    int K, int chblocks, int64_t n_units, int64_t n_edges, const T* __restrict__ Y, const T* __restrict__ h,
    const T* __restrict__ R, const EdgeList el,
    const T* __restrict__ dA, const T* __restrict__ HY, const T* __restrict__ Hh, const T* __restrict__ HR,
    T* __restrict__ ddA, T* __restrict__ d2R, T* __restrict__ d2Y_partial, T* __restrict__ d2h_edge) {
  __shared__ T stage_all[kWaves][G::kNY * kStageStride];
  const int lane = threadIdx.x & (kLanes - 1);
  const int wave = uniform(threadIdx.x / kLanes);
  T* stage = stage_all[wave];
  const int64_t unit = xcd_contiguous_block() * kWaves + wave;
  if (unit >= n_units) return;
  const size_t node = unit / chblocks;
  const int cb = static_cast<int>(unit % chblocks);
  const int ch = cb * kLanes + lane;
  const int e0 = uniform(el.first(node)), e1 = uniform(el.first(node + 1));
  T dda[G::kNout];
#pragma unroll
  for (int c = 0; c < G::kNout; ++c) dda[c] = T(0);
  if (e0 < e1) {
    T g[G::kNout];
    load_row<T, G::kNout>(dA + (node * K + ch) * G::kNout, g);
    T r0[G::kP], r1[G::kP], q0[G::kP], q1[G::kP], h0[G::kNh], h1[G::kNh], x0[G::kNh], x1[G::kNh];
    {
      const size_t j = el.snd(e0);
      load_weights<T, G::kP>(R, e0, K, ch, r0);
      load_weights<T, G::kP>(HR, e0, K, ch, q0);
      load_row<T, G::kNh>(h + (j * K + ch) * G::kNh, h0);
      load_row<T, G::kNh>(Hh + (j * K + ch) * G::kNh, x0);
    }
    int jn = (e0 + 1 < e1) ? el.raw(e0 + 1) : 0;

    auto finish_edge = [&](int e, const T (&r)[G::kP], const T (&hr)[G::kP], const T (&hh)[G::kNh],
                           const T (&hx)[G::kNh]) {
      T y[G::kNY], hy[G::kNY], d2r[G::kP], d2y[G::kNY], d2h[G::kNh];
      load_uniform<T, G::kNY>(Y, e, y);
      load_uniform<T, G::kNY>(HY, e, hy);
      G::double_backward(y, hy, hh, hx, r, hr, g, dda, d2r, d2y, d2h);
      T* out = d2R + static_cast<size_t>(e) * G::kP * K + ch;
#pragma unroll
      for (int p = 0; p < G::kP; ++p) __builtin_nontemporal_store(d2r[p], out + static_cast<size_t>(p) * K);
      store_row<T, G::kNh>(d2h_edge + (static_cast<size_t>(e) * K + ch) * G::kNh, d2h);
      lane_sum_store<T, G::kNY>(stage, lane, d2y, d2Y_partial + (static_cast<size_t>(cb) * n_edges + e) * G::kNY);
    };

    for (int e = e0; e < e1; e += 2) {
      int jn2 = 0;
      if (e + 1 < e1) {
        load_weights<T, G::kP>(R, e + 1, K, ch, r1);
        load_weights<T, G::kP>(HR, e + 1, K, ch, q1);
        load_row<T, G::kNh>(h + (el.node(jn) * K + ch) * G::kNh, h1);
        load_row<T, G::kNh>(Hh + (el.node(jn) * K + ch) * G::kNh, x1);
        if (e + 2 < e1) jn2 = el.raw(e + 2);
      }
      finish_edge(e, r0, q0, h0, x0);
      if (e + 1 < e1) {
        if (e + 2 < e1) {
          load_weights<T, G::kP>(R, e + 2, K, ch, r0);
          load_weights<T, G::kP>(HR, e + 2, K, ch, q0);
          load_row<T, G::kNh>(h + (el.node(jn2) * K + ch) * G::kNh, h0);
          load_row<T, G::kNh>(Hh + (el.node(jn2) * K + ch) * G::kNh, x0);
          if (e + 3 < e1) jn = el.raw(e + 3);
        }
        finish_edge(e + 1, r1, q1, h1, x1);
      }
    }
  }
  store_row<T, G::kNout>(ddA + (node * K + ch) * G::kNout, dda);
}

template <typename G>
bool matches(const tp_plan* plan) {
  const tp_config& c = plan->cfg;
  return c.l_Y == G::kLY && c.l_h == G::kLh && c.L_max == G::kLout && c.num_channels % kLanes == 0 &&
         static_cast<int>(plan->paths.size()) == G::kP;
}

unsigned grid_for(int64_t n_units) {
  const int64_t blocks = (n_units + kWaves - 1) / kWaves;
  return static_cast<unsigned>((blocks + kXcds - 1) / kXcds * kXcds);
}

template <typename T, typename G>
hipError_t fwd_launch(const tp_plan* plan, const FwdArgs& a, hipStream_t stream) {
  const int K = plan->cfg.num_channels, chblocks = K / kLanes;
  const int64_t n_units = a.n_out_nodes * chblocks;
  hipLaunchKernelGGL((forward_kernel<T, G>), dim3(grid_for(n_units)), dim3(kThreads), 0, stream, K, chblocks, n_units,
                     static_cast<const T*>(a.Y), static_cast<const T*>(a.h), static_cast<const T*>(a.R), EdgeList{a.sender, a.row_ptr, static_cast<int>(a.n_in), static_cast<int>(a.n_edges)}, static_cast<T*>(a.A));
  return hipGetLastError();
}

template <typename T, typename G>
hipError_t bwd_launch(const tp_plan* plan, const BwdArgs& a, hipStream_t stream) {
  const int K = plan->cfg.num_channels, chblocks = K / kLanes;
  const EdgeList el{a.sender, a.row_ptr, static_cast<int>(a.n_in), static_cast<int>(a.n_edges)};
  int32_t* receiver = static_cast<int32_t*>(a.dh_edge);   // the shares' part of the workspace is free on this path
  if (a.n_edges > 0 && a.n_out_nodes > 0) {
    hipLaunchKernelGGL(edge_receiver_kernel, dim3(static_cast<unsigned>((a.n_out_nodes + 255) / 256)), dim3(256), 0,
                       stream, a.n_out_nodes, el, receiver);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  const int64_t n_units = a.n_in * chblocks;
  // without receivers or edges no list is walked: every atom gets its zero row
  hipLaunchKernelGGL((backward_by_sender_kernel<T, G>), dim3(grid_for(n_units)), dim3(kThreads), 0, stream, K, chblocks,
                     n_units, a.n_out_nodes, a.n_out_nodes > 0 ? static_cast<int>(a.n_edges) : 0,
                     static_cast<const T*>(a.Y), static_cast<const T*>(a.h), static_cast<const T*>(a.R), a.send_ptr,
                     a.send_edge, receiver, static_cast<const T*>(a.dA), static_cast<T*>(a.dR),
                     static_cast<T*>(a.dY_partial), static_cast<T*>(a.dh));
  return hipGetLastError();
}

template <typename T, typename G>
hipError_t dbl_launch(const tp_plan* plan, const DblArgs& d, hipStream_t stream) {
  const BwdArgs& a = d.b;
  const int K = plan->cfg.num_channels, chblocks = K / kLanes;
  const int64_t n_units = a.n_out_nodes * chblocks;
  hipLaunchKernelGGL((double_backward_kernel<T, G>), dim3(grid_for(n_units)), dim3(kThreads), 0, stream, K, chblocks,
                     n_units, a.n_edges, static_cast<const T*>(a.Y), static_cast<const T*>(a.h),
                     static_cast<const T*>(a.R), EdgeList{a.sender, a.row_ptr, static_cast<int>(a.n_in), static_cast<int>(a.n_edges)}, static_cast<const T*>(a.dA),
                     static_cast<const T*>(d.HY), static_cast<const T*>(d.Hh), static_cast<const T*>(d.HR),
                     static_cast<T*>(d.ddA), static_cast<T*>(a.dR), static_cast<T*>(a.dY_partial),
                     static_cast<T*>(a.dh_edge));
  return hipGetLastError();
}

template <typename G>
void op_counts(int32_t ops[3], int32_t flops[3]) {
  for (int i = 0; i < 3; ++i) {
    ops[i] = G::kOps[i];
    flops[i] = G::kFlops[i];
  }
}

}  // namespace

int spec_lookup(const tp_plan* plan) {
  if (matches<GenTP_y3h0o3>(plan)) return 1;
  if (matches<GenTP_y3h1o3>(plan)) return 2;
  return 0;
}

void spec_op_counts(int id, int32_t ops[3], int32_t flops[3]) {
  for (int i = 0; i < 3; ++i) ops[i] = flops[i] = 0;
  if (id == 1) op_counts<GenTP_y3h0o3>(ops, flops);
  if (id == 2) op_counts<GenTP_y3h1o3>(ops, flops);
}

#define TP_DISPATCH(fn, args)                                                                        \
  const bool f64 = plan->cfg.dtype == SC_F64;                                                        \
  if (plan->specialised == 1) return f64 ? fn<double, GenTP_y3h0o3> args : fn<float, GenTP_y3h0o3> args; \
  if (plan->specialised == 2) return f64 ? fn<double, GenTP_y3h1o3> args : fn<float, GenTP_y3h1o3> args; \
  return hipErrorInvalidValue;

hipError_t launch_spec_forward(const tp_plan* plan, const FwdArgs& a, hipStream_t stream) {
  TP_DISPATCH(fwd_launch, (plan, a, stream))
}
hipError_t launch_spec_double_backward(const tp_plan* plan, const DblArgs& a, hipStream_t stream) {
  TP_DISPATCH(dbl_launch, (plan, a, stream))
}
hipError_t launch_spec_backward(const tp_plan* plan, const BwdArgs& a, hipStream_t stream) {
  TP_DISPATCH(bwd_launch, (plan, a, stream))
}

}  // namespace tp
