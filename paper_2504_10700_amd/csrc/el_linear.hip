// Per-order channel-mixing linear (see include/el.h): Y[i,k',(l,m)] = sum_k W[l,k,k'] X[i,k,(l,m)]
// (Section 4.1 of arXiv 2504.10700, the linear combination between the pooling and the
// symmetric contraction), forward and backward, on the matrix cores.
//
// One MFMA 16x16x4 multiplies a 16x4 by a 4x16 block; lane L supplies A[i = L%16][kk = L/16]
// and B[kk = L/16][j = L%16] and receives four entries of column j = L%16 of the 16x16 result
// (rows 4*(L/16)+r in fp32, 4*r + L/16 in fp64; r = 0..3).
//
// Forward (and dX, which is the same product on W transposed): rows = 16 atoms, reduction =
// input channels, columns = 16 output channels, one accumulator block per component (l,m); the
// 2l+1 components of an order share their B operand.  With the layout X[atom][channel][lm]
// the A operands of all components of one (atom, channel) are 64 contiguous bytes, and a lane
// ends up with whole 64-byte rows of the result.  Kernels: mfma_forward_lds_kernel (fp32,
// l_max = 3: X staged through LDS once per workgroup, B through a buffer descriptor, result
// rows stored as whole lines through an LDS transpose; the product lives in el_tile.h and is
// shared with the fused linear + contraction kernel) and mfma_forward_kernel (every other
// shape: operands straight from global memory through a four-deep register pipeline).
// dW: rows = 16 input channels, columns = 16 output channels, reduction = atoms (four per
// MFMA) and the components of the order; A and B operands are again 64 contiguous bytes per
// lane.  The atoms are cut into ranges, every range writes a partial dW (mfma_dw_lds_kernel:
// dY rows shared through LDS, two row tiles per wave; mfma_dw_kernel: every other shape), a
// second kernel adds the partials in a fixed order (no atomics).
// Channel counts outside the MFMA tilings run on plain vector kernels with fp64 accumulation.
#include <algorithm>
#include <atomic>
#include <string>

#include "../../include/el.h"
#include "el_tile.h"
#include "sc_internal.h"

namespace el {
namespace {

using sc::DeviceGuard;
using sc::misaligned;
using sc::set_error;

// Y[n][j][c] = sum_k X[n][k][c] * W[l(c)][k][j], W is [L][k_red][k_cols] (the dX product of the
// backward passes W transposed, so that both read their B operands along rows of W).
// One row tile = 16 atoms; wave w owns the column tiles w, w+4, ... and works on CT of them
// at a time.  The grid is persistent: every workgroup walks the row tiles blockIdx.x,
// blockIdx.x + gridDim.x, ...  With one workgroup resident per CU (the accumulators and the
// operand pipeline fill the register file) a grid of one workgroup per row tile would pay the
// launch of a workgroup, the first loads and the drain of the stores once per tile with
// nothing to overlap them (measured 27 us per workgroup against 15 us of matrix time).
// k_red % (4 * kDepth) == 0, k_cols % (64 * CT) == 0.
constexpr int kDepth = 4;  // operand sets of the forward kernel's software pipeline

template <typename T, int LMAX, int CT>
__global__ __launch_bounds__(kThreads) void mfma_forward_kernel(int64_t n_nodes, int k_red, int k_cols,
                                                                const T* __restrict__ X, const T* __restrict__ W,
                                                                T* __restrict__ Y) {
  constexpr int NC = (LMAX + 1) * (LMAX + 1), L = LMAX + 1;
  typedef typename Mma<T>::acc_t acc_t;
  const int lane = threadIdx.x & (kLanes - 1);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kLanes);
  const int kq = lane / 16;                    // position inside the reduction step
  const int steps = k_red / 4;
  const int tiles_per_wave = k_cols / (16 * kWaves);
  const int64_t row_tiles = (n_nodes + 15) / 16;
  for (int64_t tile = blockIdx.x; tile < row_tiles; tile += gridDim.x)
  for (int g = 0; g < tiles_per_wave; g += CT) {
    const int64_t n0 = tile * 16;
    int64_t na = n0 + (lane & 15);             // the atom whose A operands this lane supplies
    if (na >= n_nodes) na = n_nodes - 1;       // rows past the end compute on a valid atom and are not stored
    const T* xrow = X + (static_cast<size_t>(na) * k_red + kq) * NC;
    int jc[CT];                                // this lane's column in every tile of the group
#pragma unroll
    for (int t = 0; t < CT; ++t) jc[t] = ((g + t) * kWaves + wave) * 16 + (lane & 15);
    acc_t acc[NC][CT];
#pragma unroll
    for (int c = 0; c < NC; ++c)
#pragma unroll
      for (int t = 0; t < CT; ++t) acc[c][t] = acc_t{0, 0, 0, 0};

    auto load = [&](int s, T (&a)[NC], T (&b)[L][CT]) {
      load_row<T, NC>(xrow + static_cast<size_t>(s) * 4 * NC, a);
      const int k = s * 4 + kq;
#pragma unroll
      for (int l = 0; l < L; ++l)
#pragma unroll
        for (int t = 0; t < CT; ++t)
          b[l][t] = W[(static_cast<size_t>(l) * k_red + k) * k_cols + jc[t]];
    };
    auto multiply = [&](const T (&a)[NC], const T (&b)[L][CT]) {
#pragma unroll
      for (int c = 0; c < NC; ++c)
#pragma unroll
        for (int t = 0; t < CT; ++t) acc[c][t] = Mma<T>::mma(a[c], b[order_of(c)][t], acc[c][t]);
    };
    // kDepth operand sets in turn: the loads of step s + kDepth - 1 are issued before the
    // products of step s, so that kDepth - 1 steps of matrix work cover the load latency.
    // The loop body has no branch (steps is a multiple of kDepth; prefetches past the end
    // re-read the last step): with branches inside, the compiler's wait-count bookkeeping
    // falls back to waiting for every outstanding load at each step, which serialises the
    // pipeline (measured: 33 us instead of 15 us of matrix time per workgroup).  The scheduling
    // barriers keep the instruction scheduler from regrouping the loads of several steps, which
    // has the same effect (a wait for the newest loads at the top of every iteration).
    T a[kDepth][NC], b[kDepth][L][CT];
#pragma unroll
    for (int q = 0; q < kDepth - 1; ++q) load(q < steps ? q : steps - 1, a[q], b[q]);
    for (int s = 0; s < steps; s += kDepth) {
#pragma unroll
      for (int q = 0; q < kDepth; ++q) {
        const int nxt = s + q + kDepth - 1;
        load(nxt < steps ? nxt : steps - 1, a[(q + kDepth - 1) % kDepth], b[(q + kDepth - 1) % kDepth]);
        __builtin_amdgcn_sched_barrier(0);   // keep the loads ahead of this step's products ...
        multiply(a[q], b[q]);
        __builtin_amdgcn_sched_barrier(0);   // ... and the next step's loads behind them
      }
    }
#pragma unroll
    for (int t = 0; t < CT; ++t)
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int64_t n = n0 + Mma<T>::row(lane, r);
        if (n < n_nodes) {
          T y[NC];
#pragma unroll
          for (int c = 0; c < NC; ++c) y[c] = acc[c][t][r];
          store_row<T, NC>(Y + (static_cast<size_t>(n) * k_cols + jc[t]) * NC, y);
        }
      }
  }
}

// fp32, l_max = 3: the LDS-staged product of el_tile.h.  A full work unit = a row tile x 128
// columns (two column tiles per wave, 128 accumulator registers); see UnitSchedule for the halves.
template <int CT>
__device__ __forceinline__ void forward_lds_unit(int64_t n_nodes, int64_t n0, int g, int k_red, int k_cols,
                                                 const float* __restrict__ X, const float* __restrict__ W,
                                                 float* __restrict__ Y, float* xs) {
  constexpr int NC = 16;
  Mma<float>::acc_t acc[NC][CT];
  int jc[CT];
  lds_tile_product<CT>(n_nodes, n0, g, k_red, k_cols, X, W, xs, acc, jc);
  // (the product ends with a workgroup barrier: its buffers are free for the store stages)
  static_assert(kWaves * kStoreStageFloats <= kBuffers * 16 * kRowPad, "the store stages reuse the product's buffers");
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kLanes);
  store_tile_coalesced<CT>(Y, n_nodes, n0, k_cols, jc, acc, xs + wave * kStoreStageFloats);
}

__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(2, 2))) void mfma_forward_lds_kernel(
    int64_t n_nodes, int k_red, int k_cols, const float* __restrict__ X, const float* __restrict__ W,
    float* __restrict__ Y) {
  __shared__ __attribute__((aligned(16))) float xs[kBuffers * 16 * kRowPad];
  const int groups = k_cols / 128;                       // full units per row tile
  const UnitSchedule u = unit_schedule((n_nodes + 15) / 16 * groups, true);
  if (u.has_half)
    forward_lds_unit<1>(n_nodes, u.half_unit / groups * 16, static_cast<int>(u.half_unit % groups) * 2 + u.half, k_red,
                        k_cols, X, W, Y, xs);
  for (int64_t unit = blockIdx.x; unit < u.n_full; unit += gridDim.x)
    forward_lds_unit<2>(n_nodes, unit / groups * 16, static_cast<int>(unit % groups) * 2, k_red, k_cols, X, W, Y, xs);
}

// Partial dW of a range of atoms: part[range][l][k][j] = sum_{n in range} sum_{m in l} X[n][k][c] dY[n][j][c].
// Workgroup = (range, group of 4 row tiles, group of NT column tiles); wave w owns row tile
// 4*kgroup + w.  k_in % 64 == 0, k_out % (16 * NT) == 0, nodes_per_range % 4 == 0.
template <typename T, int LMAX, int NT>
__global__ __launch_bounds__(kThreads) void mfma_dw_kernel(int64_t n_nodes, int nodes_per_range, int k_in, int k_out,
                                                           const T* __restrict__ X, const T* __restrict__ dY,
                                                           T* __restrict__ part) {
  constexpr int NC = (LMAX + 1) * (LMAX + 1), L = LMAX + 1;
  typedef typename Mma<T>::acc_t acc_t;
  const int lane = threadIdx.x & (kLanes - 1);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kLanes);
  const int jgroups = k_out / (16 * NT), kgroups = k_in / 64;
  const int jg = blockIdx.x % jgroups;
  const int kg = (blockIdx.x / jgroups) % kgroups;
  const int64_t range = blockIdx.x / (jgroups * kgroups);
  const int64_t r0 = range * nodes_per_range;
  const int64_t r1 = (r0 + nodes_per_range < n_nodes) ? r0 + nodes_per_range : n_nodes;
  const int k = (kg * kWaves + wave) * 16 + (lane & 15);   // row (input channel) of this lane's A operands
  const int j0 = jg * NT * 16 + (lane & 15);               // column of this lane in the group's first tile
  acc_t acc[L][NT];
#pragma unroll
  for (int l = 0; l < L; ++l)
#pragma unroll
    for (int t = 0; t < NT; ++t) acc[l][t] = acc_t{0, 0, 0, 0};
  for (int64_t n4 = r0; n4 < r1; n4 += 4) {
    const int64_t n = n4 + lane / 16;          // the atom of this lane's position in the reduction step
    const bool valid = n < r1;
    const int64_t nc = valid ? n : r1 - 1;
    T a[NC];
    load_row<T, NC>(X + (static_cast<size_t>(nc) * k_in + k) * NC, a);
    if (!valid) {
#pragma unroll
      for (int c = 0; c < NC; ++c) a[c] = T(0);
    }
#pragma unroll
    for (int t = 0; t < NT; ++t) {
      T b[NC];
      load_row<T, NC>(dY + (static_cast<size_t>(nc) * k_out + j0 + t * 16) * NC, b);
#pragma unroll
      for (int c = 0; c < NC; ++c) acc[order_of(c)][t] = Mma<T>::mma(a[c], b[c], acc[order_of(c)][t]);
    }
  }
  T* out = part + static_cast<size_t>(range) * L * k_in * k_out;
  const int kt = (kg * kWaves + wave) * 16;
#pragma unroll
  for (int l = 0; l < L; ++l)
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
      for (int r = 0; r < 4; ++r)
        out[(static_cast<size_t>(l) * k_in + kt + Mma<T>::row(lane, r)) * k_out + j0 + t * 16] = acc[l][t][r];
}

// The same partial dW for fp32, l_max = 3 and k_in a multiple of 128, with more reuse per loaded
// byte: the workgroup owns 128 input channels x 64 output channels (wave w: two row tiles, 32
// input channels, against all four column tiles: 32 accumulator blocks), the dY rows of a
// reduction step (4 atoms x 64 channels x 64 B = 16 KB) are loaded once per workgroup and shared
// through LDS (two buffers, rows padded to 80 B against bank conflicts), X rows come straight from
// global memory; both are requested one step ahead.  Per MFMA a wave reads 96 B instead of 320 B.
// One workgroup per CU (the accumulators and two operand sets fill the register file).
constexpr int kDwRow = 20;   // floats per (atom, output channel) row of dY in LDS

__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(1, 1))) void mfma_dw_lds_kernel(
    int64_t n_nodes, int nodes_per_range, int k_in, int k_out, const float* __restrict__ X,
    const float* __restrict__ dY, float* __restrict__ part) {
  constexpr int NC = 16, L = 4, NT = 4, NU = 2;
  typedef Mma<float>::acc_t acc_t;
  typedef float V4 __attribute__((ext_vector_type(4)));
  __shared__ __attribute__((aligned(16))) float ys[2][4 * 64 * kDwRow];
  const int lane = threadIdx.x & (kLanes - 1);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kLanes);
  const int jgroups = k_out / 64, kgroups = k_in / 128;
  const int jg = blockIdx.x % jgroups;
  const int kg = (blockIdx.x / jgroups) % kgroups;
  const int64_t range = blockIdx.x / (jgroups * kgroups);
  const int64_t r0 = range * nodes_per_range;
  const int64_t r1 = (r0 + nodes_per_range < n_nodes) ? r0 + nodes_per_range : n_nodes;
  const int steps = static_cast<int>((r1 - r0 + 3) / 4);
  const int kt = kg * 128 + wave * 32;                       // first input channel of this wave
  const int j0 = jg * 64;                                    // first output channel of the workgroup
  const int la = lane / 16;                                  // this lane's atom within a reduction step
  // staging role of this thread: atom tid/64 of the step, output channel tid%64 of the group
  const int sa = threadIdx.x / 64, sj = threadIdx.x % 64;
  float* const swr = &ys[0][(sa * 64 + sj) * kDwRow];
  const float* const brd = &ys[0][(la * 64 + (lane & 15)) * kDwRow];   // column tile 0, this lane's row

  acc_t acc[L][NU][NT];
#pragma unroll
  for (int l = 0; l < L; ++l)
#pragma unroll
    for (int u = 0; u < NU; ++u)
#pragma unroll
      for (int t = 0; t < NT; ++t) acc[l][u][t] = acc_t{0, 0, 0, 0};

  // rows past the end of the range: a valid atom's address, A operands zeroed
  auto aload = [&](int step, V4 (&a)[NU][4]) {
    const int64_t n = r0 + step * 4 + la;
    const int64_t nc = n < r1 ? n : r1 - 1;
#pragma unroll
    for (int u = 0; u < NU; ++u) {
      const V4* p = reinterpret_cast<const V4*>(X + (static_cast<size_t>(nc) * k_in + kt + u * 16 + (lane & 15)) * NC);
#pragma unroll
      for (int i = 0; i < 4; ++i) a[u][i] = n < r1 ? p[i] : V4{0, 0, 0, 0};
    }
  };
  auto yload = [&](int step, V4 (&y)[4]) {
    const int64_t n = r0 + step * 4 + sa;
    const int64_t nc = n < r1 ? n : r1 - 1;
    const V4* p = reinterpret_cast<const V4*>(dY + (static_cast<size_t>(nc) * k_out + j0 + sj) * NC);
#pragma unroll
    for (int i = 0; i < 4; ++i) y[i] = p[i];
  };
  auto ystage = [&](int buf, const V4 (&y)[4]) {
    V4* p = reinterpret_cast<V4*>(swr + buf * 4 * 64 * kDwRow);
#pragma unroll
    for (int i = 0; i < 4; ++i) p[i] = y[i];
  };
  auto multiply = [&](int buf, const V4 (&a)[NU][4]) {
    const float* bb = brd + buf * 4 * 64 * kDwRow;
#pragma unroll
    for (int q = 0; q < 4; ++q) {             // a quarter of the components at a time
      V4 b[NT];
#pragma unroll
      for (int t = 0; t < NT; ++t) b[t] = *reinterpret_cast<const V4*>(bb + t * 16 * kDwRow + q * 4);
#pragma unroll
      for (int i = 0; i < 4; ++i)             // component c = 4 q + i; consecutive MFMAs use different accumulators
#pragma unroll
        for (int u = 0; u < NU; ++u)
#pragma unroll
          for (int t = 0; t < NT; ++t)
            acc[order_of(4 * q + i)][u][t] = Mma<float>::mma(a[u][q][i], b[t][i], acc[order_of(4 * q + i)][u][t]);
    }
  };

  // Operands are requested TWO steps before their use (a step is ~2 us of matrix work, about the
  // memory latency under load; one step of lead left ~1.5 us of stall per step).  Four A sets and
  // two dY register sets rotate with period four: the loop is unrolled by four and has no branch
  // inside (past the end of the range the A operands are zero and the addresses clamped, so the
  // padding steps add nothing), which keeps the compiler's wait counts exact.
  if (steps > 0) {
    const int padded = (steps + 3) / 4 * 4;
    V4 a[4][NU][4], yr[2][4];
    aload(0, a[0]);
    yload(0, yr[0]);
    aload(1, a[1]);
    yload(1, yr[1]);
    ystage(0, yr[0]);
    __syncthreads();
    for (int s = 0; s < padded; s += 4) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        aload(s + i + 2, a[(i + 2) & 3]);
        yload(s + i + 2, yr[i & 1]);              // (the set that held step s+i, staged a step ago)
        multiply(i & 1, a[i]);
        ystage((i + 1) & 1, yr[(i + 1) & 1]);     // step s+i+1, requested a step ago
        __syncthreads();
      }
    }
  }
  float* out = part + static_cast<size_t>(range) * L * k_in * k_out;
#pragma unroll
  for (int l = 0; l < L; ++l)
#pragma unroll
    for (int u = 0; u < NU; ++u)
#pragma unroll
      for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int r = 0; r < 4; ++r)
          out[(static_cast<size_t>(l) * k_in + kt + u * 16 + Mma<float>::row(lane, r)) * k_out + j0 + t * 16 + (lane & 15)] =
              acc[l][u][t][r];
}

// dW[i] = sum of part[r][i] over the ranges r.  A workgroup of four waves owns 64 elements; wave
// q adds the q-th quarter of the ranges (eight independent loads in flight, partial sums
// combined in a fixed tree), the four quarter sums are added in wave order: a fixed order
// altogether, so the result is bitwise reproducible.
template <typename T>
__global__ __launch_bounds__(256) void dw_reduce_kernel(int64_t n_elems, int n_ranges, const T* __restrict__ part,
                                                        T* __restrict__ dW) {
  __shared__ T quarter[4][64];
  const int lane = threadIdx.x & 63, q = threadIdx.x >> 6;
  const int64_t i = blockIdx.x * int64_t(64) + lane;
  const int ra = n_ranges * q / 4, rb = n_ranges * (q + 1) / 4;
  constexpr int U = 8;
  T a[U];
#pragma unroll
  for (int k = 0; k < U; ++k) a[k] = T(0);
  if (i < n_elems) {
    const T* src = part + i;
    int r = ra;
    for (; r + U <= rb; r += U) {
      T v[U];
#pragma unroll
      for (int k = 0; k < U; ++k) v[k] = src[static_cast<size_t>(r + k) * n_elems];
#pragma unroll
      for (int k = 0; k < U; ++k) a[k] += v[k];
    }
    for (; r < rb; ++r) a[0] += src[static_cast<size_t>(r) * n_elems];
  }
#pragma unroll
  for (int w = U / 2; w >= 1; w /= 2)
#pragma unroll
    for (int k = 0; k < w; ++k) a[k] += a[k + w];
  quarter[q][lane] = a[0];
  __syncthreads();
  if (q == 0 && i < n_elems) dW[i] = ((quarter[0][lane] + quarter[1][lane]) + quarter[2][lane]) + quarter[3][lane];
}

// ---- plain vector kernels for channel counts the MFMA tiling does not cover (fp64 accumulation)
template <typename T, bool kTrans>
__global__ void plain_forward_kernel(int64_t n_nodes, int k_red, int k_cols, int l_max, const T* __restrict__ X,
                                     const T* __restrict__ W, T* __restrict__ Y) {
  const int nc = (l_max + 1) * (l_max + 1);
  const int64_t idx = blockIdx.x * static_cast<int64_t>(blockDim.x) + threadIdx.x;
  if (idx >= n_nodes * k_cols) return;
  const int64_t n = idx / k_cols;
  const int j = static_cast<int>(idx % k_cols);
  double y[16];
  for (int c = 0; c < nc; ++c) y[c] = 0.0;
  for (int k = 0; k < k_red; ++k) {
    const T* x = X + (static_cast<size_t>(n) * k_red + k) * nc;
    for (int c = 0; c < nc; ++c) {
      const int l = order_of(c);
      const T w = kTrans ? W[(static_cast<size_t>(l) * k_cols + j) * k_red + k]
                         : W[(static_cast<size_t>(l) * k_red + k) * k_cols + j];
      y[c] += static_cast<double>(x[c]) * static_cast<double>(w);
    }
  }
  for (int c = 0; c < nc; ++c) Y[idx * nc + c] = static_cast<T>(y[c]);
}

// one thread per (l, k, j): sums over all atoms in atom order
template <typename T>
__global__ void plain_dw_kernel(int64_t n_nodes, int k_in, int k_out, int l_max, const T* __restrict__ X,
                                const T* __restrict__ dY, T* __restrict__ dW) {
  const int nc = (l_max + 1) * (l_max + 1);
  const int64_t idx = blockIdx.x * static_cast<int64_t>(blockDim.x) + threadIdx.x;
  if (idx >= static_cast<int64_t>(l_max + 1) * k_in * k_out) return;
  const int j = static_cast<int>(idx % k_out);
  const int k = static_cast<int>((idx / k_out) % k_in);
  const int l = static_cast<int>(idx / (static_cast<int64_t>(k_out) * k_in));
  double s = 0.0;
  for (int64_t n = 0; n < n_nodes; ++n)
    for (int c = l * l; c < (l + 1) * (l + 1); ++c)
      s += static_cast<double>(X[(static_cast<size_t>(n) * k_in + k) * nc + c]) *
           static_cast<double>(dY[(static_cast<size_t>(n) * k_out + j) * nc + c]);
  dW[idx] = static_cast<T>(s);
}

__global__ void zero_kernel(unsigned int* p, size_t n_words) {
  for (size_t i = blockIdx.x * static_cast<size_t>(blockDim.x) + threadIdx.x; i < n_words;
       i += static_cast<size_t>(gridDim.x) * blockDim.x)
    p[i] = 0u;
}

// Wt[l][j][k] = W[l][k][j]: the dX product then reads its B operands along rows like the forward.
template <typename T>
__global__ void transpose_w_kernel(int n_l, int k_in, int k_out, const T* __restrict__ W, T* __restrict__ Wt) {
  const int64_t idx = blockIdx.x * static_cast<int64_t>(blockDim.x) + threadIdx.x;
  if (idx >= static_cast<int64_t>(n_l) * k_in * k_out) return;
  const int k = static_cast<int>(idx % k_in);
  const int j = static_cast<int>((idx / k_in) % k_out);
  const int l = static_cast<int>(idx / (static_cast<int64_t>(k_in) * k_out));
  Wt[idx] = W[(static_cast<size_t>(l) * k_in + k) * k_out + j];
}

// ---- host side

size_t elem_size(const el_config* c) { return c->dtype == SC_F64 ? 8 : 4; }

sc_status check_config(const char* fn, const el_config* cfg, int64_t n) {
  if (!cfg) return set_error(SC_ERR_INVALID_ARG, std::string(fn) + ": cfg is NULL");
  if (cfg->struct_size != static_cast<int32_t>(sizeof(el_config)))
    return set_error(SC_ERR_INVALID_ARG, std::string(fn) + ": struct_size does not match this library's el_config");
  if (cfg->k_in < 1 || cfg->k_out < 1) return set_error(SC_ERR_INVALID_ARG, std::string(fn) + ": k_in or k_out < 1");
  if (cfg->l_max < 0 || cfg->l_max > SC_MAX_L) return set_error(SC_ERR_UNSUPPORTED, std::string(fn) + ": l_max outside 0..3");
  if (cfg->dtype != SC_F32 && cfg->dtype != SC_F64) return set_error(SC_ERR_INVALID_ARG, std::string(fn) + ": bad dtype");
  if (n < 0 || n > (int64_t(1) << 30)) return set_error(SC_ERR_INVALID_ARG, std::string(fn) + ": n_nodes outside 0..2^30");
  return SC_OK;
}

// Compute units of the current device (asked once per device).
int compute_units() {
  static std::atomic<int> cached[64];   // zero-initialised; any thread may fill an entry, all with the same value
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
  int n = cached[dev].load(std::memory_order_relaxed);
  if (n == 0) {
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n < 1) n = 256;
    cached[dev].store(n, std::memory_order_relaxed);
  }
  return n;
}

// Is the product with k_red reduction channels and k_cols output channels served by the MFMA kernel?
bool mfma_forward_ok(int k_red, int k_cols) { return k_red % (4 * kDepth) == 0 && k_cols % 64 == 0; }
bool mfma_dw_ok(const el_config* c) { return c->k_in % 64 == 0 && c->k_out % 64 == 0; }

// Is the LDS-staged dW kernel the one for this configuration?
bool dw_lds_ok(const el_config* c) { return c->dtype == SC_F32 && c->l_max == 3 && c->k_in % 128 == 0 && c->k_out % 64 == 0; }

// Atoms per range of the dW kernel: enough ranges to fill the chip about once, a multiple of 4.
int nodes_per_range(const el_config* cfg, int64_t n) {
  const int groups = (dw_lds_ok(cfg) ? cfg->k_in / 128 : cfg->k_in / 64) * (cfg->k_out / 64);
  int64_t ranges = std::max<int64_t>(1, 256 / std::max(1, groups));
  int64_t per = (n + ranges - 1) / ranges;
  per = std::max<int64_t>(16, (per + 3) / 4 * 4);
  return static_cast<int>(std::min<int64_t>(per, int64_t(1) << 20));
}

template <typename T, int LMAX, bool kTrans>
hipError_t forward_l(int64_t n, int k_red, int k_cols, const void* X, const void* W, void* Y, hipStream_t stream) {
  // The MFMA kernels read B operands along rows of W (the backward hands them W transposed).
  if constexpr (!kTrans) {
    if (mfma_forward_ok(k_red, k_cols)) {
      const int64_t tiles = (n + 15) / 16;
      const unsigned grid = static_cast<unsigned>(std::min<int64_t>(tiles, compute_units()));
      // (the LDS-staged kernel addresses W through a buffer descriptor: its bytes must fit 31 bits)
      if (sizeof(T) == 4 && LMAX == 3 && k_cols % 128 == 0 && static_cast<int64_t>(k_red) * k_cols < (int64_t(1) << 26)) {
        if constexpr (sizeof(T) == 4 && LMAX == 3) {   // the LDS-staged variant: two workgroups fit a CU
          const int64_t units = tiles * (k_cols / 128);
          const unsigned grid2 = static_cast<unsigned>(std::min<int64_t>(units, 2 * compute_units()));
          hipLaunchKernelGGL(mfma_forward_lds_kernel, dim3(grid2), dim3(kThreads), 0, stream, n, k_red, k_cols,
                             static_cast<const float*>(X), static_cast<const float*>(W), static_cast<float*>(Y));
        }
      } else if (sizeof(T) == 4 && k_cols % 128 == 0) {
        // two column tiles at a time when the accumulators fit (fp32 and at least two tiles per wave)
        hipLaunchKernelGGL((mfma_forward_kernel<T, LMAX, 2>), dim3(grid), dim3(kThreads), 0, stream, n, k_red, k_cols,
                           static_cast<const T*>(X), static_cast<const T*>(W), static_cast<T*>(Y));
      } else {
        hipLaunchKernelGGL((mfma_forward_kernel<T, LMAX, 1>), dim3(grid), dim3(kThreads), 0, stream, n, k_red, k_cols,
                           static_cast<const T*>(X), static_cast<const T*>(W), static_cast<T*>(Y));
      }
      return hipGetLastError();
    }
  }
  const int64_t total = n * k_cols;
  hipLaunchKernelGGL((plain_forward_kernel<T, kTrans>), dim3(static_cast<unsigned>((total + 255) / 256)), dim3(256), 0,
                     stream, n, k_red, k_cols, LMAX, static_cast<const T*>(X), static_cast<const T*>(W),
                     static_cast<T*>(Y));
  return hipGetLastError();
}

template <typename T, bool kTrans>
hipError_t forward_t(int l_max, int64_t n, int k_red, int k_cols, const void* X, const void* W, void* Y,
                     hipStream_t stream) {
  switch (l_max) {
    case 0: return forward_l<T, 0, kTrans>(n, k_red, k_cols, X, W, Y, stream);
    case 1: return forward_l<T, 1, kTrans>(n, k_red, k_cols, X, W, Y, stream);
    case 2: return forward_l<T, 2, kTrans>(n, k_red, k_cols, X, W, Y, stream);
    default: return forward_l<T, 3, kTrans>(n, k_red, k_cols, X, W, Y, stream);
  }
}

template <typename T, int LMAX>
hipError_t dw_l(const el_config* cfg, int64_t n, const void* X, const void* dY, void* dW, void* ws,
                hipStream_t stream) {
  const int64_t elems = static_cast<int64_t>(LMAX + 1) * cfg->k_in * cfg->k_out;
  if (!mfma_dw_ok(cfg)) {
    hipLaunchKernelGGL((plain_dw_kernel<T>), dim3(static_cast<unsigned>((elems + 255) / 256)), dim3(256), 0, stream, n,
                       cfg->k_in, cfg->k_out, LMAX, static_cast<const T*>(X), static_cast<const T*>(dY),
                       static_cast<T*>(dW));
    return hipGetLastError();
  }
  const int per = nodes_per_range(cfg, n);
  const int ranges = static_cast<int>((n + per - 1) / per);
  if constexpr (sizeof(T) == 4 && LMAX == 3) {
    if (dw_lds_ok(cfg)) {
      const unsigned grid = static_cast<unsigned>(static_cast<int64_t>(ranges) * (cfg->k_in / 128) * (cfg->k_out / 64));
      hipLaunchKernelGGL(mfma_dw_lds_kernel, dim3(grid), dim3(kThreads), 0, stream, n, per, cfg->k_in, cfg->k_out,
                         static_cast<const float*>(X), static_cast<const float*>(dY), static_cast<float*>(ws));
      hipLaunchKernelGGL((dw_reduce_kernel<T>), dim3(static_cast<unsigned>((elems + 63) / 64)), dim3(256), 0, stream,
                         elems, ranges, static_cast<const T*>(ws), static_cast<T*>(dW));
      return hipGetLastError();
    }
  }
  // column tiles per workgroup: the accumulators (orders x tiles x 4 values) must fit the registers
  constexpr int NT = sizeof(T) == 4 ? 4 : 2;
  const unsigned grid = static_cast<unsigned>(static_cast<int64_t>(ranges) * (cfg->k_in / 64) * (cfg->k_out / (16 * NT)));
  hipLaunchKernelGGL((mfma_dw_kernel<T, LMAX, NT>), dim3(grid), dim3(kThreads), 0, stream, n, per, cfg->k_in,
                     cfg->k_out, static_cast<const T*>(X), static_cast<const T*>(dY), static_cast<T*>(ws));
  hipLaunchKernelGGL((dw_reduce_kernel<T>), dim3(static_cast<unsigned>((elems + 63) / 64)), dim3(256), 0, stream, elems,
                     ranges, static_cast<const T*>(ws), static_cast<T*>(dW));
  return hipGetLastError();
}

template <typename T>
hipError_t dw_t(const el_config* cfg, int64_t n, const void* X, const void* dY, void* dW, void* ws,
                hipStream_t stream) {
  switch (cfg->l_max) {
    case 0: return dw_l<T, 0>(cfg, n, X, dY, dW, ws, stream);
    case 1: return dw_l<T, 1>(cfg, n, X, dY, dW, ws, stream);
    case 2: return dw_l<T, 2>(cfg, n, X, dY, dW, ws, stream);
    default: return dw_l<T, 3>(cfg, n, X, dY, dW, ws, stream);
  }
}

// Workspace: [ W transposed, rounded up to 256 bytes ][ partial dW per range of atoms ].
size_t wt_bytes(const el_config* cfg) {
  if (!mfma_forward_ok(cfg->k_out, cfg->k_in)) return 0;   // the plain dX kernel reads W as it is
  const size_t bytes = static_cast<size_t>(cfg->l_max + 1) * cfg->k_in * cfg->k_out * elem_size(cfg);
  return (bytes + 255) / 256 * 256;
}

size_t workspace_bytes(const el_config* cfg, int64_t n) {
  if (n == 0) return 256;
  size_t bytes = wt_bytes(cfg);
  if (mfma_dw_ok(cfg)) {
    const int per = nodes_per_range(cfg, n);
    const int64_t ranges = (n + per - 1) / per;
    bytes += static_cast<size_t>(ranges) * (cfg->l_max + 1) * cfg->k_in * cfg->k_out * elem_size(cfg);
  }
  return (bytes + 255) / 256 * 256 + 256;
}

}  // namespace
}  // namespace el

extern "C" {

sc_status el_forward(const el_config* cfg, int64_t n_nodes, const void* X, const void* W, void* Y, void* hip_stream) {
  using namespace el;
  sc_status st = check_config("el_forward", cfg, n_nodes);
  if (st != SC_OK) return st;
  if (n_nodes == 0) return SC_OK;
  if (!X || !W || !Y) return set_error(SC_ERR_INVALID_ARG, "el_forward: NULL tensor argument");
  if (misaligned(X, 16) || misaligned(W, 16) || misaligned(Y, 16))
    return set_error(SC_ERR_INVALID_ARG, "el_forward: tensor pointer not 16-byte aligned");
  DeviceGuard guard(cfg->device);
  if (!guard.ok) return set_error(SC_ERR_HIP, "el_forward: cannot make cfg->device current");
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  const hipError_t e = cfg->dtype == SC_F64
                           ? forward_t<double, false>(cfg->l_max, n_nodes, cfg->k_in, cfg->k_out, X, W, Y, stream)
                           : forward_t<float, false>(cfg->l_max, n_nodes, cfg->k_in, cfg->k_out, X, W, Y, stream);
  if (e != hipSuccess) return set_error(SC_ERR_HIP, std::string("el_forward: kernel launch: ") + hipGetErrorString(e));
  return SC_OK;
}

sc_status el_workspace_bytes(const el_config* cfg, int64_t n_nodes, size_t* bytes) {
  using namespace el;
  sc_status st = check_config("el_workspace_bytes", cfg, n_nodes);
  if (st != SC_OK) return st;
  if (!bytes) return set_error(SC_ERR_INVALID_ARG, "el_workspace_bytes: bytes is NULL");
  *bytes = workspace_bytes(cfg, n_nodes);
  return SC_OK;
}

sc_status el_backward(const el_config* cfg, int64_t n_nodes, const void* X, const void* W, const void* dY, void* dX,
                      void* dW, void* workspace, size_t workspace_bytes_given, void* hip_stream) {
  using namespace el;
  sc_status st = check_config("el_backward", cfg, n_nodes);
  if (st != SC_OK) return st;
  if (!dW) return set_error(SC_ERR_INVALID_ARG, "el_backward: dW is NULL");
  if (misaligned(dW, 16)) return set_error(SC_ERR_INVALID_ARG, "el_backward: dW not 16-byte aligned");
  DeviceGuard guard(cfg->device);
  if (!guard.ok) return set_error(SC_ERR_HIP, "el_backward: cannot make cfg->device current");
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  if (n_nodes == 0) {
    const size_t words = elem_size(cfg) / 4 * static_cast<size_t>(cfg->l_max + 1) * cfg->k_in * cfg->k_out;
    hipLaunchKernelGGL(zero_kernel, dim3(64), dim3(256), 0, stream, static_cast<unsigned int*>(dW), words);
    const hipError_t e0 = hipGetLastError();
    if (e0 != hipSuccess) return set_error(SC_ERR_HIP, std::string("el_backward: fill launch: ") + hipGetErrorString(e0));
    return SC_OK;
  }
  if (!X || !W || !dY || !dX) return set_error(SC_ERR_INVALID_ARG, "el_backward: NULL tensor argument");
  if (misaligned(X, 16) || misaligned(W, 16) || misaligned(dY, 16) || misaligned(dX, 16))
    return set_error(SC_ERR_INVALID_ARG, "el_backward: tensor pointer not 16-byte aligned");
  if (!workspace || workspace_bytes_given < workspace_bytes(cfg, n_nodes))
    return set_error(SC_ERR_WORKSPACE, "el_backward: workspace missing or smaller than el_workspace_bytes()");
  if (misaligned(workspace, 256)) return set_error(SC_ERR_WORKSPACE, "el_backward: workspace not 256-byte aligned");
  // dX = dY times W transposed: reduction over the output channels, columns = input channels.  The MFMA
  // kernels take W transposed once into the workspace (strided B operands cost a third more time).
  hipError_t e;
  if (mfma_forward_ok(cfg->k_out, cfg->k_in)) {
    const int64_t elems = static_cast<int64_t>(cfg->l_max + 1) * cfg->k_in * cfg->k_out;
    const unsigned tgrid = static_cast<unsigned>((elems + 255) / 256);
    if (cfg->dtype == SC_F64)
      hipLaunchKernelGGL((transpose_w_kernel<double>), dim3(tgrid), dim3(256), 0, stream, cfg->l_max + 1, cfg->k_in,
                         cfg->k_out, static_cast<const double*>(W), static_cast<double*>(workspace));
    else
      hipLaunchKernelGGL((transpose_w_kernel<float>), dim3(tgrid), dim3(256), 0, stream, cfg->l_max + 1, cfg->k_in,
                         cfg->k_out, static_cast<const float*>(W), static_cast<float*>(workspace));
    e = hipGetLastError();
    if (e != hipSuccess) return set_error(SC_ERR_HIP, std::string("el_backward: transpose launch: ") + hipGetErrorString(e));
    e = cfg->dtype == SC_F64
            ? forward_t<double, false>(cfg->l_max, n_nodes, cfg->k_out, cfg->k_in, dY, workspace, dX, stream)
            : forward_t<float, false>(cfg->l_max, n_nodes, cfg->k_out, cfg->k_in, dY, workspace, dX, stream);
  } else {
    e = cfg->dtype == SC_F64
            ? forward_t<double, true>(cfg->l_max, n_nodes, cfg->k_out, cfg->k_in, dY, W, dX, stream)
            : forward_t<float, true>(cfg->l_max, n_nodes, cfg->k_out, cfg->k_in, dY, W, dX, stream);
  }
  if (e != hipSuccess) return set_error(SC_ERR_HIP, std::string("el_backward: dX launch: ") + hipGetErrorString(e));
  void* partials = static_cast<char*>(workspace) + wt_bytes(cfg);
  e = cfg->dtype == SC_F64 ? dw_t<double>(cfg, n_nodes, X, dY, dW, partials, stream)
                           : dw_t<float>(cfg, n_nodes, X, dY, dW, partials, stream);
  if (e != hipSuccess) return set_error(SC_ERR_HIP, std::string("el_backward: dW launch: ") + hipGetErrorString(e));
  return SC_OK;
}

}  // extern "C"
