// Pieces of the channel-mixing linear's MFMA kernels that the fused linear + contraction kernel
// shares: operand layouts of the 16x16x4 instruction, 64-byte row access, and the LDS-staged
// product of one 16-atom row tile.
#pragma once
#include "sc_internal.h"

namespace el {

using sc::kLanes;

constexpr int kWaves = 4;
constexpr int kThreads = kWaves * kLanes;

template <typename T>
struct Mma;
template <>
struct Mma<float> {
  typedef float acc_t __attribute__((ext_vector_type(4)));
  static __device__ __forceinline__ acc_t mma(float a, float b, acc_t c) {
    return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
  }
  static __device__ __forceinline__ int row(int lane, int r) { return 4 * (lane / 16) + r; }
};
template <>
struct Mma<double> {
  typedef double acc_t __attribute__((ext_vector_type(4)));
  static __device__ __forceinline__ acc_t mma(double a, double b, acc_t c) {
    return __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, c, 0, 0, 0);
  }
  static __device__ __forceinline__ int row(int lane, int r) { return 4 * r + lane / 16; }
};

__host__ __device__ constexpr int order_of(int c) { return c >= 9 ? 3 : c >= 4 ? 2 : c >= 1 ? 1 : 0; }

// N consecutive elements (16-byte accesses when the row is a multiple of 16 bytes).
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
      *reinterpret_cast<Vec*>(p + i) = x;
    }
  } else {
#pragma unroll
    for (int i = 0; i < N; ++i) p[i] = v[i];
  }
}

// The same product for fp32 and l_max = 3 (64-byte rows) with the A operands shared through
// LDS.  In the kernel above each of the four waves reads the whole X tile itself; those
// 16-byte accesses to 32 cache lines per instruction keep the vector memory path as busy as the
// matrix cores (measured: 30 us per row tile against 15 us of matrix time).  Here the
// workgroup stages X in chunks of 16 reduction channels (16 atoms x 16 channels x 64 B = 16 KB,
// two buffers): every thread loads 64 contiguous bytes once, all waves read their A operands
// from LDS (rows padded by 16 B against bank conflicts).  B operands (this wave's columns of
// W) are read from global memory one MFMA step ahead.  k_red % 16 == 0, k_cols % 128 == 0.
constexpr int kChunk = 16;                       // reduction channels per LDS chunk
constexpr int kRowPad = kChunk * 16 + 4;         // floats per atom row in LDS
constexpr int kBuffers = 2;                      // LDS buffers of 16 * kRowPad floats per workgroup

// lds_tile_product: the accumulators of rows n0..n0+15 and of this wave's CT column tiles of column
// group g (columns jc[t] per lane); xs = the workgroup's two staging buffers.
template <int CT>
__device__ __forceinline__ void lds_tile_product(int64_t n_nodes, int64_t n0, int g, int k_red, int k_cols,
                                                 const float* __restrict__ X, const float* __restrict__ W,
                                                 float* xs /* kBuffers * 16 * kRowPad floats */, typename Mma<float>::acc_t (&acc)[16][CT],
                                                 int (&jc)[CT]) {
  constexpr int NC = 16, L = 4, SPC = kChunk / 4;   // SPC: MFMA steps per chunk
  static_assert(SPC == 4, "the B operand sets rotate with period 4");
  typedef Mma<float>::acc_t acc_t;
  typedef float V4 __attribute__((ext_vector_type(4)));
  const int lane = threadIdx.x & (kLanes - 1);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kLanes);
  const int kq = lane / 16;
  const int chunks = k_red / kChunk;
  // staging role of this thread: atom tid/16 of the tile, reduction channel tid%16 of the chunk
  const int sn = threadIdx.x / 16, sk = threadIdx.x % 16;
  float* const swr = xs + sn * kRowPad + sk * 16;
  const float* const ard = xs + (lane & 15) * kRowPad + kq * 16;   // A operands of MFMA step 0 of a chunk
  int64_t ns = n0 + sn;
  if (ns >= n_nodes) ns = n_nodes - 1;       // rows past the end stage a valid atom and are not stored
  const float* xsrc = X + (static_cast<size_t>(ns) * k_red + sk) * NC;
#pragma unroll
  for (int t = 0; t < CT; ++t) jc[t] = ((g + t) * kWaves + wave) * 16 + (lane & 15);
#pragma unroll
  for (int c = 0; c < NC; ++c)
#pragma unroll
    for (int t = 0; t < CT; ++t) acc[c][t] = acc_t{0, 0, 0, 0};

  auto gload = [&](int chunk, V4 (&x)[4]) {
    const V4* p = reinterpret_cast<const V4*>(xsrc + static_cast<size_t>(chunk) * kChunk * NC);
#pragma unroll
    for (int i = 0; i < 4; ++i) x[i] = p[i];
  };
  auto stage = [&](int buf, const V4 (&x)[4]) {
    V4* p = reinterpret_cast<V4*>(swr + buf * 16 * kRowPad);
#pragma unroll
    for (int i = 0; i < 4; ++i) p[i] = x[i];
  };
  // B operands through a buffer descriptor of W: per load one 32-bit per-lane byte offset (it
  // advances by one MFMA step = 4 rows of W) and a scalar offset for the order, no 64-bit address
  // arithmetic in the loop; a read past the end of W would return zero instead of faulting.
  unsigned boff[CT];
#pragma unroll
  for (int t = 0; t < CT; ++t) boff[t] = static_cast<unsigned>(kq * k_cols + jc[t]) * 4u;
  const unsigned bstep = static_cast<unsigned>(k_cols) * 16u;                    // bytes per MFMA step
  const unsigned lstride = static_cast<unsigned>(k_red) * k_cols * 4u;           // bytes per order
  const __amdgpu_buffer_rsrc_t wrs =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(W), 0, static_cast<int>(L * lstride), 0x00020000);
  const int steps = chunks * SPC;
  auto bload = [&](int step, float (&b)[L][CT]) {   // B operands of one MFMA step
    const unsigned so = static_cast<unsigned>(step < steps ? step : steps - 1) * bstep;   // past the end: the last step again
#pragma unroll
    for (int l = 0; l < L; ++l)
#pragma unroll
      for (int t = 0; t < CT; ++t)
        b[l][t] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(wrs, static_cast<int>(boff[t] + so),
                                                                                 static_cast<int>(l * lstride), 0));
  };

  // Two LDS buffers, one barrier per chunk; B operands are requested kBDist MFMA steps before
  // their use (four register sets, of which kBDist + 1 are live at a time).
  constexpr int kBDist = 2;
  V4 xr[4];
  float b[4][L][CT];
  __syncthreads();                           // the previous unit's reads of both buffers are done
  gload(0, xr);
#pragma unroll
  for (int d = 0; d < kBDist; ++d) bload(d, b[d]);
  stage(0, xr);
  if (chunks > 1) gload(1, xr);
  __syncthreads();
  for (int c = 0; c < chunks; ++c) {
    const float* abuf = ard + (c & 1) * 16 * kRowPad;
#pragma unroll
    for (int st = 0; st < SPC; ++st) {       // SPC == 4: the roles of the four B sets repeat per chunk
      bload(c * SPC + st + kBDist, b[(st + kBDist) & 3]);
      const V4* p = reinterpret_cast<const V4*>(abuf + st * 4 * 16);
      V4 a4[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) a4[i] = p[i];
#pragma unroll
      for (int cc = 0; cc < NC; ++cc)
#pragma unroll
        for (int t = 0; t < CT; ++t)
          acc[cc][t] = Mma<float>::mma(a4[cc / 4][cc % 4], b[st & 3][order_of(cc)][t], acc[cc][t]);
    }
    if (c + 1 < chunks) {
      stage((c + 1) & 1, xr);
      if (c + 2 < chunks) gload(c + 2, xr);
    }
    __syncthreads();
  }
}

// Store of a wave's result tile Y[n0 + 4*(lane/16) + r][jc[t]][0..15].  A lane holds whole 64-byte
// rows; stored directly, every instruction would write a quarter of each row (16-byte pieces 64
// bytes apart: partial lines, four times the write requests).  Per (t, r) the 16 rows of a
// 16-lane group are one contiguous KB of Y: they go through LDS (rows padded to 80 bytes) and
// come back so that instruction i writes the i-th contiguous 256 bytes of each KB, streamed past
// the cache.  stage: kStoreStageFloats floats of LDS owned by this wave; the caller puts a
// workgroup barrier between the last LDS read of the product and this call when the stage
// overlaps the product's buffers.  Measured on the forward kernel (10k atoms): 87 -> 73.5 us.
constexpr int kStoreRow = 20;                          // floats per staged row
constexpr int kStoreStageFloats = 4 * 16 * kStoreRow;  // per wave

template <int CT>
__device__ __forceinline__ void store_tile_coalesced(float* __restrict__ Y, int64_t n_nodes, int64_t n0, int k_cols,
                                                     const int (&jc)[CT],
                                                     const typename Mma<float>::acc_t (&acc)[16][CT], float* stage) {
  typedef float V4 __attribute__((ext_vector_type(4)));
  const int lane = threadIdx.x & (kLanes - 1);
  const int q = lane / 16, j16 = lane & 15;
  float* const mine = stage + (q * 16 + j16) * kStoreRow;
#pragma unroll
  for (int t = 0; t < CT; ++t)
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");   // the previous round's reads of the stage are done
      __builtin_amdgcn_wave_barrier();
#pragma unroll
      for (int i = 0; i < 4; ++i)
        *reinterpret_cast<V4*>(mine + 4 * i) = V4{acc[4 * i][t][r], acc[4 * i + 1][t][r], acc[4 * i + 2][t][r], acc[4 * i + 3][t][r]};
      __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");   // the other lanes' rows are visible
      __builtin_amdgcn_wave_barrier();
      const int64_t n = n0 + Mma<float>::row(lane, r);
      if (n < n_nodes) {
        float* yblock = Y + (static_cast<size_t>(n) * k_cols + (jc[t] - j16)) * 16;   // the group's KB
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int p = i * 16 + j16;                  // 16-byte piece of the KB: row p / 4, quarter p % 4
          const V4 x = *reinterpret_cast<const V4*>(stage + (q * 16 + p / 4) * kStoreRow + (p % 4) * 4);
          __builtin_nontemporal_store(x, reinterpret_cast<V4*>(yblock + p * 4));
        }
      }
    }
}

// Work of a persistent grid of S workgroups over U full units (row tile x 128 columns), two
// workgroups per CU (workgroups b and b + S/2 share a CU: read from the hardware id registers).
// Two workgroups that start together tend to stay in step: both run their matrix phase, then
// both their epilogue (stores, or the contraction).  So the second half of the grid starts with
// HALF a unit (64 columns) and is from then on half a phase away from its neighbour, whose matrix
// work then covers its epilogue and vice versa (measured: -4% on the fused kernel, about neutral
// on the plain linear).  The last n_split = min(U, S/4) full units are cut into the 2 n_split
// halves; the other units go round the workgroups as usual.  stagger = false: no halves.
struct UnitSchedule {
  bool has_half;
  int64_t half_unit;   // full unit that the half belongs to
  int half;            // which half of it (0 or 1)
  int64_t n_full;      // full units 0 .. n_full-1 are dealt blockIdx.x, blockIdx.x + gridDim.x, ...
};

__device__ __forceinline__ UnitSchedule unit_schedule(int64_t full_units, bool stagger) {
  const int S = gridDim.x, b = blockIdx.x;
  UnitSchedule u{false, 0, 0, full_units};
  if (!stagger || S % 4 != 0) return u;
  const int64_t n_split = full_units < S / 4 ? full_units : S / 4;
  u.n_full = full_units - n_split;
  const int rank = b - S / 2;
  if (rank >= 0 && rank < 2 * n_split) {
    u.has_half = true;
    u.half_unit = full_units - 1 - rank / 2;
    u.half = rank & 1;
  }
  return u;
}

}  // namespace el
