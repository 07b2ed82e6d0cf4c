// Table-driven kernels for any supported configuration (the fallback when no generated
// straight-line kernel exists).  They evaluate Algorithm 2 of arXiv 2504.10700 from the
// sparse, permutation-merged terms of every coupling path:
//
//   P_{p,M}(a) = sum_t coef_t * a[i1_t] * a[i2_t] * a[i3_t]           (terms of path p, component M)
//   B[LM]      = sum_p W[z,p,k] * P_{p,M}(a)
//   dA[i]      = sum_p W[z,p,k] * sum_t dB[col_p+M_t] * coef_t * d(monomial_t)/da[i]
//   dW'[p]     = sum_{nodes of the tile} sum_M dB[col_p+M] * P_{p,M}(a)
// and, for the second-order pass with the cotangent h of dA (D_h = derivative along h),
//   ddB[LM]    = sum_p W[z,p,k] * D_h P_{p,M}(a)
//   dA2[i]     = sum_p W[z,p,k] * sum_t dB[col_p+M_t] * coef_t * d(D_h monomial_t)/da[i]
//   dW2'[p]    = sum_{nodes of the tile} sum_M dB[col_p+M] * D_h P_{p,M}(a)
//
// One wave per tile (a run of nodes of one element) and 64-channel block; lane = channel.
// The per-node vectors a, dB/B and dA live in LDS columns (one column per lane) because
// the tables index them dynamically.  All arithmetic is done in fp64 whatever the storage
// type T: a flat fp32 sum over the ~1500 terms of a gradient component does not meet the
// 1e-5 (relative to rms) acceptance bound, and fp64 vector FMAs issue at the same rate as
// unpacked fp32 ones on this chip.
#include "sc_internal.h"

namespace sc {
namespace {

template <typename T>
__global__ __launch_bounds__(kLanes) void generic_forward_kernel(GenericTables tab, int K, int chblocks,
                                                                 const T* __restrict__ A, const T* __restrict__ W,
                                                                 T* __restrict__ B,
                                                                 const int32_t* __restrict__ ntiles,
                                                                 const TileDesc* __restrict__ tiles,
                                                                 const int32_t* __restrict__ perm) {
  extern __shared__ unsigned char lds_raw[];
  double* sA = reinterpret_cast<double*>(lds_raw);  // [n_lm][64]
  double* sB = sA + tab.n_lm * kLanes;              // [n_LM][64]
  const int lane = threadIdx.x;
  const int tile = blockIdx.x / chblocks, cb = blockIdx.x % chblocks;
  if (tile >= *ntiles) return;
  const TileDesc td = tiles[tile];
  const int ch = cb * kLanes + lane;
  const bool active = ch < K;
  const double* coef = tab.term_coef;
  const T* Wz = W + static_cast<size_t>(td.z) * tab.num_paths * K;
  for (int j = 0; j < td.count; ++j) {
    const size_t node = perm[td.start + j];
    if (active) {
      const T* a = A + (node * K + ch) * tab.n_lm;
      for (int i = 0; i < tab.n_lm; ++i) sA[i * kLanes + lane] = a[i];
    } else {
      for (int i = 0; i < tab.n_lm; ++i) sA[i * kLanes + lane] = 0.0;
    }
    for (int i = 0; i < tab.n_LM; ++i) sB[i * kLanes + lane] = 0.0;
    for (int p = 0; p < tab.num_paths; ++p) {
      const double w = active ? Wz[static_cast<size_t>(p) * K + ch] : 0.0;
      const int nu = tab.path_nu[p], col = tab.path_col[p];
      const int t0 = tab.term_begin[p], t1 = tab.term_begin[p + 1];
      int curM = -1;
      double acc = 0.0;
      for (int t = t0; t < t1; ++t) {
        const int4 ix = tab.term_idx[t];
        if (ix.x != curM) {
          if (curM >= 0) sB[(col + curM) * kLanes + lane] += w * acc;
          curM = ix.x;
          acc = 0.0;
        }
        double v = coef[t] * sA[ix.y * kLanes + lane];
        if (nu >= 2) v *= sA[ix.z * kLanes + lane];
        if (nu >= 3) v *= sA[ix.w * kLanes + lane];
        acc += v;
      }
      if (curM >= 0) sB[(col + curM) * kLanes + lane] += w * acc;
    }
    if (active) {
      T* b = B + (node * K + ch) * tab.n_LM;
      for (int i = 0; i < tab.n_LM; ++i) b[i] = static_cast<T>(sB[i * kLanes + lane]);
    }
  }
}

template <typename T>
__global__ __launch_bounds__(kLanes) void generic_backward_kernel(GenericTables tab, int K, int chblocks,
                                                                  const T* __restrict__ A, const T* __restrict__ W,
                                                                  const T* __restrict__ dB, T* __restrict__ dA,
                                                                  T* __restrict__ partial,
                                                                  const int32_t* __restrict__ ntiles,
                                                                  const TileDesc* __restrict__ tiles,
                                                                  const int32_t* __restrict__ perm) {
  extern __shared__ unsigned char lds_raw[];
  double* sA = reinterpret_cast<double*>(lds_raw);  // [n_lm][64]
  double* sG = sA + tab.n_lm * kLanes;              // [n_LM][64]  upstream gradient
  double* sD = sG + tab.n_LM * kLanes;              // [n_lm][64]  dA accumulators
  const int lane = threadIdx.x;
  const int tile = blockIdx.x / chblocks, cb = blockIdx.x % chblocks;
  if (tile >= *ntiles) return;
  const TileDesc td = tiles[tile];
  const int ch = cb * kLanes + lane;
  const bool active = ch < K;
  const double* coef = tab.term_coef;
  const T* Wz = W + static_cast<size_t>(td.z) * tab.num_paths * K;
  // this wave's private rows of the partial buffer: [tile][cb][p][lane]
  T* part = partial + (static_cast<size_t>(tile) * chblocks + cb) * tab.num_paths * kLanes;
  for (int j = 0; j < td.count; ++j) {
    const size_t node = perm[td.start + j];
    if (active) {
      const T* a = A + (node * K + ch) * tab.n_lm;
      const T* g = dB + (node * K + ch) * tab.n_LM;
      for (int i = 0; i < tab.n_lm; ++i) sA[i * kLanes + lane] = a[i];
      for (int i = 0; i < tab.n_LM; ++i) sG[i * kLanes + lane] = g[i];
    } else {
      for (int i = 0; i < tab.n_lm; ++i) sA[i * kLanes + lane] = 0.0;
      for (int i = 0; i < tab.n_LM; ++i) sG[i * kLanes + lane] = 0.0;
    }
    for (int i = 0; i < tab.n_lm; ++i) sD[i * kLanes + lane] = 0.0;
    for (int p = 0; p < tab.num_paths; ++p) {
      const double w = active ? Wz[static_cast<size_t>(p) * K + ch] : 0.0;
      const int nu = tab.path_nu[p], col = tab.path_col[p];
      const int t0 = tab.term_begin[p], t1 = tab.term_begin[p + 1];
      double gp = 0.0;
      for (int t = t0; t < t1; ++t) {
        const int4 ix = tab.term_idx[t];
        const double gc = sG[(col + ix.x) * kLanes + lane] * coef[t];
        const double a1 = sA[ix.y * kLanes + lane];
        const double a2 = (nu >= 2) ? sA[ix.z * kLanes + lane] : 1.0;
        const double a3 = (nu >= 3) ? sA[ix.w * kLanes + lane] : 1.0;
        gp += gc * a1 * a2 * a3;
        const double gw = gc * w;
        sD[ix.y * kLanes + lane] += gw * a2 * a3;
        if (nu >= 2) sD[ix.z * kLanes + lane] += gw * a1 * a3;
        if (nu >= 3) sD[ix.w * kLanes + lane] += gw * a1 * a2;
      }
      T* slot = part + static_cast<size_t>(p) * kLanes + lane;
      *slot = static_cast<T>((j == 0) ? gp : (static_cast<double>(*slot) + gp));
    }
    if (active) {
      T* d = dA + (node * K + ch) * tab.n_lm;
      for (int i = 0; i < tab.n_lm; ++i) d[i] = static_cast<T>(sD[i * kLanes + lane]);
    }
  }
}

template <typename T>
__global__ __launch_bounds__(kLanes) void generic_double_backward_kernel(
    GenericTables tab, int K, int chblocks, const T* __restrict__ A, const T* __restrict__ W,
    const T* __restrict__ dB, const T* __restrict__ H, T* __restrict__ ddB, T* __restrict__ dA2,
    T* __restrict__ partial, const int32_t* __restrict__ ntiles, const TileDesc* __restrict__ tiles,
    const int32_t* __restrict__ perm) {
  extern __shared__ unsigned char lds_raw[];
  double* sA = reinterpret_cast<double*>(lds_raw);  // [n_lm][64]
  double* sH = sA + tab.n_lm * kLanes;              // [n_lm][64]  cotangent of dA
  double* sG = sH + tab.n_lm * kLanes;              // [n_LM][64]  upstream gradient dB
  double* sD = sG + tab.n_LM * kLanes;              // [n_lm][64]  dA2 accumulators
  double* sB = sD + tab.n_lm * kLanes;              // [n_LM][64]  ddB accumulators
  const int lane = threadIdx.x;
  const int tile = blockIdx.x / chblocks, cb = blockIdx.x % chblocks;
  if (tile >= *ntiles) return;
  const TileDesc td = tiles[tile];
  const int ch = cb * kLanes + lane;
  const bool active = ch < K;
  const double* coef = tab.term_coef;
  const T* Wz = W + static_cast<size_t>(td.z) * tab.num_paths * K;
  T* part = partial + (static_cast<size_t>(tile) * chblocks + cb) * tab.num_paths * kLanes;
  for (int j = 0; j < td.count; ++j) {
    const size_t node = perm[td.start + j];
    if (active) {
      const T* a = A + (node * K + ch) * tab.n_lm;
      const T* h = H + (node * K + ch) * tab.n_lm;
      const T* g = dB + (node * K + ch) * tab.n_LM;
      for (int i = 0; i < tab.n_lm; ++i) sA[i * kLanes + lane] = a[i];
      for (int i = 0; i < tab.n_lm; ++i) sH[i * kLanes + lane] = h[i];
      for (int i = 0; i < tab.n_LM; ++i) sG[i * kLanes + lane] = g[i];
    } else {
      for (int i = 0; i < tab.n_lm; ++i) sA[i * kLanes + lane] = 0.0;
      for (int i = 0; i < tab.n_lm; ++i) sH[i * kLanes + lane] = 0.0;
      for (int i = 0; i < tab.n_LM; ++i) sG[i * kLanes + lane] = 0.0;
    }
    for (int i = 0; i < tab.n_lm; ++i) sD[i * kLanes + lane] = 0.0;
    for (int i = 0; i < tab.n_LM; ++i) sB[i * kLanes + lane] = 0.0;
    for (int p = 0; p < tab.num_paths; ++p) {
      const double w = active ? Wz[static_cast<size_t>(p) * K + ch] : 0.0;
      const int nu = tab.path_nu[p], col = tab.path_col[p];
      const int t0 = tab.term_begin[p], t1 = tab.term_begin[p + 1];
      double gp = 0.0;
      for (int t = t0; t < t1; ++t) {
        const int4 ix = tab.term_idx[t];
        const double c = coef[t];
        const double g = sG[(col + ix.x) * kLanes + lane];
        // unused slots behave as the constant 1 with tangent 0
        const double a1 = sA[ix.y * kLanes + lane], h1 = sH[ix.y * kLanes + lane];
        const double a2 = (nu >= 2) ? sA[ix.z * kLanes + lane] : 1.0, h2 = (nu >= 2) ? sH[ix.z * kLanes + lane] : 0.0;
        const double a3 = (nu >= 3) ? sA[ix.w * kLanes + lane] : 1.0, h3 = (nu >= 3) ? sH[ix.w * kLanes + lane] : 0.0;
        const double d1 = h2 * a3 + a2 * h3;  // D_h of the monomial without slot 1
        const double d2 = h1 * a3 + a1 * h3;
        const double d3 = h1 * a2 + a1 * h2;
        const double tang = c * (h1 * a2 * a3 + a1 * d1);
        sB[(col + ix.x) * kLanes + lane] += w * tang;
        gp += g * tang;
        const double gw = g * c * w;
        if (nu >= 2) {
          sD[ix.y * kLanes + lane] += gw * d1;
          sD[ix.z * kLanes + lane] += gw * d2;
        }
        if (nu >= 3) sD[ix.w * kLanes + lane] += gw * d3;
      }
      T* slot = part + static_cast<size_t>(p) * kLanes + lane;
      *slot = static_cast<T>((j == 0) ? gp : (static_cast<double>(*slot) + gp));
    }
    if (active) {
      T* d = dA2 + (node * K + ch) * tab.n_lm;
      T* b = ddB + (node * K + ch) * tab.n_LM;
      for (int i = 0; i < tab.n_lm; ++i) d[i] = static_cast<T>(sD[i * kLanes + lane]);
      for (int i = 0; i < tab.n_LM; ++i) b[i] = static_cast<T>(sB[i * kLanes + lane]);
    }
  }
}

template <typename T>
hipError_t fwd_t(const sc_plan* plan, const void* A, const void* W, void* B, const Workspace& ws,
                 const LaunchShape& shape, hipStream_t stream) {
  const GenericTables& g = plan->gen;
  const size_t lds = static_cast<size_t>(g.n_lm + g.n_LM) * kLanes * sizeof(double);
  hipLaunchKernelGGL(generic_forward_kernel<T>, dim3(shape.max_tiles * shape.chblocks), dim3(kLanes), lds, stream, g,
                     plan->cfg.num_channels, shape.chblocks, static_cast<const T*>(A), static_cast<const T*>(W),
                     static_cast<T*>(B), ws.ntiles, ws.tiles, ws.perm);
  return hipGetLastError();
}

template <typename T>
hipError_t bwd_t(const sc_plan* plan, const void* A, const void* W, const void* dB, void* dA, const Workspace& ws,
                 const LaunchShape& shape, hipStream_t stream) {
  const GenericTables& g = plan->gen;
  const size_t lds = static_cast<size_t>(2 * g.n_lm + g.n_LM) * kLanes * sizeof(double);
  hipLaunchKernelGGL(generic_backward_kernel<T>, dim3(shape.max_tiles * shape.chblocks), dim3(kLanes), lds, stream, g,
                     plan->cfg.num_channels, shape.chblocks, static_cast<const T*>(A), static_cast<const T*>(W),
                     static_cast<const T*>(dB), static_cast<T*>(dA), static_cast<T*>(ws.partial), ws.ntiles,
                     ws.tiles, ws.perm);
  return hipGetLastError();
}

template <typename T>
hipError_t dbl_t(const sc_plan* plan, const void* A, const void* W, const void* dB, const void* H, void* ddB,
                 void* dA2, const Workspace& ws, const LaunchShape& shape, hipStream_t stream) {
  const GenericTables& g = plan->gen;
  const size_t lds = static_cast<size_t>(3 * g.n_lm + 2 * g.n_LM) * kLanes * sizeof(double);
  hipLaunchKernelGGL(generic_double_backward_kernel<T>, dim3(shape.max_tiles * shape.chblocks), dim3(kLanes), lds,
                     stream, g, plan->cfg.num_channels, shape.chblocks, static_cast<const T*>(A),
                     static_cast<const T*>(W), static_cast<const T*>(dB), static_cast<const T*>(H),
                     static_cast<T*>(ddB), static_cast<T*>(dA2), static_cast<T*>(ws.partial), ws.ntiles, ws.tiles,
                     ws.perm);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_generic_forward(const sc_plan* plan, int64_t, const void* A, const void* W, void* B,
                                  const Workspace& ws, const LaunchShape& shape, hipStream_t stream) {
  return plan->cfg.dtype == SC_F64 ? fwd_t<double>(plan, A, W, B, ws, shape, stream)
                                   : fwd_t<float>(plan, A, W, B, ws, shape, stream);
}

hipError_t launch_generic_backward(const sc_plan* plan, int64_t, const void* A, const void* W, const void* dB,
                                   void* dA, const Workspace& ws, const LaunchShape& shape, hipStream_t stream) {
  return plan->cfg.dtype == SC_F64 ? bwd_t<double>(plan, A, W, dB, dA, ws, shape, stream)
                                   : bwd_t<float>(plan, A, W, dB, dA, ws, shape, stream);
}

hipError_t launch_generic_double_backward(const sc_plan* plan, int64_t, const void* A, const void* W,
                                          const void* dB, const void* H, void* ddB, void* dA2,
                                          const Workspace& ws, const LaunchShape& shape, hipStream_t stream) {
  return plan->cfg.dtype == SC_F64 ? dbl_t<double>(plan, A, W, dB, H, ddB, dA2, ws, shape, stream)
                                   : dbl_t<float>(plan, A, W, dB, H, ddB, dA2, ws, shape, stream);
}

}  // namespace sc
