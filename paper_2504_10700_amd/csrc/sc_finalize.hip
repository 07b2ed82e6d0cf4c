// Second stage of the dW reduction: sums the per-tile contributions of every element in
// tile order (fixed order => bitwise reproducible, no floating-point atomics) and maps
// the internal path basis back to the external one.
//
//   dW[e,p,k] = sum_{s} fold[p,s] * sum_{tiles t of element e} partial[t][cb(k)][s][lane(k)]
//
// Elements without nodes own no tiles and get exact zeros.
#include "sc_internal.h"

namespace sc {
namespace {

// Identity fold (table-driven kernels: internal basis == external paths).
// One wave per (element, channel block, path).
template <typename T>
__global__ __launch_bounds__(kLanes) void finalize_direct_kernel(int P, int K, int chblocks, int max_tiles,
                                                                 const T* __restrict__ partial,
                                                                 const int32_t* __restrict__ tile_off,
                                                                 T* __restrict__ dW) {
  const int lane = threadIdx.x;
  const int p = blockIdx.x % P;
  const int cb = (blockIdx.x / P) % chblocks;
  const int e = blockIdx.x / (P * chblocks);
  int t0 = tile_off[e], t1 = tile_off[e + 1];
  if (t1 > max_tiles) t1 = max_tiles;
  double acc = 0.0;
  for (int t = t0; t < t1; ++t)
    acc += static_cast<double>(partial[((static_cast<size_t>(t) * chblocks + cb) * P + p) * kLanes + lane]);
  const int ch = cb * kLanes + lane;
  if (ch < K) dW[(static_cast<size_t>(e) * P + p) * K + ch] = static_cast<T>(acc);
}

// Sparse fold (generated kernels).  One workgroup of 8 waves per (element, channel block):
// the fold table is staged in LDS, the waves reduce the S internal rows over the element's
// tiles into LDS (independent loads, four in flight per row), then every external path
// gathers its few internal rows.
constexpr int kFinalizeWaves = 8;

template <typename T>
__global__ __launch_bounds__(kFinalizeWaves * kLanes) void finalize_fold_kernel(
    FoldTables fold, int nnz, int P, int K, int chblocks, int max_tiles, const T* __restrict__ partial,
    const int32_t* __restrict__ tile_off, T* __restrict__ dW) {
  extern __shared__ double lds_d[];
  const int S = fold.S;
  double* red = lds_d;                                       // [S][64]
  double* fcoef = red + S * kLanes;                          // [nnz]
  int32_t* fsrc = reinterpret_cast<int32_t*>(fcoef + nnz);   // [nnz]
  int32_t* fbegin = fsrc + nnz;                              // [P+1]
  const int wave = threadIdx.x / kLanes, lane = threadIdx.x % kLanes;
  for (int i = threadIdx.x; i < nnz; i += blockDim.x) {
    fcoef[i] = fold.coef[i];
    fsrc[i] = fold.src[i];
  }
  for (int i = threadIdx.x; i <= P; i += blockDim.x) fbegin[i] = fold.begin[i];
  const int cb = blockIdx.x % chblocks;
  const int e = blockIdx.x / chblocks;
  int t0 = tile_off[e], t1 = tile_off[e + 1];
  if (t1 > max_tiles) t1 = max_tiles;
  const size_t tstride = static_cast<size_t>(chblocks) * S * kLanes;
  for (int s = wave; s < S; s += kFinalizeWaves) {
    const T* src = partial + (static_cast<size_t>(cb) * S + s) * kLanes + lane;
    double a0 = 0.0, a1 = 0.0, a2 = 0.0, a3 = 0.0;
    int t = t0;
    for (; t + 4 <= t1; t += 4) {
      const T v0 = src[(t + 0) * tstride], v1 = src[(t + 1) * tstride];
      const T v2 = src[(t + 2) * tstride], v3 = src[(t + 3) * tstride];
      a0 += static_cast<double>(v0);
      a1 += static_cast<double>(v1);
      a2 += static_cast<double>(v2);
      a3 += static_cast<double>(v3);
    }
    for (; t < t1; ++t) a0 += static_cast<double>(src[t * tstride]);
    red[s * kLanes + lane] = (a0 + a1) + (a2 + a3);
  }
  __syncthreads();
  const int ch = cb * kLanes + lane;
  for (int p = wave; p < P; p += kFinalizeWaves) {
    double acc = 0.0;
    for (int i = fbegin[p]; i < fbegin[p + 1]; ++i) acc += fcoef[i] * red[fsrc[i] * kLanes + lane];
    if (ch < K) dW[(static_cast<size_t>(e) * P + p) * K + ch] = static_cast<T>(acc);
  }
}

template <typename T>
hipError_t finalize_t(const sc_plan* plan, void* dW, const Workspace& ws, const LaunchShape& shape,
                      hipStream_t stream) {
  const int P = static_cast<int>(plan->table.paths.size());
  const int Z = plan->cfg.num_elements, K = plan->cfg.num_channels;
  if (plan->specialised == 0) {
    hipLaunchKernelGGL(finalize_direct_kernel<T>, dim3(Z * shape.chblocks * P), dim3(kLanes), 0, stream, P, K,
                       shape.chblocks, shape.max_tiles, static_cast<const T*>(ws.partial), ws.tile_off,
                       static_cast<T*>(dW));
  } else {
    const int nnz = plan->fold_nnz;
    const size_t lds = static_cast<size_t>(plan->fold.S) * kLanes * sizeof(double) + nnz * sizeof(double) +
                       (nnz + P + 1) * sizeof(int32_t);
    hipLaunchKernelGGL(finalize_fold_kernel<T>, dim3(Z * shape.chblocks), dim3(kFinalizeWaves * kLanes), lds, stream,
                       plan->fold, nnz, P, K, shape.chblocks, shape.max_tiles, static_cast<const T*>(ws.partial),
                       ws.tile_off, static_cast<T*>(dW));
  }
  return hipGetLastError();
}

}  // namespace

hipError_t launch_finalize(const sc_plan* plan, void* dW, const Workspace& ws, const LaunchShape& shape,
                           hipStream_t stream) {
  return plan->cfg.dtype == SC_F64 ? finalize_t<double>(plan, dW, ws, shape, stream)
                                   : finalize_t<float>(plan, dW, ws, shape, stream);
}

}  // namespace sc
