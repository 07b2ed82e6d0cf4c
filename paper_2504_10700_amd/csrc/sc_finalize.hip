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

// Sparse fold (generated kernels).  One workgroup of 4 waves per (element, channel block):
// the waves first reduce the S internal rows over the element's tiles into LDS, then
// every external path gathers its few internal rows.
template <typename T>
__global__ __launch_bounds__(4 * kLanes) void finalize_fold_kernel(FoldTables fold, int P, int K, int chblocks,
                                                                   int max_tiles, const T* __restrict__ partial,
                                                                   const int32_t* __restrict__ tile_off,
                                                                   T* __restrict__ dW) {
  extern __shared__ double red[];  // [S][64]
  const int wave = threadIdx.x / kLanes, lane = threadIdx.x % kLanes;
  const int cb = blockIdx.x % chblocks;
  const int e = blockIdx.x / chblocks;
  int t0 = tile_off[e], t1 = tile_off[e + 1];
  if (t1 > max_tiles) t1 = max_tiles;
  const int S = fold.S;
  for (int s = wave; s < S; s += 4) {
    double acc = 0.0;
    for (int t = t0; t < t1; ++t)
      acc += static_cast<double>(partial[((static_cast<size_t>(t) * chblocks + cb) * S + s) * kLanes + lane]);
    red[s * kLanes + lane] = acc;
  }
  __syncthreads();
  const int ch = cb * kLanes + lane;
  for (int p = wave; p < P; p += 4) {
    double acc = 0.0;
    for (int i = fold.begin[p]; i < fold.begin[p + 1]; ++i) acc += fold.coef[i] * red[fold.src[i] * kLanes + lane];
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
    const size_t lds = static_cast<size_t>(plan->fold.S) * kLanes * sizeof(double);
    hipLaunchKernelGGL(finalize_fold_kernel<T>, dim3(Z * shape.chblocks), dim3(4 * kLanes), lds, stream, plan->fold,
                       P, K, shape.chblocks, shape.max_tiles, static_cast<const T*>(ws.partial), ws.tile_off,
                       static_cast<T*>(dW));
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
