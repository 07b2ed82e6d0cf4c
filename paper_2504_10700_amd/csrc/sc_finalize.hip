// Second stage of the dW reduction of the table-driven kernels: sums the per-tile
// contributions of every element in tile order (fixed order => bitwise reproducible, no
// floating-point atomics):  dW[e,p,k] = sum_{tiles t of element e} partial[t][cb(k)][p][lane(k)].
// Elements without nodes own no tiles and get exact zeros.  (The generated kernels have
// their own second stage, which also maps their internal path basis to the external one.)
#include "sc_internal.h"

namespace sc {
namespace {

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

template <typename T>
hipError_t finalize_t(const sc_plan* plan, void* dW, const Workspace& ws, const LaunchShape& shape,
                      hipStream_t stream) {
  const int P = static_cast<int>(plan->table.paths.size());
  const int Z = plan->cfg.num_elements, K = plan->cfg.num_channels;
  hipLaunchKernelGGL(finalize_direct_kernel<T>, dim3(Z * shape.chblocks * P), dim3(kLanes), 0, stream, P, K,
                     shape.chblocks, shape.max_tiles, static_cast<const T*>(ws.partial), ws.tile_off,
                     static_cast<T*>(dW));
  return hipGetLastError();
}

}  // namespace

hipError_t launch_finalize(const sc_plan* plan, void* dW, const Workspace& ws, const LaunchShape& shape,
                           hipStream_t stream) {
  return plan->cfg.dtype == SC_F64 ? finalize_t<double>(plan, dW, ws, shape, stream)
                                   : finalize_t<float>(plan, dW, ws, shape, stream);
}

}  // namespace sc
