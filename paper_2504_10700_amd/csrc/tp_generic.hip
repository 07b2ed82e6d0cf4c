// Table-driven kernels of the channelwise tensor product for any supported configuration
// (the fallback when no generated straight-line kernel exists).  Algorithm 1 of
// arXiv 2504.10700 with the pooling over the receiver's edges, from the sparse terms
//
//   msg[c] += coef * R[p] * Y[a] * h[b]                     (term = (p, a, b, c, coef))
//
// lane = channel; one wave per (atom, 64-channel block) walks the atom's edges.  Per-lane
// vectors live in LDS columns because the table indexes them dynamically; arithmetic is fp64
// whatever the storage type (fp64 vector FMAs issue at the unpacked fp32 rate on this chip).
#include "tp_internal.h"

namespace tp {
namespace {

using sc::kLanes;

__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
  for (int d = kLanes / 2; d >= 1; d >>= 1) v += __shfl_xor(v, d);
  return v;
}

// A[i] = sum over the edges received by i.
template <typename T>
__global__ __launch_bounds__(kLanes) void generic_forward_kernel(TermTable tab, int K, int chblocks,
                                                                 const T* __restrict__ Y, const T* __restrict__ h,
                                                                 const T* __restrict__ R,
                                                                 const int32_t* __restrict__ sender,
                                                                 const int32_t* __restrict__ row_ptr,
                                                                 T* __restrict__ A) {
  extern __shared__ unsigned char lds_raw[];
  double* sH = reinterpret_cast<double*>(lds_raw);  // [n_h][64]
  double* sR = sH + tab.n_h * kLanes;               // [P][64]
  double* sA = sR + tab.num_paths * kLanes;         // [n_out][64]
  const int lane = threadIdx.x;
  const size_t node = blockIdx.x / chblocks;
  const int cb = blockIdx.x % chblocks;
  const int ch = cb * kLanes + lane;
  const bool active = ch < K;
  for (int c = 0; c < tab.n_out; ++c) sA[c * kLanes + lane] = 0.0;
  const int e0 = row_ptr[node], e1 = row_ptr[node + 1];
  for (int e = e0; e < e1; ++e) {
    const size_t j = sender[e];
    for (int b = 0; b < tab.n_h; ++b) sH[b * kLanes + lane] = active ? static_cast<double>(h[(j * K + ch) * tab.n_h + b]) : 0.0;
    for (int p = 0; p < tab.num_paths; ++p)
      sR[p * kLanes + lane] = active ? static_cast<double>(R[(static_cast<size_t>(e) * tab.num_paths + p) * K + ch]) : 0.0;
    const T* y = Y + static_cast<size_t>(e) * tab.n_Y;
    for (int t = 0; t < tab.n_terms; ++t) {
      const int4 ix = tab.idx[t];
      sA[ix.w * kLanes + lane] += tab.coef[t] * sR[ix.x * kLanes + lane] * static_cast<double>(y[ix.y]) * sH[ix.z * kLanes + lane];
    }
  }
  if (active)
    for (int c = 0; c < tab.n_out; ++c) A[(node * K + ch) * tab.n_out + c] = static_cast<T>(sA[c * kLanes + lane]);
}

// Receiver side of the backward: dR of every edge and the per-channel-block partial of dY.
template <typename T>
__global__ __launch_bounds__(kLanes) void generic_backward_recv_kernel(
    TermTable tab, int K, int chblocks, int64_t n_edges, const T* __restrict__ Y, const T* __restrict__ h,
    const T* __restrict__ R, const int32_t* __restrict__ sender, const int32_t* __restrict__ row_ptr,
    const T* __restrict__ dA, T* __restrict__ dR, T* __restrict__ dY_partial) {
  extern __shared__ unsigned char lds_raw[];
  double* sH = reinterpret_cast<double*>(lds_raw);  // [n_h][64]
  double* sR = sH + tab.n_h * kLanes;               // [P][64]
  double* sG = sR + tab.num_paths * kLanes;         // [n_out][64]  dA of the receiver
  double* sDR = sG + tab.n_out * kLanes;            // [P][64]
  double* sDY = sDR + tab.num_paths * kLanes;       // [n_Y][64]    this lane's share of dY
  const int lane = threadIdx.x;
  const size_t node = blockIdx.x / chblocks;
  const int cb = blockIdx.x % chblocks;
  const int ch = cb * kLanes + lane;
  const bool active = ch < K;
  for (int c = 0; c < tab.n_out; ++c)
    sG[c * kLanes + lane] = active ? static_cast<double>(dA[(node * K + ch) * tab.n_out + c]) : 0.0;
  const int e0 = row_ptr[node], e1 = row_ptr[node + 1];
  for (int e = e0; e < e1; ++e) {
    const size_t j = sender[e];
    for (int b = 0; b < tab.n_h; ++b) sH[b * kLanes + lane] = active ? static_cast<double>(h[(j * K + ch) * tab.n_h + b]) : 0.0;
    for (int p = 0; p < tab.num_paths; ++p) {
      sR[p * kLanes + lane] = active ? static_cast<double>(R[(static_cast<size_t>(e) * tab.num_paths + p) * K + ch]) : 0.0;
      sDR[p * kLanes + lane] = 0.0;
    }
    for (int a = 0; a < tab.n_Y; ++a) sDY[a * kLanes + lane] = 0.0;
    const T* y = Y + static_cast<size_t>(e) * tab.n_Y;
    for (int t = 0; t < tab.n_terms; ++t) {
      const int4 ix = tab.idx[t];
      const double gh = tab.coef[t] * sG[ix.w * kLanes + lane] * sH[ix.z * kLanes + lane];
      sDR[ix.x * kLanes + lane] += gh * static_cast<double>(y[ix.y]);
      sDY[ix.y * kLanes + lane] += gh * sR[ix.x * kLanes + lane];
    }
    if (active)
      for (int p = 0; p < tab.num_paths; ++p)
        dR[(static_cast<size_t>(e) * tab.num_paths + p) * K + ch] = static_cast<T>(sDR[p * kLanes + lane]);
    for (int a = 0; a < tab.n_Y; ++a) {
      const double s = wave_sum(sDY[a * kLanes + lane]);
      if (lane == 0) dY_partial[(static_cast<size_t>(cb) * n_edges + e) * tab.n_Y + a] = static_cast<T>(s);
    }
  }
}

// Sender side of the backward: dh[j] = sum over the edges sent by j.
template <typename T>
__global__ __launch_bounds__(kLanes) void generic_backward_send_kernel(
    TermTable tab, int K, int chblocks, const T* __restrict__ Y, const T* __restrict__ R,
    const int32_t* __restrict__ receiver, const int32_t* __restrict__ send_ptr,
    const int32_t* __restrict__ send_edge, const T* __restrict__ dA, T* __restrict__ dh) {
  extern __shared__ unsigned char lds_raw[];
  double* sR = reinterpret_cast<double*>(lds_raw);  // [P][64]
  double* sG = sR + tab.num_paths * kLanes;         // [n_out][64]
  double* sDH = sG + tab.n_out * kLanes;            // [n_h][64]
  const int lane = threadIdx.x;
  const size_t node = blockIdx.x / chblocks;
  const int cb = blockIdx.x % chblocks;
  const int ch = cb * kLanes + lane;
  const bool active = ch < K;
  for (int b = 0; b < tab.n_h; ++b) sDH[b * kLanes + lane] = 0.0;
  const int q0 = send_ptr[node], q1 = send_ptr[node + 1];
  for (int q = q0; q < q1; ++q) {
    const size_t e = send_edge[q];
    const size_t i = receiver[e];
    for (int c = 0; c < tab.n_out; ++c)
      sG[c * kLanes + lane] = active ? static_cast<double>(dA[(i * K + ch) * tab.n_out + c]) : 0.0;
    for (int p = 0; p < tab.num_paths; ++p)
      sR[p * kLanes + lane] = active ? static_cast<double>(R[(e * tab.num_paths + p) * K + ch]) : 0.0;
    const T* y = Y + e * tab.n_Y;
    for (int t = 0; t < tab.n_terms; ++t) {
      const int4 ix = tab.idx[t];
      sDH[ix.z * kLanes + lane] += tab.coef[t] * sR[ix.x * kLanes + lane] * static_cast<double>(y[ix.y]) * sG[ix.w * kLanes + lane];
    }
  }
  if (active)
    for (int b = 0; b < tab.n_h; ++b) dh[(node * K + ch) * tab.n_h + b] = static_cast<T>(sDH[b * kLanes + lane]);
}

// dY[e][a] = sum over the channel blocks of the partials, in block order.
template <typename T>
__global__ void dY_sum_kernel(int64_t n, int chblocks, const T* __restrict__ partial, T* __restrict__ dY) {
  const int64_t i = blockIdx.x * static_cast<int64_t>(blockDim.x) + threadIdx.x;
  if (i >= n) return;
  T s = partial[i];
  for (int cb = 1; cb < chblocks; ++cb) s += partial[static_cast<int64_t>(cb) * n + i];
  dY[i] = s;
}

template <typename T>
hipError_t fwd_t(const tp_plan* plan, const FwdArgs& a, hipStream_t stream) {
  const TermTable& t = plan->tab;
  const int K = plan->cfg.num_channels, chblocks = (K + kLanes - 1) / kLanes;
  const size_t lds = static_cast<size_t>(t.n_h + t.num_paths + t.n_out) * kLanes * sizeof(double);
  hipLaunchKernelGGL(generic_forward_kernel<T>, dim3(static_cast<unsigned>(a.n_out_nodes * chblocks)), dim3(kLanes), lds,
                     stream, t, K, chblocks, static_cast<const T*>(a.Y), static_cast<const T*>(a.h),
                     static_cast<const T*>(a.R), a.sender, a.row_ptr, static_cast<T*>(a.A));
  return hipGetLastError();
}

template <typename T>
hipError_t bwd_recv_t(const tp_plan* plan, const BwdArgs& a, hipStream_t stream) {
  const TermTable& t = plan->tab;
  const int K = plan->cfg.num_channels, chblocks = (K + kLanes - 1) / kLanes;
  const size_t lds = static_cast<size_t>(t.n_h + 2 * t.num_paths + t.n_out + t.n_Y) * kLanes * sizeof(double);
  hipLaunchKernelGGL(generic_backward_recv_kernel<T>, dim3(static_cast<unsigned>(a.n_out_nodes * chblocks)), dim3(kLanes),
                     lds, stream, t, K, chblocks, a.n_edges, static_cast<const T*>(a.Y), static_cast<const T*>(a.h),
                     static_cast<const T*>(a.R), a.sender, a.row_ptr, static_cast<const T*>(a.dA),
                     static_cast<T*>(a.dR), static_cast<T*>(a.dY_partial));
  return hipGetLastError();
}

template <typename T>
hipError_t bwd_send_t(const tp_plan* plan, const BwdArgs& a, hipStream_t stream) {
  const TermTable& t = plan->tab;
  const int K = plan->cfg.num_channels, chblocks = (K + kLanes - 1) / kLanes;
  const size_t lds = static_cast<size_t>(t.num_paths + t.n_out + t.n_h) * kLanes * sizeof(double);
  hipLaunchKernelGGL(generic_backward_send_kernel<T>, dim3(static_cast<unsigned>(a.n_in * chblocks)), dim3(kLanes), lds,
                     stream, t, K, chblocks, static_cast<const T*>(a.Y), static_cast<const T*>(a.R), a.receiver,
                     a.send_ptr, a.send_edge, static_cast<const T*>(a.dA), static_cast<T*>(a.dh));
  return hipGetLastError();
}

template <typename T>
hipError_t dY_sum_t(const tp_plan* plan, const BwdArgs& a, hipStream_t stream) {
  const int K = plan->cfg.num_channels, chblocks = (K + kLanes - 1) / kLanes;
  const int64_t n = a.n_edges * plan->n_Y;
  if (n == 0) return hipSuccess;
  hipLaunchKernelGGL(dY_sum_kernel<T>, dim3(static_cast<unsigned>((n + 255) / 256)), dim3(256), 0, stream, n, chblocks,
                     static_cast<const T*>(a.dY_partial), static_cast<T*>(a.dY));
  return hipGetLastError();
}

}  // namespace

hipError_t launch_generic_forward(const tp_plan* plan, const FwdArgs& a, hipStream_t stream) {
  return plan->cfg.dtype == SC_F64 ? fwd_t<double>(plan, a, stream) : fwd_t<float>(plan, a, stream);
}
hipError_t launch_generic_backward_recv(const tp_plan* plan, const BwdArgs& a, hipStream_t stream) {
  return plan->cfg.dtype == SC_F64 ? bwd_recv_t<double>(plan, a, stream) : bwd_recv_t<float>(plan, a, stream);
}
hipError_t launch_generic_backward_send(const tp_plan* plan, const BwdArgs& a, hipStream_t stream) {
  return plan->cfg.dtype == SC_F64 ? bwd_send_t<double>(plan, a, stream) : bwd_send_t<float>(plan, a, stream);
}
hipError_t launch_dY_sum(const tp_plan* plan, const BwdArgs& a, hipStream_t stream) {
  return plan->cfg.dtype == SC_F64 ? dY_sum_t<double>(plan, a, stream) : dY_sum_t<float>(plan, a, stream);
}

}  // namespace tp
