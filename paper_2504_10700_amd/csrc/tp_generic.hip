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
                                                                 const EdgeList el,
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
  const int e0 = el.first(node), e1 = el.first(node + 1);
  for (int e = e0; e < e1; ++e) {
    const size_t j = el.snd(e);
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

// Backward over the edges grouped by receiver: dR of every edge, the per-channel-block partial
// of dY and the edge's share of its sender's dh.
template <typename T>
__global__ __launch_bounds__(kLanes) void generic_backward_kernel(
    TermTable tab, int K, int chblocks, int64_t n_edges, const T* __restrict__ Y, const T* __restrict__ h,
    const T* __restrict__ R, const EdgeList el,
    const T* __restrict__ dA, T* __restrict__ dR, T* __restrict__ dY_partial, T* __restrict__ dh_edge) {
  extern __shared__ unsigned char lds_raw[];
  double* sH = reinterpret_cast<double*>(lds_raw);  // [n_h][64]
  double* sR = sH + tab.n_h * kLanes;               // [P][64]
  double* sG = sR + tab.num_paths * kLanes;         // [n_out][64]  dA of the receiver
  double* sDR = sG + tab.n_out * kLanes;            // [P][64]
  double* sDY = sDR + tab.num_paths * kLanes;       // [n_Y][64]    this lane's share of dY
  double* sDH = sDY + tab.n_Y * kLanes;             // [n_h][64]
  const int lane = threadIdx.x;
  const size_t node = blockIdx.x / chblocks;
  const int cb = blockIdx.x % chblocks;
  const int ch = cb * kLanes + lane;
  const bool active = ch < K;
  for (int c = 0; c < tab.n_out; ++c)
    sG[c * kLanes + lane] = active ? static_cast<double>(dA[(node * K + ch) * tab.n_out + c]) : 0.0;
  const int e0 = el.first(node), e1 = el.first(node + 1);
  for (int e = e0; e < e1; ++e) {
    const size_t j = el.snd(e);
    for (int b = 0; b < tab.n_h; ++b) {
      sH[b * kLanes + lane] = active ? static_cast<double>(h[(j * K + ch) * tab.n_h + b]) : 0.0;
      sDH[b * kLanes + lane] = 0.0;
    }
    for (int p = 0; p < tab.num_paths; ++p) {
      sR[p * kLanes + lane] = active ? static_cast<double>(R[(static_cast<size_t>(e) * tab.num_paths + p) * K + ch]) : 0.0;
      sDR[p * kLanes + lane] = 0.0;
    }
    for (int a = 0; a < tab.n_Y; ++a) sDY[a * kLanes + lane] = 0.0;
    const T* y = Y + static_cast<size_t>(e) * tab.n_Y;
    for (int t = 0; t < tab.n_terms; ++t) {
      const int4 ix = tab.idx[t];
      const double cg = tab.coef[t] * sG[ix.w * kLanes + lane];
      const double gh = cg * sH[ix.z * kLanes + lane];
      const double ya = static_cast<double>(y[ix.y]), rp = sR[ix.x * kLanes + lane];
      sDR[ix.x * kLanes + lane] += gh * ya;
      sDY[ix.y * kLanes + lane] += gh * rp;
      sDH[ix.z * kLanes + lane] += cg * rp * ya;
    }
    if (active) {
      for (int p = 0; p < tab.num_paths; ++p)
        dR[(static_cast<size_t>(e) * tab.num_paths + p) * K + ch] = static_cast<T>(sDR[p * kLanes + lane]);
      for (int b = 0; b < tab.n_h; ++b)
        dh_edge[(static_cast<size_t>(e) * K + ch) * tab.n_h + b] = static_cast<T>(sDH[b * kLanes + lane]);
    }
    for (int a = 0; a < tab.n_Y; ++a) {
      const double s = wave_sum(sDY[a * kLanes + lane]);
      if (lane == 0) dY_partial[(static_cast<size_t>(cb) * n_edges + e) * tab.n_Y + a] = static_cast<T>(s);
    }
  }
}

// Second-order pass over the edges grouped by receiver.  hy, hx, hr: cotangents of (dY, dh,
// dR).  Per term the derivative of the message along the cotangents is
// coef * (hr*y*x + r*hy*x + r*y*hx); ddA of the receiver sums it over the edges, and with
// psi = sum_c g[c] * (that derivative) the kernel writes d psi / d r (d2R), this channel block's
// partial of d psi / d y (d2Y) and the edge's share of d psi / d x (d2h).
template <typename T>
__global__ __launch_bounds__(kLanes) void generic_double_backward_kernel(
    TermTable tab, int K, int chblocks, int64_t n_edges, const T* __restrict__ Y, const T* __restrict__ h,
    const T* __restrict__ R, const EdgeList el,
    const T* __restrict__ dA, const T* __restrict__ HY, const T* __restrict__ Hh, const T* __restrict__ HR,
    T* __restrict__ ddA, T* __restrict__ d2R, T* __restrict__ d2Y_partial, T* __restrict__ d2h_edge) {
  extern __shared__ unsigned char lds_raw[];
  double* sH = reinterpret_cast<double*>(lds_raw);  // [n_h][64]
  double* sHH = sH + tab.n_h * kLanes;              // [n_h][64]   cotangent of dh at the sender
  double* sR = sHH + tab.n_h * kLanes;              // [P][64]
  double* sHR = sR + tab.num_paths * kLanes;        // [P][64]     cotangent of dR
  double* sG = sHR + tab.num_paths * kLanes;        // [n_out][64] dA of the receiver
  double* sDDA = sG + tab.n_out * kLanes;           // [n_out][64]
  double* sDR = sDDA + tab.n_out * kLanes;          // [P][64]
  double* sDY = sDR + tab.num_paths * kLanes;       // [n_Y][64]
  double* sDH = sDY + tab.n_Y * kLanes;             // [n_h][64]
  const int lane = threadIdx.x;
  const size_t node = blockIdx.x / chblocks;
  const int cb = blockIdx.x % chblocks;
  const int ch = cb * kLanes + lane;
  const bool active = ch < K;
  for (int c = 0; c < tab.n_out; ++c) {
    sG[c * kLanes + lane] = active ? static_cast<double>(dA[(node * K + ch) * tab.n_out + c]) : 0.0;
    sDDA[c * kLanes + lane] = 0.0;
  }
  const int e0 = el.first(node), e1 = el.first(node + 1);
  for (int e = e0; e < e1; ++e) {
    const size_t j = el.snd(e);
    for (int b = 0; b < tab.n_h; ++b) {
      sH[b * kLanes + lane] = active ? static_cast<double>(h[(j * K + ch) * tab.n_h + b]) : 0.0;
      sHH[b * kLanes + lane] = active ? static_cast<double>(Hh[(j * K + ch) * tab.n_h + b]) : 0.0;
      sDH[b * kLanes + lane] = 0.0;
    }
    for (int p = 0; p < tab.num_paths; ++p) {
      const size_t at = (static_cast<size_t>(e) * tab.num_paths + p) * K + ch;
      sR[p * kLanes + lane] = active ? static_cast<double>(R[at]) : 0.0;
      sHR[p * kLanes + lane] = active ? static_cast<double>(HR[at]) : 0.0;
      sDR[p * kLanes + lane] = 0.0;
    }
    for (int a = 0; a < tab.n_Y; ++a) sDY[a * kLanes + lane] = 0.0;
    const T* y = Y + static_cast<size_t>(e) * tab.n_Y;
    const T* hy = HY + static_cast<size_t>(e) * tab.n_Y;
    for (int t = 0; t < tab.n_terms; ++t) {
      const int4 ix = tab.idx[t];
      const double c = tab.coef[t];
      const double ya = static_cast<double>(y[ix.y]), hya = static_cast<double>(hy[ix.y]);
      const double x = sH[ix.z * kLanes + lane], hx = sHH[ix.z * kLanes + lane];
      const double r = sR[ix.x * kLanes + lane], hr = sHR[ix.x * kLanes + lane];
      const double cg = c * sG[ix.w * kLanes + lane];
      sDDA[ix.w * kLanes + lane] += c * (hr * ya * x + r * (hya * x + ya * hx));
      sDR[ix.x * kLanes + lane] += cg * (hya * x + ya * hx);
      sDY[ix.y * kLanes + lane] += cg * (hr * x + r * hx);
      sDH[ix.z * kLanes + lane] += cg * (hr * ya + r * hya);
    }
    if (active) {
      for (int p = 0; p < tab.num_paths; ++p)
        d2R[(static_cast<size_t>(e) * tab.num_paths + p) * K + ch] = static_cast<T>(sDR[p * kLanes + lane]);
      for (int b = 0; b < tab.n_h; ++b)
        d2h_edge[(static_cast<size_t>(e) * K + ch) * tab.n_h + b] = static_cast<T>(sDH[b * kLanes + lane]);
    }
    for (int a = 0; a < tab.n_Y; ++a) {
      const double s = wave_sum(sDY[a * kLanes + lane]);
      if (lane == 0) d2Y_partial[(static_cast<size_t>(cb) * n_edges + e) * tab.n_Y + a] = static_cast<T>(s);
    }
  }
  if (active)
    for (int c = 0; c < tab.n_out; ++c) ddA[(node * K + ch) * tab.n_out + c] = static_cast<T>(sDDA[c * kLanes + lane]);
}

// dh[j] = sum of the shares of the edges sent by j, in the order of send_edge.  One lane per
// (channel, component) pair: consecutive lanes read consecutive elements of an edge's row.
template <typename T>
__global__ __launch_bounds__(256) void dh_sum_kernel(int row, int64_t n_rows, int n_edges,
                                                     const int32_t* __restrict__ send_ptr,
                                                     const int32_t* __restrict__ send_edge,
                                                     const T* __restrict__ dh_edge, T* __restrict__ dh) {
  // row = K * n_h elements per node; blockIdx.y walks the row in pieces of 256 elements
  const size_t node = blockIdx.x;
  const int i = blockIdx.y * 256 + threadIdx.x;
  if (node >= static_cast<size_t>(n_rows) || i >= row) return;
  // indices clamped into their ranges (see EdgeList): no access outside the buffers for a wrong list
  auto pos = [&](int v) { return v < 0 ? 0 : (v > n_edges ? n_edges : v); };
  auto edge = [&](int q) {
    const int e = send_edge[q];
    return static_cast<size_t>(e < 0 ? 0 : (e >= n_edges ? n_edges - 1 : e));
  };
  const int q0 = pos(send_ptr[node]), q1 = pos(send_ptr[node + 1]);
  T s0 = T(0), s1 = T(0), s2 = T(0), s3 = T(0);
  int q = q0;
  for (; q + 4 <= q1; q += 4) {  // four independent loads in flight; the order of the additions is fixed
    const T v0 = dh_edge[edge(q) * row + i];
    const T v1 = dh_edge[edge(q + 1) * row + i];
    const T v2 = dh_edge[edge(q + 2) * row + i];
    const T v3 = dh_edge[edge(q + 3) * row + i];
    s0 += v0; s1 += v1; s2 += v2; s3 += v3;
  }
  for (; q < q1; ++q) s0 += dh_edge[edge(q) * row + i];
  dh[node * row + i] = (s0 + s1) + (s2 + s3);
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
                     static_cast<const T*>(a.R), EdgeList{a.sender, a.row_ptr, static_cast<int>(a.n_in), static_cast<int>(a.n_edges)}, static_cast<T*>(a.A));
  return hipGetLastError();
}

template <typename T>
hipError_t bwd_t(const tp_plan* plan, const BwdArgs& a, hipStream_t stream) {
  const TermTable& t = plan->tab;
  const int K = plan->cfg.num_channels, chblocks = (K + kLanes - 1) / kLanes;
  const size_t lds = static_cast<size_t>(2 * t.n_h + 2 * t.num_paths + t.n_out + t.n_Y) * kLanes * sizeof(double);
  if (lds > 64 * 1024) {
    const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&generic_backward_kernel<T>),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds));
    if (e != hipSuccess) return e;
  }
  hipLaunchKernelGGL(generic_backward_kernel<T>, dim3(static_cast<unsigned>(a.n_out_nodes * chblocks)), dim3(kLanes), lds,
                     stream, t, K, chblocks, a.n_edges, static_cast<const T*>(a.Y), static_cast<const T*>(a.h),
                     static_cast<const T*>(a.R), EdgeList{a.sender, a.row_ptr, static_cast<int>(a.n_in), static_cast<int>(a.n_edges)}, static_cast<const T*>(a.dA),
                     static_cast<T*>(a.dR), static_cast<T*>(a.dY_partial), static_cast<T*>(a.dh_edge));
  return hipGetLastError();
}

template <typename T>
hipError_t dbl_t(const tp_plan* plan, const DblArgs& d, hipStream_t stream) {
  const TermTable& t = plan->tab;
  const BwdArgs& a = d.b;
  const int K = plan->cfg.num_channels, chblocks = (K + kLanes - 1) / kLanes;
  const size_t lds = static_cast<size_t>(3 * t.n_h + 3 * t.num_paths + 2 * t.n_out + t.n_Y) * kLanes * sizeof(double);
  if (lds > 64 * 1024) {  // above the default dynamic LDS limit (largest l ranges): raise it for this kernel
    const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&generic_double_backward_kernel<T>),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds));
    if (e != hipSuccess) return e;
  }
  hipLaunchKernelGGL(generic_double_backward_kernel<T>, dim3(static_cast<unsigned>(a.n_out_nodes * chblocks)),
                     dim3(kLanes), lds, stream, t, K, chblocks, a.n_edges, static_cast<const T*>(a.Y),
                     static_cast<const T*>(a.h), static_cast<const T*>(a.R), EdgeList{a.sender, a.row_ptr, static_cast<int>(a.n_in), static_cast<int>(a.n_edges)},
                     static_cast<const T*>(a.dA), static_cast<const T*>(d.HY), static_cast<const T*>(d.Hh),
                     static_cast<const T*>(d.HR), static_cast<T*>(d.ddA), static_cast<T*>(a.dR),
                     static_cast<T*>(a.dY_partial), static_cast<T*>(a.dh_edge));
  return hipGetLastError();
}

template <typename T>
hipError_t dh_sum_t(const tp_plan* plan, const BwdArgs& a, hipStream_t stream) {
  const int row = plan->cfg.num_channels * plan->n_h;
  hipLaunchKernelGGL(dh_sum_kernel<T>, dim3(static_cast<unsigned>(a.n_in), (row + 255) / 256), dim3(256), 0, stream, row,
                     a.n_in, static_cast<int>(a.n_edges), a.send_ptr, a.send_edge, static_cast<const T*>(a.dh_edge),
                     static_cast<T*>(a.dh));
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
hipError_t launch_generic_backward(const tp_plan* plan, const BwdArgs& a, hipStream_t stream) {
  return plan->cfg.dtype == SC_F64 ? bwd_t<double>(plan, a, stream) : bwd_t<float>(plan, a, stream);
}
hipError_t launch_generic_double_backward(const tp_plan* plan, const DblArgs& a, hipStream_t stream) {
  return plan->cfg.dtype == SC_F64 ? dbl_t<double>(plan, a, stream) : dbl_t<float>(plan, a, stream);
}
hipError_t launch_dh_sum(const tp_plan* plan, const BwdArgs& a, hipStream_t stream) {
  return plan->cfg.dtype == SC_F64 ? dh_sum_t<double>(plan, a, stream) : dh_sum_t<float>(plan, a, stream);
}
hipError_t launch_dY_sum(const tp_plan* plan, const BwdArgs& a, hipStream_t stream) {
  return plan->cfg.dtype == SC_F64 ? dY_sum_t<double>(plan, a, stream) : dY_sum_t<float>(plan, a, stream);
}

}  // namespace tp
