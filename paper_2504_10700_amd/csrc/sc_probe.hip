// Streaming probes (measurement helper, see sc_probe_stream in include/sc.h): plain kernels
// that move a known number of bytes with no arithmetic, so that a benchmark can put the
// bandwidth this box attains next to the figures of the contraction kernels in the same run.
//
//   read / write / copy   16 bytes per lane and access, a contiguous chunk per workgroup, many
//                         independent accesses in flight: the simplest traffic there is
//   rows                  the access pattern of the fused backward kernel without its
//                         arithmetic: one wave per gathered row, 64 B per lane of one tensor
//                         (the A row of a node and 64 channels, 4 KB) and 16 B per lane of a
//                         second one (its dB row, 1 KB) in, 4 KB out in whole 1 KB pieces,
//                         the next row requested before the current one is written; a workgroup
//                         per 16 rows, a quarter of them per wave (resident workgroups that
//                         stride over the rows when there are too few rows for that)
//   forward rows          the same walk with the forward kernel's traffic: 4 KB in, 1 KB out per row,
//                         a workgroup per 32 rows
#include "sc_internal.h"

namespace sc {
namespace {

typedef float f4 __attribute__((ext_vector_type(4)));

constexpr int kProbeThreads = 256;
constexpr int kUnroll = 8;

// read / write / copy: every workgroup streams its own contiguous chunk of the buffer, 4 KB per
// instruction and workgroup, kUnroll instructions in flight; loads and the copy's stores bypass
// the cache.  (Measured against grid-stride loops, where neighbouring workgroups touch
// neighbouring 4 KB pieces: read 7.0 instead of 4.8-6.4 TB/s, write 6.0 instead of 3.9-4.4, copy
// 5.6 instead of 4.1-5.3, on one MI355X.)
__device__ __forceinline__ void probe_chunk(size_t n16, size_t& lo, size_t& hi) {
  const size_t per = (n16 + gridDim.x - 1) / gridDim.x;
  lo = blockIdx.x * per;
  hi = lo + per < n16 ? lo + per : n16;
}

__global__ __launch_bounds__(kProbeThreads) void probe_read_kernel(const f4* __restrict__ src, size_t n16,
                                                                    float* __restrict__ sink) {
  size_t lo, hi;
  probe_chunk(n16, lo, hi);
  f4 acc = {0.f, 0.f, 0.f, 0.f};
  size_t i = lo + threadIdx.x;
  for (; i + (kUnroll - 1) * kProbeThreads < hi; i += kUnroll * kProbeThreads) {
    f4 v[kUnroll];
#pragma unroll
    for (int k = 0; k < kUnroll; ++k) v[k] = __builtin_nontemporal_load(src + i + k * kProbeThreads);
#pragma unroll
    for (int k = 0; k < kUnroll; ++k) acc += v[k];
  }
  for (; i < hi; i += kProbeThreads) acc += src[i];
  // never true for finite data; keeps the loads alive
  if (acc.x + acc.y + acc.z + acc.w == 1.2345e38f) sink[0] = acc.x;
}

__global__ __launch_bounds__(kProbeThreads) void probe_write_kernel(f4* __restrict__ dst, size_t n16) {
  size_t lo, hi;
  probe_chunk(n16, lo, hi);
  const f4 v = {1.f, 2.f, 3.f, 4.f};
  for (size_t i = lo + threadIdx.x; i < hi; i += kProbeThreads) dst[i] = v;
}

__global__ __launch_bounds__(kProbeThreads) void probe_copy_kernel(const f4* __restrict__ src, f4* __restrict__ dst,
                                                                    size_t n16) {
  size_t lo, hi;
  probe_chunk(n16, lo, hi);
  size_t i = lo + threadIdx.x;
  for (; i + (kUnroll - 1) * kProbeThreads < hi; i += kUnroll * kProbeThreads) {
    f4 v[kUnroll];
#pragma unroll
    for (int k = 0; k < kUnroll; ++k) v[k] = __builtin_nontemporal_load(src + i + k * kProbeThreads);
#pragma unroll
    for (int k = 0; k < kUnroll; ++k) __builtin_nontemporal_store(v[k], dst + i + k * kProbeThreads);
  }
  for (; i < hi; i += kProbeThreads) dst[i] = src[i];
}

// rows: a[n_rows][64 lanes][4 x f4], b[n_rows][64 lanes][f4] in, out[n_rows][4][64 lanes][f4].
// One workgroup per kTile consecutive entries of perm (clamped into range), a contiguous quarter
// of them per wave - the shape of the contraction kernels, and the fastest of the walks that were
// measured (forward traffic, 400 000 rows: 366 us like this, 390-410 us with resident workgroups
// that stride over the rows).  kTile: 32 rows (forward) or 16 (backward).
// kForward: only a is read, and out is [n_rows][64 lanes][f4].
template <bool kForward>
__global__ __launch_bounds__(kProbeThreads) void probe_rows_kernel(const f4* __restrict__ a, const f4* __restrict__ b,
                                                                    f4* __restrict__ out,
                                                                    const int32_t* __restrict__ perm, int n_rows, int kTile) {
  const int lane = threadIdx.x & (kLanes - 1);
  const int wave = threadIdx.x / kLanes;
  const long long lo = static_cast<long long>(blockIdx.x) * kTile;
  const long long hi = lo + kTile < n_rows ? lo + kTile : n_rows;
  const int quarter = static_cast<int>((hi - lo + 3) / 4);
  const long long j0 = lo + static_cast<long long>(wave) * quarter;
  const long long j1 = j0 + quarter < hi ? j0 + quarter : hi;
  auto row_of = [&](long long j) {
    int r = perm[j];
    return static_cast<size_t>(r < 0 ? 0 : (r >= n_rows ? n_rows - 1 : r));
  };
  if (j0 >= j1) return;
  f4 va[4], vb = {0.f, 0.f, 0.f, 0.f}, na[4], nb = vb;
  size_t row = row_of(j0);
#pragma unroll
  for (int k = 0; k < 4; ++k) va[k] = a[(row * kLanes + lane) * 4 + k];
  if constexpr (!kForward) vb = b[row * kLanes + lane];
  for (long long j = j0; j < j1; ++j) {
    const bool more = j + 1 < j1;
    size_t next = row;
    if (more) {
      next = row_of(j + 1);
#pragma unroll
      for (int k = 0; k < 4; ++k) na[k] = a[(next * kLanes + lane) * 4 + k];
      if constexpr (!kForward) nb = b[next * kLanes + lane];
    }
    if constexpr (kForward) {
      __builtin_nontemporal_store(va[0] + va[1] + va[2] + va[3], out + row * kLanes + lane);
    } else {
#pragma unroll
      for (int k = 0; k < 4; ++k) out[(row * 4 + k) * kLanes + lane] = va[k] + vb;
    }
    if (more) {
#pragma unroll
      for (int k = 0; k < 4; ++k) va[k] = na[k];
      vb = nb;
      row = next;
    }
  }
}

// The same traffic by resident workgroups: wave w takes entries w, w + n_waves, ... of perm.  The
// faster walk when the rows are too few to fill the chip with whole tiles (20 000 rows of the
// forward's traffic: 18.8 us against 20.4 us).
template <bool kForward>
__global__ __launch_bounds__(kProbeThreads) void probe_rows_strided_kernel(const f4* __restrict__ a, const f4* __restrict__ b,
                                                                            f4* __restrict__ out,
                                                                            const int32_t* __restrict__ perm, int n_rows) {
  const int lane = threadIdx.x & (kLanes - 1);
  const int wave = (blockIdx.x * kProbeThreads + threadIdx.x) / kLanes;
  const int n_waves = gridDim.x * (kProbeThreads / kLanes);
  auto row_of = [&](int j) {
    int r = perm[j];
    return static_cast<size_t>(r < 0 ? 0 : (r >= n_rows ? n_rows - 1 : r));
  };
  if (wave >= n_rows) return;
  f4 va[4], vb = {0.f, 0.f, 0.f, 0.f}, na[4], nb = vb;
  size_t row = row_of(wave);
#pragma unroll
  for (int k = 0; k < 4; ++k) va[k] = a[(row * kLanes + lane) * 4 + k];
  if constexpr (!kForward) vb = b[row * kLanes + lane];
  for (int j = wave; j < n_rows; j += n_waves) {
    const bool more = j + n_waves < n_rows;
    size_t next = row;
    if (more) {
      next = row_of(j + n_waves);
#pragma unroll
      for (int k = 0; k < 4; ++k) na[k] = a[(next * kLanes + lane) * 4 + k];
      if constexpr (!kForward) nb = b[next * kLanes + lane];
    }
    if constexpr (kForward) {
      __builtin_nontemporal_store(va[0] + va[1] + va[2] + va[3], out + row * kLanes + lane);
    } else {
#pragma unroll
      for (int k = 0; k < 4; ++k) out[(row * 4 + k) * kLanes + lane] = va[k] + vb;
    }
    if (more) {
#pragma unroll
      for (int k = 0; k < 4; ++k) va[k] = na[k];
      vb = nb;
      row = next;
    }
  }
}

}  // namespace
}  // namespace sc

extern "C" sc_status sc_probe_stream(int32_t kind, const void* src, const void* src2, void* dst, const int32_t* perm,
                                     int64_t n, void* hip_stream) {
  using namespace sc;
  if (n < 0 || n > (int64_t(1) << 40)) return set_error(SC_ERR_INVALID_ARG, "sc_probe_stream: n out of range");
  if (n == 0) return SC_OK;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  int dev = 0, cus = 256;
  if (hipGetDevice(&dev) != hipSuccess) return set_error(SC_ERR_HIP, "sc_probe_stream: hipGetDevice");
  (void)hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
  if (cus < 1) cus = 256;
  const int grid = cus * 16;   // sixteen workgroups of four waves per compute unit
  auto bad = [](const void* p) { return !p || misaligned(p, 16); };
  switch (kind) {
    case SC_PROBE_READ:
      if (bad(src) || bad(dst) || n % 16) return set_error(SC_ERR_INVALID_ARG, "sc_probe_stream: read needs src, dst (sink), n % 16 == 0");
      hipLaunchKernelGGL(probe_read_kernel, dim3(grid), dim3(kProbeThreads), 0, stream, static_cast<const f4*>(src),
                         static_cast<size_t>(n / 16), static_cast<float*>(dst));
      break;
    case SC_PROBE_WRITE:
      if (bad(dst) || n % 16) return set_error(SC_ERR_INVALID_ARG, "sc_probe_stream: write needs dst, n % 16 == 0");
      hipLaunchKernelGGL(probe_write_kernel, dim3(grid), dim3(kProbeThreads), 0, stream, static_cast<f4*>(dst),
                         static_cast<size_t>(n / 16));
      break;
    case SC_PROBE_COPY:
      if (bad(src) || bad(dst) || n % 16) return set_error(SC_ERR_INVALID_ARG, "sc_probe_stream: copy needs src, dst, n % 16 == 0");
      hipLaunchKernelGGL(probe_copy_kernel, dim3(grid), dim3(kProbeThreads), 0, stream, static_cast<const f4*>(src),
                         static_cast<f4*>(dst), static_cast<size_t>(n / 16));
      break;
    case SC_PROBE_ROWS:
    case SC_PROBE_ROWS_FORWARD: {
      const bool fwd = kind == SC_PROBE_ROWS_FORWARD;
      if (bad(src) || (!fwd && bad(src2)) || bad(dst) || !perm || n > (int64_t(1) << 30))
        return set_error(SC_ERR_INVALID_ARG, "sc_probe_stream: rows needs src, src2 (backward pattern), dst, perm, n <= 2^30 rows");
      // whole tiles of the kernels' size where they fill the chip, else resident workgroups that stride
      const int tile = fwd ? 32 : 16;
      const int64_t tiles = (n + tile - 1) / tile, resident = static_cast<int64_t>(cus) * (fwd ? 16 : 8);
      if (tiles >= resident) {
        const dim3 grid_rows(static_cast<unsigned>(tiles));
        if (fwd)
          hipLaunchKernelGGL(probe_rows_kernel<true>, grid_rows, dim3(kProbeThreads), 0, stream, static_cast<const f4*>(src),
                             static_cast<const f4*>(src2), static_cast<f4*>(dst), perm, static_cast<int>(n), tile);
        else
          hipLaunchKernelGGL(probe_rows_kernel<false>, grid_rows, dim3(kProbeThreads), 0, stream, static_cast<const f4*>(src),
                             static_cast<const f4*>(src2), static_cast<f4*>(dst), perm, static_cast<int>(n), tile);
      } else {
        const int64_t wgs = (n + 3) / 4;
        const dim3 grid_rows(static_cast<unsigned>(wgs < resident ? wgs : resident));
        if (fwd)
          hipLaunchKernelGGL(probe_rows_strided_kernel<true>, grid_rows, dim3(kProbeThreads), 0, stream, static_cast<const f4*>(src),
                             static_cast<const f4*>(src2), static_cast<f4*>(dst), perm, static_cast<int>(n));
        else
          hipLaunchKernelGGL(probe_rows_strided_kernel<false>, grid_rows, dim3(kProbeThreads), 0, stream, static_cast<const f4*>(src),
                             static_cast<const f4*>(src2), static_cast<f4*>(dst), perm, static_cast<int>(n));
      }
      break;
    }
    default:
      return set_error(SC_ERR_INVALID_ARG, "sc_probe_stream: unknown kind");
  }
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) return set_error(SC_ERR_HIP, std::string("sc_probe_stream: launch: ") + hipGetErrorString(e));
  return SC_OK;
}
