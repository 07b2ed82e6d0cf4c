// Channel-mixing linear fused into the forward of the symmetric contraction (see include/el.h,
// el_sc_forward): B = contraction(A, z, W) with A[i,k',(l,m)] = sum_k W_lin[l,k,k'] X[i,k,(l,m)]
// (Section 4.1 of arXiv 2504.10700: the linear combination of the channels of each order and
// Algorithm 2 are consecutive steps on the receiving atom).  A never goes through memory.
//
// The MFMA 16x16x4 result layout puts, for one output channel (column lane%16 of the tile) and
// four atoms (rows 4*(lane/16)+r), every component (l,m) of A into the registers of one lane:
// exactly the operand of the generated per-(atom, channel) contraction code.  So a workgroup
// computes the A tile of 16 atoms x 128 channels with the LDS-staged product of the linear
// (el_tile.h), and each lane then evaluates the contraction for its eight (atom, channel)
// pairs from its accumulators and stores 16 bytes of B per pair.
//
// Weights: the atoms of a tile are consecutive atoms of the batch, of any element, so the folded
// weights (internal basis, S values) of a pair are read per pair, from a table [Z][K][32] that a
// small kernel writes per call; the rows of a pair are 128 contiguous bytes, requested one
// pair ahead of their use.
#include <algorithm>
#include <string>

#include "../../include/el.h"
#include "el_tile.h"
#include "sc_spec.h"

namespace sc {
namespace {

__device__ __forceinline__ float sc_fma(float x, float y, float z) { return __builtin_fmaf(x, y, z); }
__device__ __forceinline__ double sc_fma(double x, double y, double z) { return __builtin_fma(x, y, z); }

#include "generated/sc_gen_l3n3_0e1o.inc"

typedef Gen_l3n3_0e1o G;
constexpr int kWStride = 32;   // floats per (element, channel) row of the folded table
static_assert(G::kS <= kWStride && G::kNlm == 16 && G::kNLM == 4, "layout of the fused kernel");

// wf[z][ch][s] = folded weights of element z, channel ch (s < S; the rest of the row is zero).
// One wave per (element, 64 channels): the wave's rows are one contiguous 8 KB block, written
// through an LDS transpose as 256-byte pieces (per-lane rows would scatter every store over 64
// cache lines).  K % 64 == 0.
__global__ __launch_bounds__(kLanes) void fold_table_kernel(int K, const float* __restrict__ W,
                                                            float* __restrict__ wf) {
  __shared__ float t[kLanes * (kWStride + 1)];
  const int lane = threadIdx.x;
  const int chblocks = K / kLanes;
  const int z = blockIdx.x / chblocks, ch0 = (blockIdx.x % chblocks) * kLanes;
  float w[G::kS];
  G::fold(W + static_cast<size_t>(z) * G::kP * K + ch0 + lane, K, w);
#pragma unroll
  for (int s = 0; s < kWStride; ++s) t[lane * (kWStride + 1) + s] = s < G::kS ? w[s] : 0.0f;
  __syncthreads();
  float* out = wf + (static_cast<size_t>(z) * K + ch0) * kWStride;
#pragma unroll
  for (int k = 0; k < kWStride; ++k) {
    const int e = k * kLanes + lane;
    out[e] = t[(e / kWStride) * (kWStride + 1) + e % kWStride];
  }
}

template <int CT>
__device__ __forceinline__ void fused_unit(int64_t n_nodes, int64_t n0, int g, int k_in, int K, int Z,
                                           const float* __restrict__ X, const float* __restrict__ Wlin,
                                           const int32_t* __restrict__ z, const float* __restrict__ wf,
                                           float* __restrict__ B, float* xs) {
  typedef float V4 __attribute__((ext_vector_type(4)));
  typedef el::Mma<float> M;
  const int lane = threadIdx.x & (kLanes - 1);
  // elements of this lane's four atoms (rows past the end: element 0, nothing is stored); an
  // element index outside 0..Z-1 is clamped, so that it gives a wrong B row but no wild read
  int zr[4];
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    const int64_t n = n0 + M::row(lane, r);
    const int ze = n < n_nodes ? z[n] : 0;
    zr[r] = ze < 0 ? 0 : ze >= Z ? Z - 1 : ze;
  }
  M::acc_t acc[16][CT];
  int jc[CT];
  el::lds_tile_product<CT>(n_nodes, n0, g, k_in, K, X, Wlin, xs, acc, jc);

  constexpr int kPairs = CT * 4;   // pair p = (column tile p / 4, row p % 4)
  V4 wq[2][kWStride / 4];
  auto wload = [&](int p, V4 (&w)[kWStride / 4]) {
    const V4* src = reinterpret_cast<const V4*>(wf + (static_cast<size_t>(zr[p % 4]) * K + jc[p / 4]) * kWStride);
#pragma unroll
    for (int i = 0; i < kWStride / 4; ++i) w[i] = src[i];
  };
  wload(0, wq[0]);
#pragma unroll
  for (int p = 0; p < kPairs; ++p) {
    if (p + 1 < kPairs) wload(p + 1, wq[(p + 1) & 1]);
    const int t = p / 4, r = p % 4;
    const int64_t n = n0 + M::row(lane, r);
    float a[16], w[G::kS], b[4];
#pragma unroll
    for (int c = 0; c < 16; ++c) a[c] = acc[c][t][r];
#pragma unroll
    for (int s = 0; s < G::kS; ++s) w[s] = wq[p & 1][s / 4][s % 4];
    G::forward(a, w, b);
    if (n < n_nodes) {
      V4 out;
#pragma unroll
      for (int i = 0; i < 4; ++i) out[i] = b[i];
      *reinterpret_cast<V4*>(B + (static_cast<size_t>(n) * K + jc[t]) * 4) = out;
    }
  }
}

__global__ __launch_bounds__(el::kThreads) __attribute__((amdgpu_waves_per_eu(2, 2))) void fused_forward_kernel(
    int64_t n_nodes, int k_in, int K, int Z, const float* __restrict__ X, const float* __restrict__ Wlin,
    const int32_t* __restrict__ z, const float* __restrict__ wf, float* __restrict__ B) {
  __shared__ __attribute__((aligned(16))) float xs[el::kBuffers * 16 * el::kRowPad];
  const int groups = K / 128;                            // full units per row tile
  const el::UnitSchedule u = el::unit_schedule((n_nodes + 15) / 16 * groups, true);
  if (u.has_half)
    fused_unit<1>(n_nodes, u.half_unit / groups * 16, static_cast<int>(u.half_unit % groups) * 2 + u.half, k_in, K, Z,
                  X, Wlin, z, wf, B, xs);
  for (int64_t unit = blockIdx.x; unit < u.n_full; unit += gridDim.x)
    fused_unit<2>(n_nodes, unit / groups * 16, static_cast<int>(unit % groups) * 2, k_in, K, Z, X, Wlin, z, wf, B, xs);
}



// Does the fused kernel serve this plan and this number of input channels?
bool fused_ok(const sc_plan* plan, int k_in) {
  return !plan->host_only && plan->cfg.dtype == SC_F32 && spec_lookup(plan) == 1 && plan->cfg.num_channels % 128 == 0 &&
         k_in % el::kChunk == 0 && static_cast<int64_t>(k_in) * plan->cfg.num_channels < (int64_t(1) << 26);
}

size_t round256(size_t b) { return (b + 255) / 256 * 256; }
size_t fold_table_bytes(const sc_plan* plan) {
  return round256(static_cast<size_t>(plan->cfg.num_elements) * plan->cfg.num_channels * kWStride * sizeof(float));
}
size_t a_bytes(const sc_plan* plan, int64_t n) {
  const size_t nlm = static_cast<size_t>(plan->cfg.l_max + 1) * (plan->cfg.l_max + 1);
  return round256(static_cast<size_t>(n) * plan->cfg.num_channels * nlm * (plan->cfg.dtype == SC_F64 ? 8 : 4));
}

sc_status check(const char* fn, const sc_plan* plan, int32_t k_in, int64_t n) {
  if (!plan) return set_error(SC_ERR_INVALID_ARG, std::string(fn) + ": plan is NULL");
  if (plan->host_only) return set_error(SC_ERR_INVALID_ARG, std::string(fn) + ": the plan has no device");
  if (k_in < 1) return set_error(SC_ERR_INVALID_ARG, std::string(fn) + ": k_in < 1");
  if (plan->cfg.dtype == SC_BF16) return set_error(SC_ERR_UNSUPPORTED, std::string(fn) + ": plans with bfloat16 rows are not served");
  if (n < 0 || n > (int64_t(1) << 30)) return set_error(SC_ERR_INVALID_ARG, std::string(fn) + ": n_nodes outside 0..2^30");
  return SC_OK;
}

el_config linear_config(const sc_plan* plan, int32_t k_in) {
  el_config c;
  c.struct_size = static_cast<int32_t>(sizeof(el_config));
  c.k_in = k_in;
  c.k_out = plan->cfg.num_channels;
  c.l_max = plan->cfg.l_max;
  c.dtype = plan->cfg.dtype;
  c.device = plan->cfg.device;
  return c;
}

}  // namespace
}  // namespace sc

extern "C" {

int32_t el_sc_is_fused(const sc_plan* plan, int32_t k_in) {
  return plan && k_in >= 1 && sc::fused_ok(plan, k_in) ? 1 : 0;
}

sc_status el_sc_workspace_bytes(const sc_plan* plan, int32_t k_in, int64_t n_nodes, size_t* bytes) {
  using namespace sc;
  sc_status st = check("el_sc_workspace_bytes", plan, k_in, n_nodes);
  if (st != SC_OK) return st;
  if (!bytes) return set_error(SC_ERR_INVALID_ARG, "el_sc_workspace_bytes: bytes is NULL");
  if (fused_ok(plan, k_in)) {
    *bytes = fold_table_bytes(plan) + 256;
    return SC_OK;
  }
  size_t inner = 0;
  st = sc_workspace_bytes(plan, n_nodes, &inner);
  if (st != SC_OK) return st;
  *bytes = a_bytes(plan, n_nodes) + round256(inner) + 256;
  return SC_OK;
}

sc_status el_sc_forward(sc_plan* plan, int32_t k_in, int64_t n_nodes, const void* X, const void* W_lin,
                        const int32_t* z, const void* W, void* B, void* workspace, size_t workspace_bytes,
                        void* hip_stream) {
  using namespace sc;
  sc_status st = check("el_sc_forward", plan, k_in, n_nodes);
  if (st != SC_OK) return st;
  if (n_nodes == 0) return SC_OK;
  if (!X || !W_lin || !z || !W || !B) return set_error(SC_ERR_INVALID_ARG, "el_sc_forward: NULL tensor argument");
  if (misaligned(X, 16) || misaligned(W_lin, 16) || misaligned(W, 16) || misaligned(B, 16) || misaligned(z, 4))
    return set_error(SC_ERR_INVALID_ARG, "el_sc_forward: tensor pointer not aligned (16 bytes, z: 4)");
  size_t need = 0;
  st = el_sc_workspace_bytes(plan, k_in, n_nodes, &need);
  if (st != SC_OK) return st;
  if (!workspace || workspace_bytes < need)
    return set_error(SC_ERR_WORKSPACE, "el_sc_forward: workspace missing or smaller than el_sc_workspace_bytes()");
  if (misaligned(workspace, 256)) return set_error(SC_ERR_WORKSPACE, "el_sc_forward: workspace not 256-byte aligned");

  if (!fused_ok(plan, k_in)) {
    // Two steps through A in the workspace: the linear, then the contraction.
    const el_config lc = linear_config(plan, k_in);
    st = el_forward(&lc, n_nodes, X, W_lin, workspace, hip_stream);
    if (st != SC_OK) return st;
    const size_t off = a_bytes(plan, n_nodes);
    return sc_forward(plan, n_nodes, workspace, z, W, B, static_cast<char*>(workspace) + off, workspace_bytes - off, 0,
                      hip_stream);
  }

  DeviceGuard guard(plan->cfg.device);
  if (!guard.ok) return set_error(SC_ERR_HIP, "el_sc_forward: cannot make the plan's device current");
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  const int K = plan->cfg.num_channels, Z = plan->cfg.num_elements;
  float* wf = static_cast<float*>(workspace);
  hipLaunchKernelGGL(fold_table_kernel, dim3(static_cast<unsigned>(Z * (K / kLanes))), dim3(kLanes), 0, stream, K,
                     static_cast<const float*>(W), wf);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return set_error(SC_ERR_HIP, std::string("el_sc_forward: fold launch: ") + hipGetErrorString(e));
  const int64_t units = (n_nodes + 15) / 16 * (K / 128);
  const unsigned grid = static_cast<unsigned>(std::min<int64_t>(units, 2 * static_cast<int64_t>(plan->num_cus)));
  hipLaunchKernelGGL(fused_forward_kernel, dim3(grid), dim3(el::kThreads), 0, stream, n_nodes, k_in, K, Z,
                     static_cast<const float*>(X), static_cast<const float*>(W_lin), z, wf, static_cast<float*>(B));
  e = hipGetLastError();
  if (e != hipSuccess) return set_error(SC_ERR_HIP, std::string("el_sc_forward: kernel launch: ") + hipGetErrorString(e));
  return SC_OK;
}

// Workspace of el_sc_backward: A | dA | the larger of the two inner workspaces.
static size_t backward_inner_bytes(const sc_plan* plan, int32_t k_in, int64_t n, sc_status* st) {
  using namespace sc;
  size_t a = 0, b = 0;
  *st = sc_workspace_bytes(plan, n, &a);
  if (*st != SC_OK) return 0;
  const el_config lc = linear_config(plan, k_in);
  *st = el_workspace_bytes(&lc, n, &b);
  return round256(a > b ? a : b);
}

sc_status el_sc_backward_workspace_bytes(const sc_plan* plan, int32_t k_in, int64_t n_nodes, size_t* bytes) {
  using namespace sc;
  sc_status st = check("el_sc_backward_workspace_bytes", plan, k_in, n_nodes);
  if (st != SC_OK) return st;
  if (!bytes) return set_error(SC_ERR_INVALID_ARG, "el_sc_backward_workspace_bytes: bytes is NULL");
  const size_t inner = backward_inner_bytes(plan, k_in, n_nodes, &st);
  if (st != SC_OK) return st;
  *bytes = 2 * a_bytes(plan, n_nodes) + inner + 256;
  return SC_OK;
}

sc_status el_sc_backward(sc_plan* plan, int32_t k_in, int64_t n_nodes, const void* X, const void* W_lin,
                         const int32_t* z, const void* W, const void* dB, void* dX, void* dW_lin, void* dW,
                         void* workspace, size_t workspace_bytes, void* hip_stream) {
  using namespace sc;
  sc_status st = check("el_sc_backward", plan, k_in, n_nodes);
  if (st != SC_OK) return st;
  if (!dW_lin || !dW) return set_error(SC_ERR_INVALID_ARG, "el_sc_backward: dW_lin or dW is NULL");
  const el_config lc = linear_config(plan, k_in);
  if (n_nodes == 0) {   // both weight gradients are zero
    st = sc_backward(plan, 0, nullptr, nullptr, nullptr, nullptr, nullptr, dW, nullptr, 0, 0, hip_stream);
    if (st != SC_OK) return st;
    return el_backward(&lc, 0, nullptr, W_lin, nullptr, nullptr, dW_lin, nullptr, 0, hip_stream);
  }
  if (!X || !W_lin || !z || !W || !dB || !dX)
    return set_error(SC_ERR_INVALID_ARG, "el_sc_backward: NULL tensor argument");
  size_t need = 0;
  st = el_sc_backward_workspace_bytes(plan, k_in, n_nodes, &need);
  if (st != SC_OK) return st;
  if (!workspace || workspace_bytes < need)
    return set_error(SC_ERR_WORKSPACE, "el_sc_backward: workspace missing or smaller than el_sc_backward_workspace_bytes()");
  if (misaligned(workspace, 256)) return set_error(SC_ERR_WORKSPACE, "el_sc_backward: workspace not 256-byte aligned");
  char* base = static_cast<char*>(workspace);
  void* A = base;
  void* dA = base + a_bytes(plan, n_nodes);
  void* inner = base + 2 * a_bytes(plan, n_nodes);
  const size_t inner_bytes = workspace_bytes - 2 * a_bytes(plan, n_nodes);
  st = el_forward(&lc, n_nodes, X, W_lin, A, hip_stream);                                  // A again: the forward never wrote it
  if (st != SC_OK) return st;
  st = sc_backward(plan, n_nodes, A, z, W, dB, dA, dW, inner, inner_bytes, 0, hip_stream);  // dA and dW
  if (st != SC_OK) return st;
  return el_backward(&lc, n_nodes, X, W_lin, dA, dX, dW_lin, inner, inner_bytes, hip_stream);  // dX and dW_lin
}

}  // extern "C"
