// Internal declarations of the channelwise tensor product (Algorithm 1 of arXiv 2504.10700).
#pragma once
#include <hip/hip_runtime.h>

#include <array>
#include <cstdint>
#include <vector>

#include "../../include/tp.h"
#include "sc_internal.h"

namespace tp {

struct Term {  // msg[c] += coef * R[p] * Y[a] * h[b]
  int p, a, b, c;
  double coef;
};

// Device view of the sparse coupling terms, sorted by (path, c, a, b).
struct TermTable {
  int32_t n_terms, num_paths, n_Y, n_h, n_out;
  const int4* idx;      // (p, a, b, c)
  const double* coef;
};

struct Shape {
  int chblocks;  // ceil(K / 64)
};

}  // namespace tp

struct tp_plan {
  tp_config cfg;
  std::vector<std::array<int, 3>> paths;
  std::vector<tp::Term> terms;
  bool host_only = false;
  int specialised = 0;
  int n_Y = 0, n_h = 0, n_out = 0;
  bool profile = false;
  // start/stop pairs: forward, backward, dh sum, second-order kernel
  hipEvent_t ev[8] = {nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr};
  bool ev_used[4] = {false, false, false, false};
  void* dev_blob = nullptr;
  tp::TermTable tab{};
};

namespace tp {

// The caller's edge list as the kernels read it.  The index arrays are not validated on the host
// (they live on the device and the calls never synchronise); every index is clamped into its
// range where it is read, so that a wrong index gives wrong numbers for that edge but never an
// access outside the buffers.
struct EdgeList {
  const int32_t* sender;   // [n_edges]
  const int32_t* row_ptr;  // [n_out_nodes + 1]
  int n_in, n_edges;
  // A sender index is clamped where it is USED (node), not where it is read (raw): the kernels read
  // it one or two edges ahead, and a clamp at the read would wait for the load at once.
  __device__ __forceinline__ int raw(int e) const { return sender[e]; }
  __device__ __forceinline__ size_t node(int j) const { return static_cast<size_t>(j < 0 ? 0 : (j >= n_in ? n_in - 1 : j)); }
  __device__ __forceinline__ size_t snd(int e) const { return node(sender[e]); }
  __device__ __forceinline__ int first(size_t node) const {
    const int e = row_ptr[node];
    return e < 0 ? 0 : (e > n_edges ? n_edges : e);
  }
};

struct FwdArgs {
  int64_t n_in, n_out_nodes, n_edges;
  const void *Y, *h, *R;
  const int32_t *sender, *row_ptr;
  void* A;
};

struct BwdArgs {
  int64_t n_in, n_out_nodes, n_edges;
  const void *Y, *h, *R;
  const int32_t *sender, *row_ptr, *send_ptr, *send_edge;
  const void* dA;
  void *dY, *dh, *dR;
  void* dY_partial;  // [chblocks][n_edges][n_Y] of the plan's dtype
  void* dh_edge;     // [n_edges][K][n_h]: every edge's share of its sender's dh (table-driven and second-order kernels)
};

// Second-order pass: the backward's arguments (dY, dh, dR of BwdArgs receive d2Y, d2h, d2R)
// plus the cotangents and ddA.
struct DblArgs {
  BwdArgs b;
  const void *HY, *Hh, *HR;
  void* ddA;
};

hipError_t launch_generic_forward(const tp_plan* plan, const FwdArgs& a, hipStream_t stream);
hipError_t launch_generic_double_backward(const tp_plan* plan, const DblArgs& a, hipStream_t stream);
hipError_t launch_spec_double_backward(const tp_plan* plan, const DblArgs& a, hipStream_t stream);
hipError_t launch_generic_backward(const tp_plan* plan, const BwdArgs& a, hipStream_t stream);
hipError_t launch_dY_sum(const tp_plan* plan, const BwdArgs& a, hipStream_t stream);
hipError_t launch_dh_sum(const tp_plan* plan, const BwdArgs& a, hipStream_t stream);

// generated kernels (tp_spec.hip)
int spec_lookup(const tp_plan* plan);
void spec_op_counts(int id, int32_t ops[3], int32_t flops[3]);
hipError_t launch_spec_forward(const tp_plan* plan, const FwdArgs& a, hipStream_t stream);
// edges walked by sender: writes dR, the dY partials and dh itself (every atom's row, zero for atoms that send
// nothing); a.dh_edge receives the edges' receivers (int32), not shares.  Valid for n_in > 0, also without edges.
hipError_t launch_spec_backward(const tp_plan* plan, const BwdArgs& a, hipStream_t stream);

}  // namespace tp
