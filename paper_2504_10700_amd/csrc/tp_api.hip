// C ABI entry points of the channelwise tensor product (see include/tp.h): argument checks,
// plan construction (sparse coupling terms on the host) and kernel dispatch.
#include <algorithm>
#include <cstring>
#include <new>
#include <string>

#include "tp_internal.h"

namespace {

using sc::align_up;
using sc::DeviceGuard;
using sc::misaligned;
using sc::set_error;

sc_status fail_hip(hipError_t e, const char* what) {
  return set_error(SC_ERR_HIP, std::string(what) + ": " + hipGetErrorString(e));
}

size_t elem_size(const tp_plan* plan) { return plan->cfg.dtype == SC_F64 ? 8 : 4; }
int chblocks_of(const tp_plan* plan) { return (plan->cfg.num_channels + sc::kLanes - 1) / sc::kLanes; }


sc_status check_sizes(const char* fn, const tp_plan* plan, int64_t n_in, int64_t n_out, int64_t n_edges) {
  if (!plan) return set_error(SC_ERR_INVALID_ARG, std::string(fn) + ": plan is NULL");
  if (plan->host_only) return set_error(SC_ERR_UNSUPPORTED, std::string(fn) + ": plan was created with SC_PLAN_HOST_ONLY");
  const int64_t lim = int64_t(1) << 30;
  if (n_in < 0 || n_in > lim || n_out < 0 || n_out > lim || n_edges < 0 || n_edges > lim)
    return set_error(SC_ERR_INVALID_ARG, std::string(fn) + ": a size is outside 0..2^30");
  if (n_edges > 0 && (n_in == 0 || n_out == 0))
    return set_error(SC_ERR_INVALID_ARG, std::string(fn) + ": edges without nodes");
  if (n_out * chblocks_of(plan) > lim || n_in * chblocks_of(plan) > lim)
    return set_error(SC_ERR_INVALID_ARG, std::string(fn) + ": nodes x channel blocks exceeds 2^30");
  return SC_OK;
}

}  // namespace

extern "C" {

sc_status tp_plan_create(const tp_config* cfg, tp_plan** out_plan) {
  if (!cfg || !out_plan) return set_error(SC_ERR_INVALID_ARG, "tp_plan_create: NULL argument");
  *out_plan = nullptr;
  if (cfg->struct_size != static_cast<int32_t>(sizeof(tp_config)))
    return set_error(SC_ERR_INVALID_ARG, "tp_plan_create: struct_size does not match this library's tp_config");
  if (cfg->num_channels < 1) return set_error(SC_ERR_INVALID_ARG, "tp_plan_create: num_channels < 1");
  if (cfg->dtype != SC_F32 && cfg->dtype != SC_F64) return set_error(SC_ERR_INVALID_ARG, "tp_plan_create: bad dtype");
  if (cfg->l_Y < 0 || cfg->l_Y > TP_MAX_L || cfg->l_h < 0 || cfg->l_h > TP_MAX_L || cfg->L_max < 0 ||
      cfg->L_max > TP_MAX_L)
    return set_error(SC_ERR_UNSUPPORTED, "tp_plan_create: l_Y, l_h or L_max outside 0..TP_MAX_L");
  tp_plan* plan = new (std::nothrow) tp_plan();
  if (!plan) return set_error(SC_ERR_ALLOC, "tp_plan_create: out of host memory");
  plan->cfg = *cfg;
  plan->host_only = (cfg->flags & SC_PLAN_HOST_ONLY) != 0;
  plan->n_Y = (cfg->l_Y + 1) * (cfg->l_Y + 1);
  plan->n_h = (cfg->l_h + 1) * (cfg->l_h + 1);
  plan->n_out = (cfg->L_max + 1) * (cfg->L_max + 1);
  for (int l1 = 0; l1 <= cfg->l_Y; ++l1)
    for (int l2 = 0; l2 <= cfg->l_h; ++l2)
      for (int l3 = 0; l3 <= cfg->L_max; ++l3) {
        if (l3 < std::abs(l1 - l2) || l3 > l1 + l2 || (l1 + l2 + l3) % 2) continue;
        const int p = static_cast<int>(plan->paths.size());
        plan->paths.push_back({l1, l2, l3});
        const std::vector<double> C = sc::coupling_tensor(l1, l2, l3);
        const int n1 = 2 * l1 + 1, n2 = 2 * l2 + 1, n3 = 2 * l3 + 1;
        for (int m3 = 0; m3 < n3; ++m3)
          for (int m1 = 0; m1 < n1; ++m1)
            for (int m2 = 0; m2 < n2; ++m2) {
              const double c = C[(m1 * n2 + m2) * n3 + m3];
              if (std::abs(c) < 1e-14) continue;
              plan->terms.push_back(tp::Term{p, l1 * l1 + m1, l2 * l2 + m2, l3 * l3 + m3, c});
            }
      }
  plan->specialised = (cfg->flags & SC_PLAN_FORCE_GENERIC) ? 0 : tp::spec_lookup(plan);
  if (plan->host_only) {
    *out_plan = plan;
    return SC_OK;
  }
  DeviceGuard guard(cfg->device);
  if (!guard.ok) {
    delete plan;
    return set_error(SC_ERR_HIP, "tp_plan_create: cannot make cfg->device current");
  }
  const size_t nt = plan->terms.size();
  std::vector<int4> idx(nt);
  std::vector<double> coef(nt);
  for (size_t t = 0; t < nt; ++t) {
    idx[t] = make_int4(plan->terms[t].p, plan->terms[t].a, plan->terms[t].b, plan->terms[t].c);
    coef[t] = plan->terms[t].coef;
  }
  const size_t o_coef = align_up(sizeof(int4) * nt, 256);
  const size_t bytes = o_coef + align_up(sizeof(double) * nt, 256) + 256;
  std::vector<unsigned char> host(bytes, 0);
  std::memcpy(host.data(), idx.data(), sizeof(int4) * nt);
  std::memcpy(host.data() + o_coef, coef.data(), sizeof(double) * nt);
  hipError_t e = hipMalloc(&plan->dev_blob, bytes);
  if (e != hipSuccess) {
    delete plan;
    return set_error(SC_ERR_ALLOC, std::string("tp_plan_create: hipMalloc: ") + hipGetErrorString(e));
  }
  e = hipMemcpy(plan->dev_blob, host.data(), bytes, hipMemcpyHostToDevice);
  if (e != hipSuccess) {
    (void)hipFree(plan->dev_blob);
    delete plan;
    return fail_hip(e, "tp_plan_create: hipMemcpy");
  }
  plan->tab.n_terms = static_cast<int32_t>(nt);
  plan->tab.num_paths = static_cast<int32_t>(plan->paths.size());
  plan->tab.n_Y = plan->n_Y;
  plan->tab.n_h = plan->n_h;
  plan->tab.n_out = plan->n_out;
  plan->tab.idx = static_cast<const int4*>(plan->dev_blob);
  plan->tab.coef = reinterpret_cast<const double*>(static_cast<char*>(plan->dev_blob) + o_coef);
  *out_plan = plan;
  return SC_OK;
}

sc_status tp_plan_destroy(tp_plan* plan) {
  if (!plan) return SC_OK;
  sc_status st = SC_OK;
  if (!plan->host_only) {
    DeviceGuard guard(plan->cfg.device);  // events and tables belong to the plan's device
    for (int i = 0; i < 8; ++i)
      if (plan->ev[i]) (void)hipEventDestroy(plan->ev[i]);
    if (plan->dev_blob) {
      const hipError_t e = hipFree(plan->dev_blob);
      if (e != hipSuccess) st = fail_hip(e, "tp_plan_destroy: hipFree");
    }
  }
  delete plan;
  return st;
}

sc_status tp_plan_info(const tp_plan* plan, tp_info* out) {
  if (!plan || !out) return set_error(SC_ERR_INVALID_ARG, "tp_plan_info: NULL argument");
  out->n_Y = plan->n_Y;
  out->n_h = plan->n_h;
  out->n_out = plan->n_out;
  out->num_paths = static_cast<int32_t>(plan->paths.size());
  out->specialised = plan->specialised ? 1 : 0;
  tp::spec_op_counts(plan->specialised, out->ops, out->flops);
  return SC_OK;
}

sc_status tp_plan_paths(const tp_plan* plan, int32_t* paths) {
  if (!plan || !paths) return set_error(SC_ERR_INVALID_ARG, "tp_plan_paths: NULL argument");
  for (size_t p = 0; p < plan->paths.size(); ++p)
    for (int k = 0; k < 3; ++k) paths[3 * p + k] = plan->paths[p][k];
  return SC_OK;
}

sc_status tp_plan_terms(const tp_plan* plan, int32_t capacity, int32_t* n_terms, int32_t* path, int32_t* a,
                        int32_t* b, int32_t* c, double* coef) {
  if (!plan || !n_terms) return set_error(SC_ERR_INVALID_ARG, "tp_plan_terms: NULL argument");
  *n_terms = static_cast<int32_t>(plan->terms.size());
  if (capacity == 0) return SC_OK;
  if (capacity < *n_terms || !path || !a || !b || !c || !coef)
    return set_error(SC_ERR_INVALID_ARG, "tp_plan_terms: buffers missing or too small");
  for (size_t t = 0; t < plan->terms.size(); ++t) {
    path[t] = plan->terms[t].p; a[t] = plan->terms[t].a; b[t] = plan->terms[t].b; c[t] = plan->terms[t].c;
    coef[t] = plan->terms[t].coef;
  }
  return SC_OK;
}

sc_status tp_profile_enable(tp_plan* plan, int32_t on) {
  if (!plan) return set_error(SC_ERR_INVALID_ARG, "tp_profile_enable: plan is NULL");
  if (plan->host_only) return set_error(SC_ERR_UNSUPPORTED, "tp_profile_enable: host-only plan");
  DeviceGuard guard(plan->cfg.device);
  if (!guard.ok) return set_error(SC_ERR_HIP, "tp_profile_enable: cannot make the plan's device current");
  if (on && !plan->ev[0]) {
    for (int i = 0; i < 8; ++i) {
      const hipError_t e = hipEventCreate(&plan->ev[i]);
      if (e != hipSuccess) {  // all or nothing: a later call starts from scratch
        for (int k = 0; k < i; ++k) (void)hipEventDestroy(plan->ev[k]);
        for (int k = 0; k < 8; ++k) plan->ev[k] = nullptr;
        plan->profile = false;
        return fail_hip(e, "tp_profile_enable: hipEventCreate");
      }
    }
  }
  plan->profile = on != 0;
  plan->ev_used[0] = plan->ev_used[1] = plan->ev_used[2] = plan->ev_used[3] = false;
  return SC_OK;
}

sc_status tp_profile_read(tp_plan* plan, float* forward_ms, float* backward_ms, float* dh_sum_ms) {
  if (!plan || !forward_ms || !backward_ms || !dh_sum_ms)
    return set_error(SC_ERR_INVALID_ARG, "tp_profile_read: NULL argument");
  float* out[3] = {forward_ms, backward_ms, dh_sum_ms};
  for (int k = 0; k < 3; ++k) {
    *out[k] = -1.0f;
    if (!plan->ev_used[k]) continue;
    hipError_t e = hipEventSynchronize(plan->ev[2 * k + 1]);
    if (e == hipSuccess) e = hipEventElapsedTime(out[k], plan->ev[2 * k], plan->ev[2 * k + 1]);
    if (e != hipSuccess) return fail_hip(e, "tp_profile_read");
  }
  return SC_OK;
}

sc_status tp_profile_read_double_backward(tp_plan* plan, float* ms) {
  if (!plan || !ms) return set_error(SC_ERR_INVALID_ARG, "tp_profile_read_double_backward: NULL argument");
  *ms = -1.0f;
  if (!plan->ev_used[3]) return SC_OK;
  hipError_t e = hipEventSynchronize(plan->ev[7]);
  if (e == hipSuccess) e = hipEventElapsedTime(ms, plan->ev[6], plan->ev[7]);
  if (e != hipSuccess) return fail_hip(e, "tp_profile_read_double_backward");
  return SC_OK;
}

sc_status tp_forward(tp_plan* plan, int64_t n_nodes_in, int64_t n_nodes_out, int64_t n_edges, const void* Y,
                     const void* h, const void* R, const int32_t* sender, const int32_t* row_ptr, void* A,
                     void* hip_stream) {
  sc_status st = check_sizes("tp_forward", plan, n_nodes_in, n_nodes_out, n_edges);
  if (st != SC_OK) return st;
  if (n_nodes_out == 0) return SC_OK;
  if (!A || !row_ptr) return set_error(SC_ERR_INVALID_ARG, "tp_forward: A or row_ptr is NULL");
  if (n_edges > 0 && (!Y || !h || !R || !sender)) return set_error(SC_ERR_INVALID_ARG, "tp_forward: NULL tensor argument");
  if (misaligned(Y, 16) || misaligned(h, 16) || misaligned(R, 16) || misaligned(A, 16) || misaligned(sender, 4) ||
      misaligned(row_ptr, 4))
    return set_error(SC_ERR_INVALID_ARG, "tp_forward: tensor pointer not 16-byte aligned");
  DeviceGuard guard(plan->cfg.device);
  if (!guard.ok) return set_error(SC_ERR_HIP, "tp_forward: cannot make the plan's device current");
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  const tp::FwdArgs a{n_nodes_in, n_nodes_out, n_edges, Y, h, R, sender, row_ptr, A};
  if (plan->profile) (void)hipEventRecord(plan->ev[0], stream);
  const hipError_t e = plan->specialised ? tp::launch_spec_forward(plan, a, stream)
                                         : tp::launch_generic_forward(plan, a, stream);
  if (e != hipSuccess) return fail_hip(e, "tp_forward: kernel launch");
  if (plan->profile) {
    (void)hipEventRecord(plan->ev[1], stream);
    plan->ev_used[0] = true;
  }
  return SC_OK;
}

sc_status tp_workspace_bytes(const tp_plan* plan, int64_t n_edges, size_t* bytes) {
  if (!plan || !bytes) return set_error(SC_ERR_INVALID_ARG, "tp_workspace_bytes: NULL argument");
  if (n_edges < 0 || n_edges > (int64_t(1) << 30))
    return set_error(SC_ERR_INVALID_ARG, "tp_workspace_bytes: n_edges outside 0..2^30");
  *bytes = align_up(static_cast<size_t>(chblocks_of(plan)) * n_edges * plan->n_Y * elem_size(plan), 256) +
           align_up(static_cast<size_t>(n_edges) * plan->cfg.num_channels * plan->n_h * elem_size(plan), 256) + 256;
  return SC_OK;
}

sc_status tp_backward(tp_plan* plan, int64_t n_nodes_in, int64_t n_nodes_out, int64_t n_edges, const void* Y,
                      const void* h, const void* R, const int32_t* sender, const int32_t* row_ptr,
                      const int32_t* send_ptr, const int32_t* send_edge, const void* dA, void* dY, void* dh,
                      void* dR, void* workspace, size_t workspace_bytes, void* hip_stream) {
  sc_status st = check_sizes("tp_backward", plan, n_nodes_in, n_nodes_out, n_edges);
  if (st != SC_OK) return st;
  if (n_nodes_in > 0 && (!dh || !send_ptr)) return set_error(SC_ERR_INVALID_ARG, "tp_backward: dh or send_ptr is NULL");
  if (n_nodes_out > 0 && !row_ptr) return set_error(SC_ERR_INVALID_ARG, "tp_backward: row_ptr is NULL");
  if (n_edges > 0) {
    if (!Y || !h || !R || !sender || !send_edge || !dA || !dY || !dR)
      return set_error(SC_ERR_INVALID_ARG, "tp_backward: NULL tensor argument");
    size_t need = 0;
    (void)tp_workspace_bytes(plan, n_edges, &need);
    if (!workspace || workspace_bytes < need)
      return set_error(SC_ERR_WORKSPACE, "tp_backward: workspace missing or smaller than tp_workspace_bytes()");
    if (misaligned(workspace, 256)) return set_error(SC_ERR_WORKSPACE, "tp_backward: workspace not 256-byte aligned");
  }
  if (misaligned(Y, 16) || misaligned(h, 16) || misaligned(R, 16) || misaligned(dA, 16) || misaligned(dY, 16) ||
      misaligned(dh, 16) || misaligned(dR, 16) || misaligned(sender, 4) ||
      misaligned(row_ptr, 4) || misaligned(send_ptr, 4) || misaligned(send_edge, 4))
    return set_error(SC_ERR_INVALID_ARG, "tp_backward: tensor pointer not 16-byte aligned");
  DeviceGuard guard(plan->cfg.device);
  if (!guard.ok) return set_error(SC_ERR_HIP, "tp_backward: cannot make the plan's device current");
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  char* dh_edge = workspace ? static_cast<char*>(workspace) +
                                  align_up(static_cast<size_t>(chblocks_of(plan)) * n_edges * plan->n_Y * elem_size(plan), 256)
                            : nullptr;
  const tp::BwdArgs a{n_nodes_in, n_nodes_out, n_edges, Y,  h,  R,         sender,
                      row_ptr,    send_ptr,    send_edge, dA, dY, dh, dR, workspace, dh_edge};
  hipError_t e = hipSuccess;
  if (plan->specialised) {
    // generated kernels: one pass over the edges grouped by sender writes dR, the dY partials and dh itself
    if (n_nodes_in > 0) {
      if (plan->profile) (void)hipEventRecord(plan->ev[2], stream);
      e = tp::launch_spec_backward(plan, a, stream);
      if (e != hipSuccess) return fail_hip(e, "tp_backward: edge kernel launch");
      if (plan->profile) {
        (void)hipEventRecord(plan->ev[3], stream);
        plan->ev_used[1] = true;
        (void)hipEventRecord(plan->ev[4], stream);   // no separate dh sum on this path
        (void)hipEventRecord(plan->ev[5], stream);
        plan->ev_used[2] = true;
      }
    }
    if (n_nodes_out > 0 && n_edges > 0) {
      e = tp::launch_dY_sum(plan, a, stream);
      if (e != hipSuccess) return fail_hip(e, "tp_backward: dY sum launch");
    }
    return SC_OK;
  }
  if (n_nodes_out > 0 && n_edges > 0) {
    if (plan->profile) (void)hipEventRecord(plan->ev[2], stream);
    e = tp::launch_generic_backward(plan, a, stream);
    if (e != hipSuccess) return fail_hip(e, "tp_backward: edge kernel launch");
    if (plan->profile) {
      (void)hipEventRecord(plan->ev[3], stream);
      plan->ev_used[1] = true;
    }
    e = tp::launch_dY_sum(plan, a, stream);
    if (e != hipSuccess) return fail_hip(e, "tp_backward: dY sum launch");
  }
  if (n_nodes_in > 0) {
    if (plan->profile) (void)hipEventRecord(plan->ev[4], stream);
    e = tp::launch_dh_sum(plan, a, stream);
    if (e != hipSuccess) return fail_hip(e, "tp_backward: dh sum launch");
    if (plan->profile) {
      (void)hipEventRecord(plan->ev[5], stream);
      plan->ev_used[2] = true;
    }
  }
  return SC_OK;
}

sc_status tp_double_backward(tp_plan* plan, int64_t n_nodes_in, int64_t n_nodes_out, int64_t n_edges, const void* Y,
                             const void* h, const void* R, const int32_t* sender, const int32_t* row_ptr,
                             const int32_t* send_ptr, const int32_t* send_edge, const void* dA, const void* HY,
                             const void* Hh, const void* HR, void* ddA, void* d2Y, void* d2h, void* d2R,
                             void* workspace, size_t workspace_bytes, void* hip_stream) {
  sc_status st = check_sizes("tp_double_backward", plan, n_nodes_in, n_nodes_out, n_edges);
  if (st != SC_OK) return st;
  if (n_nodes_in > 0 && (!d2h || !send_ptr))
    return set_error(SC_ERR_INVALID_ARG, "tp_double_backward: d2h or send_ptr is NULL");
  if (n_nodes_out > 0 && (!row_ptr || !ddA))
    return set_error(SC_ERR_INVALID_ARG, "tp_double_backward: row_ptr or ddA is NULL");
  if (n_edges > 0) {
    if (!Y || !h || !R || !sender || !send_edge || !dA || !HY || !Hh || !HR || !d2Y || !d2R)
      return set_error(SC_ERR_INVALID_ARG, "tp_double_backward: NULL tensor argument");
    size_t need = 0;
    (void)tp_workspace_bytes(plan, n_edges, &need);
    if (!workspace || workspace_bytes < need)
      return set_error(SC_ERR_WORKSPACE, "tp_double_backward: workspace missing or smaller than tp_workspace_bytes()");
    if (misaligned(workspace, 256))
      return set_error(SC_ERR_WORKSPACE, "tp_double_backward: workspace not 256-byte aligned");
  }
  if (misaligned(Y, 16) || misaligned(h, 16) || misaligned(R, 16) || misaligned(dA, 16) || misaligned(HY, 16) ||
      misaligned(Hh, 16) || misaligned(HR, 16) || misaligned(ddA, 16) || misaligned(d2Y, 16) || misaligned(d2h, 16) ||
      misaligned(d2R, 16) || misaligned(sender, 4) || misaligned(row_ptr, 4) || misaligned(send_ptr, 4) ||
      misaligned(send_edge, 4))
    return set_error(SC_ERR_INVALID_ARG, "tp_double_backward: tensor pointer not 16-byte aligned");
  DeviceGuard guard(plan->cfg.device);
  if (!guard.ok) return set_error(SC_ERR_HIP, "tp_double_backward: cannot make the plan's device current");
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  char* dh_edge = workspace ? static_cast<char*>(workspace) +
                                  align_up(static_cast<size_t>(chblocks_of(plan)) * n_edges * plan->n_Y * elem_size(plan), 256)
                            : nullptr;
  const tp::DblArgs a{{n_nodes_in, n_nodes_out, n_edges, Y, h, R, sender, row_ptr, send_ptr, send_edge, dA, d2Y, d2h,
                       d2R, workspace, dh_edge},
                      HY, Hh, HR, ddA};
  hipError_t e = hipSuccess;
  if (n_nodes_out > 0) {  // also with no edges: ddA is zeroed
    if (plan->profile) (void)hipEventRecord(plan->ev[6], stream);
    e = plan->specialised ? tp::launch_spec_double_backward(plan, a, stream)
                          : tp::launch_generic_double_backward(plan, a, stream);
    if (e != hipSuccess) return fail_hip(e, "tp_double_backward: edge kernel launch");
    if (plan->profile) {
      (void)hipEventRecord(plan->ev[7], stream);
      plan->ev_used[3] = true;
    }
    e = tp::launch_dY_sum(plan, a.b, stream);
    if (e != hipSuccess) return fail_hip(e, "tp_double_backward: d2Y sum launch");
  }
  if (n_nodes_in > 0) {
    e = tp::launch_dh_sum(plan, a.b, stream);
    if (e != hipSuccess) return fail_hip(e, "tp_double_backward: d2h sum launch");
  }
  return SC_OK;
}

}  // extern "C"
