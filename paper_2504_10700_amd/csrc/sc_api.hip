// C ABI entry points (see include/sc.h): argument checks, plan construction, workspace
// layout and kernel dispatch.  Everything numerical happens in the kernels.
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <string>

#include "sc_internal.h"
#include "sc_spec.h"

namespace {

using sc::align_up;
using sc::DeviceGuard;
using sc::misaligned;

thread_local std::string g_last_error;

sc_status fail(sc_status code, const std::string& msg) {
  g_last_error = msg;
  return code;
}

sc_status fail_hip(hipError_t e, const char* what) {
  return fail(SC_ERR_HIP, std::string(what) + ": " + hipGetErrorString(e));
}

__global__ void fill_zero_kernel(unsigned int* p, size_t n_words) {
  for (size_t i = blockIdx.x * static_cast<size_t>(blockDim.x) + threadIdx.x; i < n_words;
       i += static_cast<size_t>(gridDim.x) * blockDim.x)
    p[i] = 0u;
}

// bytes of one element of W / dW / the per-tile dW rows (fp32 also when the per-node rows are bfloat16)
size_t elem_size(const sc_plan* plan) { return plan->cfg.dtype == SC_F64 ? 8 : 4; }

// Scratch of sc_forward_noalloc: the grouping of one call (what sc_forward keeps in the caller's
// workspace).  Every GPU the library runs on holds its own copy of this array, at its own
// address, until the process ends.  In host code the array's NAME is only a handle for
// hipGetSymbolAddress, never a device address: host code uses the pointer noalloc_scratch()
// returns and nothing else.
static __device__ __align__(256) unsigned char scratch[SC_NOALLOC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};

// Address of `scratch` on `device`, which must be the current device.  Resolved once per device.
sc_status noalloc_scratch(int device, void** out) {
  if (device < 0 || device >= kMaxDevices)
    return fail(SC_ERR_UNSUPPORTED, "sc_forward_noalloc: device ordinal outside 0..63");
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[device]) {
    void* p = nullptr;
    const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return fail_hip(e, "sc_forward_noalloc: hipGetSymbolAddress");
    if (!p) return fail(SC_ERR_HIP, "sc_forward_noalloc: hipGetSymbolAddress returned a null address");
    g_scratch_ptr[device] = p;
  }
  *out = g_scratch_ptr[device];
  return SC_OK;
}


}  // namespace

namespace sc {

sc_status set_error(sc_status code, const std::string& msg) { return fail(code, msg); }

LaunchShape launch_shape(const sc_plan* plan, int64_t n) {
  LaunchShape s{};
  s.chblocks = (plan->cfg.num_channels + kLanes - 1) / kLanes;
  const int waves_per_tile = plan->specialised ? spec_waves_per_tile() : 1;
  const int64_t work = n * s.chblocks;
  int64_t t;
  if (plan->specialised) {
    // Generated kernels: the grouped sequence is cut every t positions and at element boundaries, and the
    // pieces are processed largest first (see split_table_role).  t: a whole number of nodes per wave such
    // that the whole pieces make about one and a half workgroups per compute unit (the shorter pieces next
    // to element boundaries fill the rest), at least two and at most 24 nodes per wave.  Measured on
    // MI355X, 128 channels, 89 elements of skewed frequency, us per step against t: 3072 nodes 8 -> 37.8,
    // 16 -> 34.2, 24 -> 35.8; 5000 nodes 12 -> 53.1, 24 -> 50.1, 40 -> 52.4; 10000 nodes 24 -> 83.0, 40 -> 81.9,
    // 56 -> 80.8, 80 -> 86.2; 15000 nodes 24 -> 107.5, 80 -> 106.1, 128 -> 117.4; 40000 nodes 32 -> 250.6,
    // 96 -> 246.0, 128 -> 258.1; 200000 nodes 64 -> 1160, 96 -> 1151, 128 -> 1155.
    const int64_t target = static_cast<int64_t>(plan->num_cus) * 3 / 2;
    t = (work + target - 1) / target;
    t = (t + waves_per_tile - 1) / waves_per_tile * waves_per_tile;
    const int64_t lo = 2 * waves_per_tile, hi = 24 * waves_per_tile;
    if (t < lo) t = lo;
    if (t > hi) t = hi;
    if (plan->cfg.tile_nodes > 0) t = plan->cfg.tile_nodes;
    s.tile_nodes = static_cast<int>(t);
    s.max_tiles = static_cast<int>(n / s.tile_nodes) + 1 + plan->cfg.num_elements;
  } else {
    // Table-driven kernels: every element's nodes split evenly into tiles of at most t nodes, about eight
    // (tile x channel block) workgroups per compute unit on small batches, bounded for large ones (the
    // per-tile dW rows cost memory traffic inversely proportional to the tile size).
    const int64_t target_wgs = static_cast<int64_t>(plan->num_cus) * 8;
    t = (work + target_wgs - 1) / target_wgs;
    const int64_t lo = work <= 2560 ? 2 : work <= 12288 ? 3 : 4, hi = 32;
    if (t < lo) t = lo;
    if (t > hi) t = hi;
    if (plan->cfg.tile_nodes > 0) t = plan->cfg.tile_nodes;
    s.tile_nodes = static_cast<int>(t);
    s.max_tiles = static_cast<int>(n / s.tile_nodes) + plan->cfg.num_elements;
  }
  // Grouping: one single-workgroup launch for small batches (group_waves = 0), else three
  // launches with about four 64-node chunks per wave, at most kMaxGroupWaves waves.
  if (n <= 16384 && plan->cfg.num_elements <= 512) {  // 16 waves x 16 chunks x 64 nodes
    s.group_waves = 0;
    s.nodes_per_group_wave = 0;
  } else {
    int64_t gw = (n + 255) / 256;
    gw = (gw + kGroupWavesPerWG - 1) / kGroupWavesPerWG * kGroupWavesPerWG;
    if (gw < kGroupWavesPerWG) gw = kGroupWavesPerWG;
    if (gw > kMaxGroupWaves) gw = kMaxGroupWaves;
    s.group_waves = static_cast<int>(gw);
    s.nodes_per_group_wave = static_cast<int>((n + gw - 1) / gw);
  }
  {  // generated kernels: four 64-node chunks per wave up to kMaxGroupWaves waves, whole chunks per wave
    int64_t gw = (n + 255) / 256;
    gw = (gw + kGroupWavesPerWG - 1) / kGroupWavesPerWG * kGroupWavesPerWG;
    if (gw < kGroupWavesPerWG) gw = kGroupWavesPerWG;
    if (gw > kMaxGroupWaves) gw = kMaxGroupWaves;
    s.split_waves = static_cast<int>(gw);
    s.split_nodes_per_wave = static_cast<int>(((n + gw - 1) / gw + kLanes - 1) / kLanes * kLanes);
    if (s.split_nodes_per_wave < kLanes) s.split_nodes_per_wave = kLanes;
    s.fwd_tile_nodes = 0;   // chosen at launch from the batch size and the kernel's occupancy
  }
  return s;
}

Workspace carve_workspace(const sc_plan* plan, int64_t n, const LaunchShape& shape, void* base, bool forward_only) {
  Workspace w{};
  const int Z = plan->cfg.num_elements;
  size_t off = 0;
  auto take = [&](size_t bytes) {
    void* p = base ? static_cast<char*>(base) + off : nullptr;
    off = align_up(off + bytes, 256);
    return p;
  };
  w.ntiles = static_cast<int32_t*>(take(sizeof(int32_t)));
  w.seg_off = static_cast<int32_t*>(take(sizeof(int32_t) * (Z + 1)));
  w.tile_off = static_cast<int32_t*>(take(sizeof(int32_t) * (Z + 1)));
  w.counts = static_cast<int32_t*>(take(sizeof(int32_t) * static_cast<size_t>(kMaxGroupWaves) * Z));
  w.perm = static_cast<int32_t*>(take(sizeof(int32_t) * static_cast<size_t>(n)));
  w.tiles = static_cast<TileDesc*>(take(sizeof(TileDesc) * static_cast<size_t>(shape.max_tiles)));
  if (plan->specialised) w.wfold = take(spec_folded_bytes(plan));
  if (plan->specialised) {
    w.wnode = static_cast<int32_t*>(take(sizeof(int32_t) * static_cast<size_t>(n)));
    w.wkey = static_cast<int32_t*>(take(sizeof(int32_t) * static_cast<size_t>(n)));
  }
  if (!forward_only)  // the weight-gradient rows of the backward passes
    w.partial = take(elem_size(plan) * static_cast<size_t>(shape.max_tiles) * shape.chblocks * plan->S * kLanes);
  w.max_tiles = shape.max_tiles;
  w.bytes = off;
  return w;
}

}  // namespace sc

extern "C" {

const char* sc_last_error(void) { return g_last_error.c_str(); }

sc_status sc_coupling_tensor(int32_t l1, int32_t l2, int32_t l3, double* out) {
  if (!out) return fail(SC_ERR_INVALID_ARG, "sc_coupling_tensor: out is NULL");
  if (l1 < 0 || l2 < 0 || l3 < 0 || l1 > 2 * SC_MAX_L || l2 > 2 * SC_MAX_L || l3 > 2 * SC_MAX_L)
    return fail(SC_ERR_INVALID_ARG, "sc_coupling_tensor: l outside 0..2*SC_MAX_L");
  const std::vector<double> c = sc::coupling_tensor(l1, l2, l3);
  std::memcpy(out, c.data(), c.size() * sizeof(double));
  return SC_OK;
}

sc_status sc_plan_create(const sc_config* cfg, sc_plan** out_plan) {
  if (!cfg || !out_plan) return fail(SC_ERR_INVALID_ARG, "sc_plan_create: NULL argument");
  *out_plan = nullptr;
  if (cfg->struct_size != static_cast<int32_t>(sizeof(sc_config)))
    return fail(SC_ERR_INVALID_ARG, "sc_plan_create: struct_size does not match this library's sc_config");
  if (cfg->num_channels < 1) return fail(SC_ERR_INVALID_ARG, "sc_plan_create: num_channels < 1");
  if (cfg->tile_nodes < 0 || cfg->tile_nodes > 65536)
    return fail(SC_ERR_INVALID_ARG, "sc_plan_create: tile_nodes outside 0..65536");
  if (cfg->dtype != SC_F32 && cfg->dtype != SC_F64 && cfg->dtype != SC_BF16)
    return fail(SC_ERR_INVALID_ARG, "sc_plan_create: bad dtype");
  if (cfg->l_max < 0 || cfg->l_max > SC_MAX_L) return fail(SC_ERR_UNSUPPORTED, "sc_plan_create: l_max outside 0..3");
  if (cfg->nu_max < 1 || cfg->nu_max > SC_MAX_NU)
    return fail(SC_ERR_UNSUPPORTED, "sc_plan_create: nu_max outside 1..3");
  if (cfg->num_elements < 1 || cfg->num_elements > SC_MAX_ELEMENTS)
    return fail(SC_ERR_UNSUPPORTED, "sc_plan_create: num_elements outside 1..SC_MAX_ELEMENTS");
  if (cfg->num_out < 1 || cfg->num_out > SC_MAX_OUT)
    return fail(SC_ERR_UNSUPPORTED, "sc_plan_create: num_out outside 1..SC_MAX_OUT");
  std::vector<int> out_l, out_p;
  for (int o = 0; o < cfg->num_out; ++o) {
    if (cfg->out_l[o] < 0 || cfg->out_l[o] > SC_MAX_L)
      return fail(SC_ERR_UNSUPPORTED, "sc_plan_create: output L outside 0..3");
    if (cfg->out_parity[o] != 1 && cfg->out_parity[o] != -1)
      return fail(SC_ERR_INVALID_ARG, "sc_plan_create: out_parity must be +1 or -1");
    for (int q = 0; q < o; ++q)
      if (cfg->out_l[q] == cfg->out_l[o] && cfg->out_parity[q] == cfg->out_parity[o])
        return fail(SC_ERR_INVALID_ARG, "sc_plan_create: duplicate output irrep");
    out_l.push_back(cfg->out_l[o]);
    out_p.push_back(cfg->out_parity[o]);
  }
  sc_plan* plan = new (std::nothrow) sc_plan();
  if (!plan) return fail(SC_ERR_ALLOC, "sc_plan_create: out of host memory");
  plan->cfg = *cfg;
  plan->host_only = (cfg->flags & SC_PLAN_HOST_ONLY) != 0;
  const char* msg = nullptr;
  if (!sc::build_path_table(cfg->l_max, cfg->nu_max, out_l, out_p, &plan->table, &msg)) {
    delete plan;
    return fail(SC_ERR_UNSUPPORTED, std::string("sc_plan_create: ") + (msg ? msg : "cannot build tables"));
  }
  const sc::PathTable& T = plan->table;
  const int P = static_cast<int>(T.paths.size());
  plan->specialised = (cfg->flags & SC_PLAN_FORCE_GENERIC) ? 0 : sc::spec_lookup(plan);
  plan->S = plan->specialised ? sc::spec_basis_size(plan->specialised) : P;
  if (cfg->dtype == SC_BF16 && !plan->specialised) {
    delete plan;
    return fail(SC_ERR_UNSUPPORTED, "sc_plan_create: SC_BF16 is served by the generated kernels only (l_max = 3, nu_max = 3, "
                                    "outputs 0e, 0e+1o, 0e+1o+2e or 0e+1o+2e+3o, or the tiny configuration; channels a multiple of 8)");
  }
  if (plan->host_only) {
    *out_plan = plan;
    return SC_OK;
  }

  DeviceGuard guard(cfg->device);
  if (!guard.ok) {
    delete plan;
    return fail(SC_ERR_HIP, "sc_plan_create: cannot make cfg->device current");
  }
  hipDeviceProp_t prop;
  hipError_t e = hipGetDeviceProperties(&prop, cfg->device);
  if (e != hipSuccess) {
    delete plan;
    return fail_hip(e, "sc_plan_create: hipGetDeviceProperties");
  }
  plan->num_cus = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;

  // one device blob: path_nu | path_col | term_begin | term_idx | term_coef
  std::vector<int32_t> path_nu(P), path_col(P), term_begin(P + 1, 0);
  std::vector<int4> term_idx;
  std::vector<double> term_coef;
  for (int p = 0; p < P; ++p) {
    path_nu[p] = T.paths[p].nu;
    path_col[p] = T.out_offset[T.paths[p].out];
    term_begin[p] = static_cast<int32_t>(term_idx.size());
    for (const sc::Term& t : T.terms[p]) {
      term_idx.push_back(make_int4(t.M, t.i1, t.i2 < 0 ? 0 : t.i2, t.i3 < 0 ? 0 : t.i3));
      term_coef.push_back(t.coef);
    }
  }
  term_begin[P] = static_cast<int32_t>(term_idx.size());

  size_t off = 0;
  auto reserve = [&](size_t bytes) {
    const size_t at = off;
    off = align_up(off + bytes, 256);
    return at;
  };
  const size_t o_nu = reserve(sizeof(int32_t) * P), o_col = reserve(sizeof(int32_t) * P),
               o_tb = reserve(sizeof(int32_t) * (P + 1)), o_ti = reserve(sizeof(int4) * term_idx.size()),
               o_tc = reserve(sizeof(double) * term_coef.size());
  std::vector<unsigned char> host(off ? off : 256, 0);
  std::memcpy(host.data() + o_nu, path_nu.data(), sizeof(int32_t) * P);
  std::memcpy(host.data() + o_col, path_col.data(), sizeof(int32_t) * P);
  std::memcpy(host.data() + o_tb, term_begin.data(), sizeof(int32_t) * (P + 1));
  std::memcpy(host.data() + o_ti, term_idx.data(), sizeof(int4) * term_idx.size());
  std::memcpy(host.data() + o_tc, term_coef.data(), sizeof(double) * term_coef.size());
  e = hipMalloc(&plan->dev_blob, host.size());
  if (e != hipSuccess) {
    delete plan;
    return fail(SC_ERR_ALLOC, std::string("sc_plan_create: hipMalloc: ") + hipGetErrorString(e));
  }
  e = hipMemcpy(plan->dev_blob, host.data(), host.size(), hipMemcpyHostToDevice);
  if (e != hipSuccess) {
    (void)hipFree(plan->dev_blob);
    delete plan;
    return fail_hip(e, "sc_plan_create: hipMemcpy");
  }
  char* d = static_cast<char*>(plan->dev_blob);
  plan->gen.num_paths = P;
  plan->gen.n_lm = T.n_lm;
  plan->gen.n_LM = T.n_LM;
  plan->gen.path_nu = reinterpret_cast<const int32_t*>(d + o_nu);
  plan->gen.path_col = reinterpret_cast<const int32_t*>(d + o_col);
  plan->gen.term_begin = reinterpret_cast<const int32_t*>(d + o_tb);
  plan->gen.term_idx = reinterpret_cast<const int4*>(d + o_ti);
  plan->gen.term_coef = reinterpret_cast<const double*>(d + o_tc);
  *out_plan = plan;
  return SC_OK;
}

sc_status sc_profile_enable(sc_plan* plan, int32_t on) {
  if (!plan) return fail(SC_ERR_INVALID_ARG, "sc_profile_enable: plan is NULL");
  if (plan->host_only) return fail(SC_ERR_UNSUPPORTED, "sc_profile_enable: host-only plan");
  DeviceGuard guard(plan->cfg.device);
  if (!guard.ok) return fail(SC_ERR_HIP, "sc_profile_enable: cannot make the plan's device current");
  if (on && !plan->ev[0]) {
    for (int i = 0; i < 6; ++i) {
      const hipError_t e = hipEventCreate(&plan->ev[i]);
      if (e != hipSuccess) {  // all or nothing: a later call starts from scratch
        for (int k = 0; k < i; ++k) (void)hipEventDestroy(plan->ev[k]);
        for (int k = 0; k < 6; ++k) plan->ev[k] = nullptr;
        plan->profile = false;
        return fail_hip(e, "sc_profile_enable: hipEventCreate");
      }
    }
  }
  plan->profile = on != 0;
  plan->ev_used[0] = plan->ev_used[1] = plan->ev_used[2] = false;
  return SC_OK;
}

sc_status sc_profile_read(sc_plan* plan, float* forward_ms, float* backward_ms) {
  if (!plan || !forward_ms || !backward_ms) return fail(SC_ERR_INVALID_ARG, "sc_profile_read: NULL argument");
  *forward_ms = *backward_ms = -1.0f;
  float* out[2] = {forward_ms, backward_ms};
  for (int k = 0; k < 2; ++k) {
    if (!plan->ev_used[k]) continue;
    hipError_t e = hipEventSynchronize(plan->ev[2 * k + 1]);
    if (e == hipSuccess) e = hipEventElapsedTime(out[k], plan->ev[2 * k], plan->ev[2 * k + 1]);
    if (e != hipSuccess) return fail_hip(e, "sc_profile_read");
  }
  return SC_OK;
}

sc_status sc_profile_read_double_backward(sc_plan* plan, float* ms) {
  if (!plan || !ms) return fail(SC_ERR_INVALID_ARG, "sc_profile_read_double_backward: NULL argument");
  *ms = -1.0f;
  if (!plan->ev_used[2]) return SC_OK;
  hipError_t e = hipEventSynchronize(plan->ev[5]);
  if (e == hipSuccess) e = hipEventElapsedTime(ms, plan->ev[4], plan->ev[5]);
  if (e != hipSuccess) return fail_hip(e, "sc_profile_read_double_backward");
  return SC_OK;
}

sc_status sc_plan_destroy(sc_plan* plan) {
  if (!plan) return SC_OK;
  sc_status st = SC_OK;
  if (!plan->host_only) {
    DeviceGuard guard(plan->cfg.device);  // events and tables belong to the plan's device
    for (int i = 0; i < 6; ++i)
      if (plan->ev[i]) (void)hipEventDestroy(plan->ev[i]);
    if (plan->dev_blob) {
      const hipError_t e = hipFree(plan->dev_blob);
      if (e != hipSuccess) st = fail_hip(e, "sc_plan_destroy: hipFree");
    }
  }
  delete plan;
  return st;
}

sc_status sc_plan_info(const sc_plan* plan, sc_info* out) {
  if (!plan || !out) return fail(SC_ERR_INVALID_ARG, "sc_plan_info: NULL argument");
  out->n_lm = plan->table.n_lm;
  out->n_LM = plan->table.n_LM;
  out->num_paths = static_cast<int32_t>(plan->table.paths.size());
  out->specialised = plan->specialised ? 1 : 0;
  sc::spec_op_counts(plan->specialised, out->ops, out->flops);
  return SC_OK;
}

sc_status sc_plan_paths(const sc_plan* plan, int32_t* paths) {
  if (!plan || !paths) return fail(SC_ERR_INVALID_ARG, "sc_plan_paths: NULL argument");
  for (size_t p = 0; p < plan->table.paths.size(); ++p) {
    const sc::Path& q = plan->table.paths[p];
    int32_t* row = paths + 6 * p;
    row[0] = q.nu; row[1] = q.out; row[2] = q.l1; row[3] = q.l2; row[4] = q.l3; row[5] = q.L2;
  }
  return SC_OK;
}

sc_status sc_plan_path_terms(const sc_plan* plan, int32_t path, int32_t capacity, int32_t* n_terms, int32_t* M,
                             int32_t* i1, int32_t* i2, int32_t* i3, double* coef) {
  if (!plan || !n_terms) return fail(SC_ERR_INVALID_ARG, "sc_plan_path_terms: NULL argument");
  if (path < 0 || path >= static_cast<int32_t>(plan->table.paths.size()))
    return fail(SC_ERR_INVALID_ARG, "sc_plan_path_terms: path index out of range");
  const std::vector<sc::Term>& t = plan->table.terms[path];
  *n_terms = static_cast<int32_t>(t.size());
  if (capacity == 0) return SC_OK;
  if (capacity < *n_terms || !M || !i1 || !i2 || !i3 || !coef)
    return fail(SC_ERR_INVALID_ARG, "sc_plan_path_terms: buffers missing or too small");
  for (size_t i = 0; i < t.size(); ++i) {
    M[i] = t[i].M; i1[i] = t[i].i1; i2[i] = t[i].i2; i3[i] = t[i].i3; coef[i] = t[i].coef;
  }
  return SC_OK;
}

sc_status sc_workspace_bytes(const sc_plan* plan, int64_t n_nodes, size_t* bytes) {
  if (!plan || !bytes) return fail(SC_ERR_INVALID_ARG, "sc_workspace_bytes: NULL argument");
  if (n_nodes < 0 || n_nodes > (int64_t(1) << 30))
    return fail(SC_ERR_INVALID_ARG, "sc_workspace_bytes: n_nodes outside 0..2^30");
  const sc::LaunchShape shape = sc::launch_shape(plan, n_nodes);
  *bytes = sc::carve_workspace(plan, n_nodes, shape, nullptr).bytes;
  return SC_OK;
}

static sc_status check_common(const char* fn, const sc_plan* plan, int64_t n, const void* workspace,
                              size_t workspace_bytes, sc::LaunchShape* shape, sc::Workspace* ws) {
  if (!plan) return fail(SC_ERR_INVALID_ARG, std::string(fn) + ": plan is NULL");
  if (plan->host_only) return fail(SC_ERR_UNSUPPORTED, std::string(fn) + ": plan was created with SC_PLAN_HOST_ONLY");
  if (n < 0 || n > (int64_t(1) << 30)) return fail(SC_ERR_INVALID_ARG, std::string(fn) + ": n_nodes outside 0..2^30");
  *shape = sc::launch_shape(plan, n);
  *ws = sc::carve_workspace(plan, n, *shape, const_cast<void*>(workspace));
  if (n > 0) {
    if (!workspace || workspace_bytes < ws->bytes)
      return fail(SC_ERR_WORKSPACE, std::string(fn) + ": workspace missing or smaller than sc_workspace_bytes()");
    if (misaligned(workspace, 256)) return fail(SC_ERR_WORKSPACE, std::string(fn) + ": workspace not 256-byte aligned");
  }
  return SC_OK;
}

// What a grouped pass (backward, second-order) needs before its main kernel: the grouping and, for
// the generated kernels, the folded weights, unless the flags say the workspace still holds them.
// Records the error message itself.
static hipError_t grouped_pass_prologue(const char* fn, sc_plan* plan, int64_t n_nodes, const int32_t* z, const void* W,
                                        const sc::Workspace& ws, const sc::LaunchShape& shape, uint32_t flags,
                                        bool uses_folded_table, hipStream_t stream) {
  const bool group = !(flags & SC_REUSE_GROUPING);
  hipError_t e = hipSuccess;
  if (plan->specialised) {
    e = sc::launch_spec_prepare(plan, n_nodes, z, W, ws, shape, group, uses_folded_table && !(flags & SC_REUSE_WEIGHTS),
                                false, stream);
    if (e == hipSuccess && group) e = sc::launch_spec_scatter(plan, n_nodes, z, ws, shape, (flags & SC_Z_GROUPED) != 0, stream);
  } else if (group) {
    e = sc::launch_grouping(plan, n_nodes, z, ws, shape, stream);
  }
  if (e != hipSuccess) (void)fail_hip(e, (std::string(fn) + ": grouping / weight-fold launch").c_str());
  return e;
}

// SC_COMPONENT_MAJOR is served by the generated kernels of plans whose rows
// are stored in the arithmetic type.
static sc_status check_layout_flag(const char* fn, const sc_plan* plan, uint32_t flags) {
  if (!(flags & SC_COMPONENT_MAJOR)) return SC_OK;
  if (!plan->specialised)
    return fail(SC_ERR_UNSUPPORTED, std::string(fn) + ": SC_COMPONENT_MAJOR needs a plan served by a generated kernel (sc_info.specialised)");
  if (plan->cfg.dtype == SC_BF16)
    return fail(SC_ERR_UNSUPPORTED, std::string(fn) + ": SC_COMPONENT_MAJOR is not served for bfloat16 rows");
  return SC_OK;
}

// Checks of the tensor arguments and the launches of the forward pass, shared by sc_forward and
// sc_forward_noalloc; the plan's device is current.
static sc_status forward_launches(const char* fn, sc_plan* plan, int64_t n_nodes, const void* A, const int32_t* z,
                                  const void* W, void* B, const sc::Workspace& ws, const sc::LaunchShape& shape,
                                  uint32_t flags, hipStream_t stream) {
  if (!A || !z || !W || !B) return fail(SC_ERR_INVALID_ARG, std::string(fn) + ": NULL tensor argument");
  if (misaligned(A, 16) || misaligned(W, 16) || misaligned(B, 16) || misaligned(z, 4))
    return fail(SC_ERR_INVALID_ARG, std::string(fn) + ": tensor pointer not 16-byte aligned");
  const sc_status layout = check_layout_flag(fn, plan, flags);
  if (layout != SC_OK) return layout;
  hipError_t e = hipSuccess;
  const bool group = !(flags & SC_REUSE_GROUPING);
  // the prepare launch also orders windows of the batch by element for the forward kernel (not for a
  // batch that is ordered already, nor for small ones, where that costs more than it saves)
  const bool window_order = plan->specialised && !(flags & SC_Z_GROUPED) && ws.wnode != nullptr &&
                            (n_nodes >= SC_WINDOW_ORDER_MIN_NODES || (plan->cfg.flags & SC_PLAN_WINDOW_ORDER));
  if (plan->specialised) {
    // the forward itself needs no grouping: the two halves of it ride in the prepare and the forward launch
    e = sc::launch_spec_prepare(plan, n_nodes, z, W, ws, shape, group, !(flags & SC_REUSE_WEIGHTS), window_order, stream);
    if (e != hipSuccess) return fail_hip(e, (std::string(fn) + ": prepare launch").c_str());
  } else if (group) {
    e = sc::launch_grouping(plan, n_nodes, z, ws, shape, stream);
    if (e != hipSuccess) return fail_hip(e, (std::string(fn) + ": grouping launch").c_str());
  }
  if (plan->profile) (void)hipEventRecord(plan->ev[0], stream);
  e = plan->specialised ? sc::launch_spec_forward(plan, n_nodes, A, z, B, ws, shape,
                                                  !group ? 0 : (flags & SC_Z_GROUPED) ? 2 : 1, window_order,
                                                  (flags & SC_COMPONENT_MAJOR) != 0, stream)
                        : sc::launch_generic_forward(plan, n_nodes, A, W, B, ws, shape, stream);
  if (e != hipSuccess) return fail_hip(e, (std::string(fn) + ": kernel launch").c_str());
  if (plan->profile) {
    (void)hipEventRecord(plan->ev[1], stream);
    plan->ev_used[0] = true;
  }
  return SC_OK;
}

sc_status sc_forward(sc_plan* plan, int64_t n_nodes, const void* A, const int32_t* z, const void* W, void* B,
                     void* workspace, size_t workspace_bytes, uint32_t flags, void* hip_stream) {
  sc::LaunchShape shape;
  sc::Workspace ws;
  sc_status st = check_common("sc_forward", plan, n_nodes, workspace, workspace_bytes, &shape, &ws);
  if (st != SC_OK) return st;
  if (n_nodes == 0) return SC_OK;
  DeviceGuard guard(plan->cfg.device);
  if (!guard.ok) return fail(SC_ERR_HIP, "sc_forward: cannot make the plan's device current");
  return forward_launches("sc_forward", plan, n_nodes, A, z, W, B, ws, shape, flags, static_cast<hipStream_t>(hip_stream));
}

sc_status sc_forward_noalloc(sc_plan* plan, int64_t n_nodes, const void* A, const int32_t* z, const void* W, void* B,
                             void* hip_stream) {
  if (!plan) return fail(SC_ERR_INVALID_ARG, "sc_forward_noalloc: plan is NULL");
  if (plan->host_only) return fail(SC_ERR_UNSUPPORTED, "sc_forward_noalloc: plan was created with SC_PLAN_HOST_ONLY");
  if (n_nodes < 0) return fail(SC_ERR_INVALID_ARG, "sc_forward_noalloc: n_nodes < 0");
  if (n_nodes > SC_NOALLOC_MAX_NODES)
    return fail(SC_ERR_WORKSPACE, "sc_forward_noalloc: n_nodes = " + std::to_string(n_nodes) + " exceeds SC_NOALLOC_MAX_NODES = " +
                                      std::to_string(SC_NOALLOC_MAX_NODES) + "; use sc_forward with a workspace");
  const sc::LaunchShape shape = sc::launch_shape(plan, n_nodes);
  const size_t need = sc::carve_workspace(plan, n_nodes, shape, nullptr, true).bytes;
  if (need > SC_NOALLOC_SCRATCH_BYTES)
    return fail(SC_ERR_WORKSPACE, "sc_forward_noalloc: this plan needs " + std::to_string(need) + " bytes of scratch for " +
                                      std::to_string(n_nodes) + " nodes, more than SC_NOALLOC_SCRATCH_BYTES = " +
                                      std::to_string(SC_NOALLOC_SCRATCH_BYTES) + "; use sc_forward with a workspace");
  if (n_nodes == 0) return SC_OK;
  DeviceGuard guard(plan->cfg.device);
  if (!guard.ok) return fail(SC_ERR_HIP, "sc_forward_noalloc: cannot make the plan's device current");
  void* base = nullptr;
  const sc_status st = noalloc_scratch(plan->cfg.device, &base);
  if (st != SC_OK) return st;
  // Nothing in the scratch has to start at zero: the launches that precede the forward kernel
  // write every word it reads (the folded weights of all elements and, from
  // SC_WINDOW_ORDER_MIN_NODES nodes on, the window order of all n_nodes positions; for the
  // table-driven kernels the permutation, the offsets and all max_tiles tile descriptors),
  // whatever an earlier, larger call left there.  The generated forward kernel needs no grouping,
  // and there is no backward pass to leave one for.
  const sc::Workspace ws = sc::carve_workspace(plan, n_nodes, shape, base, true);
  return forward_launches("sc_forward_noalloc", plan, n_nodes, A, z, W, B, ws, shape,
                          plan->specialised ? SC_REUSE_GROUPING : 0u, static_cast<hipStream_t>(hip_stream));
}

sc_status sc_backward(sc_plan* plan, int64_t n_nodes, const void* A, const int32_t* z, const void* W, const void* dB,
                      void* dA, void* dW, void* workspace, size_t workspace_bytes, uint32_t flags,
                      void* hip_stream) {
  sc::LaunchShape shape;
  sc::Workspace ws;
  sc_status st = check_common("sc_backward", plan, n_nodes, workspace, workspace_bytes, &shape, &ws);
  if (st != SC_OK) return st;
  if (!dW) return fail(SC_ERR_INVALID_ARG, "sc_backward: dW is NULL");
  if (misaligned(dW, 16)) return fail(SC_ERR_INVALID_ARG, "sc_backward: dW not 16-byte aligned");
  DeviceGuard guard(plan->cfg.device);
  if (!guard.ok) return fail(SC_ERR_HIP, "sc_backward: cannot make the plan's device current");
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  if (n_nodes == 0) {
    const size_t words = elem_size(plan) / 4 * static_cast<size_t>(plan->cfg.num_elements) *
                         plan->table.paths.size() * plan->cfg.num_channels;
    hipLaunchKernelGGL(fill_zero_kernel, dim3(256), dim3(256), 0, stream, static_cast<unsigned int*>(dW), words);
    const hipError_t e0 = hipGetLastError();
    if (e0 != hipSuccess) return fail_hip(e0, "sc_backward: fill launch");
    return SC_OK;
  }
  if (!A || !z || !W || !dB || !dA) return fail(SC_ERR_INVALID_ARG, "sc_backward: NULL tensor argument");
  if (misaligned(A, 16) || misaligned(W, 16) || misaligned(dB, 16) || misaligned(dA, 16) || misaligned(z, 4))
    return fail(SC_ERR_INVALID_ARG, "sc_backward: tensor pointer not 16-byte aligned");
  st = check_layout_flag("sc_backward", plan, flags);
  if (st != SC_OK) return st;
  if (plan->specialised && (flags & SC_Z_GROUPED)) ws.perm = nullptr;   // identity: rows are read in batch order
  hipError_t e = grouped_pass_prologue("sc_backward", plan, n_nodes, z, W, ws, shape, flags, true, stream);
  if (e != hipSuccess) return SC_ERR_HIP;
  if (plan->profile) (void)hipEventRecord(plan->ev[2], stream);
  e = plan->specialised ? sc::launch_spec_backward(plan, n_nodes, A, dB, dA, ws, shape, (flags & SC_COMPONENT_MAJOR) != 0, stream)
                        : sc::launch_generic_backward(plan, n_nodes, A, W, dB, dA, ws, shape, stream);
  if (e != hipSuccess) return fail_hip(e, "sc_backward: kernel launch");
  if (plan->profile) {
    (void)hipEventRecord(plan->ev[3], stream);
    plan->ev_used[1] = true;
  }
  e = plan->specialised ? sc::launch_spec_finalize(plan, dW, ws, shape, stream)
                        : sc::launch_finalize(plan, dW, ws, shape, stream);
  if (e != hipSuccess) return fail_hip(e, "sc_backward: finalize launch");
  return SC_OK;
}

sc_status sc_double_backward(sc_plan* plan, int64_t n_nodes, const void* A, const int32_t* z, const void* W,
                             const void* dB, const void* H, void* ddB, void* dA2, void* dW2, void* workspace,
                             size_t workspace_bytes, uint32_t flags, void* hip_stream) {
  sc::LaunchShape shape;
  sc::Workspace ws;
  sc_status st = check_common("sc_double_backward", plan, n_nodes, workspace, workspace_bytes, &shape, &ws);
  if (st != SC_OK) return st;
  if (!dW2) return fail(SC_ERR_INVALID_ARG, "sc_double_backward: dW2 is NULL");
  if (misaligned(dW2, 16)) return fail(SC_ERR_INVALID_ARG, "sc_double_backward: dW2 not 16-byte aligned");
  DeviceGuard guard(plan->cfg.device);
  if (!guard.ok) return fail(SC_ERR_HIP, "sc_double_backward: cannot make the plan's device current");
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  if (n_nodes == 0) {
    const size_t words = elem_size(plan) / 4 * static_cast<size_t>(plan->cfg.num_elements) *
                         plan->table.paths.size() * plan->cfg.num_channels;
    hipLaunchKernelGGL(fill_zero_kernel, dim3(256), dim3(256), 0, stream, static_cast<unsigned int*>(dW2), words);
    const hipError_t e0 = hipGetLastError();
    if (e0 != hipSuccess) return fail_hip(e0, "sc_double_backward: fill launch");
    return SC_OK;
  }
  if (!A || !z || !W || !dB || !H || !ddB || !dA2)
    return fail(SC_ERR_INVALID_ARG, "sc_double_backward: NULL tensor argument");
  if (misaligned(A, 16) || misaligned(W, 16) || misaligned(dB, 16) || misaligned(H, 16) || misaligned(ddB, 16) ||
      misaligned(dA2, 16) || misaligned(z, 4))
    return fail(SC_ERR_INVALID_ARG, "sc_double_backward: tensor pointer not 16-byte aligned");
  st = check_layout_flag("sc_double_backward", plan, flags);
  if (st != SC_OK) return st;
  if (plan->specialised && (flags & SC_Z_GROUPED)) ws.perm = nullptr;   // identity: rows are read in batch order
  hipError_t e = grouped_pass_prologue("sc_double_backward", plan, n_nodes, z, W, ws, shape, flags, false, stream);
  if (e != hipSuccess) return SC_ERR_HIP;
  if (plan->profile) (void)hipEventRecord(plan->ev[4], stream);
  e = plan->specialised
          ? sc::launch_spec_double_backward(plan, n_nodes, A, W, dB, H, ddB, dA2, ws, shape,
                                            (flags & SC_COMPONENT_MAJOR) != 0, stream)
          : sc::launch_generic_double_backward(plan, n_nodes, A, W, dB, H, ddB, dA2, ws, shape, stream);
  if (e != hipSuccess) return fail_hip(e, "sc_double_backward: kernel launch");
  if (plan->profile) {
    (void)hipEventRecord(plan->ev[5], stream);
    plan->ev_used[2] = true;
  }
  e = plan->specialised ? sc::launch_spec_finalize(plan, dW2, ws, shape, stream)
                        : sc::launch_finalize(plan, dW2, ws, shape, stream);
  if (e != hipSuccess) return fail_hip(e, "sc_double_backward: finalize launch");
  return SC_OK;
}

}  // extern "C"
