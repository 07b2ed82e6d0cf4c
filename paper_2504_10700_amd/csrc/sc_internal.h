// Internal declarations shared by the host API and the HIP kernels.
#pragma once
#include <hip/hip_runtime.h>

#include <cstddef>
#include <cstdint>
#include <string>
#include <vector>

#include "../../include/sc.h"
#include "sc_tables.h"

namespace sc {

constexpr int kLanes = 64;          // channels per wave (one lane per channel)
constexpr int kGroupWavesPerWG = 4; // grouping kernels: waves per workgroup
constexpr int kMaxGroupWaves = 256; // grouping kernels: total waves (rows of the count matrix)

// One tile = the nodes one workgroup of a main kernel processes: a run of
// consecutive positions of `perm` that all belong to one element.  id: the tile's rank in
// (element, position) order - the index of its row set among the per-tile dW rows; the grouping
// of the generated kernels stores the descriptors largest tile first, so id differs from the
// descriptor's own index there (the table-driven kernels keep both equal and ignore it).
struct TileDesc {
  int32_t z, start, count, id;
};

// Device-side view of the workspace (all pointers into the caller's buffer).
struct Workspace {
  int32_t* ntiles;     // [1]
  int32_t* seg_off;    // [Z+1] first position in perm of each element
  int32_t* tile_off;   // [Z+1] first tile of each element
  int32_t* counts;     // [kMaxGroupWaves][Z] scratch of the counting sort
  int32_t* perm;       // [N] node indices grouped by element (stable)
  TileDesc* tiles;     // [max_tiles]
  void* wfold;         // generated kernels: weights folded into the internal basis, [Z][K][stride]
  int32_t* wnode;      // generated kernels: [N] window order of the forward pass (node per position) ...
  int32_t* wkey;       // ... and [N] its element index (Z: outside the range)
  void* partial;       // [max_tiles][chblocks][S][64] per-tile dW contributions
  int32_t max_tiles;
  size_t bytes;
};

// Table-driven ("generic") kernel tables, device pointers.
struct GenericTables {
  int32_t num_paths, n_lm, n_LM;
  const int32_t* path_nu;     // [P]
  const int32_t* path_col;    // [P] first LM column of the path's output irrep
  const int32_t* term_begin;  // [P+1]
  const int4* term_idx;       // [n_terms] (M, i1, i2, i3)
  const double* term_coef;    // [n_terms]
};

struct LaunchShape {
  int tile_nodes;   // nodes per tile (per workgroup)
  int max_tiles;    // upper bound of the tile count = grid size / chblocks
  int chblocks;     // ceil(K / 64)
  int group_waves;  // rows used of the count matrix (0: single-launch grouping)
  int nodes_per_group_wave;
  // generated kernels: grouping as roles of the prepare / forward launches, forward tiles
  int split_waves;           // waves of the counting sort (a multiple of kGroupWavesPerWG)
  int split_nodes_per_wave;  // a multiple of 64
  int fwd_tile_nodes;        // consecutive nodes per workgroup of the natural-order forward (0: chosen at launch)
};

}  // namespace sc

struct sc_plan {
  sc_config cfg;
  sc::PathTable table;
  bool host_only = false;
  int specialised = 0;          // 0 = generic, else id of a generated kernel
  int S = 0;                    // size of the internal path basis
  int num_cus = 256;
  // optional kernel timing (sc_profile_enable): start/stop pairs of the forward, backward and
  // second-order main kernels
  bool profile = false;
  hipEvent_t ev[6] = {nullptr, nullptr, nullptr, nullptr, nullptr, nullptr};
  bool ev_used[3] = {false, false, false};
  // device copies
  void* dev_blob = nullptr;
  sc::GenericTables gen{};
};

namespace sc {

// Makes `device` the current HIP device for the lifetime of the object and restores the caller's
// device afterwards; ok is false if that failed.
struct DeviceGuard {
  int prev = -1;
  bool ok = false;
  explicit DeviceGuard(int device) {
    if (hipGetDevice(&prev) != hipSuccess) return;
    ok = (prev == device) || hipSetDevice(device) == hipSuccess;
    if (prev == device) prev = -1;
  }
  ~DeviceGuard() {
    if (prev >= 0) (void)hipSetDevice(prev);
  }
};

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
inline bool misaligned(const void* p, size_t a) { return reinterpret_cast<uintptr_t>(p) % a != 0; }

// Records the calling thread's error message (what sc_last_error returns) and returns code.
sc_status set_error(sc_status code, const std::string& msg);

LaunchShape launch_shape(const sc_plan* plan, int64_t n_nodes);
// forward_only: the part the forward pass uses (the grouping), without the weight-gradient rows.
Workspace carve_workspace(const sc_plan* plan, int64_t n_nodes, const LaunchShape& shape, void* base,
                          bool forward_only = false);

// kernels (defined in the .hip files); all return hipGetLastError() of their launches
hipError_t launch_grouping(const sc_plan* plan, int64_t n, const int32_t* z, const Workspace& ws,
                           const LaunchShape& shape, hipStream_t stream);
hipError_t launch_generic_forward(const sc_plan* plan, int64_t n, const void* A, const void* W, void* B,
                                  const Workspace& ws, const LaunchShape& shape, hipStream_t stream);
hipError_t launch_generic_backward(const sc_plan* plan, int64_t n, const void* A, const void* W,
                                   const void* dB, void* dA, const Workspace& ws, const LaunchShape& shape,
                                   hipStream_t stream);
hipError_t launch_generic_double_backward(const sc_plan* plan, int64_t n, const void* A, const void* W,
                                          const void* dB, const void* H, void* ddB, void* dA2,
                                          const Workspace& ws, const LaunchShape& shape, hipStream_t stream);
hipError_t launch_finalize(const sc_plan* plan, void* dW, const Workspace& ws, const LaunchShape& shape,
                           hipStream_t stream);

}  // namespace sc
