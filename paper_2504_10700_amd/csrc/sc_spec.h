// Generated straight-line kernels for selected configurations (see sc_spec.hip).
#pragma once
#include "sc_internal.h"

namespace sc {

// Returns the id (> 0) of the generated kernel that serves this plan, 0 if none.
int spec_lookup(const sc_plan* plan);
// Size of the internal (reduced) path basis of a generated kernel.
int spec_basis_size(int id);
// VALU instructions (ops) and flops per (node, channel) of forward, backward, second-order pass.
void spec_op_counts(int id, int32_t ops[3], int32_t flops[3]);
// Waves per workgroup (= per tile) of the generated kernels.
int spec_waves_per_tile();

// Bytes of the folded-weight table wf[element][channel][stride] of a generated kernel.
size_t spec_folded_bytes(const sc_plan* plan);

// Launch 1: folds W into ws.wfold (fold) and / or counts the elements of z (count: first half
// of the grouping).  Nothing is launched if both are false.
// window_order: workgroups of the launch also write ws.wnode / ws.wkey, the order in which the forward launch of
// the same call visits the nodes.
hipError_t launch_spec_prepare(const sc_plan* plan, int64_t n, const int32_t* z, const void* W, const Workspace& ws,
                               const LaunchShape& shape, bool count, bool fold, bool window_order, hipStream_t stream);
// Second half of the grouping as a launch of its own (after launch_spec_prepare with count);
// table_only: offsets and tile table without the permutation (the batch is already grouped).
hipError_t launch_spec_scatter(const sc_plan* plan, int64_t n, const int32_t* z, const Workspace& ws,
                               const LaunchShape& shape, bool table_only, hipStream_t stream);
// Forward over the nodes in natural order from ws.wfold; group: the second half of the grouping
// rides in the same launch (0 no, 1 permutation + tile table, 2 tile table only).
// component_major: the per-node tensors are laid out [node][component][channel]
// (SC_COMPONENT_MAJOR; plans whose rows are stored in the arithmetic type only).
// window_order: the kernel follows ws.wnode / ws.wkey, written by the prepare launch of the same call.
hipError_t launch_spec_forward(const sc_plan* plan, int64_t n, const void* A, const int32_t* z, void* B,
                               const Workspace& ws, const LaunchShape& shape, int group, bool window_order,
                               bool component_major, hipStream_t stream);
// The grouped passes read ws.perm (null: the batch is already grouped, identity) and ws.tiles; the backward reads ws.wfold, the second-order pass folds W itself.
hipError_t launch_spec_backward(const sc_plan* plan, int64_t n, const void* A, const void* dB, void* dA,
                                const Workspace& ws, const LaunchShape& shape, bool component_major,
                                hipStream_t stream);
hipError_t launch_spec_double_backward(const sc_plan* plan, int64_t n, const void* A, const void* W, const void* dB,
                                       const void* H, void* ddB, void* dA2, const Workspace& ws,
                                       const LaunchShape& shape, bool component_major, hipStream_t stream);

// dW reduction over the tiles of every element and unfold to the external paths.
hipError_t launch_spec_finalize(const sc_plan* plan, void* dW, const Workspace& ws, const LaunchShape& shape,
                                hipStream_t stream);

}  // namespace sc
