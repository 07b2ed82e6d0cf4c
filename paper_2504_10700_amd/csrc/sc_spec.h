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

hipError_t launch_spec_forward(const sc_plan* plan, int64_t n, const void* A, const void* W, void* B,
                               const Workspace& ws, const LaunchShape& shape, hipStream_t stream);
hipError_t launch_spec_backward(const sc_plan* plan, int64_t n, const void* A, const void* W, const void* dB,
                                void* dA, const Workspace& ws, const LaunchShape& shape, hipStream_t stream);
hipError_t launch_spec_double_backward(const sc_plan* plan, int64_t n, const void* A, const void* W,
                                       const void* dB, const void* H, void* ddB, void* dA2, const Workspace& ws,
                                       const LaunchShape& shape, hipStream_t stream);

// dW reduction over the tiles of every element and unfold to the external paths.
hipError_t launch_spec_finalize(const sc_plan* plan, void* dW, const Workspace& ws, const LaunchShape& shape,
                                hipStream_t stream);

}  // namespace sc
