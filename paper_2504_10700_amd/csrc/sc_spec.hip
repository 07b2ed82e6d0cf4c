// Dispatch to the generated straight-line kernels.
#include "sc_spec.h"

namespace sc {

int spec_lookup(const sc_plan*) { return 0; }
int spec_basis_size(int) { return 0; }
int spec_waves_per_tile() { return 4; }
void spec_fold(int, std::vector<int32_t>*, std::vector<int32_t>*, std::vector<double>*) {}

hipError_t launch_spec_forward(const sc_plan*, int64_t, const void*, const void*, void*, const Workspace&,
                               const LaunchShape&, hipStream_t) {
  return hipErrorNotSupported;
}
hipError_t launch_spec_backward(const sc_plan*, int64_t, const void*, const void*, const void*, void*,
                                const Workspace&, const LaunchShape&, hipStream_t) {
  return hipErrorNotSupported;
}

}  // namespace sc
