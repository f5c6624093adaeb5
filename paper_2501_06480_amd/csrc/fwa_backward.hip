// Backward kernels (paper Algorithm 2) -- placeholder until implemented.
#include "fwa_internal.h"
namespace fwa {
int backward_slots(long long, int) { return 1; }
hipError_t launch_backward_bf16(const BwdArgs&, hipStream_t) { return hipErrorNotSupported; }
hipError_t launch_backward_f32(const BwdArgs&, hipStream_t) { return hipErrorNotSupported; }
}  // namespace fwa
