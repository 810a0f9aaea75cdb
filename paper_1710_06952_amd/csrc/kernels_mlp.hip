// Minibatch gradient of the two-layer perceptron (placeholder until the MFMA
// kernels land: creation of an MLP engine fails with a clear message).
#include "device_common.hpp"
#include "internal.hpp"

namespace adpsgd_impl {

size_t mlp_scratch_bytes(int32_t, int32_t, int32_t, int32_t, int32_t) { return 0; }

hipError_t launch_mlp_gradient(const MlpGradArgs&, hipStream_t, int*) { return hipErrorNotSupported; }

}  // namespace adpsgd_impl
