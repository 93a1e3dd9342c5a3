// MFMA prefill path (placeholder until the bf16 kernels land: reports "not supported" so that
// every shape takes the generic fp32 kernels).
#include "ssd_internal.hpp"

namespace ssd {
bool mfma_supported(const Dims &) { return false; }
size_t mfma_workspace_bytes(const Dims &) { return 0; }
hipError_t launch_prefill_mfma(const Dims &, const void *, const float *, const float *, const void *,
                               const void *, const float *, const float *, void *, float *, void *,
                               hipStream_t, KernelTrace *) {
  return hipErrorNotSupported;
}
}  // namespace ssd
