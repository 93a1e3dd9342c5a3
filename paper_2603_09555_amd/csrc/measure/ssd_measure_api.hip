// Entry points of the measurement library (declared in include/ssd_measure.h).  Unlike the product
// library's calls they create HIP events and wait for the device.
#include "ssd_internal.hpp"
#include "ssd_measure.h"

namespace ssd {
hipError_t run_peak_probe(int kind, int iters, int reps, void *a, void *b, size_t bytes, float *ms, double *work,
                          hipStream_t stream);
}

extern "C" {

ssd_status ssd_prefill_profile(const ssd_shape *shape, const void *x, const float *dt, const float *A,
                               const void *B, const void *C, const float *D, const float *h0, void *y,
                               float *final_state, void *workspace, size_t workspace_bytes_given,
                               void *hip_stream, int32_t max_kernels, float *kernel_ms,
                               const char **kernel_names, int32_t *num_kernels) {
  if (!kernel_ms || !kernel_names || !num_kernels || max_kernels < 1) return SSD_ERR_NULL;
  *num_kernels = 0;
  ssd::KernelTrace trace;
  int made = 0;
  for (; made <= ssd::KernelTrace::kMax; ++made)
    if (hipEventCreate(&trace.ev[made]) != hipSuccess) break;
  ssd_status st = SSD_ERR_HIP;
  if (made == ssd::KernelTrace::kMax + 1) {
    // The call is enqueued twice back to back and the second one carries the events: its launches reach a
    // busy GPU, so the first interval does not include the host's enqueue latency.  (h0 may alias
    // final_state: only then would a second run start from another state, so the first one is skipped.)
    st = h0 != nullptr && h0 == final_state
             ? SSD_OK
             : ssd::prefill_traced(shape, x, dt, A, B, C, D, h0, y, final_state, workspace, workspace_bytes_given,
                                   hip_stream, nullptr);
    if (st == SSD_OK)
      st = ssd::prefill_traced(shape, x, dt, A, B, C, D, h0, y, final_state, workspace, workspace_bytes_given,
                               hip_stream, &trace);
    if (st == SSD_OK) {
      if (trace.n > 0 && hipEventSynchronize(trace.ev[trace.n]) != hipSuccess) st = SSD_ERR_HIP;
      for (int i = 0; st == SSD_OK && i < trace.n && i < max_kernels; ++i) {
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, trace.ev[i], trace.ev[i + 1]) != hipSuccess) st = SSD_ERR_HIP;
        kernel_ms[i] = ms;
        kernel_names[i] = trace.names[i];
        *num_kernels = i + 1;
      }
    }
  }
  for (int i = 0; i < made; ++i) (void)hipEventDestroy(trace.ev[i]);
  return st;
}

ssd_status ssd_peak_probe(int32_t kind, int32_t iters, int32_t reps, void *a, void *b, size_t bytes, float *ms,
                          double *work, void *hip_stream) {
  if (!ms || !work || !a) return SSD_ERR_NULL;
  if (kind < 0 || kind > 8 || reps < 1 || reps > 100000) return SSD_ERR_SHAPE;
  const bool mfma = kind == 0 || kind >= 7;
  if (mfma && (iters < 1 || bytes < static_cast<size_t>(2048) * 256 * sizeof(float))) return SSD_ERR_SHAPE;
  if (!mfma && !b) return SSD_ERR_NULL;
  if (!mfma && bytes < 16) return SSD_ERR_SHAPE;
  if ((reinterpret_cast<uintptr_t>(a) & 15u) || (b && (reinterpret_cast<uintptr_t>(b) & 15u))) return SSD_ERR_ALIGN;
  const hipError_t e = ssd::run_peak_probe(kind, iters, reps, a, b, bytes, ms, work, static_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? SSD_OK : SSD_ERR_HIP;
}

}  // extern "C"
