/*
 * ssd_measure.h -- measurement aids around the SSD library, in a library of their own
 * (libssd_measure.so: the same sources as libssd_hip.so plus these two calls), so
 * that the product library exports only calls that allocate nothing, create nothing
 * and never synchronise.  Both calls below create and destroy HIP events and WAIT.
 */
#ifndef SSD_MEASURE_H_
#define SSD_MEASURE_H_

#include "ssd.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * ssd_prefill (Alg. 1; see ssd.h) with a HIP event recorded on `hip_stream` after
 * every kernel of the call (the prefill of Alg. 1 is several kernels).  The
 * call is enqueued twice back to back and the second run is the timed one, so
 * that no interval includes the host's enqueue latency.  Unlike
 * every other entry point it creates and destroys HIP events and WAITS for the
 * call to finish.  On return kernel_ms[i] (HOST array of max_kernels floats)
 * holds the duration in milliseconds of the i-th kernel, kernel_names[i] (HOST
 * array of max_kernels pointers) a static string naming it, *num_kernels their
 * count.  The results in y / final_state are those of ssd_prefill.
 */
SSD_API ssd_status ssd_prefill_profile(const ssd_shape *shape, const void *x, const float *dt,
                               const float *A, const void *B, const void *C,
                               const float *D, const float *h0, void *y,
                               float *final_state, void *workspace,
                               size_t workspace_bytes, void *hip_stream,
                               int32_t max_kernels, float *kernel_ms,
                               const char **kernel_names, int32_t *num_kernels);

/*
 * Machine peaks as this library's own kernels reach them, to
 * set the figures of the SSD kernels against.  Like ssd_prefill_profile it
 * creates HIP events and WAITS.
 *   kind 0   MFMA issue loop: 2048 workgroups of 4 waves, each wave `iters`
 *            times eight v_mfma_f32_32x32x16_bf16; `a` = device scratch of at
 *            least 2048*256 floats (`bytes` its size), `b` unused
 *   kind 1   streaming copy of `bytes` bytes from `a` to `b` (16 bytes per lane)
 *   kind 2   streaming read of `a` (b: 16 bytes of scratch)
 *   kind 3   streaming write of `b` (a: any valid device pointer)
 *   kind 4..6  as 1..3 with non-temporal loads and stores (what the decode step
 *            uses for a state larger than the memory-side cache)
 *   kind 7, 8  as 0 on the fp32 matrix instructions v_mfma_f32_32x32x2_f32 (what
 *            the fp32 prefill kernel uses) and v_mfma_f32_16x16x4_f32
 * One warm-up launch, then `reps` launches back to back; *ms (HOST) = their
 * total time in milliseconds, *work (HOST) = flops (kind 0) or bytes moved
 * (read + written) of ONE launch.
 * Errors: SSD_ERR_NULL, _SHAPE, _ALIGN, _HIP.
 */
SSD_API ssd_status ssd_peak_probe(int32_t kind, int32_t iters, int32_t reps, void *a, void *b,
                          size_t bytes, float *ms, double *work, void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* SSD_MEASURE_H_ */
