/*
 * ssd.h -- C ABI of the MI355X (gfx950) SSD layer-core library.
 *
 * The library computes the Mamba-2 state-space-duality layer core of
 * "Compiler-First State Space Duality and Portable O(1) Autoregressive
 * Caching": the chunked-parallel prefill (Alg. 1, lines "Discretise" to
 * "Store"; Eq. 3; appendix "Exact SSD Einsum Signatures") and the O(1) cached
 * decode step (Alg. 2, "Discretise" and "SSM step"; Eq. 2 for the output).
 *
 * Conventions shared by every entry point
 * ---------------------------------------
 *  - Every data pointer is a DEVICE pointer owned by the caller.  The library
 *    allocates nothing, frees nothing, keeps no pointer after the call and
 *    never synchronises: work is enqueued on `hip_stream` (a hipStream_t
 *    passed as void*; NULL = the default stream) and the call returns.
 *  - Tensors are dense, row-major (last index fastest), 16-byte aligned, in
 *    the axis order of the paper's einsum signatures:
 *        x, y           (batch, seqlen, nheads, headdim)      io dtype
 *        B, C           (batch, seqlen, ngroups, dstate)      io dtype
 *        dt             (batch, seqlen, nheads)               fp32, > 0: the final step
 *                       size (softplus / bias / clamp are the caller's job)
 *        A, D           (nheads)                              fp32; A <= 0 is the
 *                       already negative per-head scalar, Abar = exp(dt*A)
 *        state, h0      (batch, nheads, headdim, dstate)      fp32
 *    Head h reads B/C group h / (nheads / ngroups).
 *  - io dtype (x, B, C, y) is fp32 or bf16; bf16 values are the upper 16 bits
 *    of the fp32 pattern.  y is rounded to the io dtype with round-to-nearest-
 *    even.  All decay arithmetic (dt*A, its prefix sums, exp) and every
 *    accumulation are fp32 (section "Mapping SSD onto JAX primitives",
 *    precision rules).
 *  - Arguments are validated on the host before any HIP call; an invalid call
 *    returns a negative ssd_status and enqueues nothing.  Device data is not
 *    inspected; what it must satisfy is A <= 0 and dt >= 0 (after the optional
 *    step-size map of the *_dt entry points), nothing else: there is no upper
 *    bound on dt*|A|.  (The bf16 prefill factorises the decay mask of Eq. 3
 *    around the middle of each 64-token block; a block of a head whose decay
 *    across half the block exceeds 2^96 takes the un-factorised mask instead,
 *    whose exponents are never positive, so any step size gives the result of
 *    the recurrence.)  No C++ exception crosses this boundary.
 *  - Results do not depend on `chunk` beyond floating-point summation order.
 *    Runs are bitwise reproducible (no floating-point atomics).
 */
#ifndef SSD_H_
#define SSD_H_

#include <stddef.h>
#include <stdint.h>

#if defined(__GNUC__)
#define SSD_API __attribute__((visibility("default")))
#else
#define SSD_API
#endif

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { SSD_F32 = 0, SSD_BF16 = 1 } ssd_dtype;

typedef enum {
  SSD_OK = 0,
  SSD_ERR_NULL = -1,        /* a required pointer is NULL */
  SSD_ERR_SHAPE = -2,       /* a dimension is < 1, nheads % ngroups != 0, or a size overflows */
  SSD_ERR_DTYPE = -3,       /* io_dtype is not SSD_F32 / SSD_BF16 */
  SSD_ERR_UNSUPPORTED = -4, /* valid but not implemented (see each entry point) */
  SSD_ERR_WORKSPACE = -5,   /* workspace NULL, misaligned or smaller than required */
  SSD_ERR_HIP = -6,         /* a HIP launch reported an error */
  SSD_ERR_ALIGN = -7,       /* a tensor pointer is not 16-byte aligned */
  SSD_ERR_TOO_LARGE = -8    /* ssd_prefill_static: the shape needs more scratch than the library holds */
} ssd_status;

/* Plain data, filled by the caller; the library never keeps the pointer. */
typedef struct {
  int32_t batch;    /* Bt */
  int32_t seqlen;   /* T  (ignored by the decode entry points) */
  int32_t nheads;   /* H  */
  int32_t headdim;  /* P  */
  int32_t dstate;   /* N  */
  int32_t ngroups;  /* G, divides H */
  int32_t chunk;    /* L  (ignored by the decode entry points) */
  int32_t io_dtype; /* ssd_dtype of x, B, C, y */
} ssd_shape;

/*
 * Bytes of device scratch ssd_prefill needs for this shape (a multiple of
 * 256); 0 if the shape is invalid.  Host-only, no HIP call.
 */
SSD_API size_t ssd_prefill_workspace_bytes(const ssd_shape *shape);

/*
 * Chunked-parallel prefill (Alg. 1; Eq. 3).  With cs_l the inclusive prefix
 * sum of dt*A inside a chunk and H_c the state entering chunk c it evaluates
 *     y[cL+l] = sum_{s<=l} (C_l.B_s) exp(cs_l - cs_s) dt_s x_s      (intra-chunk, Eq. 3)
 *             + exp(cs_l) C_l.H_c                                     (state to output)
 *             + D x_l
 *     S_c     = sum_s exp(cs_{L-1} - cs_s) dt_s x_s (x) B_s           (chunk-end states)
 *     H_{c+1} = exp(cs_{L-1}) H_c + S_c,  H_0 = h0 or 0               (inter-chunk pass)
 * and stores H_{Nc} into final_state (Alg. 1, "Store").  This equals the
 * token recurrence of Eq. 2 up to rounding order.
 *
 *  x, dt, A, B, C, D   inputs (device), layouts above
 *  h0                  optional initial state (device) or NULL = zeros; may
 *                      alias final_state
 *  y                   output (device), same shape and dtype as x; must not
 *                      alias an input
 *  final_state         output (device), fp32 (batch, nheads, headdim, dstate)
 *  workspace           device scratch of at least ssd_prefill_workspace_bytes()
 *                      bytes, 256-byte aligned; contents are undefined afterwards
 *  seqlen need not be a multiple of chunk (the last chunk is short).
 *  Errors: SSD_ERR_NULL, _SHAPE, _DTYPE, _ALIGN, _WORKSPACE, _HIP.
 */
SSD_API ssd_status ssd_prefill(const ssd_shape *shape, const void *x, const float *dt,
                       const float *A, const void *B, const void *C,
                       const float *D, const float *h0, void *y,
                       float *final_state, void *workspace,
                       size_t workspace_bytes, void *hip_stream);

/*
 * ssd_prefill with the step-size activation fused in (section "Mapping SSD
 * onto JAX primitives" names softplus and clip among the elementwise
 * neighbours of the decay computation; Alg. 1, "Discretise"): the kernels read
 * the raw projection output and use
 *     dt = clamp( softplus(dt_raw + dt_bias[h]), dt_min, dt_max )
 * wherever ssd_prefill uses dt.  Each part is optional: dt_bias NULL = no bias,
 * dt_softplus 0 = no softplus, dt_max <= 0 = no clamp.  Same workspace size,
 * results, errors and aliasing rules as ssd_prefill; SSD_ERR_NULL if
 * dt_transform is NULL, SSD_ERR_SHAPE if dt_max > 0 and dt_min > dt_max.
 * The struct is read during the call only; dt_bias is a DEVICE array (nheads).
 */
typedef struct {
  const float *dt_bias;
  int32_t dt_softplus;
  float dt_min, dt_max;
} ssd_dt_transform;
SSD_API ssd_status ssd_prefill_dt(const ssd_shape *shape, const ssd_dt_transform *dt_transform,
                          const void *x, const float *dt_raw, const float *A,
                          const void *B, const void *C, const float *D,
                          const float *h0, void *y, float *final_state,
                          void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * ssd_prefill for callers that cannot allocate device memory or pass a workspace
 * along: code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  The scratch that ssd_prefill takes through its workspace argument
 * is a buffer of SSD_STATIC_SCRATCH_BYTES that the library itself holds on every
 * GPU it runs on, from the moment its code is loaded there until the process
 * ends.  The call allocates and frees nothing (its first use on a device looks
 * the buffer's address up, once).  Same arguments, results (bit for bit), errors
 * and aliasing rules as ssd_prefill, plus
 *     SSD_ERR_TOO_LARGE   ssd_prefill_workspace_bytes(shape) exceeds
 *                         SSD_STATIC_SCRATCH_BYTES (nothing is enqueued);
 *     SSD_ERR_HIP         the buffer's address could not be obtained.
 * Every call on a GPU shares that GPU's buffer: calls that overlap in time on one
 * GPU (different streams, different threads) race on it and must be serialised
 * by the caller; calls on one stream are ordered by the stream.  Nothing in the
 * buffer needs to start at zero, and nothing is kept there between calls.
 * The device that is current when the call is made must be the one that holds
 * the tensors (as for any launch on hip_stream).
 */
#define SSD_STATIC_SCRATCH_BYTES ((size_t)32 << 20)
SSD_API ssd_status ssd_prefill_static(const ssd_shape *shape, const void *x, const float *dt,
                              const float *A, const void *B, const void *C,
                              const float *D, const float *h0, void *y,
                              float *final_state, void *hip_stream);

/*
 * Prefill of a packed, variable-length batch: `batch` independent sequences
 * laid back to back along the token axis (ragged prompt batches, prompts fed in
 * pieces with their cached state as h0 -- section "The O(1) state cache":
 * prefill initialises the cache, later calls continue from it).  Each sequence
 * is an ssd_prefill of its own: the recurrence of Eq. 2 restarts from h0[q] (or
 * zero) at every boundary and nothing crosses it.
 *   shape->batch      number of sequences (nseq); shape->seqlen = total tokens
 *   cu_seqlens        DEVICE array of nseq + 1 int32: sequence q owns tokens
 *                     [cu_seqlens[q], cu_seqlens[q+1]); must be non-decreasing
 *                     within [0, seqlen].  Empty sequences are allowed (their
 *                     final state is h0[q] or zero).  The array is read on the
 *                     device only; boundaries violating the rule make the call
 *                     a no-op (nothing is written, nothing faults).
 *   x, y  (seqlen, nheads, headdim);  dt (seqlen, nheads);  B, C (seqlen, ngroups, dstate)
 *   h0 (nullable), final_state   (nseq, nheads, headdim, dstate) fp32
 *   workspace         at least ssd_prefill_varlen_workspace_bytes() bytes, 256-byte aligned
 * Tokens outside every sequence are left untouched in y.
 * Shapes of the MFMA kernel family (bf16 io, headdim a multiple of 64, dstate a
 * multiple of 8 up to 512) run on it; every other shape and fp32 io run on the
 * generic fp32 kernels, which need batch x nheads <= 65535 and
 * ceil(seqlen / chunk) + batch <= 65535 (else SSD_ERR_UNSUPPORTED, and
 * ssd_prefill_varlen_workspace_bytes returns 0).
 * Errors: SSD_ERR_NULL, _SHAPE, _DTYPE, _ALIGN, _UNSUPPORTED, _WORKSPACE, _HIP.
 */
SSD_API size_t ssd_prefill_varlen_workspace_bytes(const ssd_shape *shape);
SSD_API ssd_status ssd_prefill_varlen(const ssd_shape *shape, const int32_t *cu_seqlens,
                              const void *x, const float *dt, const float *A,
                              const void *B, const void *C, const float *D,
                              const float *h0, void *y, float *final_state,
                              void *workspace, size_t workspace_bytes,
                              void *hip_stream);

/*
 * ssd_prefill_varlen with the step-size activation of ssd_prefill_dt fused in
 * (Alg. 1, "Discretise"): dt = clamp(softplus(dt_raw + dt_bias[h]), dt_min,
 * dt_max) wherever ssd_prefill_varlen uses dt.  Same workspace size, results
 * and errors as ssd_prefill_varlen; SSD_ERR_NULL if dt_transform is NULL,
 * SSD_ERR_SHAPE if dt_max > 0 and dt_min > dt_max.
 */
SSD_API ssd_status ssd_prefill_varlen_dt(const ssd_shape *shape, const ssd_dt_transform *dt_transform,
                                 const int32_t *cu_seqlens, const void *x,
                                 const float *dt_raw, const float *A, const void *B,
                                 const void *C, const float *D, const float *h0,
                                 void *y, float *final_state, void *workspace,
                                 size_t workspace_bytes, void *hip_stream);

/*
 * One cached decode step (Alg. 2, "Discretise" + "SSM step"; output per Eq. 2),
 * for every (batch row, head):
 *     dA      = exp(dt * A_h)
 *     h[p][n] = dA * h[p][n] + (dt * x[p]) * B[n]        state updated IN PLACE
 *     y[p]    = sum_n C[n] * h[p][n] + D_h * x[p]        (updated h)
 *  state (batch, nheads, headdim, dstate) fp32 in/out; x, y (batch, nheads,
 *  headdim) io dtype; dt (batch, nheads) fp32; B, C (batch, ngroups, dstate) io
 *  dtype; A, D (nheads) fp32.  shape->seqlen and shape->chunk are ignored.
 *  y must not alias an input; state must not alias anything else.
 *  Errors: SSD_ERR_NULL, _SHAPE, _DTYPE, _ALIGN, _HIP.
 */
SSD_API ssd_status ssd_decode_step(const ssd_shape *shape, float *state, const void *x,
                           const float *dt, const float *A, const void *B,
                           const void *C, const float *D, void *y,
                           void *hip_stream);

/*
 * The same step for `nlayers` independent layers in ONE launch: every array of
 * ssd_decode_step gains a leading [nlayers] axis (A and D become
 * (nlayers, nheads)).  Exists because one layer's state is far too small to
 * amortise a kernel launch (the analogue of the paper's compiled on-device
 * loop body, section "Mapping SSD onto JAX primitives").
 */
SSD_API ssd_status ssd_decode_step_layers(int32_t nlayers, const ssd_shape *shape,
                                  float *state, const void *x, const float *dt,
                                  const float *A, const void *B, const void *C,
                                  const float *D, void *y, void *hip_stream);

/*
 * `nsteps` consecutive decode steps of `nlayers` independent layers in ONE
 * launch, for callers that know the inputs of all steps up front (a short
 * continuation of a cached prompt, draft tokens to be verified): the analogue
 * of the paper's compiled on-device decode loop (section "Mapping SSD onto JAX
 * primitives"; Alg. 2 applied nsteps times).  Every per-step array of
 * ssd_decode_step_layers gains a leading [nsteps] axis:
 *     x, y (nsteps, nlayers, batch, nheads, headdim);  dt (nsteps, nlayers, batch, nheads);
 *     B, C (nsteps, nlayers, batch, ngroups, dstate);  A, D (nlayers, nheads);
 *     state (nlayers, batch, nheads, headdim, dstate) in/out: the state after the last step.
 * The result equals nsteps calls of ssd_decode_step_layers up to the order of
 * the fp32 summation over dstate.  For
 * the common head shapes the state stays on chip between the steps and moves
 * through memory once per call instead of once per step.
 * Errors: as ssd_decode_step_layers (only the base pointers need 16-byte alignment).
 */
SSD_API ssd_status ssd_decode_steps_layers(int32_t nsteps, int32_t nlayers, const ssd_shape *shape,
                                   float *state, const void *x, const float *dt,
                                   const float *A, const void *B, const void *C,
                                   const float *D, void *y, void *hip_stream);

/*
 * The two decode entry points above with the step-size activation fused in
 * (Alg. 2, "Discretise": the step applies softplus to the projected dt plus its
 * bias before it forms exp(dt * A)): the kernels read the raw projection output
 * and use dt = clamp(softplus(dt_raw + dt_bias[layer][h]), dt_min, dt_max).
 * dt_transform as for ssd_prefill_dt, except that dt_bias is a DEVICE array
 * (nlayers, nheads).  Errors as the plain entry points, plus SSD_ERR_NULL if
 * dt_transform is NULL and SSD_ERR_SHAPE if dt_max > 0 and dt_min > dt_max.
 */
SSD_API ssd_status ssd_decode_step_layers_dt(int32_t nlayers, const ssd_shape *shape,
                                     const ssd_dt_transform *dt_transform, float *state,
                                     const void *x, const float *dt_raw, const float *A,
                                     const void *B, const void *C, const float *D,
                                     void *y, void *hip_stream);
SSD_API ssd_status ssd_decode_steps_layers_dt(int32_t nsteps, int32_t nlayers, const ssd_shape *shape,
                                      const ssd_dt_transform *dt_transform, float *state,
                                      const void *x, const float *dt_raw, const float *A,
                                      const void *B, const void *C, const float *D,
                                      void *y, void *hip_stream);

/*
 * The step in front of the SSD core: the depthwise causal convolution of a
 * Mamba-2 block with its rolling cache (Alg. 2, "Update conv state" and
 * "DepthwiseConv"; section "The O(1) state cache": the cache holds the k-1
 * inputs before the current token, shape (batch, channels, k-1)).  Per channel c
 *     window_t = [ the k-1 inputs before token t, u_t ]
 *     z[t][c]  = act( bias[c] + sum_{j<k} weight[c][j] * window_t[j] )
 * so weight[c][k-1] multiplies the current input.  ssd_conv1d_prefill filters a
 * whole prompt (inputs before it come from conv_state_in, or are zero when it
 * is NULL) and stores the last k-1 inputs to conv_state_out (nullable);
 * ssd_conv1d_step is the one-token case and updates conv_state in place.
 *   u                 (batch, seqlen, channels) / (batch, channels), io dtype, channels-last
 *   weight            (channels, ksize) fp32;  bias (channels) fp32 or NULL;  2 <= ksize <= 8
 *   conv_state*       (batch, channels, ksize-1), io dtype; conv_state_in must
 *                     not be conv_state_out
 *   split[3], z0..z2  the output is scattered by channel range into up to three
 *                     dense tensors (batch, seqlen, split[i]) -- a Mamba-2 block
 *                     feeds the ranges x | B | C to the SSD core as separate
 *                     tensors; channels = split[0] + split[1] + split[2];
 *                     split[1], split[2] may be 0 (then z1, z2 are ignored).
 *                     split is a HOST array.
 *   activation        0 = none, 1 = SiLU (the paper does not name one; Mamba-2
 *                     applies SiLU here)
 * Arithmetic is fp32; z is rounded to the io dtype (RNE).  All pointers except
 * split are device pointers, 16-byte aligned.
 * Errors: SSD_ERR_NULL, _SHAPE, _DTYPE, _ALIGN, _HIP.
 */
SSD_API ssd_status ssd_conv1d_prefill(int32_t batch, int32_t seqlen, int32_t ksize, int32_t io_dtype,
                              const int32_t *split, const void *u, const float *weight,
                              const float *bias, const void *conv_state_in,
                              void *z0, void *z1, void *z2, void *conv_state_out,
                              int32_t activation, void *hip_stream);
SSD_API ssd_status ssd_conv1d_step(int32_t batch, int32_t ksize, int32_t io_dtype,
                           const int32_t *split, void *conv_state, const void *u,
                           const float *weight, const float *bias,
                           void *z0, void *z1, void *z2, int32_t activation,
                           void *hip_stream);

/*
 * Name of the kernel family ssd_prefill would use for this shape:
 * "mfma_bf16" (bf16 io: bf16 MFMA contractions over LDS-staged tiles, fp32
 * accumulation), "mfma_f32" (fp32 io, headdim a multiple of 32, dstate a multiple
 * of 8 up to 128: fp32 MFMA contractions, one launch, the workspace is not
 * touched), "generic_f32" (plain fp32 vector kernels, any shape), or "invalid".
 * Host-only.
 */
SSD_API const char *ssd_prefill_path(const ssd_shape *shape);

/* Human-readable name of a status code (static storage). */
SSD_API const char *ssd_status_string(ssd_status status);

/* Library version: major*10000 + minor*100 + patch. */
SSD_API int ssd_version(void);

#ifdef __cplusplus
}
#endif
#endif /* SSD_H_ */
