// Internal declarations shared by the translation units of the SSD library.
// Nothing here is part of the C ABI (see include/ssd.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "ssd.h"

namespace ssd {

// Optional map from the caller's dt values to the step size (section "Mapping SSD onto JAX
// primitives" lists softplus and clip among the elementwise neighbours that must fuse with the
// decay computation): dt = clamp(softplus(raw + bias[h]), lo, hi).  Default: dt is used as given.
struct DtXform {
  const float *bias = nullptr;  // (nheads) -- decode: (nlayers, nheads) --, device; nullptr = none
  int softplus = 0;
  float lo = 0.f, hi = 0.f;     // clamp to [lo, hi] if hi > 0
  bool identity() const { return bias == nullptr && softplus == 0 && !(hi > 0.f); }
};
// (bias already fetched: kernels that apply the map step after step read it once)
__device__ __forceinline__ float dt_apply_biased(float v, float bias, const DtXform &t) {
  v += bias;
  if (t.softplus) v = v > 20.f ? v : log1pf(expf(v));
  if (t.hi > 0.f) v = fminf(fmaxf(v, t.lo), t.hi);
  return v;
}
__device__ __forceinline__ float dt_apply(float v, int h, const DtXform &t) {
  return dt_apply_biased(v, t.bias != nullptr ? t.bias[h] : 0.f, t);
}
// The same map without a branch (hardware exp2 / log2, relative error about 2e-7), for code whose loads
// must not wait at a join: softplus(v) = max(v, 0) + log(1 + exp(-|v|)).
__device__ __forceinline__ float dt_apply_branchless(float v, float bias, const DtXform &t) {
  v += bias;
  const float e = __builtin_amdgcn_exp2f(-fabsf(v) * 1.4426950408889634f);
  const float sp = fmaxf(v, 0.f) + 0.6931471805599453f * __builtin_amdgcn_logf(1.f + e);
  v = t.softplus ? sp : v;
  const float cl = fminf(fmaxf(v, t.lo), t.hi);
  return t.hi > 0.f ? cl : v;
}

// Validated problem dimensions (host side).
struct Dims {
  int Bt, T, H, P, N, G, L;
  int Nc;     // number of chunks, ceil(T / L)
  int hpg;    // heads per B/C group
  bool bf16;  // io dtype of x, B, C, y
  DtXform dtx;  // step-size map of the *_dt entry points (identity otherwise)
};

// ---- bf16 <-> fp32 (bf16 = upper half of the fp32 pattern, round-to-nearest-even) ----
__device__ __forceinline__ float bf16_bits_to_f32(uint16_t v) {
  return __uint_as_float(static_cast<uint32_t>(v) << 16);
}
__device__ __forceinline__ uint16_t f32_to_bf16_bits(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return static_cast<uint16_t>((u >> 16) | 0x0040u);  // quiet NaN
  u += 0x7fffu + ((u >> 16) & 1u);
  return static_cast<uint16_t>(u >> 16);
}

// Element access for the two io dtypes.
struct IoF32 {
  using type = float;
  static __device__ __forceinline__ float load(const void *p, size_t i) {
    return static_cast<const float *>(p)[i];
  }
  static __device__ __forceinline__ void store(void *p, size_t i, float v) {
    static_cast<float *>(p)[i] = v;
  }
};
struct IoBf16 {
  using type = uint16_t;
  static __device__ __forceinline__ float load(const void *p, size_t i) {
    return bf16_bits_to_f32(static_cast<const uint16_t *>(p)[i]);
  }
  static __device__ __forceinline__ void store(void *p, size_t i, float v) {
    static_cast<uint16_t *>(p)[i] = f32_to_bf16_bits(v);
  }
};

// Optional per-kernel timing (used only by the measurement library): an event is recorded on the
// launch stream after every kernel of a prefill call.
struct KernelTrace {
  static constexpr int kMax = 8;
  int n = 0;
  hipEvent_t ev[kMax + 1];
  const char *names[kMax];
};
inline void trace_mark(KernelTrace *t, hipStream_t s, const char *name) {
  if (t && t->n < KernelTrace::kMax) {
    (void)hipEventRecord(t->ev[t->n + 1], s);
    t->names[t->n++] = name;
  }
}

// Process-wide overrides of choices the library otherwise makes by itself; set only through the
// test-only entry points of include/ssd_testing.h (nothing reads the environment).
struct Knobs {
  int force_generic = 0;   // 1: every prefill takes the generic fp32 kernels
  int seg_chunks = 0;      // > 0: chunks per segment of the MFMA prefill
  int seg_blocks = 0;      // > 0: 64-token blocks per segment (if seg_chunks is not set)
  int seg_parts = 0;       // > 0: pieces per segment in the states-only pass
  int y_stream = -1;       // 0 / 1: ordinary / non-temporal stores of y in the full scan
  int decode_stream = -1;  // 0 / 1: ordinary / non-temporal accesses to the decode state
  int force_mfma_f32 = 0;  // 1: fp32 io takes the fp32 MFMA kernel whenever the shape is eligible
  int f32_segments = 0;    // > 0: time segments per sequence in the fp32 MFMA kernel
  int fold_max_slots = 3;  // most state slots a segment sums by itself instead of a pass over segment states (0: never)
};
Knobs &knobs();

// ---- launchers (each returns the first HIP error it sees) ----
hipError_t launch_decode(int nlayers, const Dims &d, float *state, const void *x, const float *dt,
                         const float *A, const void *B, const void *C, const float *D, void *y,
                         hipStream_t stream);

hipError_t launch_decode_steps(int nsteps, int nlayers, const Dims &d, float *state, const void *x,
                               const float *dt, const float *A, const void *B, const void *C, const float *D,
                               void *y, hipStream_t stream);

size_t generic_workspace_bytes(const Dims &d);
hipError_t launch_prefill_generic(const Dims &d, const void *x, const float *dt, const float *A,
                                  const void *B, const void *C, const float *D, const float *h0,
                                  void *y, float *final_state, void *workspace, hipStream_t stream,
                                  KernelTrace *trace = nullptr);

// How the bf16 MFMA prefill cuts a call up (for the launcher and for the test-only plan query).
struct SlicePlan {
  int seg_blocks, segments, parts, fold;
};
SlicePlan mfma_plan(const Dims &d, bool h0_aliases_final_state);
int mfma_f32_time_segments(const Dims &d);
bool mfma_supported(const Dims &d);
size_t mfma_workspace_bytes(const Dims &d);
hipError_t launch_prefill_mfma(const Dims &d, const void *x, const float *dt, const float *A,
                               const void *B, const void *C, const float *D, const float *h0,
                               void *y, float *final_state, void *workspace, hipStream_t stream,
                               KernelTrace *trace = nullptr);

// fp32 io on fp32 MFMA (one launch, no workspace); see ssd_prefill_mfma_f32.hip.
bool mfma_f32_supported(const Dims &d, bool whenever_eligible);  // false: only where it is expected to win
hipError_t launch_prefill_mfma_f32(const Dims &d, const void *x, const float *dt, const float *A, const void *B,
                                   const void *C, const float *D, const float *h0, void *y, float *final_state,
                                   hipStream_t stream, KernelTrace *trace = nullptr);

// Device-side tables of a packed variable-length batch (all int32; see ssd_prefill_mfma.hip, "tables of a
// variable-length call").  tok0 == nullptr: plain batch.
struct VarPlan {
  const int32_t *tok0, *len, *blk0, *item0, *slot0, *blk_seq, *item_seq;
  int nseq, nb_cap, slot_cap;
};
void launch_varlen_tables(const int32_t *cu, int total, int blk_len, int seg_blocks, int item_cap, const VarPlan &vp,
                          hipStream_t stream);
size_t generic_varlen_workspace_bytes(const Dims &d);
hipError_t launch_prefill_generic_varlen(const Dims &d, const int32_t *cu_seqlens, const void *x, const float *dt,
                                         const float *A, const void *B, const void *C, const float *D,
                                         const float *h0, void *y, float *final_state, void *workspace,
                                         hipStream_t stream);

// Packed variable-length batch (d.Bt sequences, d.T tokens in total, cu_seqlens on the device).
bool mfma_varlen_supported(const Dims &d);
size_t mfma_varlen_workspace_bytes(const Dims &d);
hipError_t launch_prefill_mfma_varlen(const Dims &d, const int32_t *cu_seqlens, const void *x, const float *dt,
                                      const float *A, const void *B, const void *C, const float *D, const float *h0,
                                      void *y, float *final_state, void *workspace, hipStream_t stream,
                                      KernelTrace *trace = nullptr);

// Depthwise causal convolution (channels-last); z / width: up to three dense outputs by channel range.
hipError_t launch_conv_prefill(int Bt, int T, int ksize, bool bf16, const void *u, const float *w, const float *bias,
                               const void *state_in, void *const z[3], const int width[3], void *state_out, int act,
                               hipStream_t stream);
hipError_t launch_conv_step(int Bt, int ksize, bool bf16, void *state, const void *u, const float *w, const float *bias,
                            void *const z[3], const int width[3], int act, hipStream_t stream);

// ssd_prefill with an event recorded after every kernel (the measurement library's ssd_prefill_profile).
ssd_status prefill_traced(const ssd_shape *shape, const void *x, const float *dt, const float *A, const void *B,
                          const void *C, const float *D, const float *h0, void *y, float *final_state,
                          void *workspace, size_t workspace_bytes_given, void *hip_stream, KernelTrace *trace);

inline size_t round_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

}  // namespace ssd
