// C ABI of the SSD library (declared in include/ssd.h): host-side validation and dispatch.
// Every check runs before the first HIP call, so an invalid call enqueues nothing.
#include <cstring>
#include <limits>
#include <mutex>

#include "ssd_internal.hpp"
#include "ssd_testing.h"

namespace ssd {
Knobs &knobs() {
  static Knobs k;
  return k;
}
}  // namespace ssd

namespace {

using ssd::Dims;

ssd_status make_dims(const ssd_shape *s, bool decode, Dims *out, bool packed = false) {
  if (!s) return SSD_ERR_NULL;
  if (s->io_dtype != SSD_F32 && s->io_dtype != SSD_BF16) return SSD_ERR_DTYPE;
  if (s->batch < 1 || s->nheads < 1 || s->headdim < 1 || s->dstate < 1 || s->ngroups < 1)
    return SSD_ERR_SHAPE;
  if (!decode && (s->seqlen < 1 || s->chunk < 1)) return SSD_ERR_SHAPE;
  if (s->nheads % s->ngroups != 0) return SSD_ERR_SHAPE;
  Dims d;
  d.Bt = s->batch;
  d.T = decode ? 1 : s->seqlen;
  d.H = s->nheads;
  d.P = s->headdim;
  d.N = s->dstate;
  d.G = s->ngroups;
  d.L = decode ? 1 : s->chunk;
  d.Nc = (d.T + d.L - 1) / d.L;
  d.hpg = d.H / d.G;
  d.bf16 = s->io_dtype == SSD_BF16;
  // Every tensor must be addressable with comfortable head-room in size_t / 32-bit grids.
  const long double lim = 1.0e15L;
  const long double bt = d.Bt, t = d.T, h = d.H, p = d.P, n = d.N;
  if (bt * t * h * p > lim || bt * h * p * n > lim || bt * t * d.G * n > lim) return SSD_ERR_SHAPE;
  if (bt * h > 65535.0L && !decode && !packed) return SSD_ERR_UNSUPPORTED;  // grid y/z limit of the prefill kernels
  if (d.Nc > 65535) return SSD_ERR_UNSUPPORTED;
  *out = d;
  return SSD_OK;
}

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

bool force_generic() { return ssd::knobs().force_generic != 0; }

bool use_mfma(const Dims &d) { return !force_generic() && ssd::mfma_supported(d); }
bool use_mfma_f32(const Dims &d) { return !force_generic() && ssd::mfma_f32_supported(d, ssd::knobs().force_mfma_f32 != 0); }

// Enough for either kernel family that may run the shape, so that which one does (a test may force the
// generic one between the query and the call) never invalidates a size the caller was given.
size_t workspace_bytes(const Dims &d) {
  const size_t generic = ssd::generic_workspace_bytes(d);
  if (!ssd::mfma_supported(d)) return generic;
  const size_t mfma = ssd::mfma_workspace_bytes(d);
  return mfma > generic ? mfma : generic;
}

// Copies the caller's step-size map into the validated dimensions (nullptr: dt is used as given).
ssd_status set_dt_transform(Dims *d, const ssd_dt_transform *dtx) {
  if (dtx == nullptr) return SSD_OK;
  if (dtx->dt_max > 0.f && !(dtx->dt_min <= dtx->dt_max)) return SSD_ERR_SHAPE;
  d->dtx.bias = dtx->dt_bias;
  d->dtx.softplus = dtx->dt_softplus != 0;
  d->dtx.lo = dtx->dt_min;
  d->dtx.hi = dtx->dt_max;
  return SSD_OK;
}

ssd_status prefill_impl(const ssd_shape *shape, const void *x, const float *dt, const float *A,
                        const void *B, const void *C, const float *D, const float *h0, void *y,
                        float *final_state, void *workspace, size_t workspace_bytes_given,
                        void *hip_stream, ssd::KernelTrace *trace, const ssd_dt_transform *dtx = nullptr) {
  Dims d;
  const ssd_status st = make_dims(shape, false, &d);
  if (st != SSD_OK) return st;
  const ssd_status sx = set_dt_transform(&d, dtx);
  if (sx != SSD_OK) return sx;
  if (!x || !dt || !A || !B || !C || !D || !y || !final_state) return SSD_ERR_NULL;
  if (!aligned16(x) || !aligned16(dt) || !aligned16(B) || !aligned16(C) || !aligned16(y) ||
      !aligned16(final_state) || (h0 && !aligned16(h0)))
    return SSD_ERR_ALIGN;
  const size_t need = workspace_bytes(d);
  if (!workspace || workspace_bytes_given < need || (reinterpret_cast<uintptr_t>(workspace) & 255u))
    return SSD_ERR_WORKSPACE;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  if (trace) (void)hipEventRecord(trace->ev[0], stream);
  const hipError_t e =
      use_mfma(d)
          ? ssd::launch_prefill_mfma(d, x, dt, A, B, C, D, h0, y, final_state, workspace, stream, trace)
      : use_mfma_f32(d)
          ? ssd::launch_prefill_mfma_f32(d, x, dt, A, B, C, D, h0, y, final_state, stream, trace)
          : ssd::launch_prefill_generic(d, x, dt, A, B, C, D, h0, y, final_state, workspace, stream,
                                        trace);
  return e == hipSuccess ? SSD_OK : SSD_ERR_HIP;
}

}  // namespace

namespace ssd {
ssd_status prefill_traced(const ssd_shape *shape, const void *x, const float *dt, const float *A, const void *B,
                          const void *C, const float *D, const float *h0, void *y, float *final_state,
                          void *workspace, size_t workspace_bytes_given, void *hip_stream, KernelTrace *trace) {
  return prefill_impl(shape, x, dt, A, B, C, D, h0, y, final_state, workspace, workspace_bytes_given, hip_stream,
                      trace);
}
}  // namespace ssd

extern "C" {

size_t ssd_prefill_workspace_bytes(const ssd_shape *shape) {
  Dims d;
  if (make_dims(shape, false, &d) != SSD_OK) return 0;
  return workspace_bytes(d);
}

const char *ssd_prefill_path(const ssd_shape *shape) {
  Dims d;
  if (make_dims(shape, false, &d) != SSD_OK) return "invalid";
  return use_mfma(d) ? "mfma_bf16" : use_mfma_f32(d) ? "mfma_f32" : "generic_f32";
}

ssd_status ssd_testing_prefill_plan(const ssd_shape *shape, int32_t h0_aliases_final_state, int32_t plan[8]) {
  Dims d;
  if (shape == nullptr || plan == nullptr) return SSD_ERR_NULL;
  if (const ssd_status st = make_dims(shape, false, &d); st != SSD_OK) return st;
  for (int i = 0; i < 8; ++i) plan[i] = 0;
  if (use_mfma(d)) {
    const ssd::SlicePlan pl = ssd::mfma_plan(d, h0_aliases_final_state != 0);
    plan[0] = 1;
    plan[1] = pl.seg_blocks;
    plan[2] = pl.segments;
    plan[3] = pl.parts;
    plan[4] = pl.fold;
  } else if (use_mfma_f32(d)) {
    plan[0] = 2;
    plan[5] = ssd::mfma_f32_time_segments(d);
  }
  return SSD_OK;
}

ssd_status ssd_prefill(const ssd_shape *shape, const void *x, const float *dt, const float *A,
                       const void *B, const void *C, const float *D, const float *h0, void *y,
                       float *final_state, void *workspace, size_t workspace_bytes_given,
                       void *hip_stream) {
  return prefill_impl(shape, x, dt, A, B, C, D, h0, y, final_state, workspace, workspace_bytes_given,
                      hip_stream, nullptr);
}

namespace {
// Scratch of ssd_prefill_static: one copy per GPU, part of the library's device image.  In host code the
// array's name is only a handle for hipGetSymbolAddress; the address of a device's copy is looked up once,
// with that device current, and kept.
static __device__ __align__(256) unsigned char scratch[SSD_STATIC_SCRATCH_BYTES];
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[kMaxDevices] = {};

ssd_status static_scratch(void **out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return SSD_ERR_HIP;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (g_scratch_ptr[dev] == nullptr) {
    void *ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || ptr == nullptr) return SSD_ERR_HIP;
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return SSD_OK;
}
}  // namespace

ssd_status ssd_prefill_static(const ssd_shape *shape, const void *x, const float *dt, const float *A,
                              const void *B, const void *C, const float *D, const float *h0, void *y,
                              float *final_state, void *hip_stream) {
  Dims d;
  const ssd_status st = make_dims(shape, false, &d);
  if (st != SSD_OK) return st;
  if (workspace_bytes(d) > SSD_STATIC_SCRATCH_BYTES) return SSD_ERR_TOO_LARGE;
  if (!x || !dt || !A || !B || !C || !D || !y || !final_state) return SSD_ERR_NULL;  // before any HIP call
  void *ws = nullptr;
  const ssd_status sp = static_scratch(&ws);
  if (sp != SSD_OK) return sp;
  return prefill_impl(shape, x, dt, A, B, C, D, h0, y, final_state, ws, SSD_STATIC_SCRATCH_BYTES, hip_stream,
                      nullptr);
}

ssd_status ssd_prefill_dt(const ssd_shape *shape, const ssd_dt_transform *dt_transform, const void *x,
                          const float *dt_raw, const float *A, const void *B, const void *C, const float *D,
                          const float *h0, void *y, float *final_state, void *workspace,
                          size_t workspace_bytes_given, void *hip_stream) {
  if (!dt_transform) return SSD_ERR_NULL;
  return prefill_impl(shape, x, dt_raw, A, B, C, D, h0, y, final_state, workspace, workspace_bytes_given, hip_stream,
                      nullptr, dt_transform);
}

namespace {
// The generic kernels take a packed batch while (sequences x heads) and the chunk capacity fit a grid axis.
bool generic_varlen_ok(const Dims &d) {
  const long long cap = (static_cast<long long>(d.T) + d.L - 1) / d.L + d.Bt;
  return static_cast<long long>(d.Bt) * d.H <= 65535 && cap <= 65535;
}
bool use_mfma_varlen(const Dims &d) { return !force_generic() && ssd::mfma_varlen_supported(d); }
}  // namespace

size_t ssd_prefill_varlen_workspace_bytes(const ssd_shape *shape) {
  Dims d;
  if (make_dims(shape, false, &d, true) != SSD_OK) return 0;
  // enough for either family that may run it (see workspace_bytes); 0: neither family takes this shape
  const size_t generic = generic_varlen_ok(d) ? ssd::generic_varlen_workspace_bytes(d) : 0;
  const size_t mfma = ssd::mfma_varlen_supported(d) ? ssd::mfma_varlen_workspace_bytes(d) : 0;
  return mfma > generic ? mfma : generic;
}

namespace {
ssd_status varlen_impl(const ssd_shape *shape, const ssd_dt_transform *dtx, const int32_t *cu_seqlens, const void *x,
                       const float *dt, const float *A, const void *B, const void *C, const float *D, const float *h0,
                       void *y, float *final_state, void *workspace, size_t workspace_bytes_given, void *hip_stream) {
  Dims d;  // batch = number of sequences, seqlen = total tokens
  const ssd_status st = make_dims(shape, false, &d, true);
  if (st != SSD_OK) return st;
  const ssd_status sx = set_dt_transform(&d, dtx);
  if (sx != SSD_OK) return sx;
  if (!cu_seqlens || !x || !dt || !A || !B || !C || !D || !y || !final_state) return SSD_ERR_NULL;
  if (!aligned16(x) || !aligned16(dt) || !aligned16(B) || !aligned16(C) || !aligned16(y) ||
      !aligned16(final_state) || (h0 && !aligned16(h0)) || (reinterpret_cast<uintptr_t>(cu_seqlens) & 3u))
    return SSD_ERR_ALIGN;
  const bool mfma = use_mfma_varlen(d);
  if (!mfma && !generic_varlen_ok(d)) return SSD_ERR_UNSUPPORTED;
  const size_t need = ssd_prefill_varlen_workspace_bytes(shape);
  if (!workspace || workspace_bytes_given < need || (reinterpret_cast<uintptr_t>(workspace) & 255u))
    return SSD_ERR_WORKSPACE;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  const hipError_t e =
      mfma ? ssd::launch_prefill_mfma_varlen(d, cu_seqlens, x, dt, A, B, C, D, h0, y, final_state, workspace, stream)
           : ssd::launch_prefill_generic_varlen(d, cu_seqlens, x, dt, A, B, C, D, h0, y, final_state, workspace,
                                                stream);
  return e == hipSuccess ? SSD_OK : SSD_ERR_HIP;
}
}  // namespace

ssd_status ssd_prefill_varlen(const ssd_shape *shape, const int32_t *cu_seqlens, const void *x, const float *dt,
                              const float *A, const void *B, const void *C, const float *D, const float *h0,
                              void *y, float *final_state, void *workspace, size_t workspace_bytes_given,
                              void *hip_stream) {
  return varlen_impl(shape, nullptr, cu_seqlens, x, dt, A, B, C, D, h0, y, final_state, workspace,
                     workspace_bytes_given, hip_stream);
}

ssd_status ssd_prefill_varlen_dt(const ssd_shape *shape, const ssd_dt_transform *dt_transform,
                                 const int32_t *cu_seqlens, const void *x, const float *dt_raw, const float *A,
                                 const void *B, const void *C, const float *D, const float *h0, void *y,
                                 float *final_state, void *workspace, size_t workspace_bytes_given,
                                 void *hip_stream) {
  if (!dt_transform) return SSD_ERR_NULL;
  return varlen_impl(shape, dt_transform, cu_seqlens, x, dt_raw, A, B, C, D, h0, y, final_state, workspace,
                     workspace_bytes_given, hip_stream);
}

namespace {
ssd_status decode_impl(int32_t nsteps, int32_t nlayers, const ssd_shape *shape, const ssd_dt_transform *dtx,
                       float *state, const void *x, const float *dt, const float *A, const void *B, const void *C,
                       const float *D, void *y, void *hip_stream, bool multi);
}  // namespace

ssd_status ssd_decode_step_layers(int32_t nlayers, const ssd_shape *shape, float *state, const void *x,
                                  const float *dt, const float *A, const void *B, const void *C,
                                  const float *D, void *y, void *hip_stream) {
  return decode_impl(1, nlayers, shape, nullptr, state, x, dt, A, B, C, D, y, hip_stream, false);
}

ssd_status ssd_decode_step_layers_dt(int32_t nlayers, const ssd_shape *shape, const ssd_dt_transform *dt_transform,
                                     float *state, const void *x, const float *dt_raw, const float *A,
                                     const void *B, const void *C, const float *D, void *y, void *hip_stream) {
  if (!dt_transform) return SSD_ERR_NULL;
  return decode_impl(1, nlayers, shape, dt_transform, state, x, dt_raw, A, B, C, D, y, hip_stream, false);
}

ssd_status ssd_decode_steps_layers(int32_t nsteps, int32_t nlayers, const ssd_shape *shape, float *state,
                                   const void *x, const float *dt, const float *A, const void *B, const void *C,
                                   const float *D, void *y, void *hip_stream) {
  return decode_impl(nsteps, nlayers, shape, nullptr, state, x, dt, A, B, C, D, y, hip_stream, true);
}

ssd_status ssd_decode_steps_layers_dt(int32_t nsteps, int32_t nlayers, const ssd_shape *shape,
                                      const ssd_dt_transform *dt_transform, float *state, const void *x,
                                      const float *dt_raw, const float *A, const void *B, const void *C,
                                      const float *D, void *y, void *hip_stream) {
  if (!dt_transform) return SSD_ERR_NULL;
  return decode_impl(nsteps, nlayers, shape, dt_transform, state, x, dt_raw, A, B, C, D, y, hip_stream, true);
}

namespace {
ssd_status decode_impl(int32_t nsteps, int32_t nlayers, const ssd_shape *shape, const ssd_dt_transform *dtx,
                       float *state, const void *x, const float *dt, const float *A, const void *B, const void *C,
                       const float *D, void *y, void *hip_stream, bool multi) {
  Dims d;
  const ssd_status st = make_dims(shape, true, &d);
  if (st != SSD_OK) return st;
  const ssd_status sx = set_dt_transform(&d, dtx);
  if (sx != SSD_OK) return sx;
  if (nlayers < 1 || nsteps < 1) return SSD_ERR_SHAPE;
  const long double pairs = static_cast<long double>(nlayers) * d.Bt * d.H;
  if (pairs > 2.0e9L || pairs * d.P * nsteps > 1.0e15L) return SSD_ERR_SHAPE;  // one workgroup per (layer, batch row, head)
  if (!state || !x || !dt || !A || !B || !C || !D || !y) return SSD_ERR_NULL;
  if (!aligned16(state) || !aligned16(x) || !aligned16(B) || !aligned16(C) || !aligned16(y))
    return SSD_ERR_ALIGN;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  const hipError_t e = multi ? ssd::launch_decode_steps(nsteps, nlayers, d, state, x, dt, A, B, C, D, y, stream)
                             : ssd::launch_decode(nlayers, d, state, x, dt, A, B, C, D, y, stream);
  return e == hipSuccess ? SSD_OK : SSD_ERR_HIP;
}
}  // namespace

ssd_status ssd_decode_step(const ssd_shape *shape, float *state, const void *x, const float *dt,
                           const float *A, const void *B, const void *C, const float *D, void *y,
                           void *hip_stream) {
  return ssd_decode_step_layers(1, shape, state, x, dt, A, B, C, D, y, hip_stream);
}

namespace {
// Shared checks of the two convolution entry points.  Returns SSD_OK and fills z / width.
ssd_status conv_args(int32_t batch, int32_t ksize, int32_t io_dtype, const int32_t *split, const void *u,
                     const float *weight, void *z0, void *z1, void *z2, int32_t activation, void *z[3], int width[3]) {
  if (io_dtype != SSD_F32 && io_dtype != SSD_BF16) return SSD_ERR_DTYPE;
  if (!split) return SSD_ERR_NULL;
  if (batch < 1 || ksize < 2 || ksize > 8 || split[0] < 1 || split[1] < 0 || split[2] < 0) return SSD_ERR_SHAPE;
  if (activation != 0 && activation != 1) return SSD_ERR_SHAPE;
  const long double chans = static_cast<long double>(split[0]) + split[1] + split[2];
  if (chans > 1.0e9L || chans * batch > 2.0e11L) return SSD_ERR_SHAPE;
  z[0] = z0;
  z[1] = z1;
  z[2] = z2;
  for (int i = 0; i < 3; ++i) {
    width[i] = split[i];
    if (width[i] > 0 && !z[i]) return SSD_ERR_NULL;
    if (width[i] > 0 && !aligned16(z[i])) return SSD_ERR_ALIGN;
  }
  if (!u || !weight) return SSD_ERR_NULL;
  if (!aligned16(u)) return SSD_ERR_ALIGN;
  return SSD_OK;
}
}  // namespace

ssd_status ssd_conv1d_prefill(int32_t batch, int32_t seqlen, int32_t ksize, int32_t io_dtype, const int32_t *split,
                              const void *u, const float *weight, const float *bias, const void *conv_state_in,
                              void *z0, void *z1, void *z2, void *conv_state_out, int32_t activation,
                              void *hip_stream) {
  void *z[3];
  int width[3];
  const ssd_status st = conv_args(batch, ksize, io_dtype, split, u, weight, z0, z1, z2, activation, z, width);
  if (st != SSD_OK) return st;
  if (seqlen < 1 || batch > 65535) return SSD_ERR_SHAPE;
  // one thread per (run of tokens, channel): the thread count of a batch row must fit 32 bits
  if (static_cast<long double>(seqlen) * (static_cast<long double>(split[0]) + split[1] + split[2]) > 3.0e10L)
    return SSD_ERR_SHAPE;
  if (conv_state_in && conv_state_in == conv_state_out) return SSD_ERR_SHAPE;  // read and written by different threads
  const hipError_t e = ssd::launch_conv_prefill(batch, seqlen, ksize, io_dtype == SSD_BF16, u, weight, bias,
                                                conv_state_in, z, width, conv_state_out, activation,
                                                static_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? SSD_OK : SSD_ERR_HIP;
}

ssd_status ssd_conv1d_step(int32_t batch, int32_t ksize, int32_t io_dtype, const int32_t *split, void *conv_state,
                           const void *u, const float *weight, const float *bias, void *z0, void *z1, void *z2,
                           int32_t activation, void *hip_stream) {
  void *z[3];
  int width[3];
  const ssd_status st = conv_args(batch, ksize, io_dtype, split, u, weight, z0, z1, z2, activation, z, width);
  if (st != SSD_OK) return st;
  if (!conv_state) return SSD_ERR_NULL;
  const hipError_t e = ssd::launch_conv_step(batch, ksize, io_dtype == SSD_BF16, conv_state, u, weight, bias, z, width,
                                             activation, static_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? SSD_OK : SSD_ERR_HIP;
}

ssd_status ssd_testing_set_knob(int32_t knob, int32_t value) {
  ssd::Knobs &k = ssd::knobs();
  switch (knob) {
    case SSD_KNOB_FORCE_GENERIC: k.force_generic = value > 0 ? 1 : 0; return SSD_OK;
    case SSD_KNOB_SEG_CHUNKS: k.seg_chunks = value > 0 ? value : 0; return SSD_OK;
    case SSD_KNOB_SEG_BLOCKS: k.seg_blocks = value > 0 ? value : 0; return SSD_OK;
    case SSD_KNOB_SEG_PARTS: k.seg_parts = value > 0 ? value : 0; return SSD_OK;
    case SSD_KNOB_Y_STREAM: k.y_stream = value < 0 ? -1 : (value != 0); return SSD_OK;
    case SSD_KNOB_DECODE_STREAM: k.decode_stream = value < 0 ? -1 : (value != 0); return SSD_OK;
    case SSD_KNOB_FORCE_MFMA_F32: k.force_mfma_f32 = value > 0 ? 1 : 0; return SSD_OK;
    case SSD_KNOB_F32_SEGMENTS: k.f32_segments = value > 0 ? value : 0; return SSD_OK;
    case SSD_KNOB_FOLD_MAX_SLOTS: k.fold_max_slots = value > 0 ? value : 0; return SSD_OK;
    default: return SSD_ERR_SHAPE;
  }
}

void ssd_testing_reset_knobs(void) { ssd::knobs() = ssd::Knobs(); }

const char *ssd_status_string(ssd_status status) {
  switch (status) {
    case SSD_OK: return "ok";
    case SSD_ERR_NULL: return "a required pointer is NULL";
    case SSD_ERR_SHAPE: return "invalid shape";
    case SSD_ERR_DTYPE: return "invalid io dtype";
    case SSD_ERR_UNSUPPORTED: return "shape not supported";
    case SSD_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case SSD_ERR_HIP: return "HIP launch error";
    case SSD_ERR_ALIGN: return "tensor pointer not 16-byte aligned";
    case SSD_ERR_TOO_LARGE: return "shape needs more scratch than the library's static buffer holds";
  }
  return "unknown status";
}

int ssd_version(void) { return 100; }

}  // extern "C"
