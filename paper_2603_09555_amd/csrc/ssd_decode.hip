// Cached decode step (Alg. 2, "Discretise" + "SSM step"; output per Eq. 2):
//     dA = exp(dt*A_h);  h[p][n] = dA*h[p][n] + (dt*x[p])*B[n];  y[p] = sum_n C[n]*h[p][n] + D_h*x[p]
//
// The step moves 8 bytes of fp32 state per 5 flops, so it is bound by HBM bandwidth.  The
// kernel streams the state exactly once: one workgroup per (layer, batch row, head), each
// lane owns four consecutive n of a row (one 16-byte load and one 16-byte store per row),
// N/4 consecutive lanes form a row, and all loads of a pass are issued before the first use
// so that each lane keeps eight 16-byte requests in flight.  The C.h reduction runs across
// the N/4 lanes of a row with wave shuffles; nothing but the state round-trips memory.
#include <cstdlib>
#include "ssd_internal.hpp"

// Multiply-adds are written as explicit fmaf so that the single-step and the multi-step kernels
// round identically (the compiler's own choice of what to fuse differs between kernels).
namespace ssd {
namespace {

constexpr int kDecodeThreads = 256;
constexpr int kDecodeUnroll = 8;  // rows per lane whose loads are in flight together

template <typename Io>
__device__ __forceinline__ float4 load4(const void *base, size_t elem_index);
template <>
__device__ __forceinline__ float4 load4<IoF32>(const void *base, size_t i) {
  return *reinterpret_cast<const float4 *>(static_cast<const float *>(base) + i);
}
template <>
__device__ __forceinline__ float4 load4<IoBf16>(const void *base, size_t i) {
  const uint2 v = *reinterpret_cast<const uint2 *>(static_cast<const uint16_t *>(base) + i);
  float4 r;
  r.x = __uint_as_float(v.x << 16);
  r.y = __uint_as_float(v.x & 0xffff0000u);
  r.z = __uint_as_float(v.y << 16);
  r.w = __uint_as_float(v.y & 0xffff0000u);
  return r;
}

// Four consecutive io values as loaded (kept packed while they wait in registers), and their conversion.
template <typename Io>
struct Raw4;
template <>
struct Raw4<IoF32> {
  float4 v;
  __device__ __forceinline__ void load(const void *base, size_t i) {
    v = *reinterpret_cast<const float4 *>(static_cast<const float *>(base) + i);
  }
  __device__ __forceinline__ float4 get() const { return v; }
};
template <>
struct Raw4<IoBf16> {
  uint2 v;
  __device__ __forceinline__ void load(const void *base, size_t i) {
    v = *reinterpret_cast<const uint2 *>(static_cast<const uint16_t *>(base) + i);
  }
  __device__ __forceinline__ float4 get() const {
    float4 r;
    r.x = __uint_as_float(v.x << 16);
    r.y = __uint_as_float(v.x & 0xffff0000u);
    r.z = __uint_as_float(v.y << 16);
    r.w = __uint_as_float(v.y & 0xffff0000u);
    return r;
  }
};

// Four state values of a lane.  kStream marks the accesses non-temporal: a state that does not fit the
// 256 MiB memory-side cache cannot be found there by the next step anyway, and streaming it past the
// caches was measured 7-12 % faster (64 layers, batch 2..16); a state that fits (batch 1, 160 MiB) is
// served from that cache step after step and loses 15 % when it is streamed.
typedef float f32x4_t __attribute__((ext_vector_type(4)));
template <bool kStream>
__device__ __forceinline__ float4 load_h4(const float *p) {
  if constexpr (kStream) {
    const f32x4_t q = __builtin_nontemporal_load(reinterpret_cast<const f32x4_t *>(p));
    return make_float4(q.x, q.y, q.z, q.w);
  } else {
    return *reinterpret_cast<const float4 *>(p);
  }
}
template <bool kStream>
__device__ __forceinline__ void store_h4(float *p, const float4 v) {
  if constexpr (kStream) {
    const f32x4_t q = {v.x, v.y, v.z, v.w};
    __builtin_nontemporal_store(q, reinterpret_cast<f32x4_t *>(p));
  } else {
    *reinterpret_cast<float4 *>(p) = v;
  }
}

// LPR = lanes per state row = N / 4 (a power of two, <= 64).
template <typename Io, int LPR, bool kStream>
__global__ __launch_bounds__(kDecodeThreads) void decode_vec_kernel(
    float *__restrict__ state, const void *__restrict__ x, const float *__restrict__ dt,
    const float *__restrict__ A, const void *__restrict__ B, const void *__restrict__ C,
    const float *__restrict__ D, void *__restrict__ y, int BtH, int H, int P, int G, int hpg,
    const DtXform dtx) {
  constexpr int N = LPR * 4;
  constexpr int RPP = kDecodeThreads / LPR;  // rows per pass
  const size_t pair = blockIdx.x;            // (layer*Bt + b)*H + h
  // blockIdx.y: with few (layer, row, head) units the rows of a state are shared out over gridDim.y
  // workgroups (contiguous ranges of whole passes), so that a small launch still fills the chip
  const int rows_per_wg = (P + gridDim.y - 1) / gridDim.y;
  const int p_begin = blockIdx.y * rows_per_wg, p_end = min(P, p_begin + rows_per_wg);
  const int h = static_cast<int>(pair % H);
  const size_t lb = pair / H;                // layer*Bt + b
  const int layer = static_cast<int>(pair / BtH);
  const int lane_n = threadIdx.x % LPR;
  const int row0 = threadIdx.x / LPR;

  const float dtv = dt_apply(dt[pair], layer * H + h, dtx);
  const float Ah = A[static_cast<size_t>(layer) * H + h];
  const float Dh = D[static_cast<size_t>(layer) * H + h];
  const float dA = expf(dtv * Ah);
  const size_t bc = (lb * G + h / hpg) * N + lane_n * 4;
  const float4 Bv = load4<Io>(B, bc);
  const float4 Cv = load4<Io>(C, bc);

  float *hbase = state + pair * static_cast<size_t>(P) * N + lane_n * 4;
  for (int p0 = p_begin + row0; p0 < p_end; p0 += RPP * kDecodeUnroll) {
    float4 hv[kDecodeUnroll];
    float xv[kDecodeUnroll];
#pragma unroll
    for (int u = 0; u < kDecodeUnroll; ++u) {
      const int p = p0 + u * RPP;
      if (p < p_end) {
        hv[u] = load_h4<kStream>(hbase + static_cast<size_t>(p) * N);
        xv[u] = Io::load(x, pair * P + p);
      }
    }
#pragma unroll
    for (int u = 0; u < kDecodeUnroll; ++u) {
      const int p = p0 + u * RPP;
      if (p < p_end) {
        const float ux = dtv * xv[u];
        float4 v = hv[u];
        v.x = fmaf(dA, v.x, ux * Bv.x);
        v.y = fmaf(dA, v.y, ux * Bv.y);
        v.z = fmaf(dA, v.z, ux * Bv.z);
        v.w = fmaf(dA, v.w, ux * Bv.w);
        store_h4<kStream>(hbase + static_cast<size_t>(p) * N, v);
        float part = fmaf(Cv.w, v.w, fmaf(Cv.z, v.z, fmaf(Cv.y, v.y, Cv.x * v.x)));
#pragma unroll
        for (int m = LPR / 2; m >= 1; m >>= 1) part += __shfl_xor(part, m, 64);
        if (lane_n == 0) Io::store(y, pair * P + p, fmaf(Dh, xv[u], part));
      }
    }
  }
}

// Any N: one wave per row, lanes stride over n.
template <typename Io>
__global__ __launch_bounds__(kDecodeThreads) void decode_any_kernel(
    float *__restrict__ state, const void *__restrict__ x, const float *__restrict__ dt,
    const float *__restrict__ A, const void *__restrict__ B, const void *__restrict__ C,
    const float *__restrict__ D, void *__restrict__ y, int BtH, int H, int P, int N, int G, int hpg,
    const DtXform dtx) {
  const size_t pair = blockIdx.x;
  const int h = static_cast<int>(pair % H);
  const size_t lb = pair / H;
  const int layer = static_cast<int>(pair / BtH);
  const int lane = threadIdx.x % 64;
  const int wave = threadIdx.x / 64;
  const float dtv = dt_apply(dt[pair], layer * H + h, dtx);
  const float dA = expf(dtv * A[static_cast<size_t>(layer) * H + h]);
  const float Dh = D[static_cast<size_t>(layer) * H + h];
  const size_t bc = (lb * G + h / hpg) * static_cast<size_t>(N);
  for (int p = wave; p < P; p += kDecodeThreads / 64) {
    const float xv = Io::load(x, pair * P + p);
    const float ux = dtv * xv;
    float *hp = state + (pair * P + p) * static_cast<size_t>(N);
    float part = 0.f;
    for (int n = lane; n < N; n += 64) {
      const float v = fmaf(dA, hp[n], ux * Io::load(B, bc + n));
      hp[n] = v;
      part = fmaf(Io::load(C, bc + n), v, part);
    }
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) part += __shfl_xor(part, m, 64);
    if (lane == 0) Io::store(y, pair * P + p, fmaf(Dh, xv, part));
  }
}

// Several steps in one launch (inputs of all steps known up front, e.g. a short continuation of a
// cached prompt): the state of a (layer, batch row, head) stays in registers across the steps, so
// it is read and written once instead of once per step, and the per-step traffic shrinks to the
// step's inputs and its output row.  What then bounds the kernel is the vector ALU, so the layout
// minimises instructions per state element: LPR (<= 16) lanes share a row, each lane owns NV groups
// of four consecutive n (group v covers n = 4 (v LPR + lane) ..), so a row's C.h is reduced inside a
// 16-lane DPP row by four single add-with-lane-permute instructions, without LDS traffic.
// ROWS = rows per lane = P / (256 / LPR).  The inputs of step s+1 are requested before step s is
// computed.
template <int CTRL>
__device__ __forceinline__ float dpp_mov(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, false));
}
// Sum over the LPR lanes of a row (LPR a power of two <= 16, rows aligned to LPR lanes); every lane
// of the row receives the sum.  Lane permutations: swap neighbours, swap pairs, mirror inside 8,
// mirror inside 16 (after the first two steps the mirrors act like swaps of quads and of halves).
template <int LPR>
__device__ __forceinline__ float row_sum(float v) {
  if (LPR >= 2) v += dpp_mov<0xB1>(v);   // quad_perm [1,0,3,2]
  if (LPR >= 4) v += dpp_mov<0x4E>(v);   // quad_perm [2,3,0,1]
  if (LPR >= 8) v += dpp_mov<0x141>(v);  // row_half_mirror
  if (LPR >= 16) v += dpp_mov<0x140>(v); // row_mirror
  return v;
}

template <typename Io, int LPR, int NV, int ROWS>
__global__ __launch_bounds__(kDecodeThreads) void decode_steps_kernel(
    float *__restrict__ state, const void *__restrict__ x, const float *__restrict__ dt,
    const float *__restrict__ A, const void *__restrict__ B, const void *__restrict__ C,
    const float *__restrict__ D, void *__restrict__ y, int nsteps, size_t npairs, size_t nbc, int BtH,
    int H, int G, int hpg, const DtXform dtx) {
  constexpr int N = LPR * 4 * NV;
  constexpr int RPP = kDecodeThreads / LPR;
  constexpr int P = ROWS * RPP;
  const size_t pair = blockIdx.x;
  const int h = static_cast<int>(pair % H);
  const size_t lb = pair / H;
  const int layer = static_cast<int>(pair / BtH);
  const int lane_n = threadIdx.x % LPR;
  const int row0 = threadIdx.x / LPR;
  const float Ah = A[static_cast<size_t>(layer) * H + h];
  const float Dh = D[static_cast<size_t>(layer) * H + h];
  const float dt_bias = dtx.bias != nullptr ? dtx.bias[static_cast<size_t>(layer) * H + h] : 0.f;
  const size_t bc = (lb * G + h / hpg) * N + lane_n * 4;
  const size_t bc_step = nbc * N;  // elements of B (or C) per step

  float *hbase = state + pair * static_cast<size_t>(P) * N + lane_n * 4;
  float4 hv[ROWS][NV];
#pragma unroll
  for (int u = 0; u < ROWS; ++u)
#pragma unroll
    for (int v = 0; v < NV; ++v)
      hv[u][v] = *reinterpret_cast<const float4 *>(hbase + static_cast<size_t>(row0 + u * RPP) * N + v * (4 * LPR));

  // Inputs of a step: two sets, one consumed while the other is in flight; B and C stay packed in
  // the io dtype until they are used (registers decide how many waves a SIMD holds).  Two steps per
  // loop trip, so that the set index is a compile-time constant and no set is ever copied.  (Three
  // sets, two steps ahead, took 168 registers and measured 10 % slower.)
  struct StepIn {
    float dt;
    Raw4<Io> B[NV], C[NV];
    float x[ROWS];
  } in[2];
  auto request = [&](StepIn &d, int s) __attribute__((always_inline)) {
    d.dt = dt[s * npairs + pair];
#pragma unroll
    for (int v = 0; v < NV; ++v) {
      d.B[v].load(B, s * bc_step + bc + v * (4 * LPR));
      d.C[v].load(C, s * bc_step + bc + v * (4 * LPR));
    }
#pragma unroll
    for (int u = 0; u < ROWS; ++u) d.x[u] = Io::load(x, (s * npairs + pair) * P + row0 + u * RPP);
  };
  auto step = [&](int s, const StepIn &c, StepIn &n) __attribute__((always_inline)) {
    request(n, s + 1 < nsteps ? s + 1 : s);  // the surplus loads of the last step are not used
    const float dtv = dt_apply_biased(c.dt, dt_bias, dtx);
    const float dA = expf(dtv * Ah);
    float4 Bv[NV], Cv[NV];
#pragma unroll
    for (int v = 0; v < NV; ++v) {
      Bv[v] = c.B[v].get();
      Cv[v] = c.C[v].get();
    }
#pragma unroll
    for (int u = 0; u < ROWS; ++u) {
      const float ux = dtv * c.x[u];
      float part = 0.f;
#pragma unroll
      for (int v = 0; v < NV; ++v) {
        float4 w = hv[u][v];
        w.x = fmaf(dA, w.x, ux * Bv[v].x);
        w.y = fmaf(dA, w.y, ux * Bv[v].y);
        w.z = fmaf(dA, w.z, ux * Bv[v].z);
        w.w = fmaf(dA, w.w, ux * Bv[v].w);
        hv[u][v] = w;
        part = fmaf(Cv[v].w, w.w, fmaf(Cv[v].z, w.z, fmaf(Cv[v].y, w.y, fmaf(Cv[v].x, w.x, part))));
      }
      part = row_sum<LPR>(part);
      if (lane_n == 0) Io::store(y, (s * npairs + pair) * P + row0 + u * RPP, fmaf(Dh, c.x[u], part));
    }
  };
  request(in[0], 0);
  int s = 0;
  for (; s + 1 < nsteps; s += 2) {
    step(s, in[0], in[1]);
    step(s + 1, in[1], in[0]);
  }
  if (s < nsteps) step(s, in[0], in[1]);
#pragma unroll
  for (int u = 0; u < ROWS; ++u)
#pragma unroll
    for (int v = 0; v < NV; ++v)
      *reinterpret_cast<float4 *>(hbase + static_cast<size_t>(row0 + u * RPP) * N + v * (4 * LPR)) = hv[u][v];
}

template <typename Io>
hipError_t launch_typed(int nlayers, const Dims &d, float *state, const void *x, const float *dt,
                        const float *A, const void *B, const void *C, const float *D, void *y,
                        hipStream_t stream) {
  const size_t npairs = static_cast<size_t>(nlayers) * d.Bt * d.H;
  const dim3 grid(static_cast<unsigned>(npairs)), block(kDecodeThreads);
  const int BtH = d.Bt * d.H;
  // Small launches (a single layer at a small batch) split each state over several workgroups: the
  // step is latency bound there, and 80 workgroups leave most of the 256 CUs idle.
  auto split_for = [&](int rows_per_pass) {
    int split = 1;
    while (npairs * split < 1024 && d.P / (2 * split) >= rows_per_pass && split < 8) split *= 2;
    return split;
  };
  // the states of this call against the memory-side cache (see load_h4); the decode_stream knob overrides
  bool stream_state = npairs * static_cast<size_t>(d.P) * d.N * sizeof(float) > (256ull << 20);
  if (knobs().decode_stream >= 0) stream_state = knobs().decode_stream != 0;
#define SSD_DECODE_CASE(LPR_)                                                                            \
  case LPR_:                                                                                             \
    if (stream_state)                                                                                    \
      hipLaunchKernelGGL((decode_vec_kernel<Io, LPR_, true>),                                            \
                         dim3(static_cast<unsigned>(npairs), split_for(kDecodeThreads / LPR_)), block, 0, \
                         stream, state, x, dt, A, B, C, D, y, BtH, d.H, d.P, d.G, d.hpg, d.dtx);         \
    else                                                                                                 \
      hipLaunchKernelGGL((decode_vec_kernel<Io, LPR_, false>),                                           \
                         dim3(static_cast<unsigned>(npairs), split_for(kDecodeThreads / LPR_)), block, 0, \
                         stream, state, x, dt, A, B, C, D, y, BtH, d.H, d.P, d.G, d.hpg, d.dtx);         \
    break;
  if (d.N % 4 == 0) {
    switch (d.N / 4) {
      SSD_DECODE_CASE(1)
      SSD_DECODE_CASE(2)
      SSD_DECODE_CASE(4)
      SSD_DECODE_CASE(8)
      SSD_DECODE_CASE(16)
      SSD_DECODE_CASE(32)
      SSD_DECODE_CASE(64)
      default:
        hipLaunchKernelGGL((decode_any_kernel<Io>), grid, block, 0, stream, state, x, dt, A, B, C, D, y,
                           BtH, d.H, d.P, d.N, d.G, d.hpg, d.dtx);
    }
  } else {
    hipLaunchKernelGGL((decode_any_kernel<Io>), grid, block, 0, stream, state, x, dt, A, B, C, D, y, BtH,
                       d.H, d.P, d.N, d.G, d.hpg, d.dtx);
  }
#undef SSD_DECODE_CASE
  return hipGetLastError();
}

// Register-resident multi-step kernel for the shapes whose state fits (at most 64 values per lane); returns false for any other shape.
template <typename Io>
bool launch_steps_resident(int nsteps, int nlayers, const Dims &d, float *state, const void *x, const float *dt,
                           const float *A, const void *B, const void *C, const float *D, void *y,
                           hipStream_t stream) {
  const size_t npairs = static_cast<size_t>(nlayers) * d.Bt * d.H;
  const size_t nbc = static_cast<size_t>(nlayers) * d.Bt * d.G;
  const dim3 grid(static_cast<unsigned>(npairs)), block(kDecodeThreads);
  const int BtH = d.Bt * d.H;
#define SSD_STEPS_CASE(LPR_, NV_, ROWS_)                                                                      \
  if (d.N == 4 * LPR_ * NV_ && d.P == ROWS_ * (kDecodeThreads / LPR_)) {                                      \
    hipLaunchKernelGGL((decode_steps_kernel<Io, LPR_, NV_, ROWS_>), grid, block, 0, stream, state, x, dt, A, B, \
                       C, D, y, nsteps, npairs, nbc, BtH, d.H, d.G, d.hpg, d.dtx);                             \
    return true;                                                                                              \
  }
  SSD_STEPS_CASE(16, 2, 4)  // P 64,  N 128
  SSD_STEPS_CASE(16, 2, 8)  // P 128, N 128
  SSD_STEPS_CASE(16, 2, 2)  // P 32,  N 128
  SSD_STEPS_CASE(16, 1, 4)  // P 64,  N 64
  SSD_STEPS_CASE(16, 1, 8)  // P 128, N 64
  SSD_STEPS_CASE(16, 4, 4)  // P 64,  N 256
  SSD_STEPS_CASE(4, 1, 1)   // P 64,  N 16
  SSD_STEPS_CASE(4, 1, 2)   // P 128, N 16
#undef SSD_STEPS_CASE
  return false;
}

}  // namespace

hipError_t launch_decode(int nlayers, const Dims &d, float *state, const void *x, const float *dt,
                         const float *A, const void *B, const void *C, const float *D, void *y,
                         hipStream_t stream) {
  return d.bf16 ? launch_typed<IoBf16>(nlayers, d, state, x, dt, A, B, C, D, y, stream)
                : launch_typed<IoF32>(nlayers, d, state, x, dt, A, B, C, D, y, stream);
}

hipError_t launch_decode_steps(int nsteps, int nlayers, const Dims &d, float *state, const void *x,
                               const float *dt, const float *A, const void *B, const void *C, const float *D,
                               void *y, hipStream_t stream) {
  const bool resident =
      d.bf16 ? launch_steps_resident<IoBf16>(nsteps, nlayers, d, state, x, dt, A, B, C, D, y, stream)
             : launch_steps_resident<IoF32>(nsteps, nlayers, d, state, x, dt, A, B, C, D, y, stream);
  if (resident) return hipGetLastError();
  // any other shape: one single-step launch per step
  const size_t esz = d.bf16 ? 2 : 4;
  const size_t npairs = static_cast<size_t>(nlayers) * d.Bt * d.H;
  const size_t nbc = static_cast<size_t>(nlayers) * d.Bt * d.G;
  for (int s = 0; s < nsteps; ++s) {
    const hipError_t e = launch_decode(
        nlayers, d, state, static_cast<const char *>(x) + s * npairs * d.P * esz, dt + s * npairs, A,
        static_cast<const char *>(B) + s * nbc * d.N * esz, static_cast<const char *>(C) + s * nbc * d.N * esz, D,
        static_cast<char *>(y) + s * npairs * d.P * esz, stream);
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

}  // namespace ssd
