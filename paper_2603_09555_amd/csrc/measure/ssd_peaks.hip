// Measured machine peaks to put the kernels' figures next to: an MFMA issue loop and plain streaming
// kernels.  Measurement aids only (exported as ssd_peak_probe); nothing in the SSD path calls them.
#include "ssd_internal.hpp"

namespace ssd {
namespace {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));

// Every wave issues iters x 8 independent-enough v_mfma_f32_32x32x16_bf16 (eight accumulators, so the
// 8-pass latency of one instruction is covered by the others).  The result is stored so that nothing is
// optimised away.
__global__ __launch_bounds__(256) void mfma_loop_kernel(float *__restrict__ sink, int iters) {
  bf16x8_t a, b;
#pragma unroll
  for (int k = 0; k < 8; ++k) {
    a[k] = static_cast<__bf16>(0.001f * static_cast<float>((threadIdx.x + k) & 7));
    b[k] = static_cast<__bf16>(0.002f * static_cast<float>((threadIdx.x * 3 + k) & 7));
  }
  f32x16_t acc[8];
#pragma unroll
  for (int j = 0; j < 8; ++j)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[j][i] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[j], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int j = 0; j < 8; ++j)
#pragma unroll
    for (int i = 0; i < 16; ++i) s += acc[j][i];
  sink[static_cast<size_t>(blockIdx.x) * blockDim.x + threadIdx.x] = s;
}

// The same loop on the fp32 matrix instructions: kShape 0 = v_mfma_f32_32x32x2_f32 (what the fp32 prefill
// kernel is written on), 1 = v_mfma_f32_16x16x4_f32.  Eight accumulators per wave again.
typedef float f32x4_t __attribute__((ext_vector_type(4)));
template <int kShape>
__global__ __launch_bounds__(256) void mfma_f32_loop_kernel(float *__restrict__ sink, int iters) {
  const float a = 0.001f * static_cast<float>(threadIdx.x & 7), b = 0.002f * static_cast<float>((threadIdx.x * 3) & 7);
  float s = 0.f;
  if constexpr (kShape == 0) {
    f32x16_t acc[8];
#pragma unroll
    for (int j = 0; j < 8; ++j)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[j][i] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
      for (int j = 0; j < 8; ++j) acc[j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc[j], 0, 0, 0);
    }
#pragma unroll
    for (int j = 0; j < 8; ++j)
#pragma unroll
      for (int i = 0; i < 16; ++i) s += acc[j][i];
  } else {
    f32x4_t acc[8];
#pragma unroll
    for (int j = 0; j < 8; ++j)
#pragma unroll
      for (int i = 0; i < 4; ++i) acc[j][i] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
      for (int j = 0; j < 8; ++j) acc[j] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, acc[j], 0, 0, 0);
    }
#pragma unroll
    for (int j = 0; j < 8; ++j)
#pragma unroll
      for (int i = 0; i < 4; ++i) s += acc[j][i];
  }
  sink[static_cast<size_t>(blockIdx.x) * blockDim.x + threadIdx.x] = s;
}

typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
template <bool kNt>
__device__ __forceinline__ uint4 ld16(const uint4 *p) {
  if constexpr (kNt) {
    const u32x4_t q = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t *>(p));
    return make_uint4(q.x, q.y, q.z, q.w);
  } else {
    return *p;
  }
}
template <bool kNt>
__device__ __forceinline__ void st16(uint4 *p, const uint4 v) {
  if constexpr (kNt) {
    const u32x4_t q = {v.x, v.y, v.z, v.w};
    __builtin_nontemporal_store(q, reinterpret_cast<u32x4_t *>(p));
  } else {
    *p = v;
  }
}

// 16 bytes per lane per step, consecutive lanes on consecutive addresses; eight steps are requested
// before the first is used.  mode 0: copy (read src, write dst); 1: read only (a sum is
// written once per thread); 2: write only.  kNt: non-temporal loads and stores, the accesses the
// decode step uses for a state that no cache can hold.
template <bool kNt>
__global__ __launch_bounds__(256) void stream_kernel(const uint4 *__restrict__ src, uint4 *__restrict__ dst, size_t n,
                                                     int mode) {
  // a workgroup takes 32 KB slabs (eight consecutive 4 KB rows of 256 lanes x 16 bytes), grid-stride
  const size_t slab = 8 * 256;
  const size_t slabs = n / slab;
  uint32_t keep = 0;
  for (size_t sidx = blockIdx.x; sidx < slabs; sidx += gridDim.x) {
    const size_t i = sidx * slab + threadIdx.x;
    uint4 v[8];
    if (mode != 2) {
#pragma unroll
      for (int k = 0; k < 8; ++k) v[k] = ld16<kNt>(src + i + k * 256);
    } else {
#pragma unroll
      for (int k = 0; k < 8; ++k) v[k] = make_uint4(static_cast<uint32_t>(i), k, 2, 3);
    }
    if (mode != 1) {
#pragma unroll
      for (int k = 0; k < 8; ++k) st16<kNt>(dst + i + k * 256, v[k]);
    } else {
#pragma unroll
      for (int k = 0; k < 8; ++k) keep += v[k].x ^ v[k].y ^ v[k].z ^ v[k].w;
    }
  }
  for (size_t i = slabs * slab + static_cast<size_t>(blockIdx.x) * 256 + threadIdx.x; i < n;
       i += static_cast<size_t>(gridDim.x) * 256) {
    uint4 v = mode != 2 ? ld16<kNt>(src + i) : make_uint4(static_cast<uint32_t>(i), 1, 2, 3);
    if (mode != 1) st16<kNt>(dst + i, v); else keep += v.x ^ v.y ^ v.z ^ v.w;
  }
  if (mode == 1 && keep == 0x12345678u) dst[0] = make_uint4(keep, 0, 0, 0);  // (practically never) keeps the loads alive
}

}  // namespace

// kind 0: MFMA loop (work = iters; buffer a: at least 2048 * 256 floats); kinds 7, 8: the same on the fp32 matrix
// instructions 32x32x2 / 16x16x4.  kinds 1..3: copy / read /
// write of `bytes` bytes (a = source, b = destination); kinds 4..6: the same, non-temporal.  Returns the elapsed milliseconds of `reps`
// back-to-back launches in *ms and the work of ONE launch (flops or bytes moved) in *work.
hipError_t run_peak_probe(int kind, int iters, int reps, void *a, void *b, size_t bytes, float *ms, double *work,
                          hipStream_t stream) {
  hipEvent_t e0, e1;
  hipError_t e = hipEventCreate(&e0);
  if (e != hipSuccess) return e;
  e = hipEventCreate(&e1);
  if (e != hipSuccess) {
    (void)hipEventDestroy(e0);
    return e;
  }
  const int wgs = 2048;  // eight workgroups of four waves per CU
  auto once = [&]() {
    if (kind == 0)
      hipLaunchKernelGGL(mfma_loop_kernel, dim3(wgs), dim3(256), 0, stream, static_cast<float *>(a), iters);
    else if (kind == 7)
      hipLaunchKernelGGL(mfma_f32_loop_kernel<0>, dim3(wgs), dim3(256), 0, stream, static_cast<float *>(a), iters);
    else if (kind == 8)
      hipLaunchKernelGGL(mfma_f32_loop_kernel<1>, dim3(wgs), dim3(256), 0, stream, static_cast<float *>(a), iters);
    else if (kind <= 3)
      hipLaunchKernelGGL(stream_kernel<false>, dim3(wgs * 2), dim3(256), 0, stream, static_cast<const uint4 *>(a),
                         static_cast<uint4 *>(b), bytes / 16, kind - 1);
    else
      hipLaunchKernelGGL(stream_kernel<true>, dim3(wgs * 2), dim3(256), 0, stream, static_cast<const uint4 *>(a),
                         static_cast<uint4 *>(b), bytes / 16, kind - 4);
  };
  once();  // warm-up
  (void)hipEventRecord(e0, stream);
  for (int r = 0; r < reps; ++r) once();
  (void)hipEventRecord(e1, stream);
  e = hipEventSynchronize(e1);
  if (e == hipSuccess) e = hipEventElapsedTime(ms, e0, e1);
  if (e == hipSuccess) e = hipGetLastError();
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  if (kind == 0)
    *work = static_cast<double>(wgs) * 4.0 * iters * 8.0 * (2.0 * 32 * 32 * 16);
  else if (kind == 7)
    *work = static_cast<double>(wgs) * 4.0 * iters * 8.0 * (2.0 * 32 * 32 * 2);
  else if (kind == 8)
    *work = static_cast<double>(wgs) * 4.0 * iters * 8.0 * (2.0 * 16 * 16 * 4);
  else
    *work = static_cast<double>(bytes / 16 * 16) * (kind == 1 || kind == 4 ? 2.0 : 1.0);
  return e;
}

}  // namespace ssd
