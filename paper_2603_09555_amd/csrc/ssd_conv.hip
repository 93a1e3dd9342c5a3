// Depthwise causal convolution in front of the SSD core (Alg. 2, "Update conv state" and
// "DepthwiseConv"; section "The O(1) state cache": a sliding window of k-1 cached inputs per channel).
//
//   window_t = [ the k-1 inputs before token t , u_t ]                    (k values per channel)
//   z[t][c]  = act( bias[c] + sum_j w[c][j] * window_t[j][c] ),  j = 0 .. k-1, w[c][k-1] multiplies u_t
//   cache    <- the last k-1 inputs                                        (batch, channels, k-1)
//
// Prefill runs the same filter over a whole prompt (inputs before the prompt come from the cache, or
// are zero) and leaves the cache that the first decode step needs; the decode step is the one-token
// case.  Both are pure streams (one read of u, one write of z), so the kernels are laid out for HBM:
// channels-last tensors, a lane owns 8 consecutive channels (16 bytes of bf16), a thread walks a run
// of tokens with the window in registers, and the weights of its channels stay in registers.
// The output can be scattered into up to three dense tensors by channel range, which is how a
// Mamba-2 block consumes it (x | B | C go to the SSD core as separate tensors).
#include "ssd_internal.hpp"

namespace ssd {
namespace {

constexpr int kConvThreads = 256;
constexpr int kRun = 32;  // tokens per thread in the prefill kernel

__device__ __forceinline__ float act_apply(float v, int act) {
  return act == 1 ? v / (1.f + __expf(-v)) : v;  // 1: SiLU
}

struct ConvOut {
  void *ptr[3];  // dense (batch, T, width[i]) tensors
  int begin[4];  // channel ranges [begin[i], begin[i+1])
};

// Output address of channel c (c is a multiple of VEC and ranges are multiples of VEC).
template <typename Io>
__device__ __forceinline__ typename Io::type *out_ptr(const ConvOut &o, size_t row, int c) {
  const int part = c >= o.begin[2] ? 2 : (c >= o.begin[1] ? 1 : 0);
  const int width = o.begin[part + 1] - o.begin[part];
  return static_cast<typename Io::type *>(o.ptr[part]) + row * width + (c - o.begin[part]);
}

// One thread: VEC consecutive channels, kRun consecutive tokens.  grid (ceil(C / (VEC*256)), ceil(T / kRun), Bt).
template <typename Io, int VEC, int K>
__global__ __launch_bounds__(kConvThreads) void conv_prefill_kernel(
    const void *__restrict__ u, const float *__restrict__ w, const float *__restrict__ bias,
    const void *__restrict__ state_in, ConvOut out, void *__restrict__ state_out, int T, int C, int act) {
  using E = typename Io::type;
  const int c0 = (blockIdx.x * kConvThreads + threadIdx.x) * VEC;
  if (c0 >= C) return;
  const int b = blockIdx.z;
  const int t0 = blockIdx.y * kRun;
  const int t1 = min(T, t0 + kRun);
  float wt[VEC][K], bs[VEC];
#pragma unroll
  for (int v = 0; v < VEC; ++v) {
#pragma unroll
    for (int j = 0; j < K; ++j) wt[v][j] = w[static_cast<size_t>(c0 + v) * K + j];
    bs[v] = bias ? bias[c0 + v] : 0.f;
  }
  // window[j] = input at token t - (K-1) + j; tokens before the prompt come from the cache
  float win[K][VEC];
  const E *ub = static_cast<const E *>(u) + static_cast<size_t>(b) * T * C + c0;
  const E *sb = state_in ? static_cast<const E *>(state_in) + (static_cast<size_t>(b) * C + c0) * (K - 1) : nullptr;
  auto input_at = [&](int t, int v) -> float {  // t may be negative: cache entry K-1+t
    if (t >= 0) return Io::load(ub, static_cast<size_t>(t) * C + v);
    return sb ? Io::load(sb, static_cast<size_t>(v) * (K - 1) + (K - 1 + t)) : 0.f;
  };
#pragma unroll
  for (int j = 1; j < K; ++j)
#pragma unroll
    for (int v = 0; v < VEC; ++v) win[j][v] = input_at(t0 - K + j, v);
  for (int t = t0; t < t1; ++t) {
#pragma unroll
    for (int j = 0; j + 1 < K; ++j)
#pragma unroll
      for (int v = 0; v < VEC; ++v) win[j][v] = win[j + 1][v];
    if constexpr (VEC == 8 && sizeof(E) == 2) {
      const uint4 q = *reinterpret_cast<const uint4 *>(ub + static_cast<size_t>(t) * C);
      const uint32_t qq[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        win[K - 1][2 * k] = __uint_as_float(qq[k] << 16);
        win[K - 1][2 * k + 1] = __uint_as_float(qq[k] & 0xffff0000u);
      }
    } else {
#pragma unroll
      for (int v = 0; v < VEC; ++v) win[K - 1][v] = Io::load(ub, static_cast<size_t>(t) * C + v);
    }
    float z[VEC];
#pragma unroll
    for (int v = 0; v < VEC; ++v) {
      float a = bs[v];
#pragma unroll
      for (int j = 0; j < K; ++j) a = fmaf(wt[v][j], win[j][v], a);
      z[v] = act_apply(a, act);
    }
    E *zp = out_ptr<Io>(out, static_cast<size_t>(b) * T + t, c0);
    if constexpr (VEC == 8 && sizeof(E) == 2) {
      uint32_t pk[4];
#pragma unroll
      for (int k = 0; k < 4; ++k)
        pk[k] = static_cast<uint32_t>(f32_to_bf16_bits(z[2 * k])) | (static_cast<uint32_t>(f32_to_bf16_bits(z[2 * k + 1])) << 16);
      *reinterpret_cast<uint4 *>(zp) = make_uint4(pk[0], pk[1], pk[2], pk[3]);
    } else {
#pragma unroll
      for (int v = 0; v < VEC; ++v) Io::store(zp, v, z[v]);
    }
  }
  // the thread that owns the last tokens leaves the cache: inputs T-(K-1) .. T-1
  if (t1 == T && state_out) {
    E *so = static_cast<E *>(state_out) + (static_cast<size_t>(b) * C + c0) * (K - 1);
#pragma unroll
    for (int v = 0; v < VEC; ++v)
#pragma unroll
      for (int j = 0; j + 1 < K; ++j) Io::store(so, static_cast<size_t>(v) * (K - 1) + j, input_at(T - (K - 1) + j, v));
  }
}

// Decode step: one thread per channel.  cache (batch, C, K-1) in place.
template <typename Io, int K>
__global__ __launch_bounds__(kConvThreads) void conv_step_kernel(void *__restrict__ state, const void *__restrict__ u,
                                                                 const float *__restrict__ w,
                                                                 const float *__restrict__ bias, ConvOut out,
                                                                 size_t n, int C, int act) {
  using E = typename Io::type;
  const size_t i = static_cast<size_t>(blockIdx.x) * kConvThreads + threadIdx.x;  // b * C + c
  if (i >= n) return;
  const int c = static_cast<int>(i % C);
  const size_t b = i / C;
  E *s = static_cast<E *>(state) + i * (K - 1);
  float win[K];
#pragma unroll
  for (int j = 0; j + 1 < K; ++j) win[j] = Io::load(s, j);
  win[K - 1] = Io::load(u, i);
  float a = bias ? bias[c] : 0.f;
#pragma unroll
  for (int j = 0; j < K; ++j) a = fmaf(w[static_cast<size_t>(c) * K + j], win[j], a);
#pragma unroll
  for (int j = 0; j + 1 < K; ++j) Io::store(s, j, win[j + 1]);
  const int part = c >= out.begin[2] ? 2 : (c >= out.begin[1] ? 1 : 0);
  const int width = out.begin[part + 1] - out.begin[part];
  Io::store(out.ptr[part], b * width + (c - out.begin[part]), act_apply(a, act));
}

template <typename Io, int K>
hipError_t prefill_typed(int Bt, int T, int C, bool vec8, const void *u, const float *w, const float *bias,
                         const void *state_in, const ConvOut &out, void *state_out, int act, hipStream_t stream) {
  const int runs = (T + kRun - 1) / kRun;
  if (vec8) {
    const dim3 grid((C / 8 + kConvThreads - 1) / kConvThreads, runs, Bt);
    hipLaunchKernelGGL((conv_prefill_kernel<Io, 8, K>), grid, dim3(kConvThreads), 0, stream, u, w, bias, state_in, out,
                       state_out, T, C, act);
  } else {
    const dim3 grid((C + kConvThreads - 1) / kConvThreads, runs, Bt);
    hipLaunchKernelGGL((conv_prefill_kernel<Io, 1, K>), grid, dim3(kConvThreads), 0, stream, u, w, bias, state_in, out,
                       state_out, T, C, act);
  }
  return hipGetLastError();
}

template <typename Io, int K>
hipError_t step_typed(int Bt, int C, void *state, const void *u, const float *w, const float *bias, const ConvOut &out,
                      int act, hipStream_t stream) {
  const size_t n = static_cast<size_t>(Bt) * C;
  hipLaunchKernelGGL((conv_step_kernel<Io, K>), dim3(static_cast<unsigned>((n + kConvThreads - 1) / kConvThreads)),
                     dim3(kConvThreads), 0, stream, state, u, w, bias, out, n, C, act);
  return hipGetLastError();
}

ConvOut make_out(void *const z[3], const int width[3]) {
  ConvOut o;
  int c = 0;
  for (int i = 0; i < 3; ++i) {
    o.ptr[i] = z[i];
    o.begin[i] = c;
    c += width[i];
  }
  o.begin[3] = c;
  return o;
}

}  // namespace

#define SSD_CONV_DISPATCH(FN, ...)                                         \
  switch (ksize) {                                                         \
    case 2: return bf16 ? FN<IoBf16, 2>(__VA_ARGS__) : FN<IoF32, 2>(__VA_ARGS__); \
    case 3: return bf16 ? FN<IoBf16, 3>(__VA_ARGS__) : FN<IoF32, 3>(__VA_ARGS__); \
    case 4: return bf16 ? FN<IoBf16, 4>(__VA_ARGS__) : FN<IoF32, 4>(__VA_ARGS__); \
    case 5: return bf16 ? FN<IoBf16, 5>(__VA_ARGS__) : FN<IoF32, 5>(__VA_ARGS__); \
    case 6: return bf16 ? FN<IoBf16, 6>(__VA_ARGS__) : FN<IoF32, 6>(__VA_ARGS__); \
    case 7: return bf16 ? FN<IoBf16, 7>(__VA_ARGS__) : FN<IoF32, 7>(__VA_ARGS__); \
    case 8: return bf16 ? FN<IoBf16, 8>(__VA_ARGS__) : FN<IoF32, 8>(__VA_ARGS__); \
    default: return hipErrorInvalidValue;                                  \
  }

hipError_t launch_conv_prefill(int Bt, int T, int ksize, bool bf16, const void *u, const float *w, const float *bias,
                               const void *state_in, void *const z[3], const int width[3], void *state_out, int act,
                               hipStream_t stream) {
  const ConvOut out = make_out(z, width);
  const int C = out.begin[3];
  // the vector kernel wants 16-byte pieces that do not straddle two output tensors
  const bool vec8 = bf16 && width[0] % 8 == 0 && width[1] % 8 == 0 && width[2] % 8 == 0;
  SSD_CONV_DISPATCH(prefill_typed, Bt, T, C, vec8, u, w, bias, state_in, out, state_out, act, stream)
}

hipError_t launch_conv_step(int Bt, int ksize, bool bf16, void *state, const void *u, const float *w, const float *bias,
                            void *const z[3], const int width[3], int act, hipStream_t stream) {
  const ConvOut out = make_out(z, width);
  const int C = out.begin[3];
  SSD_CONV_DISPATCH(step_typed, Bt, C, state, u, w, bias, out, act, stream)
}

}  // namespace ssd
