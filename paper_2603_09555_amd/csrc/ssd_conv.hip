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
constexpr int kRunMin = 16, kRunMax = 192;  // tokens per thread in the prefill kernel: chosen per launch

// SiLU v / (1 + exp(-v)) with the hardware exp2 and reciprocal (each within 1 ulp): the kernels are
// streams, and an IEEE division per element would make them ALU bound.
__device__ __forceinline__ float act_apply(float v, int act) {
  if (act != 1) return v;
  const float e = __builtin_amdgcn_exp2f(v * -1.4426950408889634f);
  return v * __builtin_amdgcn_rcpf(1.f + e);
}
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {  // two fp32 -> packed bf16, RNE
  f32x2_t v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
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

// One thread: VEC consecutive channels, `run` consecutive tokens.  Threads are numbered over (run of
// tokens, channel group) without padding, channel group fastest: grid (ceil(runs * C / VEC / 256), 1, Bt).
template <typename Io, int VEC, int K>
__global__ __launch_bounds__(kConvThreads) void conv_prefill_kernel(
    const void *__restrict__ u, const float *__restrict__ w, const float *__restrict__ bias,
    const void *__restrict__ state_in, ConvOut out, void *__restrict__ state_out, int T, int C, int act,
    int run_len) {
  using E = typename Io::type;
  const int groups = C / VEC;
  const unsigned gid = blockIdx.x * kConvThreads + threadIdx.x;
  const int run = static_cast<int>(gid / groups);
  const int t0 = run * run_len;
  if (t0 >= T) return;
  const int c0 = static_cast<int>(gid % groups) * VEC;
  const int b = blockIdx.z;
  const int t1 = min(T, t0 + run_len);
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
  constexpr bool kVec = VEC > 1 && sizeof(E) == 2;
  static_assert(VEC == 1 || (kVec && (VEC == 4 || VEC == 8)), "one channel per thread, or 4 / 8 bf16 channels");
  struct Raw {
    uint32_t w[VEC > 1 ? VEC / 2 : 1];  // VEC bf16 values
  };
  // The input is read with non-temporal loads: it is used once, and what the memory-side cache holds
  // after the kernel should be the outputs, which the SSD core reads next (measured on convolution ->
  // prefill at 16384 tokens x 5376 channels: 6-8 % less for the pair, 16 % when the cache starts dirty).
  typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
  typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));
  auto load_raw = [&](const E *ptr) {
    Raw r;
    if constexpr (VEC == 8) {
      const u32x4_t q = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t *>(ptr));
      r.w[0] = q.x, r.w[1] = q.y, r.w[2] = q.z, r.w[3] = q.w;
    } else if constexpr (VEC == 4) {
      const u32x2_t q = __builtin_nontemporal_load(reinterpret_cast<const u32x2_t *>(ptr));
      r.w[0] = q.x, r.w[1] = q.y;
    }
    return r;
  };
  auto unpack_row = [&](const Raw &q, float *dst) {  // bf16 -> fp32
#pragma unroll
    for (int k = 0; k < VEC / 2; ++k) {
      dst[2 * k] = __uint_as_float(q.w[k] << 16);
      dst[2 * k + 1] = __uint_as_float(q.w[k] & 0xffff0000u);
    }
  };
#pragma unroll
  for (int j = 1; j < K; ++j) {
    const int t = t0 - K + j;
    if (kVec && t >= 0) {
      unpack_row(load_raw(ub + static_cast<size_t>(t) * C), win[j]);
    } else {
#pragma unroll
      for (int v = 0; v < VEC; ++v) win[j][v] = input_at(t, v);
    }
  }
  // Tokens are taken kBatch at a time, and the rows of the next batch are requested before the
  // current one is computed, so a thread has kBatch to 2 kBatch 16-byte requests in flight all the
  // time.  Rows stay raw until they enter the window: registers decide how many waves a SIMD can
  // hold.  Two batches per loop trip, so that the buffer index is a compile-time constant.
  constexpr int kBatch = 4;
  struct Rows {
    Raw q[kBatch];
    float s[kBatch];
  } buf[2];
  auto request = [&](Rows &r, int tb) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < kBatch; ++i) {
      const int t = min(tb + i, t1 - 1);  // surplus requests beyond the run repeat its last row
      if constexpr (kVec)
        r.q[i] = load_raw(ub + static_cast<size_t>(t) * C);
      else
        r.s[i] = Io::load(ub, static_cast<size_t>(t) * C);
    }
  };
  auto process = [&](const Rows &r, int tb) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < kBatch; ++i) {
      const int t = tb + i;
      if (t < t1) {
#pragma unroll
        for (int j = 0; j + 1 < K; ++j)
#pragma unroll
          for (int v = 0; v < VEC; ++v) win[j][v] = win[j + 1][v];
        if constexpr (kVec)
          unpack_row(r.q[i], win[K - 1]);
        else
          win[K - 1][0] = r.s[i];
        float z[VEC];
#pragma unroll
        for (int v = 0; v < VEC; ++v) {
          float a = bs[v];
#pragma unroll
          for (int j = 0; j < K; ++j) a = fmaf(wt[v][j], win[j][v], a);
          z[v] = act_apply(a, act);
        }
        E *zp = out_ptr<Io>(out, static_cast<size_t>(b) * T + t, c0);
        if constexpr (kVec) {
          uint32_t pk[VEC / 2];
#pragma unroll
          for (int k = 0; k < VEC / 2; ++k) pk[k] = pack_bf16x2(z[2 * k], z[2 * k + 1]);
          if constexpr (VEC == 8)
            *reinterpret_cast<uint4 *>(zp) = make_uint4(pk[0], pk[1], pk[2], pk[3]);
          else
            *reinterpret_cast<uint2 *>(zp) = make_uint2(pk[0], pk[1]);
        } else {
#pragma unroll
          for (int v = 0; v < VEC; ++v) Io::store(zp, v, z[v]);
        }
      }
    }
  };
  request(buf[0], t0);
  for (int tb = t0; tb < t1; tb += 2 * kBatch) {
    request(buf[1], tb + kBatch);
    process(buf[0], tb);
    request(buf[0], tb + 2 * kBatch);
    process(buf[1], tb + kBatch);
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

// Tokens per thread: long runs amortise the k-1 rows a thread reads in front of its own and the
// weights it loads, but the threads should also fill the chip a whole number of times: the length in
// [kRunMin, kRunMax] with the least (rounds of waves) x (rows read per run).  `blocks_per_cu` is what the
// runtime reports for the kernel (its register count decides it).
int choose_run(int T, size_t groups_total, int ksize, int blocks_per_cu) {
  const double slots = 256.0 * blocks_per_cu * kConvThreads;  // threads resident at once
  int best = kRunMin;
  double best_cost = 0.0;
  for (int len = kRunMin; len <= kRunMax; ++len) {
    const double runs = (T + len - 1) / len;
    const double rounds = static_cast<double>(static_cast<long long>((runs * groups_total + slots - 1) / slots));
    const double cost = rounds * (len + ksize - 1 + 4);  // + about four rows' worth of start-up per thread
    if (len == kRunMin || cost < best_cost) {
      best = len;
      best_cost = cost;
    }
  }
  return best;
}

template <typename Io, int VEC, int K>
int resident_blocks() {
  static const int blocks = [] {
    int n = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, conv_prefill_kernel<Io, VEC, K>, kConvThreads, 0) != hipSuccess ||
        n < 1)
      n = 4;
    return n;
  }();
  return blocks;
}

template <typename Io, int K>
hipError_t prefill_typed(int Bt, int T, int C, bool vec8, const void *u, const float *w, const float *bias,
                         const void *state_in, const ConvOut &out, void *state_out, int act, hipStream_t stream) {
  if constexpr (sizeof(typename Io::type) == 2) {
    if (vec8) {
      constexpr int kV = 4;
      const int run_len = choose_run(T, static_cast<size_t>(Bt) * (C / kV), K, resident_blocks<Io, kV, K>());
      const int runs = (T + run_len - 1) / run_len;
      const dim3 grid(static_cast<unsigned>((static_cast<size_t>(runs) * (C / kV) + kConvThreads - 1) / kConvThreads), 1, Bt);
      hipLaunchKernelGGL((conv_prefill_kernel<Io, kV, K>), grid, dim3(kConvThreads), 0, stream, u, w, bias, state_in,
                         out, state_out, T, C, act, run_len);
      return hipGetLastError();
    }
  }
  {
    const int run_len = choose_run(T, static_cast<size_t>(Bt) * C, K, resident_blocks<Io, 1, K>());
    const int runs = (T + run_len - 1) / run_len;
    const dim3 grid(static_cast<unsigned>((static_cast<size_t>(runs) * C + kConvThreads - 1) / kConvThreads), 1, Bt);
    hipLaunchKernelGGL((conv_prefill_kernel<Io, 1, K>), grid, dim3(kConvThreads), 0, stream, u, w, bias, state_in, out,
                       state_out, T, C, act, run_len);
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
