// MFMA prefill for the Mamba-2 head shape (headdim 64, dstate 128, bf16 io, chunk % 64 == 0).
//
// The chunked algorithm (Alg. 1; Eq. 3) is evaluated on 64-token blocks.  Inside a chunk the
// decay mask of Eq. 3 is lower triangular and, below the diagonal 64x64 blocks, has rank one
// per block pair (exp(cs_l - cs_s) = exp(cs_l - cs_ref) * exp(cs_ref - cs_s) with every exponent
// <= 0).  The off-diagonal part of the masked product therefore equals "C_l . (state entering
// the block)", so one workgroup walks its blocks in order with the fp32 state H (headdim x
// dstate) resident in MFMA accumulators -- the inter-chunk state pass happens in registers,
// wave-synchronously, with no per-chunk launch -- and only the diagonal blocks need the
// element-wise mask.  Per block and head:
//     Y^T  = H C^T                      (state -> output, K = dstate)          8 MFMA / wave
//     Y^T  = exp(cs_l) o Y^T + X'^T M^T (M = G o exp(segsum) masked, K = 64)   <=4 MFMA / wave
//     y    = Y + D x                                                            epilogue
//     H^T  = exp(cs_63) H^T + Bt X''    (chunk-state accumulation, K = 64)     8 MFMA / wave
// with X' = dt o x, X'' = exp(cs_63 - cs_s) o X', all MFMAs v_mfma_f32_32x32x16_bf16 with fp32
// accumulation.  The mask exp2(cs_l - cs_s) is generated in registers from the block-relative
// fp32 prefix sums and never stored; masked entries are exact zeros.
//
// Kernels:
//   scores_bt      per (batch, group, block): G = C B^T (diagonal 64x64 blocks only, bf16) and a
//                  transposed copy of B, both shared by all heads of the group.
//   segment_states per (batch, head, segment): the segment's local end state from a zero start
//                  (only the chunk-state accumulation), so that segments can run in parallel.
//   segment_pass   sequential pass over segment end states -> state entering each segment.
//   chunk_scan     per (batch, head, segment): everything above, from the entering state.
// A segment is a whole number of chunks; with one segment only chunk_scan (and scores_bt) run.
#include <cstdlib>

#include "ssd_internal.hpp"

namespace ssd {
namespace {

constexpr int kBlk = 64;   // tokens per block
constexpr int kP = 64;     // headdim
constexpr int kN = 128;    // dstate
constexpr int kThreads = 256;
constexpr int kCStride = kN + 8;     // LDS row strides in bf16 elements (16-byte pad against
constexpr int kBtStride = kBlk + 8;  // bank conflicts of the row-per-lane operand reads)
constexpr int kXStride = kBlk + 8;
constexpr float kLog2e = 1.4426950408889634f;

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

// One MFMA input operand: 8 bf16 per lane.
union Operand {
  bf16x8 v;
  uint4 q;
  uint2 d[2];
  uint32_t u[4];
};

__device__ __forceinline__ uint32_t pack2(float lo, float hi) {  // two fp32 -> packed bf16, RNE
  f32x2 v = {lo, hi};
  bf16x2 b = __builtin_convertvector(v, bf16x2);
  return __builtin_bit_cast(uint32_t, b);
}
__device__ __forceinline__ float bf_lo(uint32_t u) { return __uint_as_float(u << 16); }
__device__ __forceinline__ float bf_hi(uint32_t u) { return __uint_as_float(u & 0xffff0000u); }
__device__ __forceinline__ float fast_exp2(float v) { return __builtin_amdgcn_exp2f(v); }

// D(32x32) += A(32x16) * B(16x32).  Lane (r = lane%32, kg = lane/32) supplies A[r][8kg..8kg+7] and
// B[8kg..8kg+7][r]; it receives D[(i/4)*8 + 4kg + i%4][r] in element i.
__device__ __forceinline__ f32x16 mfma(const Operand &a, const Operand &b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a.v, b.v, c, 0, 0, 0);
}

// ---- scores_bt: G = C B^T on the diagonal blocks, and B transposed ------------------------------
// grid (NB, Bt*G).  Gd: (Bt*G, NB, 64 l, 64 s) bf16.  Btr: (Bt*G, NB, 128 n, 64 s) bf16.
__global__ __launch_bounds__(kThreads) void scores_bt_kernel(const uint16_t *__restrict__ B,
                                                             const uint16_t *__restrict__ C,
                                                             uint16_t *__restrict__ Gd,
                                                             uint16_t *__restrict__ Btr, int T, int G,
                                                             int NB) {
  __shared__ __align__(16) uint16_t sB[kBlk * (kN + 2)];
  const int jb = blockIdx.x;
  const int bg = blockIdx.y;
  const int b = bg / G, g = bg % G;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int ws = wave >> 1, wl = wave & 1;
  const int r = lane & 31, kg = lane >> 5;
  const int t0 = jb * kBlk;

  // G^T tile (rows s, columns l): lane ends up with four consecutive s for its l.
  const int srow = t0 + 32 * ws + r, lrow = t0 + 32 * wl + r;
  const uint16_t *Bp = B + ((static_cast<size_t>(b) * T + srow) * G + g) * kN + 8 * kg;
  const uint16_t *Cp = C + ((static_cast<size_t>(b) * T + lrow) * G + g) * kN + 8 * kg;
  f32x16 acc = {};
#pragma unroll
  for (int q = 0; q < kN / 16; ++q) {
    Operand a, c;
    a.q = make_uint4(0, 0, 0, 0);
    c.q = make_uint4(0, 0, 0, 0);
    if (srow < T) a.q = *reinterpret_cast<const uint4 *>(Bp + 16 * q);
    if (lrow < T) c.q = *reinterpret_cast<const uint4 *>(Cp + 16 * q);
    acc = mfma(a, c, acc);
  }
  uint16_t *Gout = Gd + (static_cast<size_t>(bg) * NB + jb) * kBlk * kBlk;
  const int l = 32 * wl + r;
#pragma unroll
  for (int i4 = 0; i4 < 4; ++i4) {
    const int s = 32 * ws + i4 * 8 + 4 * kg;
    uint2 v;
    v.x = pack2(acc[4 * i4 + 0], acc[4 * i4 + 1]);
    v.y = pack2(acc[4 * i4 + 2], acc[4 * i4 + 3]);
    *reinterpret_cast<uint2 *>(Gout + l * kBlk + s) = v;
  }

  // B^T: stage the block row-major, write it back n-major.
  for (int c = threadIdx.x; c < kBlk * (kN / 8); c += kThreads) {
    const int row = c / (kN / 8), ch = c % (kN / 8);
    uint4 v = make_uint4(0, 0, 0, 0);
    if (t0 + row < T)
      v = *reinterpret_cast<const uint4 *>(B + ((static_cast<size_t>(b) * T + t0 + row) * G + g) * kN + 8 * ch);
    uint32_t *dst = reinterpret_cast<uint32_t *>(sB + row * (kN + 2) + 8 * ch);
    dst[0] = v.x;
    dst[1] = v.y;
    dst[2] = v.z;
    dst[3] = v.w;
  }
  __syncthreads();
  uint16_t *Bout = Btr + (static_cast<size_t>(bg) * NB + jb) * kN * kBlk;
  for (int c = threadIdx.x; c < kN * (kBlk / 8); c += kThreads) {
    const int n = c / (kBlk / 8), s0 = (c % (kBlk / 8)) * 8;
    uint32_t w[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const uint32_t lo = sB[(s0 + 2 * k) * (kN + 2) + n], hi = sB[(s0 + 2 * k + 1) * (kN + 2) + n];
      w[k] = lo | (hi << 16);
    }
    *reinterpret_cast<uint4 *>(Bout + n * kBlk + s0) = make_uint4(w[0], w[1], w[2], w[3]);
  }
}

// ---- chunk_scan / segment_states ----------------------------------------------------------------
struct ScanParams {
  const uint16_t *x;
  const float *dt;
  const float *A;
  const uint16_t *C;
  const float *D;
  const uint16_t *Gd;
  const uint16_t *Btr;
  uint16_t *y;
  const float *Hin;        // state entering each segment, or nullptr = zeros
  size_t hin_bh_stride;    // elements between consecutive (b, h) in Hin
  float *final_state;      // (Bt, H, P, N): written by the last segment
  float *seg_state;        // states-only: (Bt, H, S, P, N); local end state of segment sg -> slot sg+1
  float *seg_decay;        // states-only: (Bt, H, S) log2 of the segment's total decay
  int T, H, G, hpg, NB, seg_blocks, S;
};

template <bool kStatesOnly>
__global__ __launch_bounds__(kThreads, 2) void chunk_scan_kernel(const ScanParams p) {
  __shared__ __align__(16) uint16_t sC[kStatesOnly ? 8 : kBlk * kCStride];  // C, n permuted per 16
  __shared__ __align__(16) uint16_t sBt[kN * kBtStride];                    // B^T [n][s]
  __shared__ __align__(16) uint16_t sX1[kStatesOnly ? 8 : kP * kXStride];   // (dt o x)^T [p][s]
  __shared__ __align__(16) uint16_t sX2[kP * kXStride];                     // decayed (dt o x)^T
  __shared__ __align__(16) uint4 sExch[kStatesOnly ? 1 : 4][4][64];         // bf16 state operands
  __shared__ __align__(16) float sCs[2][kBlk];  // block-relative inclusive prefix sum of dt*A*log2(e)
  __shared__ __align__(16) float sDt[2][kBlk];  // dt_s
  __shared__ __align__(16) float sW[2][kBlk];   // dt_s * exp2(cs_63 - cs_s)

  const int h = blockIdx.x, sg = blockIdx.y, b = blockIdx.z;
  const int g = h / p.hpg;
  const size_t bh = static_cast<size_t>(b) * p.H + h;
  const size_t bg = static_cast<size_t>(b) * p.G + g;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wn = wave >> 1, wp = wave & 1;  // wn doubles as the row-block index wl of the outputs
  const int r = lane & 31, kg = lane >> 5;
  const int jb0 = sg * p.seg_blocks;
  const int jb1 = min(p.NB, jb0 + p.seg_blocks);
  const float a_scale = p.A[h] * kLog2e;

  // Block-relative prefix sums for block jb into buffer `buf` (wave 0 only; lane = token).
  auto block_cumsum = [&](int jb, int buf) -> float {
    const int t = jb * kBlk + lane;
    const float dtv = (t < p.T) ? p.dt[(static_cast<size_t>(b) * p.T + t) * p.H + h] : 0.f;
    float v = dtv * a_scale;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
      const float up = __shfl_up(v, off, 64);
      if (lane >= off) v += up;
    }
    const float total = __shfl(v, 63, 64);
    sCs[buf][lane] = v;
    sDt[buf][lane] = dtv;
    sW[buf][lane] = dtv * fast_exp2(total - v);
    return total;
  };

  // ---- state accumulators: Hacc[t][i] = H^T[n = 64wn + 32t + (i/4)*8 + 4kg + i%4][p = 32wp + r] ----
  f32x16 Hacc[2];
  if (!kStatesOnly && p.Hin != nullptr) {
    const float *hp = p.Hin + bh * p.hin_bh_stride + static_cast<size_t>(sg) * kP * kN +
                      static_cast<size_t>(32 * wp + r) * kN;
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int i4 = 0; i4 < 4; ++i4) {
        const float4 v = *reinterpret_cast<const float4 *>(hp + 64 * wn + 32 * t + i4 * 8 + 4 * kg);
        Hacc[t][4 * i4 + 0] = v.x;
        Hacc[t][4 * i4 + 1] = v.y;
        Hacc[t][4 * i4 + 2] = v.z;
        Hacc[t][4 * i4 + 3] = v.w;
      }
  } else {
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int i = 0; i < 16; ++i) Hacc[t][i] = 0.f;
  }

  // bf16 copies of the state as MFMA operands: own[2t+u] covers n = 64wn + 32t + 16u + {4kg..4kg+3,
  // 8+4kg..8+4kg+3}; the other n half comes from the partner wave through LDS.
  Operand own[4], partner[4];
  auto pack_state = [&]() {
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int u = 0; u < 2; ++u)
#pragma unroll
        for (int k = 0; k < 4; ++k)
          own[2 * t + u].u[k] = pack2(Hacc[t][8 * u + 2 * k], Hacc[t][8 * u + 2 * k + 1]);
  };
  auto publish_state = [&]() {
#pragma unroll
    for (int k = 0; k < 4; ++k) sExch[wave][k][lane] = own[k].q;
  };

  float seg_total = 0.f;
  if (wave == 0 && jb0 < jb1) seg_total = block_cumsum(jb0, 0);
  if (!kStatesOnly) {
    pack_state();
    publish_state();
  }
  __syncthreads();

  for (int jb = jb0; jb < jb1; ++jb) {
    const int buf = (jb - jb0) & 1;
    const int tb = jb * kBlk;

    // ================= staging phase (between the end barrier of the previous block and A) ======
    Operand Gop[4];
    if (!kStatesOnly) {
      // partner's state operands (published before the previous barrier)
#pragma unroll
      for (int k = 0; k < 4; ++k) partner[k].q = sExch[wave ^ 2][k][lane];
      // G rows for this lane's output column l = 32wn + r, straight into operand registers
      const uint16_t *gp = p.Gd + ((bg * p.NB + jb) * kBlk + 32 * wn + r) * kBlk + 8 * kg;
#pragma unroll
      for (int q = 0; q < 4; ++q)
        if (q <= 2 * wn + 1) Gop[q].q = *reinterpret_cast<const uint4 *>(gp + 16 * q);
      // C tile, columns permuted inside each group of 16 so that one 16-byte read yields
      // n-offsets {4kg..4kg+3, 8+4kg..8+4kg+3}
      for (int c = threadIdx.x; c < kBlk * (kN / 8); c += kThreads) {
        const int row = c / (kN / 8), ch = c % (kN / 8);
        uint4 v = make_uint4(0, 0, 0, 0);
        if (tb + row < p.T)
          v = *reinterpret_cast<const uint4 *>(
              p.C + ((static_cast<size_t>(b) * p.T + tb + row) * p.G + g) * kN + 8 * ch);
        uint16_t *dst = sC + row * kCStride + 16 * (ch >> 1) + 4 * (ch & 1);
        *reinterpret_cast<uint2 *>(dst) = make_uint2(v.x, v.y);
        *reinterpret_cast<uint2 *>(dst + 8) = make_uint2(v.z, v.w);
      }
    }
    {
      const uint16_t *bp = p.Btr + (bg * p.NB + jb) * kN * kBlk;
      for (int c = threadIdx.x; c < kN * (kBlk / 8); c += kThreads) {
        const int n = c / (kBlk / 8), ch = c % (kBlk / 8);
        *reinterpret_cast<uint4 *>(sBt + n * kBtStride + 8 * ch) =
            *reinterpret_cast<const uint4 *>(bp + n * kBlk + 8 * ch);
      }
    }
    // x tile -> X'^T and X''^T: each task takes 4 tokens x 2 columns and writes 2 x 8 bytes per tile
    for (int task = threadIdx.x; task < 16 * 32; task += kThreads) {
      const int pp = task & 31, sq = task >> 5;
      uint32_t v[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int t = tb + 4 * sq + i;
        v[i] = 0;
        if (t < p.T)
          v[i] = *reinterpret_cast<const uint32_t *>(p.x + ((static_cast<size_t>(b) * p.T + t) * p.H + h) * kP +
                                                     2 * pp);
      }
      const float4 w2 = *reinterpret_cast<const float4 *>(&sW[buf][4 * sq]);
      *reinterpret_cast<uint2 *>(sX2 + (2 * pp) * kXStride + 4 * sq) =
          make_uint2(pack2(w2.x * bf_lo(v[0]), w2.y * bf_lo(v[1])), pack2(w2.z * bf_lo(v[2]), w2.w * bf_lo(v[3])));
      *reinterpret_cast<uint2 *>(sX2 + (2 * pp + 1) * kXStride + 4 * sq) =
          make_uint2(pack2(w2.x * bf_hi(v[0]), w2.y * bf_hi(v[1])), pack2(w2.z * bf_hi(v[2]), w2.w * bf_hi(v[3])));
      if (!kStatesOnly) {
        const float4 w1 = *reinterpret_cast<const float4 *>(&sDt[buf][4 * sq]);
        *reinterpret_cast<uint2 *>(sX1 + (2 * pp) * kXStride + 4 * sq) = make_uint2(
            pack2(w1.x * bf_lo(v[0]), w1.y * bf_lo(v[1])), pack2(w1.z * bf_lo(v[2]), w1.w * bf_lo(v[3])));
        *reinterpret_cast<uint2 *>(sX1 + (2 * pp + 1) * kXStride + 4 * sq) = make_uint2(
            pack2(w1.x * bf_hi(v[0]), w1.y * bf_hi(v[1])), pack2(w1.z * bf_hi(v[2]), w1.w * bf_hi(v[3])));
      }
    }
    __syncthreads();  // ---- barrier A: tiles of block jb are in LDS ----

    // prefix sums of the next block, into the other buffer (read only after the end barrier)
    if (wave == 0 && jb + 1 < jb1) seg_total += block_cumsum(jb + 1, buf ^ 1);

    if (!kStatesOnly) {
      const int l = 32 * wn + r;  // this lane's output token inside the block
      const float cs_l = sCs[buf][l];
      // ---- state -> output: Y^T[p][l] = sum_n H[p][n] C[l][n] ----
      f32x16 Y = {};
      const uint16_t *crow = sC + l * kCStride + 8 * kg;
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        Operand c;
        c.q = *reinterpret_cast<const uint4 *>(crow + 16 * (4 * wn + k));
        Y = mfma(own[k], c, Y);
      }
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        Operand c;
        c.q = *reinterpret_cast<const uint4 *>(crow + 16 * (4 * (wn ^ 1) + k));
        Y = mfma(partner[k], c, Y);
      }
      {
        const float e = fast_exp2(cs_l);
#pragma unroll
        for (int i = 0; i < 16; ++i) Y[i] *= e;
      }
      // ---- intra-block: Y^T[p][l] += sum_{s<=l} X'[s][p] * G[l][s] exp2(cs_l - cs_s) ----
      const uint16_t *x1row = sX1 + (32 * wp + r) * kXStride + 8 * kg;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        if (q <= 2 * wn + 1) {
          const int s0 = 16 * q + 8 * kg;
          const float4 ca = *reinterpret_cast<const float4 *>(&sCs[buf][s0]);
          const float4 cb = *reinterpret_cast<const float4 *>(&sCs[buf][s0 + 4]);
          const float css[8] = {ca.x, ca.y, ca.z, ca.w, cb.x, cb.y, cb.z, cb.w};
          Operand m;
#pragma unroll
          for (int k = 0; k < 4; ++k) {
            const float e0 = (s0 + 2 * k <= l) ? fast_exp2(cs_l - css[2 * k]) : 0.f;
            const float e1 = (s0 + 2 * k + 1 <= l) ? fast_exp2(cs_l - css[2 * k + 1]) : 0.f;
            m.u[k] = pack2(bf_lo(Gop[q].u[k]) * e0, bf_hi(Gop[q].u[k]) * e1);
          }
          Operand xo;
          xo.q = *reinterpret_cast<const uint4 *>(x1row + 16 * q);
          Y = mfma(xo, m, Y);
        }
      }
      // ---- epilogue: y[l][p] = Y + D x, four consecutive p per 8-byte store ----
      const int t = tb + l;
      if (t < p.T) {
        const float Dh = p.D[h];
        const size_t row = ((static_cast<size_t>(b) * p.T + t) * p.H + h) * kP + 32 * wp + 4 * kg;
#pragma unroll
        for (int i4 = 0; i4 < 4; ++i4) {
          const uint2 xv = *reinterpret_cast<const uint2 *>(p.x + row + 8 * i4);
          uint2 o;
          o.x = pack2(Y[4 * i4 + 0] + Dh * bf_lo(xv.x), Y[4 * i4 + 1] + Dh * bf_hi(xv.x));
          o.y = pack2(Y[4 * i4 + 2] + Dh * bf_lo(xv.y), Y[4 * i4 + 3] + Dh * bf_hi(xv.y));
          *reinterpret_cast<uint2 *>(p.y + row + 8 * i4) = o;
        }
      }
    }

    // ---- state update: H^T[n][p] = exp2(cs_63) H^T[n][p] + sum_s B^T[n][s] X''[s][p] ----
    {
      const float d = fast_exp2(sCs[buf][kBlk - 1]);
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int i = 0; i < 16; ++i) Hacc[t][i] *= d;
      const uint16_t *x2row = sX2 + (32 * wp + r) * kXStride + 8 * kg;
      const uint16_t *btrow = sBt + (64 * wn + r) * kBtStride + 8 * kg;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        Operand xo, b0, b1;
        xo.q = *reinterpret_cast<const uint4 *>(x2row + 16 * q);
        b0.q = *reinterpret_cast<const uint4 *>(btrow + 16 * q);
        b1.q = *reinterpret_cast<const uint4 *>(btrow + 32 * kBtStride + 16 * q);
        Hacc[0] = mfma(b0, xo, Hacc[0]);
        Hacc[1] = mfma(b1, xo, Hacc[1]);
      }
    }
    if (!kStatesOnly) {
      pack_state();
      publish_state();
    }
    __syncthreads();  // ---- end barrier: tiles may be overwritten, published state is visible ----
  }

  // ---- write the state out (canonical (p, n) layout, four consecutive n per 16-byte store) ----
  float *out = nullptr;
  if (kStatesOnly) {
    out = p.seg_state + (bh * p.S + sg + 1) * kP * kN;
    if (threadIdx.x == 0) p.seg_decay[bh * p.S + sg] = seg_total;
  } else if (sg == p.S - 1) {
    out = p.final_state + bh * kP * kN;
  }
  if (out != nullptr) {
    float *op = out + static_cast<size_t>(32 * wp + r) * kN;
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int i4 = 0; i4 < 4; ++i4)
        *reinterpret_cast<float4 *>(op + 64 * wn + 32 * t + i4 * 8 + 4 * kg) =
            make_float4(Hacc[t][4 * i4 + 0], Hacc[t][4 * i4 + 1], Hacc[t][4 * i4 + 2], Hacc[t][4 * i4 + 3]);
  }
}

// ---- segment_pass: slot[0] = h0; slot[sg] = exp2(decay[sg-1]) * slot[sg-1] + local[sg-1] --------
// grid (P*N/256, Bt*H).  seg_state slot sg (sg >= 1) holds the local end state of segment sg-1 on
// entry and the state entering segment sg on exit.
__global__ __launch_bounds__(kThreads) void segment_pass_kernel(float *__restrict__ seg_state,
                                                                const float *__restrict__ seg_decay,
                                                                const float *__restrict__ h0, int S) {
  const int e = blockIdx.x * kThreads + threadIdx.x;
  const size_t bh = blockIdx.y;
  float run = h0 ? h0[bh * kP * kN + e] : 0.f;
  float *sp = seg_state + bh * S * kP * kN + e;
  sp[0] = run;
  for (int sg = 1; sg < S; ++sg) {
    run = fast_exp2(seg_decay[bh * S + sg - 1]) * run + sp[static_cast<size_t>(sg) * kP * kN];
    sp[static_cast<size_t>(sg) * kP * kN] = run;
  }
}

// Blocks per segment: a whole number of chunks, as few segments as keep >= ~4 workgroups per CU.
int choose_seg_blocks(const Dims &d) {
  const int chunk_blocks = d.L / kBlk;
  const int nchunks = d.Nc;
  int k = 0;
  if (const char *e = std::getenv("SSD_SEG_CHUNKS")) k = std::atoi(e);
  if (k < 1) {
    const long target = 1024;
    const long bh = static_cast<long>(d.Bt) * d.H;
    long want_segs = (target + bh - 1) / bh;       // segments needed to reach the target
    if (want_segs < 1) want_segs = 1;
    if (want_segs > nchunks) want_segs = nchunks;
    k = static_cast<int>((nchunks + want_segs - 1) / want_segs);  // chunks per segment
  }
  if (k > nchunks) k = nchunks;
  if (k < 1) k = 1;
  return k * chunk_blocks;
}

struct Layout {
  int NB, S_max;
  size_t off_G, off_Bt, off_state, off_decay, total;
};

Layout make_layout(const Dims &d) {
  Layout w;
  w.NB = (d.T + kBlk - 1) / kBlk;
  w.S_max = d.Nc;  // a segment is at least one chunk
  const size_t BG = static_cast<size_t>(d.Bt) * d.G, BH = static_cast<size_t>(d.Bt) * d.H;
  size_t off = 0;
  w.off_G = off;
  off += round_up(BG * w.NB * kBlk * kBlk * sizeof(uint16_t), 256);
  w.off_Bt = off;
  off += round_up(BG * w.NB * kN * kBlk * sizeof(uint16_t), 256);
  w.off_state = off;
  off += round_up(BH * w.S_max * kP * kN * sizeof(float), 256);
  w.off_decay = off;
  off += round_up(BH * w.S_max * sizeof(float), 256);
  w.total = off;
  return w;
}

}  // namespace

bool mfma_supported(const Dims &d) {
  return d.bf16 && d.P == kP && d.N == kN && d.L % kBlk == 0 && d.Bt <= 65535 && d.H <= 65535;
}

size_t mfma_workspace_bytes(const Dims &d) { return make_layout(d).total; }

hipError_t launch_prefill_mfma(const Dims &d, const void *x, const float *dt, const float *A, const void *B,
                               const void *C, const float *D, const float *h0, void *y, float *final_state,
                               void *workspace, hipStream_t stream, KernelTrace *trace) {
  const Layout w = make_layout(d);
  char *ws = static_cast<char *>(workspace);
  uint16_t *Gd = reinterpret_cast<uint16_t *>(ws + w.off_G);
  uint16_t *Btr = reinterpret_cast<uint16_t *>(ws + w.off_Bt);
  float *seg_state = reinterpret_cast<float *>(ws + w.off_state);
  float *seg_decay = reinterpret_cast<float *>(ws + w.off_decay);
  const int seg_blocks = choose_seg_blocks(d);
  const int S = (w.NB + seg_blocks - 1) / seg_blocks;

  hipLaunchKernelGGL(scores_bt_kernel, dim3(w.NB, d.Bt * d.G), dim3(kThreads), 0, stream,
                     static_cast<const uint16_t *>(B), static_cast<const uint16_t *>(C), Gd, Btr, d.T, d.G,
                     w.NB);
  trace_mark(trace, stream, "scores_bt");

  ScanParams p;
  p.x = static_cast<const uint16_t *>(x);
  p.dt = dt;
  p.A = A;
  p.C = static_cast<const uint16_t *>(C);
  p.D = D;
  p.Gd = Gd;
  p.Btr = Btr;
  p.y = static_cast<uint16_t *>(y);
  p.final_state = final_state;
  p.seg_state = seg_state;
  p.seg_decay = seg_decay;
  p.T = d.T;
  p.H = d.H;
  p.G = d.G;
  p.hpg = d.hpg;
  p.NB = w.NB;
  p.seg_blocks = seg_blocks;
  p.S = S;
  if (S > 1) {
    p.Hin = nullptr;
    p.hin_bh_stride = 0;
    hipLaunchKernelGGL((chunk_scan_kernel<true>), dim3(d.H, S - 1, d.Bt), dim3(kThreads), 0, stream, p);
    trace_mark(trace, stream, "segment_states");
    hipLaunchKernelGGL(segment_pass_kernel, dim3(kP * kN / kThreads, d.Bt * d.H), dim3(kThreads), 0, stream,
                       seg_state, seg_decay, h0, S);
    trace_mark(trace, stream, "segment_pass");
    p.Hin = seg_state;
    p.hin_bh_stride = static_cast<size_t>(S) * kP * kN;
  } else {
    p.Hin = h0;
    p.hin_bh_stride = static_cast<size_t>(kP) * kN;
  }
  hipLaunchKernelGGL((chunk_scan_kernel<false>), dim3(d.H, S, d.Bt), dim3(kThreads), 0, stream, p);
  trace_mark(trace, stream, "chunk_scan");
  return hipGetLastError();
}

}  // namespace ssd
