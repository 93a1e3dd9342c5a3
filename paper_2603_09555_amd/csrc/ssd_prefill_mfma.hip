// MFMA prefill for the Mamba-2 head shape (headdim 64, dstate 128, bf16 io, chunk % 64 == 0).
//
// The chunked algorithm (Alg. 1; Eq. 3) is evaluated on 64-token blocks.  Below the diagonal
// blocks the decay mask of Eq. 3 has rank one per block pair, so the off-diagonal part of the
// masked product equals "C_l . (state entering the block)": one workgroup walks its blocks in
// order with the fp32 state H (headdim x dstate) resident in MFMA accumulators -- the
// inter-chunk state pass happens in registers with no per-chunk launch -- and only the
// diagonal 64x64 blocks need the mask.  Inside a diagonal block the mask is factorised around a
// reference point per 32-token half (ref_0 = block start, ref_1 = token 31):
//     exp(cs_l - cs_s) = exp(cs_l - ref_I) * exp(ref_I - ref_J) * exp(ref_J - cs_s),   J <= I
// The last factor is folded into the input once per token (Xc = dt_s exp(ref_J - cs_s) x_s), the
// middle one is a scalar applied to the accumulators between MFMA groups, the first one scales
// output rows, and what remains of the mask -- the causal zero pattern -- is head independent
// and baked into G = tril(C B^T), computed once per group.  So the mask is never materialised,
// costs no per-element work per head, and every exponent that is evaluated is bounded by the
// decay of 32 tokens (clamped at 2^100, far beyond dt*|A| = 1.6 per token).  Per block and head:
//     Y^T  = H C^T                      (state -> output, K = dstate)          8 MFMA / wave
//     Y^T += Xc^T G^T                   (intra-block, K <= 64)                 2-4 MFMA / wave
//     y    = rowfactor o Y + D x                                               epilogue
//     H^T  = d1 (d0 (H^T + Bt Xc[0:32]) + Bt Xc[32:64])                        8 MFMA / wave
// all MFMAs v_mfma_f32_32x32x16_bf16 with fp32 accumulation; decay arithmetic is fp32.
//
// Kernels:
//   scores_bt      per (batch, group, block): G = tril(C B^T) (diagonal blocks only, bf16) and a
//                  transposed copy of B, both shared by all heads of the group.
//   block_cumsum   per (batch, head, block): prefix sums of dt*A and the per-token input factors.
//   segment_states per (batch, head, segment): the segment's local end state from a zero start
//                  (only the chunk-state accumulation), so that segments can run in parallel.
//   segment_pass   sequential pass over segment end states -> state entering each segment.
//   chunk_scan     per (batch, head, segment): everything above, from the entering state.
// A segment is a whole number of chunks; with one segment only the first two and chunk_scan run.
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
// Native vectors (not the HIP struct types: copies of those go through memcpy and may end up in
// scratch memory instead of registers).
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ u32x4 mk4(uint32_t a, uint32_t b, uint32_t c, uint32_t d) { return u32x4{a, b, c, d}; }
__device__ __forceinline__ u32x2 mk2(uint32_t a, uint32_t b) { return u32x2{a, b}; }

// One MFMA input operand: 8 bf16 per lane.
union Operand {
  bf16x8 v;
  u32x4 q;
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

// ---- scores_bt: G = tril(C B^T) on the diagonal blocks, and B transposed ------------------------------
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
    a.q = mk4(0, 0, 0, 0);
    c.q = mk4(0, 0, 0, 0);
    if (srow < T) a.q = *reinterpret_cast<const u32x4 *>(Bp + 16 * q);
    if (lrow < T) c.q = *reinterpret_cast<const u32x4 *>(Cp + 16 * q);
    acc = mfma(a, c, acc);
  }
  uint16_t *Gout = Gd + (static_cast<size_t>(bg) * NB + jb) * kBlk * kBlk;
  const int l = 32 * wl + r;
#pragma unroll
  for (int i4 = 0; i4 < 4; ++i4) {
    const int s = 32 * ws + i4 * 8 + 4 * kg;
    u32x2 v;  // causal zero pattern: keep s <= l
    v.x = pack2(s + 0 <= l ? acc[4 * i4 + 0] : 0.f, s + 1 <= l ? acc[4 * i4 + 1] : 0.f);
    v.y = pack2(s + 2 <= l ? acc[4 * i4 + 2] : 0.f, s + 3 <= l ? acc[4 * i4 + 3] : 0.f);
    *reinterpret_cast<u32x2 *>(Gout + l * kBlk + s) = v;
  }

  // B^T: stage the block row-major, write it back n-major.
  for (int c = threadIdx.x; c < kBlk * (kN / 8); c += kThreads) {
    const int row = c / (kN / 8), ch = c % (kN / 8);
    u32x4 v = mk4(0, 0, 0, 0);
    if (t0 + row < T)
      v = *reinterpret_cast<const u32x4 *>(B + ((static_cast<size_t>(b) * T + t0 + row) * G + g) * kN + 8 * ch);
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
    *reinterpret_cast<u32x4 *>(Bout + n * kBlk + s0) = mk4(w[0], w[1], w[2], w[3]);
  }
}

// ---- block_cumsum: per (batch, head, block) decay bookkeeping ----------------------------------
// grid (NB, ceil(H/16), Bt).  For every head writes one 128-float record per block:
//   [0,64)    cs_s  block-relative inclusive prefix sum of dt*A*log2(e)   (the "segsum" input)
//   [64,128)  f_s = dt_s * exp2(min(ref - cs_s, 100)), ref = 0 for s < 32 and cs_31 otherwise
// Tokens beyond the sequence get dt = 0 (state-neutral padding).  dt is read in its
// (batch, token, head) layout and transposed through LDS.
constexpr int kRec = 2 * kBlk;
constexpr int kCumHeads = 16;
constexpr float kMaxExp = 100.f;
__global__ __launch_bounds__(kThreads) void block_cumsum_kernel(const float *__restrict__ dt,
                                                                const float *__restrict__ A,
                                                                float *__restrict__ prep, int T, int H,
                                                                int NB) {
  __shared__ float tile[kBlk][kCumHeads + 1];
  const int jb = blockIdx.x, h0 = blockIdx.y * kCumHeads, b = blockIdx.z;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int tb = jb * kBlk;
  for (int i = threadIdx.x; i < kBlk * kCumHeads; i += kThreads) {
    const int tok = i / kCumHeads, hh = i % kCumHeads;
    float v = 0.f;
    if (tb + tok < T && h0 + hh < H) v = dt[(static_cast<size_t>(b) * T + tb + tok) * H + h0 + hh];
    tile[tok][hh] = v;
  }
  __syncthreads();
  for (int hh = wave; hh < kCumHeads && h0 + hh < H; hh += kThreads / 64) {
    const int h = h0 + hh;
    const float dtv = tile[lane][hh];
    float v = dtv * (A[h] * kLog2e);
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
      const float up = __shfl_up(v, off, 64);
      if (lane >= off) v += up;
    }
    const float c31 = __shfl(v, 31, 64);  // executed by every lane: the source lane must be active
    const float ref = (lane < 32) ? 0.f : c31;
    float *rec = prep + ((static_cast<size_t>(b) * H + h) * NB + jb) * kRec;
    rec[lane] = v;
    rec[kBlk + lane] = dtv * fast_exp2(fminf(ref - v, kMaxExp));
  }
}

// ---- chunk_scan / segment_states ----------------------------------------------------------------
struct ScanParams {
  const uint16_t *x;
  const uint16_t *C;
  const float *D;
  const uint16_t *Gd;
  const uint16_t *Btr;
  const float *prep;
  uint16_t *y;
  const float *Hin;        // state entering each segment, or nullptr = zeros
  size_t hin_bh_stride;    // elements between consecutive (b, h) in Hin
  float *final_state;      // (Bt, H, P, N): written by the last segment
  float *seg_state;        // states-only: (Bt, H, S, P, N); local end state of segment sg -> slot sg+1
  float *seg_decay;        // states-only: (Bt, H, S) log2 of the segment's total decay
  int T, H, G, hpg, NB, seg_blocks, S;
};

// Register budget: two workgroups (8 waves) per CU for the full kernel, up to four for the
// states-only one; pinned so that the compiler neither spills to reach a higher occupancy
// nor exceeds what two resident workgroups allow.
template <bool kStatesOnly>
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(2, kStatesOnly ? 4 : 2)))
void chunk_scan_kernel(const ScanParams p) {
  __shared__ __align__(16) uint16_t sC[kStatesOnly ? 8 : kBlk * kCStride];  // C, n permuted per 16
  __shared__ __align__(16) uint16_t sBt[kN * kBtStride];                    // B^T [n][s]
  __shared__ __align__(16) uint16_t sXc[kP * kXStride];                     // Xc^T [p][s]
  __shared__ __align__(16) u32x4 sExch[kStatesOnly ? 1 : 4][4][64];         // bf16 state operands
  __shared__ __align__(16) float sCs[kBlk];  // block-relative inclusive prefix sum of dt*A*log2(e)

  const int h = blockIdx.x, sg = blockIdx.y, b = blockIdx.z;
  const int g = h / p.hpg;
  const size_t bh = static_cast<size_t>(b) * p.H + h;
  const size_t bg = static_cast<size_t>(b) * p.G + g;
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int wn = wave >> 1, wp = wave & 1;  // wn doubles as the row-block index of the outputs
  const int r = lane & 31, kg = lane >> 5;
  const int jb0 = sg * p.seg_blocks;
  const int jb1 = min(p.NB, jb0 + p.seg_blocks);
  const int pp = tid & 31, sq0 = tid >> 5;  // x staging: columns 2pp, 2pp+1; tokens 4sq..4sq+3

  // Everything the workgroup needs for one block is held in registers while the previous block
  // is being computed (global-load latency is hidden behind that block's MFMA work).
  u32x4 r_c[4];          // C tile, 16-byte chunks
  u32x4 r_bt[4] = {};    // B^T tile
  uint32_t r_x[2][4];    // x: 2 tasks x 4 tokens x 2 columns
  f32x4 r_f4[2];        // per-token input factors of the two tasks
  f32x4 r_cs4 = {};     // threads 0..15: the block's prefix sums
  u32x4 r_g[4];          // G rows in operand layout

  auto load_block = [&](int jb) {
    const int tb = jb * kBlk;
    const float *rec = p.prep + (bh * p.NB + jb) * kRec;
#pragma unroll
    for (int k = 0; k < 2; ++k) {
      const int sq = sq0 + 8 * k;
      r_f4[k] = *reinterpret_cast<const f32x4 *>(rec + kBlk + 4 * sq);
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int t = tb + 4 * sq + i;
        r_x[k][i] = 0;
        if (t < p.T)
          r_x[k][i] = *reinterpret_cast<const uint32_t *>(
              p.x + ((static_cast<size_t>(b) * p.T + t) * p.H + h) * kP + 2 * pp);
      }
    }
    if (tid < 16) r_cs4 = *reinterpret_cast<const f32x4 *>(rec + 4 * tid);
    const uint16_t *bp = p.Btr + (bg * p.NB + jb) * kN * kBlk;
#pragma unroll
    for (int k = 0; k < 4; ++k) r_bt[k] = *reinterpret_cast<const u32x4 *>(bp + 8 * (tid + kThreads * k));
    if constexpr (!kStatesOnly) {
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        const int c = tid + kThreads * k, row = c >> 4, ch = c & 15;
        r_c[k] = mk4(0, 0, 0, 0);
        if (tb + row < p.T)
          r_c[k] = *reinterpret_cast<const u32x4 *>(
              p.C + ((static_cast<size_t>(b) * p.T + tb + row) * p.G + g) * kN + 8 * ch);
      }
      const uint16_t *gp = p.Gd + ((bg * p.NB + jb) * kBlk + 32 * wn + r) * kBlk + 8 * kg;
#pragma unroll
      for (int q = 0; q < 4; ++q)
        if (q <= 2 * wn + 1) r_g[q] = *reinterpret_cast<const u32x4 *>(gp + 16 * q);
    }
  };

  auto store_block = [&]() {
    if (tid < 16) *reinterpret_cast<f32x4 *>(&sCs[4 * tid]) = r_cs4;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const int c = tid + kThreads * k, n = c >> 3, ch = c & 7;
      *reinterpret_cast<u32x4 *>(sBt + n * kBtStride + 8 * ch) = r_bt[k];
    }
#pragma unroll
    for (int k = 0; k < 2; ++k) {
      const int sq = sq0 + 8 * k;
      const f32x4 f = r_f4[k];
      const uint32_t v0 = r_x[k][0], v1 = r_x[k][1], v2 = r_x[k][2], v3 = r_x[k][3];
      *reinterpret_cast<u32x2 *>(sXc + (2 * pp) * kXStride + 4 * sq) =
          mk2(pack2(f.x * bf_lo(v0), f.y * bf_lo(v1)), pack2(f.z * bf_lo(v2), f.w * bf_lo(v3)));
      *reinterpret_cast<u32x2 *>(sXc + (2 * pp + 1) * kXStride + 4 * sq) =
          mk2(pack2(f.x * bf_hi(v0), f.y * bf_hi(v1)), pack2(f.z * bf_hi(v2), f.w * bf_hi(v3)));
    }
    if constexpr (!kStatesOnly) {
      // C columns are permuted inside each group of 16 so that one 16-byte read yields
      // n-offsets {4kg..4kg+3, 8+4kg..8+4kg+3}
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        const int c = tid + kThreads * k, row = c >> 4, ch = c & 15;
        uint16_t *dst = sC + row * kCStride + 16 * (ch >> 1) + 4 * (ch & 1);
        *reinterpret_cast<u32x2 *>(dst) = mk2(r_c[k].x, r_c[k].y);
        *reinterpret_cast<u32x2 *>(dst + 8) = mk2(r_c[k].z, r_c[k].w);
      }
    }
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
        const f32x4 v = *reinterpret_cast<const f32x4 *>(hp + 64 * wn + 32 * t + i4 * 8 + 4 * kg);
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
  Operand own[4], partner[4], Gop[4];
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
  if (jb0 < jb1) load_block(jb0);
  if constexpr (!kStatesOnly) {
    pack_state();
    publish_state();
  }
  if (jb0 < jb1) {
    store_block();
    if constexpr (!kStatesOnly) {
#pragma unroll
      for (int q = 0; q < 4; ++q) Gop[q].q = r_g[q];
    }
  }
  __syncthreads();

  for (int jb = jb0; jb < jb1; ++jb) {
    const int tb = jb * kBlk;
    const bool more = jb + 1 < jb1;
    // ---- issue the next block's global loads; they land while this block is computed ----
    if (more) load_block(jb + 1);
    const int l = 32 * wn + r;  // this lane's output token inside the block
    const int t = tb + l;
    u32x2 xepi[4];
    size_t yrow = 0;
    if constexpr (!kStatesOnly) {
      // partner's state operands (published between the two barriers that end the previous block)
#pragma unroll
      for (int k = 0; k < 4; ++k) partner[k].q = sExch[wave ^ 2][k][lane];
      yrow = ((static_cast<size_t>(b) * p.T + min(t, p.T - 1)) * p.H + h) * kP + 32 * wp + 4 * kg;
#pragma unroll
      for (int i4 = 0; i4 < 4; ++i4) xepi[i4] = *reinterpret_cast<const u32x2 *>(p.x + yrow + 8 * i4);
    }
    const float c31 = sCs[31], c63 = sCs[kBlk - 1];
    const float d0 = fast_exp2(c31);        // decay over tokens 0..31
    const float d1 = fast_exp2(c63 - c31);  // decay over tokens 32..63
    if (kStatesOnly) seg_total += c63;
    const uint16_t *xrow = sXc + (32 * wp + r) * kXStride + 8 * kg;
    Operand xo[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) xo[q].q = *reinterpret_cast<const u32x4 *>(xrow + 16 * q);

    if constexpr (!kStatesOnly) {
      // ---- state -> output: Y^T[p][l] = sum_n H[p][n] C[l][n] ----
      f32x16 Y = {};
      const uint16_t *crow = sC + l * kCStride + 8 * kg;
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        Operand c;
        c.q = *reinterpret_cast<const u32x4 *>(crow + 16 * (4 * wn + k));
        Y = mfma(own[k], c, Y);
      }
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        Operand c;
        c.q = *reinterpret_cast<const u32x4 *>(crow + 16 * (4 * (wn ^ 1) + k));
        Y = mfma(partner[k], c, Y);
      }
      // ---- intra-block: Y^T[p][l] += sum_{s<=l} Xc[s][p] G[l][s], half by half ----
      Y = mfma(xo[0], Gop[0], Y);
      Y = mfma(xo[1], Gop[1], Y);
      float rowf = sCs[l];
      if (wn == 1) {
#pragma unroll
        for (int i = 0; i < 16; ++i) Y[i] *= d0;
        Y = mfma(xo[2], Gop[2], Y);
        Y = mfma(xo[3], Gop[3], Y);
        rowf -= c31;
      }
      rowf = fast_exp2(rowf);
      // ---- epilogue: y[l][p] = rowf * Y + D x, four consecutive p per 8-byte store ----
      if (t < p.T) {
        const float Dh = p.D[h];
#pragma unroll
        for (int i4 = 0; i4 < 4; ++i4) {
          const u32x2 xv = xepi[i4];
          u32x2 o;
          o.x = pack2(rowf * Y[4 * i4 + 0] + Dh * bf_lo(xv.x), rowf * Y[4 * i4 + 1] + Dh * bf_hi(xv.x));
          o.y = pack2(rowf * Y[4 * i4 + 2] + Dh * bf_lo(xv.y), rowf * Y[4 * i4 + 3] + Dh * bf_hi(xv.y));
          *reinterpret_cast<u32x2 *>(p.y + yrow + 8 * i4) = o;
        }
      }
    }

    // ---- state update: H^T = d1 (d0 (H^T + Bt Xc[0:32]) + Bt Xc[32:64]) ----
    {
      const uint16_t *btrow = sBt + (64 * wn + r) * kBtStride + 8 * kg;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        if (q == 2) {
#pragma unroll
          for (int tt = 0; tt < 2; ++tt)
#pragma unroll
            for (int i = 0; i < 16; ++i) Hacc[tt][i] *= d0;
        }
        Operand b0, b1;
        b0.q = *reinterpret_cast<const u32x4 *>(btrow + 16 * q);
        b1.q = *reinterpret_cast<const u32x4 *>(btrow + 32 * kBtStride + 16 * q);
        Hacc[0] = mfma(b0, xo[q], Hacc[0]);
        Hacc[1] = mfma(b1, xo[q], Hacc[1]);
      }
#pragma unroll
      for (int tt = 0; tt < 2; ++tt)
#pragma unroll
        for (int i = 0; i < 16; ++i) Hacc[tt][i] *= d1;
    }
    if (!kStatesOnly) pack_state();
    __syncthreads();  // ---- everyone is done reading this block's tiles and the published state ----
    if (!kStatesOnly) publish_state();
    if (more) {
      store_block();
      if constexpr (!kStatesOnly) {
#pragma unroll
        for (int q = 0; q < 4; ++q) Gop[q].q = r_g[q];
      }
    }
    __syncthreads();  // ---- next block's tiles and the published state are visible ----
  }

  // ---- write the state out (canonical (p, n) layout, four consecutive n per 16-byte store) ----
  float *out = nullptr;
  if (kStatesOnly) {
    out = p.seg_state + (bh * p.S + sg + 1) * kP * kN;
    if (tid == 0) p.seg_decay[bh * p.S + sg] = seg_total;
  } else if (sg == p.S - 1) {
    out = p.final_state + bh * kP * kN;
  }
  if (out != nullptr) {
    float *op = out + static_cast<size_t>(32 * wp + r) * kN;
#pragma unroll
    for (int tt = 0; tt < 2; ++tt)
#pragma unroll
      for (int i4 = 0; i4 < 4; ++i4)
        *reinterpret_cast<f32x4 *>(op + 64 * wn + 32 * tt + i4 * 8 + 4 * kg) =
            f32x4{Hacc[tt][4 * i4 + 0], Hacc[tt][4 * i4 + 1], Hacc[tt][4 * i4 + 2], Hacc[tt][4 * i4 + 3]};
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
  size_t off_G, off_Bt, off_prep, off_state, off_decay, total;
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
  w.off_prep = off;
  off += round_up(BH * w.NB * kRec * sizeof(float), 256);
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
  float *prep = reinterpret_cast<float *>(ws + w.off_prep);
  float *seg_state = reinterpret_cast<float *>(ws + w.off_state);
  float *seg_decay = reinterpret_cast<float *>(ws + w.off_decay);
  const int seg_blocks = choose_seg_blocks(d);
  const int S = (w.NB + seg_blocks - 1) / seg_blocks;

  hipLaunchKernelGGL(scores_bt_kernel, dim3(w.NB, d.Bt * d.G), dim3(kThreads), 0, stream,
                     static_cast<const uint16_t *>(B), static_cast<const uint16_t *>(C), Gd, Btr, d.T, d.G,
                     w.NB);
  trace_mark(trace, stream, "scores_bt");
  hipLaunchKernelGGL(block_cumsum_kernel, dim3(w.NB, (d.H + kCumHeads - 1) / kCumHeads, d.Bt), dim3(kThreads),
                     0, stream, dt, A, prep, d.T, d.H, w.NB);
  trace_mark(trace, stream, "block_cumsum");

  ScanParams p;
  p.x = static_cast<const uint16_t *>(x);
  p.C = static_cast<const uint16_t *>(C);
  p.D = D;
  p.Gd = Gd;
  p.Btr = Btr;
  p.prep = prep;
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
