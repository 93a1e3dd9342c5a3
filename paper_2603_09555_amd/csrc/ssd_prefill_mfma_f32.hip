// MFMA prefill for fp32 io (x, B, C, y in fp32): the chunked SSD algorithm (Alg. 1; Eq. 3) with every
// contraction on v_mfma_f32_32x32x2_f32 -- fp32 operands, fp32 accumulation, so the results sit at fp32
// rounding level (the 1e-4 tolerance of fp32 inputs is out of reach of bf16 operands).
// Shapes: headdim a multiple of 32, dstate a multiple of 8 up to 128.
//
// One kernel, one launch, no workspace.  A workgroup of four waves owns (batch row, head, 32 columns of
// headdim) and walks the sequence in 64-token blocks with its 32 x dstate slice of the state carried in
// MFMA accumulators: the inter-chunk state pass (Alg. 1, "Inter-chunk scan") happens in registers and
// the result does not depend on the chunk argument.
// When that leaves most of the chip idle, the sequence is also cut into time segments, one workgroup
// each: a workgroup walks from the first block of the sequence, but up to its own segment it only updates
// the state (no scores, no output, the update shared by all four waves: a fraction of a block's time), then
// computes the outputs of its segment.  The states are recomputed rather than handed over, so there is still one launch, no workspace
// and no waiting on another workgroup; the last segment's workgroup writes the final state.
// Per block, with cs_l the block-relative inclusive prefix sum of dt*A and S the state entering the block:
//   scores      G[l][s] = C_l . B_s for s <= l                     three 32 x 32 tiles, K = dstate   (waves 0-2)
//   mask        GM[l][s] = G[l][s] * dt_s * exp(cs_l - cs_s)      in registers, on the accumulators; the
//               exponent is never positive, so any step size is exact; to LDS as the next operand
//   output      y[l][p] = sum_s GM[l][s] x[s][p] + exp(cs_l) sum_n C[l][n] S[p][n] + D x[l][p]       (waves 0, 1)
//   state       S'[p][n] = exp(cs_63) S[p][n] + sum_s dt_s exp(cs_63 - cs_s) x[s][p] B[s][n]         (waves 2, 3)
// The tiles of a block (C and B row-major, B and x transposed too: every MFMA operand needs its k index
// contiguous per lane) live in LDS, rows padded by 16 bytes so that the 16-byte operand reads of
// consecutive rows fall into different banks; the global loads of the next block are issued into
// registers before the current block is computed.
//
// v_mfma_f32_32x32x2_f32: D(32x32) += A(32x2) B(2x32); lane (r = lane % 32, k = lane / 32) supplies A[r][k]
// and B[k][r] and receives D[(e/4)*8 + 4k + e%4][r] in element e.  A group of four consecutive steps reads
// one 16-byte piece per operand: lane (r, k) takes contraction indices 8m + 4k .. 8m + 4k + 3 of group m --
// a permutation of the contraction index that both operands share.
#include "ssd_internal.hpp"

namespace ssd {
namespace {

constexpr int kTok = 64;        // tokens per block
constexpr int kCols = 32;       // headdim columns per workgroup
constexpr int kF32Threads = 256;
constexpr int kPad = 4;         // floats of padding per LDS row
constexpr float kLog2e = 1.4426950408889634f;

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ f32x16 mfma2(float a, float b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c, 0, 0, 0);
}
__device__ __forceinline__ f32x16 mfma_group(const f32x4 a, const f32x4 b, f32x16 c) {
  c = mfma2(a.x, b.x, c);
  c = mfma2(a.y, b.y, c);
  c = mfma2(a.z, b.z, c);
  return mfma2(a.w, b.w, c);
}
__device__ __forceinline__ float exp2_fast(float v) { return __builtin_amdgcn_exp2f(v); }

template <int kCtrl, int kRowMask>
__device__ __forceinline__ float dpp_or_zero(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), kCtrl, kRowMask, 0xF, false));
}
// Inclusive prefix sum over the 64 lanes of a wave (data-parallel-primitive moves: shifts inside rows of
// 16 lanes, then the last lane of row 0 / 2 into row 1 / 3 and the last lane of row 1 into rows 2 and 3).
__device__ __forceinline__ float wave_prefix_sum(float v) {
  v += dpp_or_zero<0x111, 0xF>(v);  // row_shr:1
  v += dpp_or_zero<0x112, 0xF>(v);  // row_shr:2
  v += dpp_or_zero<0x114, 0xF>(v);  // row_shr:4
  v += dpp_or_zero<0x118, 0xF>(v);  // row_shr:8
  v += dpp_or_zero<0x142, 0xA>(v);  // row_bcast:15 -> rows 1 and 3
  v += dpp_or_zero<0x143, 0xC>(v);  // row_bcast:31 -> rows 2 and 3
  return v;
}

// Buffer addressing: a (base, size) descriptor in scalar registers plus a 32-bit byte offset per lane, which
// the hardware checks against the size -- loads beyond it return zero, stores beyond it are dropped.  Rows
// beyond the sequence and columns beyond dstate are masked that way, with no branch around a memory
// operation: the compiler can then leave the loads of the next block in flight across the whole loop body
// (with a branch in the way it waits for them at the next join).
using Rsrc = __amdgpu_buffer_rsrc_t;
__device__ __forceinline__ Rsrc make_rsrc(const void *base, uint32_t bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(base), 0, static_cast<int>(bytes), 0x00020000);
}
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ f32x4 buf_load4(Rsrc rs, uint32_t voff) {
  return __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(rs, voff, 0, 0));
}
__device__ __forceinline__ float buf_load1(Rsrc rs, uint32_t voff) {
  return __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rs, voff, 0, 0));
}
__device__ __forceinline__ void buf_store1(Rsrc rs, uint32_t voff, float v) {
  __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(uint32_t, v), rs, voff, 0, 0);
}
constexpr uint32_t kNowhere = 0xFFFFFF00u;  // an offset beyond any descriptor

struct F32Params {
  const float *x, *dt, *A, *B, *C, *D, *h0;
  float *y, *final_state;
  int T, H, P, N, G, hpg;
  int tseg;  // time segments per sequence (>= 1), each a workgroup of its own
  DtXform dtx;
};

// NT: 32-column tiles of the state (dstate <= 32 NT; columns beyond dstate are zero padding).
template <int NT>
__global__ __launch_bounds__(kF32Threads) void prefill_f32_kernel(const F32Params p) {
  constexpr int N32 = 32 * NT;
  constexpr int kRowN = N32 + kPad;   // row stride of the tiles indexed [token][n] and of the state [col][n]
  constexpr int kRowT = kTok + kPad;  // row stride of the tiles indexed [..][token]
  constexpr int kVecN = kTok * (N32 / 4) / kF32Threads;  // 16-byte pieces of a C (or B) tile per thread
  static_assert(kVecN * kF32Threads == kTok * (N32 / 4), "the threads share a tile evenly");
  __shared__ __align__(16) float sC[kTok * kRowN];    // C [l][n]
  __shared__ __align__(16) float sB[kTok * kRowN];    // B [s][n]
  __shared__ __align__(16) float sBT[N32 * kRowT];    // B^T [n][s]
  __shared__ __align__(16) float sXT[kCols * kRowT];  // x^T [col][s]
  __shared__ __align__(16) float sGM[kTok * kRowT];   // masked scores [l][s]
  __shared__ __align__(16) float sS[kCols * kRowN];   // state entering the block [col][n]
  __shared__ __align__(16) float sCs[kTok], sDt[kTok], sW[kTok], sEl[kTok];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int r = lane & 31, kk = lane >> 5;
  const int slices = p.P / kCols;
  const int seg = blockIdx.x % p.tseg, owner = blockIdx.x / p.tseg;
  const int ps = owner % slices;
  const int h = (owner / slices) % p.H;
  const int b = owner / (slices * p.H);
  const int g = h / p.hpg;
  const int nblocks = (p.T + kTok - 1) / kTok;
  // this workgroup's blocks: the state alone up to out0, everything from out0 to walk_end
  const int seg_len = (nblocks + p.tseg - 1) / p.tseg;
  const int out0 = min(nblocks, seg * seg_len), walk_end = min(nblocks, out0 + seg_len);
  const bool last_seg = walk_end == nblocks && (out0 < walk_end || seg == 0);  // writes the final state
  if (out0 >= walk_end && !last_seg) return;  // more segments than blocks (uniform over the workgroup)
  const size_t tok0 = static_cast<size_t>(b) * p.T;
  const float alog = p.A[h] * kLog2e;
  const float Dh = p.D[h];
  const float dbias = p.dtx.bias != nullptr ? p.dtx.bias[h] : 0.f;
  const uint32_t xrow = static_cast<uint32_t>(p.H) * p.P * 4;  // bytes per token of x / y
  const uint32_t brow = static_cast<uint32_t>(p.G) * p.N * 4;  // bytes per token of B / C
  const uint32_t drow = static_cast<uint32_t>(p.H) * 4;        // bytes per token of dt
  const uint32_t xoff = (static_cast<uint32_t>(h) * p.P + kCols * ps) * 4, boff = static_cast<uint32_t>(g) * p.N * 4;
  const uint8_t *const xb = reinterpret_cast<const uint8_t *>(p.x) + tok0 * xrow + xoff;
  uint8_t *const yb = reinterpret_cast<uint8_t *>(p.y) + tok0 * xrow + xoff;
  const uint8_t *const Bb = reinterpret_cast<const uint8_t *>(p.B) + tok0 * brow + boff;
  const uint8_t *const Cb = reinterpret_cast<const uint8_t *>(p.C) + tok0 * brow + boff;
  const uint8_t *const dtb = reinterpret_cast<const uint8_t *>(p.dt) + tok0 * drow + static_cast<uint32_t>(h) * 4;
  // descriptors start at the block and end with the batch row's last token
  const uint32_t T = static_cast<uint32_t>(p.T);
  auto rsrc_at = [&](const uint8_t *base, uint32_t row_bytes, uint32_t lead, int jb) {
    const uint32_t t0 = static_cast<uint32_t>(jb) * kTok;
    return make_rsrc(base + static_cast<size_t>(t0) * row_bytes, (T - t0) * row_bytes - lead);
  };

  // ---- registers holding the next block's global data ----
  f32x4 r_c[kVecN], r_b[kVecN], r_x[2];
  float r_dt = 0.f;
  // thread -> (token row, 16-byte piece) of the C / B tiles and of the x tile, tid-major
  // (B is also written transposed, n-major: there the 16 lanes of a quarter wave take 16 consecutive token
  // rows of one piece, so that their scalar writes fall into 16 consecutive banks -- with the row-major
  // assignment of C they would share four)
  auto b_piece = [&](int k, int &row, int &n0) {
    const int c = tid + kF32Threads * k;
    row = 16 * ((c >> 4) / (N32 / 4)) + (c & 15);
    n0 = 4 * ((c >> 4) % (N32 / 4));
  };
  uint32_t v_bc[kVecN], v_b[kVecN], v_x[2];
#pragma unroll
  for (int k = 0; k < kVecN; ++k) {
    const int c = tid + kF32Threads * k;
    const int row = c / (N32 / 4), n0 = 4 * (c % (N32 / 4));
    v_bc[k] = n0 < p.N ? static_cast<uint32_t>(row) * brow + 4 * n0 : kNowhere;  // dstate is a multiple of 8
    int rb, nb;
    b_piece(k, rb, nb);
    v_b[k] = nb < p.N ? static_cast<uint32_t>(rb) * brow + 4 * nb : kNowhere;
  }
#pragma unroll
  for (int k = 0; k < 2; ++k) {
    const int c = tid + kF32Threads * k;
    v_x[k] = static_cast<uint32_t>(c >> 3) * xrow + 16 * (c & 7);
  }
  const uint32_t v_dt = static_cast<uint32_t>(lane) * drow;  // every wave fetches the block's 64 step sizes; wave 0 uses them
  // (with_c, uniform: a block of which only the state is wanted needs no C -- its loads are pointed beyond the
  // descriptor, where they cost nothing, rather than put behind a branch)
  auto load_block = [&](int jb, bool with_c = true) __attribute__((always_inline)) {
    const Rsrc rc = rsrc_at(Cb, brow, boff, jb), rb = rsrc_at(Bb, brow, boff, jb);
#pragma unroll
    for (int k = 0; k < kVecN; ++k) {
      r_c[k] = buf_load4(rc, with_c ? v_bc[k] : kNowhere);
      r_b[k] = buf_load4(rb, v_b[k]);
    }
    const Rsrc rx = rsrc_at(xb, xrow, xoff, jb);
#pragma unroll
    for (int k = 0; k < 2; ++k) r_x[k] = buf_load4(rx, v_x[k]);
    r_dt = buf_load1(rsrc_at(dtb, drow, static_cast<uint32_t>(h) * 4, jb), v_dt);
  };
  // registers -> LDS tiles; wave 0 also turns dt into the block's decay bookkeeping
  // (full, uniform: the row-major C and B tiles serve the scores only)
  auto stage_block = [&](int jb_staged, bool full = true) __attribute__((always_inline)) {
#pragma unroll
    for (int k = 0; k < kVecN; ++k) {
      const int c = tid + kF32Threads * k;
      const int row = c / (N32 / 4), n0 = 4 * (c % (N32 / 4));
      int rb, nb;
      b_piece(k, rb, nb);
      if (full) {
        *reinterpret_cast<f32x4 *>(&sC[row * kRowN + n0]) = r_c[k];
        *reinterpret_cast<f32x4 *>(&sB[rb * kRowN + nb]) = r_b[k];
      }
#pragma unroll
      for (int j = 0; j < 4; ++j) sBT[(nb + j) * kRowT + rb] = r_b[k][j];
    }
#pragma unroll
    for (int k = 0; k < 2; ++k) {
      const int c = tid + kF32Threads * k;
      const int row = c >> 3, c0 = 4 * (c & 7);
#pragma unroll
      for (int j = 0; j < 4; ++j) sXT[(c0 + j) * kRowT + row] = r_x[k][j];
    }
    if (wave == 0) {  // lane = token; tokens beyond the sequence have step size zero (state-neutral)
      const float dtv = static_cast<uint32_t>(jb_staged * kTok + lane) < T ? dt_apply_branchless(r_dt, dbias, p.dtx) : 0.f;
      const float cs = wave_prefix_sum(dtv * alog);
      const float c63 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, cs), 63));
      sCs[lane] = cs;
      sDt[lane] = dtv;
      sW[lane] = dtv * exp2_fast(c63 - cs);  // input weight relative to the end of the block
      sEl[lane] = exp2_fast(cs);             // decay from the start of the block to token l
    }
  };
  auto ld4 = [](const float *ptr) { return *reinterpret_cast<const f32x4 *>(ptr); };

  // ---- the state: waves 2 and 3 carry it in accumulators, tile nt = wave - 2 (+ 2); D[i = col][j = n] ----
  constexpr int kTilesPerWave = (NT + 1) / 2;
  f32x16 Sacc[kTilesPerWave];
#pragma unroll
  for (int k = 0; k < kTilesPerWave; ++k)
#pragma unroll
    for (int e = 0; e < 16; ++e) Sacc[k][e] = 0.f;
  auto state_tile = [&](int k) { return (wave - 2) + 2 * k; };  // meaningful for waves 2, 3
  if (wave >= 2) {
#pragma unroll
    for (int k = 0; k < kTilesPerWave; ++k) {
      const int n = 32 * state_tile(k) + r;
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int col = (e >> 2) * 8 + 4 * kk + (e & 3);
        const bool live = p.h0 != nullptr && state_tile(k) < NT && n < p.N;
        Sacc[k][e] = live ? p.h0[((static_cast<size_t>(b) * p.H + h) * p.P + kCols * ps + col) * p.N + n] : 0.f;
      }
    }
  }
  auto put_state = [&]() __attribute__((always_inline)) {  // accumulators -> sS (waves 2, 3)
#pragma unroll
    for (int k = 0; k < kTilesPerWave; ++k)
      if (state_tile(k) < NT) {
#pragma unroll
        for (int e = 0; e < 16; ++e) sS[((e >> 2) * 8 + 4 * kk + (e & 3)) * kRowN + 32 * state_tile(k) + r] = Sacc[k][e];
      }
  };

  if (walk_end > 0) load_block(0, out0 == 0);
  if (out0 > 0) {
    // ---- the blocks before the segment: the state alone.  All four waves share the update -- wave w takes
    //      tokens 16 w .. 16 w + 15 of every block, for every state tile -- in accumulators of their own, which
    //      are summed once, at the end (the update is linear in the state); the initial state rides in the
    //      accumulators of the wave that owns the tile afterwards. ----
    f32x16 Spart[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
      const bool mine = wave == 2 + (nt & 1);
#pragma unroll
      for (int e = 0; e < 16; ++e) Spart[nt][e] = mine ? Sacc[nt >> 1][e] : 0.f;
    }
    for (int jb = 0; jb < out0; ++jb) {
      __syncthreads();  // the previous block's readers are done with every tile
      stage_block(jb, false);
      load_block(jb + 1, jb + 1 == out0);  // (out0 < walk_end: block jb + 1 exists)
      __syncthreads();
      const float e63 = sEl[kTok - 1];
      const float *ap = &sXT[r * kRowT + 4 * kk];
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) {
#pragma unroll
        for (int e = 0; e < 16; ++e) Spart[nt][e] *= e63;
      }
#pragma unroll
      for (int mm = 0; mm < 2; ++mm) {
        const int m = 2 * wave + mm;
        f32x4 a = ld4(ap + 8 * m);
        const f32x4 w = ld4(&sW[8 * m + 4 * kk]);
        a = f32x4{a.x * w.x, a.y * w.y, a.z * w.z, a.w * w.w};
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) Spart[nt] = mfma_group(a, ld4(&sBT[(32 * nt + r) * kRowT + 4 * kk + 8 * m]), Spart[nt]);
      }
    }
    // the sum, tile by tile, through what will be the masked-score tile: three waves put, the owner adds
    static_assert(3 * 1024 <= kTok * kRowT, "three partial tiles fit in the masked-score tile");
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
      const int owner_wave = 2 + (nt & 1);
      __syncthreads();
      if (wave != owner_wave) {
        float *dst = &sGM[(wave - (wave > owner_wave)) * 1024 + 4 * lane];
#pragma unroll
        for (int e4 = 0; e4 < 4; ++e4)
          *reinterpret_cast<f32x4 *>(dst + 256 * e4) = f32x4{Spart[nt][4 * e4], Spart[nt][4 * e4 + 1], Spart[nt][4 * e4 + 2], Spart[nt][4 * e4 + 3]};
      }
      __syncthreads();
      if (wave == owner_wave) {
#pragma unroll
        for (int e4 = 0; e4 < 4; ++e4) {
          f32x4 sum = f32x4{Spart[nt][4 * e4], Spart[nt][4 * e4 + 1], Spart[nt][4 * e4 + 2], Spart[nt][4 * e4 + 3]};
#pragma unroll
          for (int q = 0; q < 3; ++q) {
            const f32x4 v = ld4(&sGM[q * 1024 + 256 * e4 + 4 * lane]);
            sum = f32x4{sum.x + v.x, sum.y + v.y, sum.z + v.z, sum.w + v.w};
          }
          Sacc[nt >> 1][4 * e4] = sum.x;
          Sacc[nt >> 1][4 * e4 + 1] = sum.y;
          Sacc[nt >> 1][4 * e4 + 2] = sum.z;
          Sacc[nt >> 1][4 * e4 + 3] = sum.w;
        }
      }
    }
  }
  for (int jb = out0; jb < walk_end; ++jb) {
    __syncthreads();  // the previous block's readers are done with every tile
    stage_block(jb);
    if (wave >= 2) put_state();
    load_block(min(jb + 1, walk_end - 1));  // (after the last block: a harmless repeat, no branch)
    __syncthreads();

    // ---- scores and mask: wave w < 3 owns tile (lt, st) = (0,0), (1,0), (1,1) ----
    if (wave < 3) {
      const int lt = wave > 0, st = wave > 1;
      // (two accumulators, summed at the end: consecutive matrix instructions then do not wait for each other)
      f32x16 acc, acc2;
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[e] = acc2[e] = 0.f;
      const float *ap = &sC[(32 * lt + r) * kRowN + 4 * kk], *bp = &sB[(32 * st + r) * kRowN + 4 * kk];
#pragma unroll
      for (int m = 0; m < N32 / 8; m += 2) {
        acc = mfma_group(ld4(ap + 8 * m), ld4(bp + 8 * m), acc);
        acc2 = mfma_group(ld4(ap + 8 * m + 8), ld4(bp + 8 * m + 8), acc2);
      }
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[e] += acc2[e];
      // element e: l = 32 lt + (e/4)*8 + 4kk + e%4, s = 32 st + r
      const int s = 32 * st + r;
      const float cs_s = sCs[s], dt_s = sDt[s];
#pragma unroll
      for (int e4 = 0; e4 < 4; ++e4) {
        const int l0 = 32 * lt + 8 * e4 + 4 * kk;
        const f32x4 cs_l = ld4(&sCs[l0]);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const int l = l0 + j;
          const float m = dt_s * exp2_fast(fminf(cs_l[j] - cs_s, 0.f));
          sGM[l * kRowT + s] = s <= l ? acc[4 * e4 + j] * m : 0.f;
        }
      }
    }
    __syncthreads();

    if (wave < 2) {
      // ---- output rows 32 wave .. 32 wave + 31: Y[i = l][j = col] ----
      const int lt = wave;
      f32x16 acc, acc2;  // the state -> output term and the intra-block term, summed at the end
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[e] = acc2[e] = 0.f;
      {
        const float el = sEl[32 * lt + r];
        const float *ap = &sC[(32 * lt + r) * kRowN + 4 * kk], *bp = &sS[r * kRowN + 4 * kk];     // (exp(cs_l) C[l][n]) S[col][n]
        const float *gp = &sGM[(32 * lt + r) * kRowT + 4 * kk], *xp = &sXT[r * kRowT + 4 * kk];  // GM[l][s] x[s][col], s <= l
        // the first row tile needs the first 32 tokens only; the two products are interleaved
        constexpr int kOff = N32 / 8;
#pragma unroll
        for (int m = 0; m < (kOff > 8 ? kOff : 8); ++m) {
          if (m < kOff) {
            f32x4 a = ld4(ap + 8 * m);
            a = f32x4{a.x * el, a.y * el, a.z * el, a.w * el};
            acc = mfma_group(a, ld4(bp + 8 * m), acc);
          }
          if (m < 8 && (lt == 1 || m < 4)) acc2 = mfma_group(ld4(gp + 8 * m), ld4(xp + 8 * m), acc2);
        }
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[e] += acc2[e];
      }
      // epilogue: + D x, store (lane r = column, elements = 16 rows; rows beyond the sequence are dropped)
      const Rsrc ry = rsrc_at(yb, xrow, xoff, jb);
#pragma unroll
      for (int e4 = 0; e4 < 4; ++e4) {
        const int l0 = 32 * lt + 8 * e4 + 4 * kk;
        const f32x4 xv = ld4(&sXT[r * kRowT + l0]);
#pragma unroll
        for (int j = 0; j < 4; ++j)
          buf_store1(ry, static_cast<uint32_t>(l0 + j) * xrow + 4 * r, acc[4 * e4 + j] + Dh * xv[j]);
      }
    } else {
      // ---- state update: S'[i = col][j = n] = exp(c63) S + sum_s (w_s x[s][col]) B[s][n] ----
      const float e63 = sEl[kTok - 1];
#pragma unroll
      for (int k = 0; k < kTilesPerWave; ++k)
        if (state_tile(k) < NT) {
#pragma unroll
          for (int e = 0; e < 16; ++e) Sacc[k][e] *= e63;
          f32x16 acc2;
#pragma unroll
          for (int e = 0; e < 16; ++e) acc2[e] = 0.f;
          const float *ap = &sXT[r * kRowT + 4 * kk], *bp = &sBT[(32 * state_tile(k) + r) * kRowT + 4 * kk];
#pragma unroll
          for (int m = 0; m < kTok / 8; ++m) {
            f32x4 a = ld4(ap + 8 * m);
            const f32x4 w = ld4(&sW[8 * m + 4 * kk]);
            a = f32x4{a.x * w.x, a.y * w.y, a.z * w.z, a.w * w.w};
            if (m & 1)
              acc2 = mfma_group(a, ld4(bp + 8 * m), acc2);
            else
              Sacc[k] = mfma_group(a, ld4(bp + 8 * m), Sacc[k]);
          }
#pragma unroll
          for (int e = 0; e < 16; ++e) Sacc[k][e] += acc2[e];
        }
    }
  }

  // ---- final state (Alg. 1, "Store") ----
  if (wave >= 2 && last_seg) {
#pragma unroll
    for (int k = 0; k < kTilesPerWave; ++k) {
      const int n = 32 * state_tile(k) + r;
      if (state_tile(k) < NT && n < p.N) {
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const int col = (e >> 2) * 8 + 4 * kk + (e & 3);
          p.final_state[((static_cast<size_t>(b) * p.H + h) * p.P + kCols * ps + col) * p.N + n] = Sacc[k][e];
        }
      }
    }
  }
}

}  // namespace

// Time per block of a workgroup (microseconds on MI355X; fits to a handful of timings): a full block, and a
// block of which only the state update runs.  nt = 32-column tiles of the state.
double f32_block_us(int nt) { return 1.7 + 1.39 * nt; }
double f32_state_block_us(int nt) { return 0.29 + 0.47 * nt; }
// Time segments per sequence, and the modelled time of the walk that results.  More segments shorten the
// stretch of full blocks of the longest walk -- the last segment's, which first carries the state over
// everything before it -- as long as the workgroups still run side by side (one round of 256).
int f32_time_segments(const Dims &d, double *walk_us) {
  const unsigned long long wgs = static_cast<unsigned long long>(d.Bt) * d.H * (d.P / kCols);
  const int nblocks = (d.T + kTok - 1) / kTok, nt = (d.N + 31) / 32;
  const double rounds = static_cast<double>((wgs + 255) / 256);
  int best = 1;
  double best_us = rounds * nblocks * f32_block_us(nt);
  const int forced = knobs().f32_segments;
  for (int s = 2; s <= nblocks && s <= 64 && (forced > 0 || wgs * s <= 256); ++s) {
    const int len = (nblocks + s - 1) / s;
    const double us = static_cast<double>((wgs * s + 255) / 256) * ((nblocks - len) * f32_state_block_us(nt) + len * f32_block_us(nt));
    if (forced > 0 ? s <= forced : us < best_us) {
      best = s;
      best_us = us;
    }
  }
  if (walk_us != nullptr) *walk_us = best_us;
  return best;
}

// Shapes the kernel takes, and among them those it is expected to win on.  It walks a sequence block by block
// with one workgroup per (batch row, head, 32 columns, time segment), so its time is (rounds of 256
// workgroups) x (the longest walk, see above); the generic fp32 kernels are chunk-parallel
// over the whole chip, cost four launches and then time proportional to the work.  A long sequence with few
// heads is theirs.  Both estimates are fits to a handful of timings on MI355X (microseconds); where they are
// within a tenth of each other the MFMA kernel is taken.
bool mfma_f32_supported(const Dims &d, bool whenever_eligible) {
  const unsigned long long wgs = static_cast<unsigned long long>(d.Bt) * d.H * (d.P / kCols);
  // one batch row of x and of B / C must be addressable with 32-bit byte offsets
  const unsigned long long lim = 0xFFFF0000ull, t = static_cast<unsigned long long>(d.T);
  if (d.bf16 || d.P % kCols != 0 || d.N % 8 != 0 || d.N > 128 || wgs > 0x7fffffffull / 64 || t * d.H * d.P * 4 > lim ||
      t * d.G * d.N * 4 > lim)
    return false;
  if (whenever_eligible) return true;
  double walk_us;
  f32_time_segments(d, &walk_us);
  const double mfma_us = 8.0 + walk_us;
  const double token_heads = static_cast<double>(d.Bt) * d.T * d.H;
  const double generic_us = 33.0 + token_heads * (0.9 + 0.0005 * d.P * d.N) * 1e-3;
  return mfma_us <= 1.1 * generic_us;
}

int mfma_f32_time_segments(const Dims &d) { return f32_time_segments(d, nullptr); }

hipError_t launch_prefill_mfma_f32(const Dims &d, const void *x, const float *dt, const float *A, const void *B,
                                   const void *C, const float *D, const float *h0, void *y, float *final_state,
                                   hipStream_t stream, KernelTrace *trace) {
  F32Params p;
  p.x = static_cast<const float *>(x);
  p.dt = dt;
  p.A = A;
  p.B = static_cast<const float *>(B);
  p.C = static_cast<const float *>(C);
  p.D = D;
  p.h0 = h0;
  p.y = static_cast<float *>(y);
  p.final_state = final_state;
  p.T = d.T;
  p.H = d.H;
  p.P = d.P;
  p.N = d.N;
  p.G = d.G;
  p.hpg = d.hpg;
  p.dtx = d.dtx;
  p.tseg = f32_time_segments(d, nullptr);
  const dim3 grid(static_cast<unsigned>(d.Bt) * d.H * (d.P / kCols) * p.tseg), block(kF32Threads);
  const int nt = (d.N + 31) / 32;
  switch (nt) {
    case 1: hipLaunchKernelGGL(prefill_f32_kernel<1>, grid, block, 0, stream, p); break;
    case 2: hipLaunchKernelGGL(prefill_f32_kernel<2>, grid, block, 0, stream, p); break;
    case 3: hipLaunchKernelGGL(prefill_f32_kernel<3>, grid, block, 0, stream, p); break;
    default: hipLaunchKernelGGL(prefill_f32_kernel<4>, grid, block, 0, stream, p); break;
  }
  trace_mark(trace, stream, "prefill_f32");
  return hipGetLastError();
}

}  // namespace ssd
