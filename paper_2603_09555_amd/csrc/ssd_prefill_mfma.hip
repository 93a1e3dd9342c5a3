// MFMA prefill for the Mamba-2 head shape (headdim 64 or a multiple of it, dstate 128 -- other state
// sizes are mapped onto it, see "state slices" at the launcher -- bf16 io; any chunk length, any number of
// heads per group).  A head with headdim 64 k is
// processed as k independent heads of 64 columns ("head" below means such a 64-column slice): its
// columns never interact, x, y and the state are laid out exactly as those of k narrower heads, and
// the slices share the head's decay records, A and D.
//
// The chunked algorithm (Alg. 1; Eq. 3) is evaluated on 64-token blocks.  Below the diagonal
// blocks the decay mask of Eq. 3 has rank one per block pair, so the off-diagonal part of the
// masked product equals "C_l . (state entering the block)": a wave walks the blocks of its
// head in order with the fp32 state H (headdim x dstate) resident in MFMA accumulators -- the
// inter-chunk state pass happens in registers with no per-chunk launch -- and only the
// diagonal 64x64 blocks need the mask.  Inside a diagonal block the mask is factorised around
// the middle of the block (c31 = prefix sum at token 31):
//     exp(cs_l - cs_s) = exp(cs_l - c31) * exp(c31 - cs_s)
// The second factor is folded into the input once per token (Xm = dt_s exp(c31 - cs_s) x_s),
// the first one scales output rows, and what remains of the mask -- the causal zero pattern --
// is head independent and baked into G = tril(C B^T), computed once per group.  So the mask is
// never materialised, costs no per-element work per head, and every exponent that is evaluated
// is bounded by the decay of 32 tokens; blocks where that leaves the fp32 range ("steep" blocks, far beyond
// the benchmark's dt*|A| <= 1.6 per token) keep the mask un-factorised, see block_cumsum_block.
// With Ht = exp(c31) * (state entering the block), per block and head:
//     Y^T  = Ht C^T + Xm^T G^T            (state -> output, K = dstate; intra-block, K <= 64)
//     y    = exp(cs_l - c31) o Y + D x     (epilogue)
//     H'   = Ht + B^T Xm                   (chunk-state accumulation, K = 64)
//     Ht_next = exp(c63 - c31) exp(c31_next) H'
// all on v_mfma_f32_32x32x16_bf16 with fp32 accumulation (76 MFMAs per block and head); decay
// arithmetic is fp32.
//
// Work decomposition: one WAVE per (head, half of headdim), four heads of one B/C group per
// workgroup of eight waves, one workgroup per CU (two waves per SIMD).  A wave owns a 128 x 32
// slice of the state and never exchanges data with another wave.  The C, B^T and G tiles are
// staged once per workgroup in double-buffered LDS and shared by the four heads; each wave
// stages its own slice of the scaled input.  Global loads for block j+2 are issued while block
// j+1 is being computed; two barriers per block (tiles of the next block visible; both halves of the
// output rows in LDS).
//
// Kernels (launch order):
//   block_prep     one launch for both preparation steps: per (batch, group, block) G = tril(C B^T)
//                  (diagonal blocks only, bf16) and a transposed copy of B, both shared by all heads of
//                  the group; per (batch, head, block) the prefix sums of dt*A turned into per-token
//                  input factors, per-row output factors and per-block state factors.
//   chunk_scan<true>  ("segment_states") per (batch, 4 heads, segment): the segment's end state from a
//                  zero start (only the chunk-state accumulation), so that segments can run in parallel.
//   segment_pass   sequential pass over segment end states -> state entering each segment.
//   chunk_scan<false> per (batch, 4 heads, segment): everything above, from the entering state.
// A segment is a whole number of 64-token blocks; with one segment only the first and the last kernel
// run, and with few segments segment_pass does not: the last kernel sums the few states itself.
#include <type_traits>

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

// ---- state slices ----------------------------------------------------------------------------------
// The kernels are written for 128 state columns.  A launch works on columns [off, off + valid) of a
// dstate axis of `width` columns (valid <= 128; columns beyond `valid` are zero padding): dstate 64 is
// one padded slice, dstate 256 is two slices, each an SSD of its own with the same x and dt, whose
// outputs add up (everything is linear in the triple B, C, state).
struct NSlice {
  int width, off, valid;
};

// ---- tables of a variable-length call -----------------------------------------------------------
// A packed batch (sequences back to back along the token axis, boundaries in a device array of
// cumulative lengths) is handled as a batch whose rows differ in length: every sequence gets whole
// 64-token blocks of its own (the ragged last block of each is masked by the buffer descriptors, as
// for a plain batch) and one or more segments.  Two tiny kernels turn the boundaries into tables:
//   tok0[q], len[q]      first token and length of sequence q
//   blk0[q], item0[q]    number of blocks / segments of the sequences before q (entry nseq: totals)
//   slot0[q]             number of state slots before q: a sequence of several segments has one slot
//                        per segment, a sequence of one segment needs none
//   blk_seq[i], item_seq[i]   sequence that block i / entry i of the segment list belongs to
// Blocks and segments are numbered over the whole batch; workspace arrays are indexed by those
// numbers (capacities nb_cap, slot_cap are upper bounds that the host can compute from the token
// count and the number of sequences alone).  Boundaries that are not non-decreasing within
// [0, total] give empty tables: every later kernel then finds nothing to do.

__global__ __launch_bounds__(256) void varlen_scan_kernel(const int32_t *__restrict__ cu, int nseq, int total,
                                                          int blk_len, int seg_blocks, int32_t *__restrict__ tok0,
                                                          int32_t *__restrict__ len, int32_t *__restrict__ blk0,
                                                          int32_t *__restrict__ item0, int32_t *__restrict__ slot0) {
  __shared__ int sblk[256], sitem[256], sslot[256];
  __shared__ int bad;
  const int tid = threadIdx.x;
  const int per = (nseq + 255) / 256;
  const int q0 = min(nseq, tid * per), q1 = min(nseq, q0 + per);
  if (tid == 0) bad = 0;
  __syncthreads();
  int nb = 0, ni = 0, ns = 0;
  bool mine_bad = false;
  for (int q = q0; q < q1; ++q) {
    const int a = cu[q], b = cu[q + 1];
    if (a < 0 || b < a || b > total) mine_bad = true;
    const int n = (b - a + blk_len - 1) / blk_len;
    const int segs = max(1, (n + seg_blocks - 1) / seg_blocks);
    nb += n;
    ni += segs;
    ns += segs > 1 ? segs : 0;
  }
  if (mine_bad) atomicOr(&bad, 1);
  sblk[tid] = nb;
  sitem[tid] = ni;
  sslot[tid] = ns;
  __syncthreads();
  if (tid == 0) {  // exclusive prefix over the 256 partial sums
    int a = 0, b = 0, c = 0;
    for (int i = 0; i < 256; ++i) {
      const int t = sblk[i], u = sitem[i], v = sslot[i];
      sblk[i] = a;
      sitem[i] = b;
      sslot[i] = c;
      a += t;
      b += u;
      c += v;
    }
    blk0[nseq] = bad ? 0 : a;
    item0[nseq] = bad ? 0 : b;
    slot0[nseq] = bad ? 0 : c;
  }
  __syncthreads();
  int rb = sblk[tid], ri = sitem[tid], rs = sslot[tid];
  for (int q = q0; q < q1; ++q) {
    const int a = cu[q], l = cu[q + 1] - a;
    const int n = (l + blk_len - 1) / blk_len;
    const int segs = max(1, (n + seg_blocks - 1) / seg_blocks);
    tok0[q] = bad ? 0 : a;
    len[q] = bad ? 0 : l;
    blk0[q] = bad ? 0 : rb;
    item0[q] = bad ? 0 : ri;
    slot0[q] = bad ? 0 : rs;
    rb += n;
    ri += segs;
    rs += segs > 1 ? segs : 0;
  }
}

// Largest q in [0, nseq) with first[q] <= i: the sequence that contains block (or segment) i.
__device__ __forceinline__ int owner_of(const int32_t *__restrict__ first, int nseq, int i) {
  int lo = 0, hi = nseq;
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (first[mid] <= i) lo = mid; else hi = mid;
  }
  return lo;
}
// Segments are listed with every sequence's non-last segments first (all of them are full length,
// seg_blocks blocks) and the last segment of every sequence after them (any length from empty to
// full), longest first while the batch has at most kSortMax sequences (rank by counting, quadratic
// but tiny): workgroups are dispatched in list order, so the long ones start first and the short
// ones fill the gaps; and the states-only pass, which needs no last segment, takes a prefix of the
// list.  Sequence q has item0[q] - q non-last segments before it.
constexpr int kSortMax = 2048;
__global__ __launch_bounds__(256) void varlen_fill_kernel(const int32_t *__restrict__ blk0,
                                                          const int32_t *__restrict__ item0, int nseq,
                                                          int seg_blocks, int32_t *__restrict__ blk_seq,
                                                          int32_t *__restrict__ item_seq) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i < blk0[nseq]) blk_seq[i] = owner_of(blk0, nseq, i);
  const int n_items = item0[nseq], n_full = n_items - nseq;
  if (i < n_full) {
    int lo = 0, hi = nseq;
    while (hi - lo > 1) {
      const int mid = (lo + hi) >> 1;
      if (item0[mid] - mid <= i) lo = mid; else hi = mid;
    }
    item_seq[i] = lo;
  }
  // (no early return above: the barrier below is reached by every thread)
  __shared__ int16_t last_blocks[kSortMax];  // blocks in the last segment of every sequence (<= seg_blocks)
  const bool sort = nseq <= kSortMax && seg_blocks < 32768;
  const bool ranks_here = static_cast<int>(blockIdx.x) * 256 < n_items && static_cast<int>(blockIdx.x) * 256 + 256 > n_full;
  if (sort && ranks_here)
    for (int k = threadIdx.x; k < nseq; k += 256)
      last_blocks[k] = static_cast<int16_t>((blk0[k + 1] - blk0[k]) - (item0[k + 1] - item0[k] - 1) * seg_blocks);
  __syncthreads();
  if (i >= n_full && i < n_items) {
    const int q = i - n_full;
    int rank = q;
    if (sort) {
      const int mine = last_blocks[q];
      rank = 0;
      for (int k = 0; k < nseq; ++k) {
        const int other = last_blocks[k];
        rank += (other > mine || (other == mine && k < q)) ? 1 : 0;
      }
    }
    item_seq[n_full + rank] = q;
  }
}

// Buffer addressing: a 128-bit descriptor (base, size) in scalar registers plus a 32-bit byte offset
// per lane.  The hardware checks the per-lane offset against the size: loads beyond it return zero
// and stores beyond it are dropped, which is how the ragged last block is handled (a descriptor
// that ends at the last token of the batch row) without clamps or branches.
using Rsrc = __amdgpu_buffer_rsrc_t;
__device__ __forceinline__ Rsrc make_rsrc(const void *base, uint32_t bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(base), 0, static_cast<int>(bytes), 0x00020000);
}
__device__ __forceinline__ u32x4 buf_load16(Rsrc r, uint32_t voff, uint32_t soff) {
  return __builtin_amdgcn_raw_buffer_load_b128(r, voff, soff, 0);
}
// kPolicy is the instruction's cache-policy field: 0 = default (write-back through L2 and the memory-side
// cache), kStreamStore = sc0 | nt, a non-temporal store that does not displace what those caches hold.
constexpr int kStreamStore = 3;
constexpr int kYPlain = 0, kYStream = 1, kYAdd = 2;
template <int kPolicy = 0>
__device__ __forceinline__ void buf_store16(Rsrc r, uint32_t voff, u32x4 v) {
  __builtin_amdgcn_raw_buffer_store_b128(v, r, voff, 0, kPolicy);
}

// A 64-bit value that is the same in every lane, moved to scalar registers.
__device__ __forceinline__ size_t uniform_size(size_t v) {
  const uint32_t lo = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(v));
  const uint32_t hi = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(v >> 32));
  return (static_cast<size_t>(hi) << 32) | lo;
}

// ---- scores_bt: G = tril(C B^T) on the diagonal blocks, and B transposed ------------------------------
// One workgroup per (block, group).  The block covers rows [row0, row0 + 64) of the (tokens, G, N)
// arrays B and C, of which only rows below row_end belong to its sequence; its results go to tile
// number `tile` of Gd (64 l x 64 s, bf16) and of Btr (128 n x 64 s, bf16).  ns: which columns of the
// dstate axis this launch works on (see NSlice); with a slice that is not the whole axis, the slice of C
// is also copied, zero padded to 128 columns, to Cpad (tokens, G, 128), from which the scan then reads it.
// Both tiles are read once, 16 consecutive bytes per thread and whole rows per 16 threads (a lane per
// row, which is what the MFMA operands want, would fetch every 128-byte line of the tiles four times,
// 32 bytes at a time: measured four times slower with many groups), and go through LDS -- B whole, C one
// half of the dstate axis (64 columns) at a time, from the registers that hold the whole tile: the
// workgroup's LDS is what limits how many of these short, latency-bound workgroups a CU holds (six this
// way; four with both tiles whole, which put the launch through two rounds at the benchmark shapes).
//   sB  kBlk rows of kN + 2 elements: the odd dword stride makes the transposed read-back conflict free
//   sC  kBlk rows of 64 + 8 elements, read as operands with 16-byte reads; once the products are done
//       it holds G on its way out (rows of kBlk + 8 elements), so that G too is stored in whole rows
constexpr int kHalfN = kN / 2;
constexpr int kSbStride = kN + 2, kScStride = kHalfN + 8;
constexpr int kGtStride = kBlk + 8;
constexpr int kSbElems = kBlk * kSbStride, kScElems = kBlk * kScStride;
static_assert(kBlk * kGtStride <= kScElems, "G fits where the half tile of C was");
__device__ __forceinline__ void scores_bt_block(uint16_t *sB, uint16_t *sC, size_t row0, size_t row_end, size_t tile,
                                                int g, const uint16_t *__restrict__ B, const uint16_t *__restrict__ C,
                                                uint16_t *__restrict__ Gd, uint16_t *__restrict__ Btr, int G,
                                                const NSlice ns, uint16_t *__restrict__ Cpad) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int ws = wave >> 1, wl = wave & 1;
  const int r = lane & 31, kg = lane >> 5;

  // The block's rows of the group's slice of B and of C, addressed as row * row_bytes + 2 * column.  The
  // descriptors end with the slice of the last row that belongs to the sequence, so later rows read as
  // zero; a column beyond the slice is given an offset no descriptor covers.  No load sits behind a
  // branch, so all of them are in flight together.
  const uint32_t row_bytes = static_cast<uint32_t>(G) * ns.width * 2;
  const uint32_t rows_here = row_end > row0 ? static_cast<uint32_t>(row_end - row0 < kBlk ? row_end - row0 : kBlk) : 0;
  // (readfirstlane: 64-bit comparisons are vector instructions, and a descriptor with a part in vector
  // registers is accessed through a loop over the lanes' values)
  const uint32_t span = __builtin_amdgcn_readfirstlane(rows_here ? (rows_here - 1) * row_bytes + static_cast<uint32_t>(ns.valid) * 2 : 0);
  const size_t first = (row0 * G + g) * ns.width + ns.off;
  const Rsrc rB = make_rsrc(B + first, span), rC = make_rsrc(C + first, span);
  constexpr uint32_t kNowhere = 0xFFFFFF00u;
  constexpr int kPieces = kBlk * (kN / 8) / kThreads;
  // thread -> 16-byte piece `ch` of the rows row_first + 16 i
  const int ch = threadIdx.x % (kN / 8), row_first = threadIdx.x / (kN / 8);
  static_assert(kThreads % (kN / 8) == 0, "a thread keeps its piece of the row over its rows");
  constexpr int kRowStep = kThreads / (kN / 8);
  u32x4 vb[kPieces], vc[kPieces];
#pragma unroll
  for (int i = 0; i < kPieces; ++i) {
    const int row = row_first + i * kRowStep;
    const uint32_t off = 8 * ch < ns.valid ? row * row_bytes + ch * 16 : kNowhere;  // columns beyond the slice: zero
    vb[i] = buf_load16(rB, off, 0);
    vc[i] = buf_load16(rC, off, 0);
  }
  if (Cpad != nullptr) {
#pragma unroll
    for (int i = 0; i < kPieces; ++i) {
      const int row = row_first + i * kRowStep;
      if (row0 + row < row_end) *reinterpret_cast<u32x4 *>(Cpad + ((row0 + row) * G + g) * kN + 8 * ch) = vc[i];
    }
  }
#pragma unroll
  for (int i = 0; i < kPieces; ++i) {
    uint32_t *dst = reinterpret_cast<uint32_t *>(sB + (row_first + i * kRowStep) * kSbStride + 8 * ch);
    dst[0] = vb[i].x;
    dst[1] = vb[i].y;
    dst[2] = vb[i].z;
    dst[3] = vb[i].w;
  }
  // G^T tile (rows s, columns l): lane ends up with four consecutive s for its l.
  f32x16 acc = {};
#pragma unroll
  for (int half = 0; half < 2; ++half) {
    if (half) __syncthreads();  // the first half's operands have been read
    if (ch / (kHalfN / 8) == half) {
#pragma unroll
      for (int i = 0; i < kPieces; ++i)
        *reinterpret_cast<u32x4 *>(sC + (row_first + i * kRowStep) * kScStride + 8 * (ch % (kHalfN / 8))) = vc[i];
    }
    __syncthreads();
    const uint32_t *bp = reinterpret_cast<const uint32_t *>(sB + (32 * ws + r) * kSbStride + kHalfN * half + 8 * kg);
    const uint16_t *cp = sC + (32 * wl + r) * kScStride + 8 * kg;
#pragma unroll
    for (int q = 0; q < kHalfN / 16; ++q) {
      Operand a, c;
      a.q = mk4(bp[8 * q], bp[8 * q + 1], bp[8 * q + 2], bp[8 * q + 3]);
      c.q = *reinterpret_cast<const u32x4 *>(cp + 16 * q);
      acc = mfma(a, c, acc);
    }
  }
  // B^T: the staged block read back n-major
  uint16_t *Bout = Btr + tile * kN * kBlk;
#pragma unroll
  for (int i = 0; i < kN * (kBlk / 8) / kThreads; ++i) {
    const int c8 = threadIdx.x + i * kThreads, n = c8 / (kBlk / 8), s0 = (c8 % (kBlk / 8)) * 8;
    uint32_t w[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const uint32_t lo = sB[(s0 + 2 * k) * kSbStride + n], hi = sB[(s0 + 2 * k + 1) * kSbStride + n];
      w[k] = lo | (hi << 16);
    }
    *reinterpret_cast<u32x4 *>(Bout + n * kBlk + s0) = mk4(w[0], w[1], w[2], w[3]);
  }
  __syncthreads();  // every wave has read its operands: sC may take G
  uint16_t *sGt = sC;
  const int l = 32 * wl + r;
#pragma unroll
  for (int i4 = 0; i4 < 4; ++i4) {
    const int s = 32 * ws + i4 * 8 + 4 * kg;
    u32x2 v;  // causal zero pattern: keep s <= l
    v.x = pack2(s + 0 <= l ? acc[4 * i4 + 0] : 0.f, s + 1 <= l ? acc[4 * i4 + 1] : 0.f);
    v.y = pack2(s + 2 <= l ? acc[4 * i4 + 2] : 0.f, s + 3 <= l ? acc[4 * i4 + 3] : 0.f);
    *reinterpret_cast<u32x2 *>(sGt + l * kGtStride + s) = v;
  }
  __syncthreads();
  // G in whole rows
  uint16_t *Gout = Gd + tile * kBlk * kBlk;
#pragma unroll
  for (int i = 0; i < kBlk * (kBlk / 8) / kThreads; ++i) {
    const int ch16 = threadIdx.x + i * kThreads, row = ch16 / (kBlk / 8), piece = ch16 % (kBlk / 8);
    *reinterpret_cast<u32x4 *>(Gout + row * kBlk + 8 * piece) =
        *reinterpret_cast<const u32x4 *>(sGt + row * kGtStride + 8 * piece);
  }
}

// ---- block_cumsum: per (head, block) decay bookkeeping ------------------------------------------
// One workgroup per (block, 16 heads starting at h0).  With cs_s the block-relative inclusive prefix
// sum of dt*A*log2(e) (the "segsum" input) and c31, c63 its values at tokens 31 and 63, every head
// gets one record of kRec floats per block:
//   [0,64)     rowf_l = exp2(cs_l - c31)                   output-row factor of the decay mask
//   [64,128)   f_s    = dt_s * exp2(c31 - cs_s)            input factor of the decay mask
//   [128]      exp2(c63 - c31)     state: middle of the block -> end of the block
//   [129]      c63                 log2 of the block's total decay
//   [130]      exp2(c31)           state: start of the block -> middle of the block
//   [131]      [128] * [130] of the next block: middle of the block -> middle of the next block
// The two mask factors evaluate exponents as large as the decay across half a block.  A block of a head
// whose decay across either half exceeds 2^kSteepExp is STEEP: the factors would leave the fp32 range
// (their product would be wrong by O(1) with nothing non-finite to show for it), so the mask is not
// factorised there -- the full kernel applies exp2(cs_l - cs_s), whose exponent is never positive, to
// the scores of that head in registers (see chunk_scan_kernel) -- and the record holds instead
//   [0,64)     dt_l
//   [64,128)   dt_s * exp2(c63 - cs_s)    input weight relative to the END of the block (never > dt_s)
//   [128]      1     [129] c63     [130] -1 (marks the record)     [131] A * log2(e)
// With these the states-only pass, which multiplies [64,128) by [128] and by the decay of the later
// blocks, needs no change.  No benchmark input is steep (dt <= 0.1, |A| <= 16: 74 at most).
// The block covers rows [row0, row0 + 64) of dt (tokens, H); rows from row_end on are not part of
// the sequence and count as dt = 0 (state-neutral padding).  The caller's dt values pass through
// dt_apply (optional bias, softplus, clamp) as they are read.  dt is transposed through LDS, 64 tokens
// of the block plus the first 32 of the next one (for [131]).  Head h's record goes to record number
// h * rec_stride + rec_off.
constexpr int kRec = 2 * kBlk + 4;
constexpr int kCumHeads = 16;
constexpr float kSteepExp = 96.f;
__device__ __forceinline__ void block_cumsum_block(float (*tile)[kCumHeads + 1], size_t row0, size_t row_end, int h0,
                                                   size_t rec_stride, size_t rec_off, const float *__restrict__ dt,
                                                   const float *__restrict__ A, float *__restrict__ prep, int H,
                                                   const DtXform dtx) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  // dt of the block's 64 tokens and of the first 32 of the next block, 16 heads each: six values per
  // thread, requested together (no load sits behind a branch).  The descriptor covers the rows from
  // row0 to the end of the sequence, so later rows read as zero; a head beyond H is given an offset
  // outside it.  Padding must end up as dt = 0 whatever the step-size map makes of a zero.
  constexpr int kTileToks = kBlk + kBlk / 2, kLoads = kTileToks * kCumHeads / kThreads;
  const size_t rows_left = row_end > row0 ? row_end - row0 : 0;
  const Rsrc rdt = make_rsrc(dt + row0 * H, __builtin_amdgcn_readfirstlane(static_cast<uint32_t>((rows_left < kTileToks ? rows_left : kTileToks) * H * 4)));
  constexpr int kPer = kCumHeads / (kThreads / 64);
  float a_head[kPer];  // A of the wave's heads (see below), requested with everything else
#pragma unroll
  for (int k = 0; k < kPer; ++k) a_head[k] = A[min(h0 + wave + k * (kThreads / 64), H - 1)];
  float raw[kLoads], bias[kLoads];
#pragma unroll
  for (int k = 0; k < kLoads; ++k) {
    const int i = threadIdx.x + k * kThreads, tok = i / kCumHeads, hh = i % kCumHeads;
    const bool head_ok = h0 + hh < H;
    raw[k] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(
                                           rdt, head_ok ? static_cast<uint32_t>(tok * H + h0 + hh) * 4u : 0xFFFFFF00u, 0, 0));
    bias[k] = dtx.bias != nullptr ? dtx.bias[head_ok ? h0 + hh : H - 1] : 0.f;
  }
#pragma unroll
  for (int k = 0; k < kLoads; ++k) {
    const int i = threadIdx.x + k * kThreads, tok = i / kCumHeads, hh = i % kCumHeads;
    const bool there = static_cast<size_t>(tok) < rows_left && h0 + hh < H;
    tile[tok][hh] = there ? dt_apply_branchless(raw[k], bias[k], dtx) : 0.f;
  }
  __syncthreads();
  // A wave takes the heads wave, wave + 4, wave + 8, wave + 12 of the group of 16.  Their prefix sums
  // are four independent chains of cross-lane steps, written side by side so that the latency of one
  // chain's step is covered by the steps of the others.
  float dtv[kPer], v[kPer], nx[kPer], ah[kPer];
  bool live[kPer];
#pragma unroll
  for (int k = 0; k < kPer; ++k) {
    const int hh = wave + k * (kThreads / 64);
    live[k] = h0 + hh < H;
    ah[k] = live[k] ? a_head[k] * kLog2e : 0.f;
    dtv[k] = tile[lane][hh];
    v[k] = dtv[k] * ah[k];
    // prefix sum at token 31 of the next block: the sum of its first 32 terms
    nx[k] = lane < kBlk / 2 ? tile[kBlk + lane][hh] * ah[k] : 0.f;
  }
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
#pragma unroll
    for (int k = 0; k < kPer; ++k) {
      const float up = __shfl_up(v[k], off, 64);
      if (lane >= off) v[k] += up;
    }
  }
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) {
#pragma unroll
    for (int k = 0; k < kPer; ++k) nx[k] += __shfl_xor(nx[k], m, 64);
  }
#pragma unroll
  for (int k = 0; k < kPer; ++k) {
    const float c0 = __shfl(v[k], 0, 64);
    const float c31 = __shfl(v[k], 31, 64);
    const float c63 = __shfl(v[k], 63, 64);
    if (live[k]) {
      const int h = h0 + wave + k * (kThreads / 64);
      float *rec = prep + (static_cast<size_t>(h) * rec_stride + rec_off) * kRec;
      // (negated test: a NaN prefix sum also takes the steep form, which has no exponent to overflow)
      const bool steep = !(c0 - c31 <= kSteepExp && c31 - c63 <= kSteepExp);
      if (!steep) {
        rec[lane] = fast_exp2(v[k] - c31);
        rec[kBlk + lane] = dtv[k] * fast_exp2(c31 - v[k]);
        if (lane < 4)
          rec[2 * kBlk + lane] = lane == 0   ? fast_exp2(c63 - c31)
                                 : lane == 1 ? c63
                                 : lane == 2 ? fast_exp2(c31)
                                             : fast_exp2(c63 - c31) * fast_exp2(nx[k]);
      } else {
        rec[lane] = dtv[k];
        rec[kBlk + lane] = dtv[k] * fast_exp2(c63 - v[k]);
        if (lane < 4) rec[2 * kBlk + lane] = lane == 0 ? 1.f : lane == 1 ? c63 : lane == 2 ? -1.f : ah[k];
      }
    }
  }
}

// Both preparation steps in one launch (they are independent of each other and each is far too
// small to fill the chip): the first n_scores workgroups compute G and B^T, the others the decay
// records.  NB = blocks per batch row (plain batch) or the block capacity (variable-length batch,
// where workgroups beyond the actual number of blocks have nothing to do).
// grid (n_scores + NB * ceil(H/16) * Bt), n_scores = NB * Bt * G; Bt = 1 for a variable-length batch.
// Workspace tiles are numbered (b * G + g) * NB + block, records (b * H + h) * NB + block.
__global__ __launch_bounds__(kThreads) void block_prep_kernel(const uint16_t *__restrict__ B,
                                                              const uint16_t *__restrict__ C,
                                                              uint16_t *__restrict__ Gd,
                                                              uint16_t *__restrict__ Btr,
                                                              const float *__restrict__ dt,
                                                              const float *__restrict__ A,
                                                              float *__restrict__ prep, int T, int H, int G,
                                                              int NB, int n_scores, const VarPlan vp,
                                                              const NSlice ns, uint16_t *__restrict__ Cpad,
                                                              const DtXform dtx) {
  // score workgroups: the B and C tiles; decay workgroups: the transposed dt (in the same memory)
  __shared__ __align__(16) uint16_t sB[kSbElems];
  __shared__ __align__(16) uint16_t sC[kScElems];
  static_assert(sizeof(float) * (kBlk + kBlk / 2) * (kCumHeads + 1) <= sizeof(uint16_t) * kScElems, "dt tile fits");
  float (*tile)[kCumHeads + 1] = reinterpret_cast<float (*)[kCumHeads + 1]>(sC);
  const int wg = blockIdx.x;
  const bool scores = wg < n_scores;
  const int i = scores ? wg : wg - n_scores;
  // Workgroups that read neighbouring pieces of the same rows of B and C (the groups of a block) or of dt
  // (the sets of 16 heads of a block) have consecutive numbers, so that they run at about the same time.
  const int hgroups = (H + kCumHeads - 1) / kCumHeads;
  const int fan = scores ? G : hgroups;
  const int part = i % fan;          // group, or set of 16 heads
  const int jb = (i / fan) % NB;     // block inside the batch row, or block of the packed batch
  const int b = i / (fan * NB);
  size_t row0, row_end;
  if (vp.tok0 != nullptr) {
    if (jb >= vp.blk0[vp.nseq]) return;
    const int q = vp.blk_seq[jb];
    row0 = static_cast<size_t>(vp.tok0[q]) + static_cast<size_t>(jb - vp.blk0[q]) * kBlk;
    row_end = static_cast<size_t>(vp.tok0[q]) + vp.len[q];
  } else {
    row0 = static_cast<size_t>(b) * T + static_cast<size_t>(jb) * kBlk;
    row_end = static_cast<size_t>(b) * T + T;
  }
  // (the tables are read with vector loads: tell the compiler that the rows are the same for every lane,
  // or every buffer descriptor built from them costs a loop over the lanes' values per access)
  row0 = uniform_size(row0);
  row_end = uniform_size(row_end);
  if (scores)
    scores_bt_block(sB, sC, row0, row_end, (static_cast<size_t>(b) * G + part) * NB + jb, part,
                    B, C, Gd, Btr, G, ns, Cpad);
  else
    block_cumsum_block(tile, row0, row_end, part * kCumHeads, NB, static_cast<size_t>(b) * H * NB + jb, dt, A, prep, H,
                       dtx);
}

// ---- chunk_scan / segment_states ----------------------------------------------------------------
struct ScanParams {
  const uint8_t *x;
  const uint8_t *C;
  const float *D;
  const uint8_t *Gd;
  const uint8_t *Btr;
  const float *prep;
  uint8_t *y;
  const float *h0;         // (sequences, H, P, N) initial states, or nullptr = zeros (read by one-segment sequences)
  const float *Hin;        // state entering each segment of a sequence of several: one slot per segment
  float *final_state;      // (sequences, H, P, N): written by the last segment of each sequence
  float *seg_state;        // states-only: local end state of a segment -> the slot of the NEXT segment
  float *seg_decay;        // states-only: log2 of the segment's total decay, one per slot
  int T, H, G, hpg, NB, seg_blocks, S;  // H, hpg count 64-column slices
  int cpg;                 // workgroups ("head groups of four") per B/C group: ceil(hpg / 4); the slots of the
                           // last one beyond hpg repeat the group's last slice with every store suppressed
  // The states-only pass may cut every segment into `parts` pieces of `part_blocks` blocks (more,
  // shorter workgroups when the segments alone would leave most of the chip idle); the pass over
  // segment states then chains the pieces, and a sequence has `slots` state slots, of which segment
  // sg of the full scan starts from slot sg * parts.  Plain batches only; parts = 1 otherwise.
  int parts, part_blocks, slots;
  // fold != 0 (plain batches of few segments): no pass over segment states has run.  The first segment
  // starts from h0 itself; segment sg sums the local end states of the pieces before it (slots 1 .. sg
  // parts) and h0, each times the decay of the pieces after it, as it loads them.
  int fold;
  int pdiv, Hrec;          // slices per head (headdim / 64); heads (owners of decay records, A, D)
  NSlice ns;               // columns of h0 / final_state (rows of ns.width floats) this launch works on
  int cols, segs, total, per_xcd;  // workgroup mapping, see wg_coords
  VarPlan vp;              // tok0 == nullptr: plain batch
};

// Where a workgroup works: head group `col`, segment `sg` of `S` of sequence `b`, whose `nb` blocks
// start at token `tok0` of the packed token axis (`len` tokens), at workspace tile / record number
// `blk0` (per group / per head: stride `blk_stride`), and whose state slots (one per segment, per
// head: stride `slot_stride`) start at `slot0`.
struct SeqView {
  int col, sg, S, b, nb;
  size_t tok0, blk0, blk_stride, slot0, slot_stride;
  uint32_t len;
};

// Workgroup -> (head group, segment, sequence).  The chip dispatches consecutive workgroup ids to
// its eight XCDs in turn, and each XCD has its own L2.  The workgroups that share C / B^T / G tiles
// (all head groups of one segment of one sequence) are therefore given ids that are congruent
// modulo 8, so that they run on one XCD and the tiles are fetched into one L2 instead of eight:
// XCD k owns the contiguous range [k * per_xcd, (k + 1) * per_xcd) of the (sequence, segment, head
// group) list, head group fastest.  Ids beyond the list (the grid is rounded up to 8 * per_xcd) idle.
// `last_too`: whether the last segment of a sequence is in the list (not for the states-only pass).
constexpr int kXcds = 8;
__device__ __forceinline__ bool wg_coords_varlen(const ScanParams &p, bool last_too, SeqView &v);
__device__ __forceinline__ bool wg_coords(const ScanParams &p, bool last_too, SeqView &v) {
  if (p.vp.tok0 != nullptr) return wg_coords_varlen(p, last_too, v);
  const int id = blockIdx.x;
  const int w = (id % kXcds) * p.per_xcd + id / kXcds;
  if (w >= p.total) return false;
  v.col = w % p.cols;
  v.sg = (w / p.cols) % p.segs;
  v.b = w / (p.cols * p.segs);
  v.S = p.S;
  v.nb = p.NB;
  v.tok0 = static_cast<size_t>(v.b) * p.T;
  v.len = static_cast<uint32_t>(p.T);
  v.blk0 = static_cast<size_t>(v.b) * p.NB;   // times G (tiles) or H (records) in the caller's stride
  v.blk_stride = p.NB;
  v.slot0 = static_cast<size_t>(v.b) * p.slots;
  v.slot_stride = p.slots;
  return true;
}
// Variable-length batch: the list (see varlen_fill_kernel) and with it the split over the XCDs come
// from the device-side tables; the grid was sized for the host's upper bound on its length.
__device__ __forceinline__ bool wg_coords_varlen(const ScanParams &p, bool last_too, SeqView &v) {
  const int n_items = p.vp.item0[p.vp.nseq];
  const int n_full = n_items - p.vp.nseq;
  const int n_list = last_too ? n_items : n_full;
  // The same contiguous split over the XCDs as for a plain batch, so that every XCD gets the same
  // number of workgroups.  The list is sorted by length; for the full pass (whose entries differ in
  // length) it is first dealt into eight hands, hand k holding entries k, k + 8, ..., and the hands
  // are laid end to end: every XCD then works on the same mix of long and short entries, long first.
  const int total = n_list * p.cols;
  const int per_xcd = (total + kXcds - 1) / kXcds;
  const int id = blockIdx.x;
  if (id / kXcds >= per_xcd) return false;
  const int w = (id % kXcds) * per_xcd + id / kXcds;
  if (w >= total) return false;
  v.col = w % p.cols;
  int item = w / p.cols;
  if (last_too) {
    const int base = n_list / kXcds, rem = n_list % kXcds;  // hands 0..rem-1 hold base + 1 entries
    const int big = rem * (base + 1);
    const int hand = item < big ? item / (base + 1) : rem + (item - big) / base;
    const int pos = item < big ? item % (base + 1) : (item - big) % base;
    item = pos * kXcds + hand;
  }
  const int q = p.vp.item_seq[item];
  const int first = p.vp.item0[q];
  v.b = q;
  v.S = p.vp.item0[q + 1] - first;
  v.sg = item < n_full ? item - (first - q) : v.S - 1;
  v.len = static_cast<uint32_t>(p.vp.len[q]);
  v.nb = static_cast<int>((v.len + kBlk - 1) / kBlk);
  v.tok0 = static_cast<size_t>(p.vp.tok0[q]);
  v.blk0 = static_cast<size_t>(p.vp.blk0[q]);
  v.blk_stride = static_cast<size_t>(p.vp.nb_cap);
  v.slot0 = static_cast<size_t>(p.vp.slot0[q]);
  v.slot_stride = static_cast<size_t>(p.vp.slot_cap);
  return true;
}

constexpr int kHeadsPerWg = 4;
constexpr int kScanThreads = 2 * 64 * kHeadsPerWg;  // two waves per head, one per half of headdim
constexpr int kGStride = kBlk + 8;

// Waits until no vector memory operation of the wave is outstanding.  Used once, at the end of a
// loop prologue: the compiler places its waits for the worst case over all paths into a loop, and the
// order in which a prologue happened to request its loads would otherwise dictate (too strict) waits
// to every iteration.  (vmcnt = 0, expcnt and lgkmcnt not waited for.)
__device__ __forceinline__ void wait_all_loads() { __builtin_amdgcn_s_waitcnt(0x0F70); }

// The MFMA writes row m of a 32-row result to lane group kg = (m >> 2) & 1, element 4 (m >> 3) + (m & 3).
// Giving MFMA row m the headdim column pi(m) = 16 kg + element makes every lane own 16 consecutive
// columns of its token: 32 contiguous bytes of y per lane instead of four 8-byte pieces.
__device__ __forceinline__ int pi_of_row(int m) { return 16 * ((m >> 2) & 1) + 4 * (m >> 3) + (m & 3); }

// One wave per (head, half of headdim): the wave owns a 128 x 32 slice of the state (64
// accumulator registers), a 64 x 32 output tile (32) and its input operands (16); with the next
// block's data in flight it stays under 256 registers, so the eight waves of a workgroup run two
// per SIMD and one wave's MFMAs overlap the other's vector work and memory waits.
//
// What bounds the kernel is the memory path (every CU has to pull its share of x and push its share
// of y, and a CU sustains only ~1/256 of the chip's bandwidth), so the loop is arranged to keep
// requests outstanding all the time and to move no byte twice: the skip term D x reads x from a raw
// copy that the staging step leaves in LDS instead of loading it again, the loads of the block after
// next are issued in the middle of an iteration, as soon as their registers are free, and the stores
// of y are spread over the second half.
#ifndef SSD_ROW_STORES
#define SSD_ROW_STORES 1
#endif
// y leaves as whole 128-byte rows (the two waves of a head exchange their halves through LDS, one more
// barrier per block) instead of 64-byte half rows per wave.
constexpr bool kRowStores = SSD_ROW_STORES != 0;
constexpr int kRawStride = 40;                       // raw x rows: 32 columns + 16 bytes, in bf16 elements
constexpr int kGLowStride = 32 + 8;                  // G rows 0..31 keep only columns 0..31 (the rest is masked)
constexpr int kGTile = 32 * kGLowStride + 32 * kGStride;  // elements of a compacted G tile
// HPW = heads per workgroup (two waves each).  Both kernels take four heads: the full kernel's LDS tiles
// fill the CU; the states-only kernel could run two smaller workgroups per CU, but its grid then no
// longer divides evenly over the CUs and the measured time was worse.
// kYMode, how y leaves: kYPlain -- ordinary stores; kYStream -- non-temporal stores, so that writing y does not
// evict x, which the states-only pass has just pulled into the memory-side cache, before this kernel reads it
// again (chosen per launch, see stream_y()); kYAdd -- added to what y already holds (the later state slices
// of a dstate above 128: the sum of the slices' outputs is formed where the last one is stored).
// The LDS tiles of a scan workgroup, as pointers that keep their address space across a function call.
typedef __attribute__((address_space(3))) uint16_t lds_u16;
struct LdsTiles {
  lds_u16 *sC, *sBt, *sG, *sXm, *sRaw;
};
template <bool kStatesOnly, int HPW>
struct ScanLds {
  static constexpr int kCElems = kStatesOnly ? 8 : kBlk * kCStride, kCBufs = kStatesOnly ? 1 : 2;
  static constexpr int kBtElems = kN * kBtStride;
  static constexpr int kGElems = kStatesOnly ? 8 : kGTile, kGBufs = kStatesOnly ? 1 : 2;
  static constexpr int kXmElems = kP * kXStride;
  static constexpr int kXmBufs = kStatesOnly ? 2 : 1;  // the states-only pass reads the other wave's half: two copies
  static constexpr int kRawElems = kStatesOnly ? 8 : kBlk * kRawStride, kRawBufs = kStatesOnly ? 1 : 2 * HPW;
};

// The walk of one workgroup over its blocks.  kMixed: the walk may meet steep blocks (see
// block_cumsum_block) and chooses the form block by block; otherwise every block has the common form.
template <bool kStatesOnly, int HPW, int kYMode, bool kMixed>
__device__ __forceinline__ void scan_walk(const ScanParams &p, const SeqView &sv, const LdsTiles lds) {
  static_assert(!(kStatesOnly && kYMode != kYPlain), "the states-only pass writes no y");
  static_assert(!(kStatesOnly && kMixed), "the states-only pass needs no second form");
  static_assert(kStatesOnly || HPW == kHeadsPerWg, "the full kernel is written for four heads per workgroup");
  constexpr int kThr = 128 * HPW;
  constexpr int kBtPieces = kN * kBlk * 2 / 16 / kThr;  // 16-byte pieces of the B^T tile per thread
  using L = ScanLds<kStatesOnly, HPW>;
  // (generic pointers derived from the address-space pointers: the compiler keeps them LDS accesses)
  uint16_t (*const sC)[L::kCElems] = reinterpret_cast<uint16_t (*)[L::kCElems]>((uint16_t *)lds.sC);
  uint16_t (*const sBt)[L::kBtElems] = reinterpret_cast<uint16_t (*)[L::kBtElems]>((uint16_t *)lds.sBt);  // B^T [n][s]
  uint16_t (*const sG)[L::kGElems] = reinterpret_cast<uint16_t (*)[L::kGElems]>((uint16_t *)lds.sG);
  uint16_t (*const sXm)[L::kXmElems] = reinterpret_cast<uint16_t (*)[L::kXmElems]>((uint16_t *)lds.sXm);  // Xm^T [row][s], per head
  uint16_t (*const sRaw)[L::kRawElems] = reinterpret_cast<uint16_t (*)[L::kRawElems]>((uint16_t *)lds.sRaw);  // x [s][col], per wave

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // uniform: addresses derived from it stay scalar
  const int hw = wave >> 1, ph = wave & 1;  // head inside the workgroup, half of headdim
  // Waves w and w + 4 of the workgroup share a SIMD.  Giving one of the two the higher issue priority
  // for the whole kernel lets it run ahead between barriers instead of both contending for the same
  // pipe in the same phase (measured: 3 % on 8 x 4096 tokens x 48 heads, nothing lost elsewhere).
  if (wave >= 4) __builtin_amdgcn_s_setprio(1);
  const int col = sv.col, sg = sv.sg;
  // The heads of a workgroup share one B/C group.  A group whose number of (64-column) slices is not a
  // multiple of four leaves slots of its last workgroup without a slice: those waves repeat the group's last
  // slice -- they take part in the shared staging and the barriers like any other -- and write nothing.
  const int g = col / p.cpg;
  const int slot = (col % p.cpg) * HPW + hw;
  const bool live = slot < p.hpg;
  const int h = g * p.hpg + min(slot, p.hpg - 1);
  // workspace numbering: tiles (b, g, block), records (b, h, block), state slots (b, h, segment) for a
  // plain batch; (g, block), (h, block), (h, segment) with batch-wide block / segment numbers otherwise
  const bool plain = p.vp.tok0 == nullptr;
  const size_t tile0 = plain ? (sv.blk0 * p.G + static_cast<size_t>(g) * sv.blk_stride) : (g * sv.blk_stride + sv.blk0);
  const int hrec = h / p.pdiv;  // the head this slice belongs to
  const size_t rec0 = plain ? (sv.blk0 * p.Hrec + static_cast<size_t>(hrec) * sv.blk_stride) : (hrec * sv.blk_stride + sv.blk0);
  const size_t slot0 = plain ? (sv.slot0 * p.H + static_cast<size_t>(h) * sv.slot_stride) : (h * sv.slot_stride + sv.slot0);
  const size_t bh = static_cast<size_t>(sv.b) * p.H + h;  // row of final_state
  const int r = lane & 31, kg = lane >> 5;
  // (the states-only pass walks a piece of a segment, the full scan a whole segment)
  const int walk = kStatesOnly ? p.part_blocks : p.seg_blocks;
  const int jb0 = min(sv.nb, sg * walk);
  const int jb1 = min(sv.nb, jb0 + walk);
  const int cg = lane & 3, tg = lane >> 2;  // x staging: columns 8cg..8cg+7 of the half, tokens 4tg..4tg+3
  uint16_t *const myX = sXm[hw] + 32 * ph * kXStride;  // this wave's 32 rows of Xm^T
  uint16_t *const myRaw = sRaw[kStatesOnly ? 0 : wave];

  // ---- addressing: scalar bases, per-lane byte offsets that never change ----
  const uint32_t xrow = static_cast<uint32_t>(p.H) * (kP * 2);   // bytes per token of x / y
  const uint32_t crow = static_cast<uint32_t>(p.G) * (kN * 2);   // bytes per token of C
  const uint32_t xbytes = sv.len * xrow;                         // the sequence's rows of x / y
  const uint32_t cbytes = sv.len > 0 ? sv.len * crow - static_cast<uint32_t>(g) * (kN * 2) : 0;
  const uint8_t *const xb = p.x + sv.tok0 * xrow;
  uint8_t *const yb = p.y + sv.tok0 * xrow;
  const uint8_t *const cb = p.C + (sv.tok0 * p.G + g) * (kN * 2);
  const Rsrc rs_bt = make_rsrc(p.Btr + tile0 * (kN * kBlk * 2), static_cast<uint32_t>(sv.nb) * (kN * kBlk * 2));
  const Rsrc rs_g = make_rsrc(p.Gd + tile0 * (kBlk * kBlk * 2), static_cast<uint32_t>(sv.nb) * (kBlk * kBlk * 2));
  const float *const prep_bh = p.prep + rec0 * kRec;
  const Rsrc rs_prep = make_rsrc(prep_bh, static_cast<uint32_t>(sv.nb) * (kRec * 4));
  // descriptors of x, y and C start at the block and end at the sequence's last token
  auto x_rsrc = [&](int jb) { return make_rsrc(xb + static_cast<size_t>(jb) * kBlk * xrow, xbytes - static_cast<uint32_t>(jb) * kBlk * xrow); };
  auto y_rsrc = [&](int jb) { return make_rsrc(yb + static_cast<size_t>(jb) * kBlk * xrow, live ? xbytes - static_cast<uint32_t>(jb) * kBlk * xrow : 0u); };
  auto c_rsrc = [&](int jb) { return make_rsrc(cb + static_cast<size_t>(jb) * kBlk * crow, cbytes - static_cast<uint32_t>(jb) * kBlk * crow); };
  const uint32_t vt = static_cast<uint32_t>(tid) * 16;  // shared tiles: 16 bytes per thread, tid-major
  const uint32_t xcol = static_cast<uint32_t>(h) * (kP * 2) + 64 * ph;
  uint32_t vx[4], vc[2], ve[2];
#pragma unroll
  for (int i = 0; i < 4; ++i) vx[i] = static_cast<uint32_t>(4 * tg + i) * xrow + xcol + 16 * cg;
#pragma unroll
  for (int k = 0; k < 2; ++k) {
    const int c = tid + kThr * k;
    vc[k] = static_cast<uint32_t>(c >> 4) * crow + 16 * (c & 15);
    ve[k] = static_cast<uint32_t>(r + 32 * k) * xrow + xcol + 32 * kg;  // output layout: token r + 32k, 32 bytes
  }
  const uint32_t vf = static_cast<uint32_t>(kBlk + 4 * tg) * 4;  // input factors of this thread's four tokens
  // G: thread -> (row, 16-byte piece); in rows 0..31 only pieces 0..3 are kept (s <= l < 32), the
  // threads of the other pieces duplicate a kept one (same data to the same place)
  const int g_row = tid >> 3, g_pc = (g_row < 32) ? (tid & 3) : (tid & 7);
  const uint32_t vg = static_cast<uint32_t>(g_row * kBlk + 8 * g_pc) * 2;

  // ---- data of a block in flight (registers) ----
  u32x4 r_c[2], r_bt[kBtPieces], r_g;  // shared tiles: this thread's 16-byte pieces
  // own slice: 4 tokens x 8 columns, and the input factors of the 4 tokens (fp32 bits); two blocks
  // of them are in flight (x comes from HBM and is the stream that must never run dry)
  constexpr int kSets = 2;
  u32x4 r_x[kSets][4];
  u32x4 r_f[kSets];

  // Global loads of block jb, in three portions so that they can be spread over the instruction stream.
  auto load_part = [&](int part, int jb, int set = 0) __attribute__((always_inline)) {
    if (part == 0) {
      const Rsrc rx = x_rsrc(jb);
#pragma unroll
      for (int i = 0; i < 4; ++i) r_x[set][i] = buf_load16(rx, vx[i], 0);
      r_f[set] = buf_load16(rs_prep, vf, jb * (kRec * 4));
    } else if (part == 1) {
#pragma unroll
      for (int k = 0; k < kBtPieces; ++k) r_bt[k] = buf_load16(rs_bt, vt, jb * (kN * kBlk * 2) + k * (kThr * 16));
    } else if (!kStatesOnly) {
      const Rsrc rc = c_rsrc(jb);
#pragma unroll
      for (int k = 0; k < 2; ++k) r_c[k] = buf_load16(rc, vc[k], 0);
      r_g = buf_load16(rs_g, vg, jb * (kBlk * kBlk * 2));
    }
  };

  // LDS destinations of this thread's pieces (fixed)
  uint32_t lds_bt[kBtPieces], lds_c[2];
#pragma unroll
  for (int k = 0; k < kBtPieces; ++k) {
    const int c = tid + kThr * k;
    lds_bt[k] = (c >> 3) * kBtStride + 8 * (c & 7);
  }
#pragma unroll
  for (int k = 0; k < 2; ++k) {
    const int c = tid + kThr * k;
    // C columns are permuted inside each group of 16 so that one 16-byte read yields
    // n-offsets {4kg..4kg+3, 8+4kg..8+4kg+3}
    lds_c[k] = (c >> 4) * kCStride + 16 * ((c & 15) >> 1) + 4 * (c & 1);
  }
  const uint32_t lds_g = (g_row < 32 ? g_row * kGLowStride : 32 * kGLowStride + (g_row - 32) * kGStride) + 8 * g_pc;
  // Xm^T: column 8cg + c of the half goes to row pi^-1(8cg + c) = 16 (cg & 1) + 4 (cg >> 1) + 8 (c >> 2) + (c & 3)
  uint16_t *const xm_dst = myX + (16 * (cg & 1) + 4 * (cg >> 1)) * kXStride + 4 * tg;
  uint16_t *const raw_dst = myRaw + (4 * tg) * kRawStride + 8 * cg;

  // Registers -> LDS for the block in flight, in slices.  Slice c < 8 computes column c of the own
  // slice, Xm^T[row][s] = f_s x[s][col] (four tokens per 8-byte write).
  // (xbuf: which copy of Xm^T, for the states-only pass; the full kernel has one)
  auto stage_column = [&](int c, int set = 0, int xbuf = 0) __attribute__((always_inline)) {
    const float f0 = __uint_as_float(r_f[set].x), f1 = __uint_as_float(r_f[set].y),
                f2 = __uint_as_float(r_f[set].z), f3 = __uint_as_float(r_f[set].w);
    const int w = c >> 1;
    const uint32_t a0 = r_x[set][0][w], a1 = r_x[set][1][w], a2 = r_x[set][2][w], a3 = r_x[set][3][w];
    uint16_t *dst = xm_dst + xbuf * (HPW * L::kXmElems) + (8 * (c >> 2) + (c & 3)) * kXStride;
    if (c & 1)
      *reinterpret_cast<u32x2 *>(dst) =
          mk2(pack2(f0 * bf_hi(a0), f1 * bf_hi(a1)), pack2(f2 * bf_hi(a2), f3 * bf_hi(a3)));
    else
      *reinterpret_cast<u32x2 *>(dst) =
          mk2(pack2(f0 * bf_lo(a0), f1 * bf_lo(a1)), pack2(f2 * bf_lo(a2), f3 * bf_lo(a3)));
  };
  auto stage_tile = [&](int piece, int buf) {  // pieces 0,1: B^T; 2,3: C; 4: G
    if (piece < 2) {
      *reinterpret_cast<u32x4 *>(&sBt[buf][lds_bt[piece]]) = r_bt[piece];
    } else if constexpr (!kStatesOnly) {
      if (piece < 4) {
        uint16_t *d2 = &sC[buf][lds_c[piece - 2]];
        *reinterpret_cast<u32x2 *>(d2) = mk2(r_c[piece - 2].x, r_c[piece - 2].y);
        *reinterpret_cast<u32x2 *>(d2 + 8) = mk2(r_c[piece - 2].z, r_c[piece - 2].w);
      } else {
        *reinterpret_cast<u32x4 *>(&sG[buf][lds_g]) = r_g;
      }
    }
  };
  auto stage_raw = [&](int set = 0) __attribute__((always_inline)) {  // the unscaled rows, for the skip term of the block's epilogue
    if constexpr (!kStatesOnly) {
#pragma unroll
      for (int i = 0; i < 4; ++i) *reinterpret_cast<u32x4 *>(raw_dst + i * kRawStride) = r_x[set][i];
    }
  };

  // Per-block state factors (record entries 128..131): uniform over the wave, but fetched with
  // ordinary (broadcast) vector loads and requested well ahead of their use.  A scalar load would share
  // its counter with the LDS operations and, returning out of order, turn every LDS wait into a wait
  // for everything including the scalar load's trip to memory.
  auto factor_ptr = [&](int jb) { return prep_bh + static_cast<size_t>(jb) * kRec + 2 * kBlk; };
  // Output-row factors of this lane's two tokens (r, 32 + r): of the current block, and of the next
  // one.  The next block's are requested early in an iteration, BEFORE the stores of y and the loads
  // of x: vector memory operations complete in order, so a small load issued after them could only be
  // waited for together with them.
  float rowf0 = 0.f, rowf1 = 0.f, rowf0n = 0.f, rowf1n = 0.f;
  auto load_rowf = [&](int jb) __attribute__((always_inline)) {
    if constexpr (!kStatesOnly) {
      const float *rec = prep_bh + static_cast<size_t>(jb) * kRec;
      rowf0n = rec[r];
      rowf1n = rec[32 + r];
    }
  };

  // ---- state slice: Hacc[nt][i] = Ht^T[n = 32nt + (i/4)*8 + 4kg + i%4][headdim column 32 ph + pi_of_row(r)] ----
  f32x16 Hacc[4];
  u32x4 hraw[16];          // the entering state as loaded (full kernel)
  bool has_state = false;  // uniform over the workgroup
  // Everything the prologue needs from memory -- D, the entering state, the first block factor and (below)
  // the first block -- is requested before any of it is waited for: one trip to memory instead of one each.
  float Dh = kStatesOnly || p.D == nullptr ? 0.f : p.D[hrec];
  if constexpr (!kStatesOnly) {
    // A sequence of one segment starts from h0 itself (this workgroup reads it here and is the only
    // one to write final_state, so the two may share memory); with several segments every segment,
    // the first included, starts from the slot that the pass over segment states has filled.
    // Rows of hrow floats of which hvalid columns exist; no state at all: an empty descriptor, whose
    // loads return zero.
    const float *hbase = nullptr;
    uint32_t hrow = kN, hvalid = kN;
    if (sv.S > 1 && !(p.fold && sg == 0)) {
      hbase = p.Hin + (slot0 + static_cast<size_t>(sg) * p.parts) * (kP * kN);
    } else if (p.h0 != nullptr) {
      hbase = p.h0 + bh * kP * p.ns.width + p.ns.off;
      hrow = static_cast<uint32_t>(p.ns.width);
      hvalid = static_cast<uint32_t>(p.ns.valid);
    }
    const Rsrc rs_h = make_rsrc(hbase != nullptr ? hbase : p.prep, hbase != nullptr ? ((kP - 1) * hrow + hvalid) * 4u : 0u);
    // Requested in whole row segments (16 lanes x 16 bytes = 64 state columns of one headdim column, four
    // columns per instruction); the accumulator layout -- 16-byte pieces of 32 different rows per lane --
    // is reached through LDS below (turn_state), once the first block's loads are on their way as well.
    has_state = hbase != nullptr;
#pragma unroll
    for (int k = 0; k < 16; ++k) {
      const uint32_t row = 32 * ph + 4 * (k & 7) + (lane >> 4), n0 = 64 * (k >> 3) + 4 * (lane & 15);
      hraw[k] = buf_load16(rs_h, n0 < hvalid ? (row * hrow + n0) * 4u : 0xFFFFFF00u, 0);
    }
  } else {
#pragma unroll
    for (int nt = 0; nt < 4; ++nt)
#pragma unroll
      for (int i = 0; i < 16; ++i) Hacc[nt][i] = 0.f;
  }
  // The accumulators hold the state up to a factor that is applied lazily: `pending` takes the state
  // from where the previous block left it (the middle of that block) to the middle of the current
  // block.  It is multiplied in eight elements at a time, right where those elements are converted
  // to an MFMA operand, so the multiplies hide under the matrix instructions of the same loop.
  float pending = jb0 < jb1 && !kStatesOnly ? factor_ptr(jb0)[2] : 1.f;
  // A steep block (see block_cumsum_block) marks its record with a negative entry there; it starts from
  // the state as it is at the start of the block.  Uniform over the wave, kept in a scalar register.
  bool steep_cur = false;
  if constexpr (kMixed) {
    steep_cur = __builtin_amdgcn_readfirstlane(__float_as_int(pending)) < 0;
    if (steep_cur) pending = 1.f;
  }

  // LDS operand addresses of this lane (element offsets inside a tile)
  const uint32_t a_c = r * kCStride + 8 * kg;    // + 32 rows for the second token half, + 16 kk
  const uint32_t a_g0 = r * kGLowStride + 8 * kg;                     // token r, + 16 q (q < 2)
  const uint32_t a_g1 = 32 * kGLowStride + r * kGStride + 8 * kg;     // token 32 + r, + 16 q
  const uint32_t a_bt = r * kBtStride + 8 * kg;  // + 32 nt rows, + 16 q
  const uint16_t *const raw_src = myRaw + r * kRawStride + 16 * kg;   // + 32 rows for the second half, + 8 c
  uint16_t *const raw_rw = myRaw + r * kRawStride + 16 * kg;
  // output rows.  Half rows: lane i handles 16 bytes of token i/4 (+16k) of the wave's own half.  Whole
  // rows: the wave handles tokens 32ph + i/8 (+8k), lane i the 16-byte piece i%8 of the 128-byte row --
  // pieces 0..3 come from the tile of the head's first wave, 4..7 from that of its second wave.
  const uint16_t *const raw_dst_row =
      kRowStores && !kStatesOnly
          ? sRaw[kStatesOnly ? 0 : 2 * hw + ((lane & 7) >> 2)] + (32 * ph + (lane >> 3)) * kRawStride + 8 * (lane & 3)
          : myRaw + (lane >> 2) * kRawStride + 8 * (lane & 3);
  const uint32_t vy = kRowStores ? static_cast<uint32_t>(32 * ph + (lane >> 3)) * xrow +
                                       static_cast<uint32_t>(h) * (kP * 2) + 16 * (lane & 7)
                                 : static_cast<uint32_t>(lane >> 2) * xrow + xcol + 16 * (lane & 3);
  constexpr int kRowStep = kRowStores ? 8 : 16;  // tokens between a lane's four pieces
  auto lds16 = [](const uint16_t *ptr) {
    Operand o;
    o.q = *reinterpret_cast<const u32x4 *>(ptr);
    return o;
  };

  float seg_total = 0.f;
  // The loop body below is free of branches around memory operations (block indices are clamped to
  // the segment instead, redundant loads in the last two iterations are harmless): the hardware
  // counts outstanding loads and stores in order, and only with straight-line code can the compiler
  // wait for exactly the older ones and leave the newer ones in flight.
  // It is written as an explicit software pipeline: every group of matrix instructions is preceded by
  // the LDS reads of the NEXT group's operands and accompanied by independent vector work (state
  // scaling and conversion and the staging of the next block in the first phase, the output epilogue
  // in the second); the scheduling fences keep the compiler from undoing that order.
  const int jlast = jb1 - 1;
  if constexpr (kStatesOnly) {
    // ---- states only: the segment's end state from a zero start, H = sum_s w_s x_s (x) B_s with
    //      w_s = dt_s * (decay from token s to the END OF THE SEGMENT).  Taking the weights relative
    //      to the segment end (every exponent <= 0: nothing overflows, what has decayed away
    //      underflows to zero as it should) means the accumulators are never rescaled: per block only
    //      H += B^T Xm.  w_s = f_s * (middle -> end of its block) * exp2(decay of the blocks after it).
    //      The kernel is a pure stream of x (plus the shared B^T tile), so x is requested two blocks
    //      ahead: block k's iteration stages block k+1 from one register set and then refills that set
    //      with block k+3.  Two iterations are written out per loop trip so that the set index is a
    //      compile-time constant. ----
    auto at = [&](int j) { return min(j, jlast); };
    auto load_factors = [&](int j) { return *reinterpret_cast<const f32x2 *>(factor_ptr(j)); };
    // {middle -> end, log2 of the total decay} of the block to be staged next, fetched one iteration
    // before it is used
    f32x2 sf_stage = {1.f, 0.f};
    // The first TWO blocks are requested at once, together with the decays that are summed next: the second
    // block's B^T pieces land in registers of their own until the first block's have gone to LDS, so the
    // prologue costs one trip to memory, not two.
    f32x2 sf_second = {1.f, 0.f};
    u32x4 r_bt_second[kBtPieces];
    if (jb0 < jb1) {
      load_part(0, jb0, 0);
      load_part(1, jb0);
      load_part(0, at(jb0 + 1), 1);
#pragma unroll
      for (int k = 0; k < kBtPieces; ++k)
        r_bt_second[k] = buf_load16(rs_bt, vt, at(jb0 + 1) * (kN * kBlk * 2) + k * (kThr * 16));
      sf_stage = load_factors(jb0);
      sf_second = load_factors(at(jb0 + 1));
    }
    for (int j = jb0; j < jb1; j += 64) {  // the segment's total log2 decay: one lane per block
      float v = j + lane < jb1 ? factor_ptr(j + lane)[1] : 0.f;
#pragma unroll
      for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m, 64);
      seg_total += v;
    }
    float rest = seg_total;  // log2 decay of the blocks after the one being staged
    float ws = 0.f;
    auto next_weight = [&]() __attribute__((always_inline)) {
      rest -= sf_stage.y;
      ws = sf_stage.x * fast_exp2(rest);
    };
    auto weigh = [&](int set) __attribute__((always_inline)) {
#pragma unroll
      for (int i = 0; i < 4; ++i) r_f[set][i] = __float_as_uint(__uint_as_float(r_f[set][i]) * ws);
    };
    if (jb0 < jb1) {
      next_weight();
      weigh(0);
      sf_stage = sf_second;
#pragma unroll
      for (int c = 0; c < 8; ++c) stage_column(c, 0);
#pragma unroll
      for (int k = 0; k < kBtPieces; ++k) *reinterpret_cast<u32x4 *>(&sBt[0][lds_bt[k]]) = r_bt[k];
#pragma unroll
      for (int k = 0; k < kBtPieces; ++k) r_bt[k] = r_bt_second[k];
      wait_all_loads();  // (everything so far is needed by now: nothing is lost)
      load_part(0, at(jb0 + 2), 0);
    }
    __syncthreads();
    auto body = [&](int par, int jb) __attribute__((always_inline)) {
      const int buf = par, set = par ^ 1;  // block jb sits in LDS buffer `par`; block jb+1 in register set par^1
      const uint16_t *const tBt = sBt[buf];
      next_weight();                          // weight of block jb+1 from the factors fetched an iteration ago
      sf_stage = load_factors(at(jb + 2));    // for the next iteration
      // This pass is bound by its LDS operand reads (without them it takes half the time), so its two
      // waves per head split the state differently from the full kernel: wave `ph` owns state columns
      // [64 ph, 64 ph + 64) for all 64 headdim columns -- two n tiles x two column tiles, 2 + 2 operand
      // reads per group of four matrix instructions where four n tiles x one column tile need 4 + 1.
      // (Staging is unchanged: wave `ph` stages headdim half `ph` of Xm^T; the other half comes from the
      // head's other wave, through the barrier that every block has anyway -- and since that wave may
      // already be staging the next block while this one still reads, Xm^T has two copies in this pass.)
      Operand xo[4][2], bto[4][2];
      const uint16_t *const headX = sXm[buf * HPW + hw];  // block jb's copy; the next block is staged into the other
      auto request = [&](int q) __attribute__((always_inline)) {
#pragma unroll
        for (int pt = 0; pt < 2; ++pt) xo[q][pt] = lds16(headX + (32 * pt + r) * kXStride + 16 * q + 8 * kg);
#pragma unroll
        for (int nt = 0; nt < 2; ++nt) bto[q][nt] = lds16(tBt + a_bt + 32 * (2 * ph + nt) * kBtStride + 16 * q);
      };
      // Hacc[2 pt + nt]: headdim columns 32 pt + pi(r), state columns 32 (2 ph + nt) + row of the element
      auto multiply = [&](int q) __attribute__((always_inline)) {
#pragma unroll
        for (int pt = 0; pt < 2; ++pt)
#pragma unroll
          for (int nt = 0; nt < 2; ++nt) Hacc[2 * pt + nt] = mfma(bto[q][nt], xo[q][pt], Hacc[2 * pt + nt]);
      };
      // The two waves of a SIMD (w and w + 4) take the two halves of an iteration in opposite order: while
      // one reads its operands and keeps the matrix pipe busy, the other stages the next block on the vector
      // ALU.  Both halves only need what the barrier at the end of the previous iteration has published
      // (the matrix half reads LDS copy `buf`, the staging half writes copy `buf ^ 1`), so their order is
      // free; with every wave in the same half at the same time the pipes would take turns idling.
      auto matrix_half = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int q = 0; q < 4; ++q) request(q);
#pragma unroll
        for (int q = 0; q < 4; ++q) multiply(q);
      };
      const bool matrix_first = wave < 4;
      if (matrix_first) matrix_half();
      __builtin_amdgcn_sched_barrier(0);
      // the next block is staged, then its registers are refilled (tile of block jb+2, x of block jb+3)
      weigh(set);
#pragma unroll
      for (int c = 0; c < 8; ++c) stage_column(c, set, buf ^ 1);
#pragma unroll
      for (int k = 0; k < kBtPieces; ++k) *reinterpret_cast<u32x4 *>(&sBt[buf ^ 1][lds_bt[k]]) = r_bt[k];
      load_part(1, at(jb + 2));
      load_part(0, at(jb + 3), set);
      __builtin_amdgcn_sched_barrier(0);
      if (!matrix_first) matrix_half();
      __syncthreads();
    };
    // pairs of blocks, then the odd one: with the test between the two halves of a pair the compiler
    // would also have to allow for "first half, then first half again", where the set staged at the
    // top has only just been requested, and would wait for the newest loads in every iteration
    int jb = jb0;
    for (; jb + 1 < jb1; jb += 2) {
      body(0, jb);
      body(1, jb + 1);
    }
    if (jb < jb1) body(0, jb);
  }
  if constexpr (!kStatesOnly) {
    auto at = [&](int j) { return min(j, jlast); };
    if (jb0 < jb1) {
      // ---- prologue: block jb0 into LDS buffer 0; blocks jb0+1 and jb0+2 in flight ----
#pragma unroll
      for (int part = 0; part < 3; ++part) load_part(part, jb0, 0);
    }
    // The entering state into the accumulators: every wave turns its 32 x 128 tile, half at a time, through
    // a private piece of LDS (waves 0-3 in what will be the B^T buffers, waves 4-7 in the C buffers; rows of
    // 64 state columns padded by 16 bytes).  The barrier hands those buffers over to the staging below.
    if (has_state) {
      constexpr int kTurnStride = 64 + 4;  // floats
      float *const turn = reinterpret_cast<float *>(wave < 4 ? &sBt[0][0] : &sC[0][0]) + (wave & 3) * (32 * kTurnStride);
#pragma unroll
      for (int half = 0; half < 2; ++half) {
#pragma unroll
        for (int k = 0; k < 8; ++k)
          *reinterpret_cast<u32x4 *>(turn + (4 * k + (lane >> 4)) * kTurnStride + 4 * (lane & 15)) = hraw[8 * half + k];
#pragma unroll
        for (int nt = 0; nt < 2; ++nt)
#pragma unroll
          for (int i4 = 0; i4 < 4; ++i4) {
            const f32x4 v = *reinterpret_cast<const f32x4 *>(turn + pi_of_row(r) * kTurnStride + 32 * nt + 8 * i4 + 4 * kg);
            Hacc[2 * half + nt][4 * i4 + 0] = v.x;
            Hacc[2 * half + nt][4 * i4 + 1] = v.y;
            Hacc[2 * half + nt][4 * i4 + 2] = v.z;
            Hacc[2 * half + nt][4 * i4 + 3] = v.w;
          }
      }
      if (p.fold && sg >= 1) {
        // What was loaded is the local end state of the piece that ends where this segment begins; the
        // earlier pieces' (slots sg parts - 1 .. 1) and h0 follow, one at a time through the same registers,
        // each weighted by the decay of everything after it.  (Uniform over the workgroup.)
        float log2_decay = 0.f;
        for (int k = sg * p.parts - 1; k >= 0; --k) {
          log2_decay += p.seg_decay[slot0 + k];
          if (k == 0 && p.h0 == nullptr) break;
          const float *base = k > 0 ? p.Hin + (slot0 + k) * (kP * kN) : p.h0 + bh * kP * p.ns.width + p.ns.off;
          const uint32_t trow = k > 0 ? kN : static_cast<uint32_t>(p.ns.width);
          const uint32_t tvalid = k > 0 ? kN : static_cast<uint32_t>(p.ns.valid);
          const Rsrc rs_t = make_rsrc(base, ((kP - 1) * trow + tvalid) * 4u);
          const float wgt = fast_exp2(log2_decay);
#pragma unroll
          for (int i = 0; i < 16; ++i) {
            const uint32_t row = 32 * ph + 4 * (i & 7) + (lane >> 4), n0 = 64 * (i >> 3) + 4 * (lane & 15);
            hraw[i] = buf_load16(rs_t, n0 < tvalid ? (row * trow + n0) * 4u : 0xFFFFFF00u, 0);
          }
#pragma unroll
          for (int half = 0; half < 2; ++half) {
#pragma unroll
            for (int i = 0; i < 8; ++i)
              *reinterpret_cast<u32x4 *>(turn + (4 * i + (lane >> 4)) * kTurnStride + 4 * (lane & 15)) = hraw[8 * half + i];
#pragma unroll
            for (int nt = 0; nt < 2; ++nt)
#pragma unroll
              for (int i4 = 0; i4 < 4; ++i4) {
                const f32x4 v = *reinterpret_cast<const f32x4 *>(turn + pi_of_row(r) * kTurnStride + 32 * nt + 8 * i4 + 4 * kg);
                Hacc[2 * half + nt][4 * i4 + 0] += wgt * v.x;
                Hacc[2 * half + nt][4 * i4 + 1] += wgt * v.y;
                Hacc[2 * half + nt][4 * i4 + 2] += wgt * v.z;
                Hacc[2 * half + nt][4 * i4 + 3] += wgt * v.w;
              }
          }
        }
      }
      __syncthreads();
    } else {
#pragma unroll
      for (int nt = 0; nt < 4; ++nt)
#pragma unroll
        for (int i = 0; i < 16; ++i) Hacc[nt][i] = 0.f;
    }
    if (jb0 < jb1) {
#pragma unroll
      for (int c = 0; c < 8; ++c) stage_column(c, 0);
#pragma unroll
      for (int piece = 0; piece < 5; ++piece) stage_tile(piece, 0);
      if constexpr (!kRowStores) stage_raw(0);
      // the following blocks are requested in the order the loop requests blocks (shared tiles, own
      // slices, row factors): the compiler derives its waits from the order of outstanding loads,
      // and they stay exact only if the path into the loop and the path around it agree on it
      load_part(1, at(jb0 + 1));
      load_part(2, at(jb0 + 1));
      load_part(0, at(jb0 + 1), 1);
      if constexpr (!kRowStores) load_part(0, at(jb0 + 2), 0);
      load_rowf(jb0);
    }
    wait_all_loads();
    // Pin the two as "arrived": otherwise the wait for them is placed at their first use inside the
    // loop, where it also waits for every younger load of every iteration.
    asm volatile("" : "+v"(Dh));
    asm volatile("" : "+v"(pending));
    rowf0 = rowf0n;
    rowf1 = rowf1n;
    __syncthreads();

    // One block.  `par` is the parity of the block inside the segment, a compile-time constant (two
    // iterations are written out per loop trip): block jb sits in LDS buffer par, block jb+1 in
    // register set par^1 (it is staged during this iteration, and the set then refilled with block
    // jb+3), block jb+2 in register set par.
    // steep_tag: the block is steep (a compile-time constant per instantiation; the loop below picks the
    // instantiation block by block).  Both forms issue the same memory operations in the same order, so
    // the waits the compiler derives for the common form are not affected by the other.  The steep form
    // differs in four places: the state -> output term is scaled by exp2(cs_l) as soon as it is complete;
    // the masked product takes the raw x and, as its other operand, the scores times
    // dt_s exp2(cs_l - cs_s) -- the un-factorised mask, exponent never positive, applied in registers to
    // this lane's eight scores per operand; the state is taken to the end of the block before the update
    // (whose operand carries end-relative weights, see the record); the output rows need no factor.
    // In a mixed walk the factor owed to the accumulators at the end of the block depends on the form of
    // the next block.
    auto body = [&](int par, int jb, auto steep_tag) __attribute__((always_inline)) {
      constexpr bool kSteep = decltype(steep_tag)::value;
      static_assert(kMixed || !kSteep, "a steep block is only met in the mixed walk");
      float pend_next = 0.f;
      const int buf = par, setA = par ^ 1;
      const bool more = jb < jlast;
      f32x4 fac = {0.f, 0.f, 0.f, 0.f};  // record entries 128..131 of this block
      float nf = 0.f;                    // entry 130 of the next block
      const uint16_t *const tC = sC[buf], *const tG = sG[buf], *const tBt = sBt[buf];
      float dt_t = 0.f, cs_t = 0.f;      // steep: step size and inclusive prefix sum of dt*A*log2(e) of token `lane`
      if constexpr (kSteep) {
        const float alog = factor_ptr(jb)[3];
        dt_t = kg ? rowf1 : rowf0;
        cs_t = dt_t * alog;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
          const float up = __shfl_up(cs_t, off, 64);
          if (lane >= off) cs_t += up;
        }
      }

      if constexpr (kRowStores) {
        // the raw rows of this block go to LDS only now: until the barrier that ended the previous
        // iteration the other wave of the head was still reading the previous block's y from this
        // tile.  Then the register set is refilled with the block after next.
        stage_raw(par);
        load_part(0, at(jb + 2), par);
      }
      Operand xo[4];  // Xm^T[row r][s = 16q + 8kg ..]
      if constexpr (!kSteep) {
#pragma unroll
        for (int q = 0; q < 4; ++q) xo[q] = lds16(myX + r * kXStride + 16 * q + 8 * kg);
      }
      Operand bto[2][4];  // operands of the state update, double buffered over q
      f32x16 Y[2] = {};

      // ---- phase 1: Y^T[row][l] = sum_n Ht[row][n] C[l][n]  +  sum_{s<=l} Xm[s][row] G[l][s];
      //      alongside, the next block moves from registers to the other LDS buffer, and as soon as
      //      the registers of its shared tiles are free the tiles of block jb+2 are requested ----
      Operand co[2][2], go[2][2];
      co[0][0] = lds16(tC + a_c);
      co[0][1] = lds16(tC + a_c + 32 * kCStride);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int kk = 0; kk < 8; ++kk) {
        if (kk < 7) {
          co[(kk + 1) & 1][0] = lds16(tC + a_c + 16 * (kk + 1));
          co[(kk + 1) & 1][1] = lds16(tC + a_c + 32 * kCStride + 16 * (kk + 1));
        } else {
          go[0][1] = lds16(tG + a_g1);
          go[0][0] = lds16(tG + a_g0);
        }
        // bf16 copy of a 16-column slice of Ht as an MFMA operand: slice 2nt+u covers n = 32nt + 16u +
        // {4kg..4kg+3, 8+4kg..8+4kg+3} (the order in which sC stores each group of 16 columns)
        f32x16 &hv = Hacc[kk >> 1];
        const int u = kk & 1;
        Operand ho;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          hv[8 * u + 2 * k] *= pending;
          hv[8 * u + 2 * k + 1] *= pending;
          ho.u[k] = pack2(hv[8 * u + 2 * k], hv[8 * u + 2 * k + 1]);
        }
        Y[0] = mfma(ho, co[kk & 1][0], Y[0]);
        Y[1] = mfma(ho, co[kk & 1][1], Y[1]);
        if (kk < 5) stage_tile(kk, buf ^ 1);
        if (kk == 4) {
          load_rowf(at(jb + 1));
          if constexpr (kMixed) {
            fac = *reinterpret_cast<const f32x4 *>(factor_ptr(jb));
            nf = factor_ptr(at(jb + 1))[2];
          } else {
            // to the middle of the next block; after the last block only the way to its end is left
            pend_next = factor_ptr(jb)[more ? 3 : 0];
          }
        }
        if (kk == 5) load_part(1, at(jb + 2));
        if (kk == 6) load_part(2, at(jb + 2));
        // (steep: the state update is the only user of this block's scaled input, which the next block's
        // would overwrite here; it is staged after that update instead)
        if constexpr (!kSteep) stage_column(kk, setA);
        __builtin_amdgcn_sched_barrier(0);
      }
      // the masked product
      u32x4 xe;  // x of the block in output layout (token r + 32lt, columns 32ph + 16kg + 8c ..), read from
                 // the raw copy at the start of the group whose end uses it
      if constexpr (kSteep) {
        const float csl[2] = {__shfl(cs_t, r, 64), __shfl(cs_t, 32 + r, 64)};
        {
          const float s0 = fast_exp2(csl[0]), s1 = fast_exp2(csl[1]);
#pragma unroll
          for (int i = 0; i < 16; ++i) {
            Y[0][i] *= s0;
            Y[1][i] *= s1;
          }
        }
        const uint16_t *const xcol_src = myRaw + pi_of_row(r);  // this lane's column of the raw rows
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          float cs_s[8], dt_s[8];
          Operand xr;  // raw x^T[row r][s = 16q + 8kg ..]
#pragma unroll
          for (int j = 0; j < 8; ++j) {
            const int src = 16 * q + 8 * kg + j;
            cs_s[j] = __shfl(cs_t, src, 64);
            dt_s[j] = __shfl(dt_t, src, 64);
          }
#pragma unroll
          for (int k = 0; k < 4; ++k) {
            const uint32_t lo = xcol_src[(16 * q + 8 * kg + 2 * k) * kRawStride];
            const uint32_t hi = xcol_src[(16 * q + 8 * kg + 2 * k + 1) * kRawStride];
            xr.u[k] = lo | (hi << 16);
          }
#pragma unroll
          for (int lt = (q < 2 ? 0 : 1); lt < 2; ++lt) {
            const Operand gq = lds16(lt ? tG + a_g1 + 16 * q : tG + a_g0 + 16 * q);
            Operand gh;
#pragma unroll
            for (int k = 0; k < 4; ++k) {
              const float w0 = dt_s[2 * k] * fast_exp2(fminf(csl[lt] - cs_s[2 * k], 0.f));
              const float w1 = dt_s[2 * k + 1] * fast_exp2(fminf(csl[lt] - cs_s[2 * k + 1], 0.f));
              gh.u[k] = pack2(bf_lo(gq.u[k]) * w0, bf_hi(gq.u[k]) * w1);
            }
            Y[lt] = mfma(xr, gh, Y[lt]);
          }
        }
#pragma unroll
        for (int q = 0; q < 4; ++q) xo[q] = lds16(myX + r * kXStride + 16 * q + 8 * kg);
#pragma unroll
        for (int nt = 0; nt < 4; ++nt) bto[0][nt] = lds16(tBt + a_bt + 32 * nt * kBtStride);
        const float e63 = fast_exp2(fac.y);  // the state, so far at the start of the block, to its end
#pragma unroll
        for (int nt = 0; nt < 4; ++nt)
#pragma unroll
          for (int i = 0; i < 16; ++i) Hacc[nt][i] *= e63;
        __builtin_amdgcn_sched_barrier(0);
      }
#pragma unroll
      for (int q = 0; q < (kSteep ? 0 : 4); ++q) {
        if (q < 3) {
          go[(q + 1) & 1][1] = lds16(tG + a_g1 + 16 * (q + 1));
          if (q + 1 < 2) go[(q + 1) & 1][0] = lds16(tG + a_g0 + 16 * (q + 1));
        } else {
#pragma unroll
          for (int nt = 0; nt < 4; ++nt) bto[0][nt] = lds16(tBt + a_bt + 32 * nt * kBtStride);
        }
        if (q < 2) Y[0] = mfma(xo[q], go[q & 1][0], Y[0]);
        Y[1] = mfma(xo[q], go[q & 1][1], Y[1]);
        __builtin_amdgcn_sched_barrier(0);
      }

      // ---- phase 2: H'^T[n][col] = Ht^T[n][col] + sum_s B^T[n][s] Xm[s][col]; alongside, the output
      //      epilogue of the block (y[l][col] = rowf_l Y + D x; element i of the lane is column
      //      32ph + 16kg + i), one quarter per group ----
      const Rsrc ry = y_rsrc(jb);
      const float rowf[2] = {kSteep ? 1.f : rowf0, kSteep ? 1.f : rowf1};
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        if (q < 3) {
#pragma unroll
          for (int nt = 0; nt < 4; ++nt) bto[(q + 1) & 1][nt] = lds16(tBt + a_bt + 32 * nt * kBtStride + 16 * (q + 1));
        }
        xe = lds16(raw_src + 32 * (q >> 1) * kRawStride + 8 * (q & 1)).q;
#pragma unroll
        for (int nt = 0; nt < 4; ++nt) Hacc[nt] = mfma(bto[q & 1][nt], xo[q], Hacc[nt]);
        const int lt = q >> 1, c = q & 1;
        const f32x16 &Yt = Y[lt];
        const u32x4 xv = xe;
        u32x4 o;
#pragma unroll
        for (int w = 0; w < 4; ++w)
          o[w] = pack2(rowf[lt] * Yt[8 * c + 2 * w] + Dh * bf_lo(xv[w]),
                       rowf[lt] * Yt[8 * c + 2 * w + 1] + Dh * bf_hi(xv[w]));
        // the quarter replaces, in place, the x it was computed from: y leaves through the raw copy
        *reinterpret_cast<u32x4 *>(raw_rw + 32 * lt * kRawStride + 8 * c) = o;
        __builtin_amdgcn_sched_barrier(0);
      }

      // ---- y goes out in row layout, read back from LDS: the output layout of the MFMA would give
      //      32-byte pieces, which the memory system handles much worse next to the concurrent reads of
      //      x than 64-byte half rows, and those worse than whole 128-byte rows.  For whole rows the
      //      two waves of a head wait for each other's halves (the barrier below) and each stores the
      //      rows of 32 tokens; the raw rows of the next block then go to LDS at the top of the next
      //      iteration instead of here.  Tokens beyond the sequence are beyond the descriptor and are
      //      dropped. ----
      if constexpr (kSteep) {
#pragma unroll
        for (int c = 0; c < 8; ++c) stage_column(c, setA);
      }
      u32x4 yprev[4];  // kYAdd: what y holds so far, requested before the barrier
      if constexpr (kYMode == kYAdd) {
#pragma unroll
        for (int k = 0; k < 4; ++k) yprev[k] = buf_load16(ry, vy + static_cast<uint32_t>(kRowStep * k) * xrow, 0);
      }
      if constexpr (kRowStores) __syncthreads();  // both halves of every row of y are in LDS
      {
        u32x4 yo[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) yo[k] = *reinterpret_cast<const u32x4 *>(raw_dst_row + kRowStep * k * kRawStride);
        if constexpr (kYMode == kYAdd) {
#pragma unroll
          for (int k = 0; k < 4; ++k)
#pragma unroll
            for (int w = 0; w < 4; ++w)
              yo[k][w] = pack2(bf_lo(yo[k][w]) + bf_lo(yprev[k][w]), bf_hi(yo[k][w]) + bf_hi(yprev[k][w]));
        }
#pragma unroll
        for (int k = 0; k < 4; ++k)
          buf_store16<kYMode == kYStream ? kStreamStore : 0>(ry, vy + static_cast<uint32_t>(kRowStep * k) * xrow, yo[k]);
      }
      if constexpr (!kRowStores) {
        stage_raw(setA);
        load_part(0, at(jb + 3), setA);
      }
      // The factor still owed to the accumulators: from the middle of this block (steep: from its end) to
      // the middle of the next block -- to its start if that one is steep; after the last block only the
      // way to its end is left.
      if constexpr (kMixed) {
        const bool next_steep = more && __builtin_amdgcn_readfirstlane(__float_as_int(nf)) < 0;
        if constexpr (kSteep)
          pending = more && !next_steep ? nf : 1.f;
        else
          pending = more && !next_steep ? fac.w : fac.x;
        steep_cur = next_steep;
      } else {
        pending = pend_next;
      }
      rowf0 = rowf0n;
      rowf1 = rowf1n;
      __syncthreads();  // block jb's tiles may be overwritten; block jb+1's tiles are visible
    };
    // pairs of blocks, then the odd one: with the test between the two halves of a pair the compiler
    // would also have to allow for "first half, then first half again", where the set staged at the
    // top has only just been requested, and would wait for the newest loads in every iteration
    if constexpr (!kMixed) {
      int jb = jb0;
      for (; jb + 1 < jb1; jb += 2) {
        body(0, jb, std::false_type{});
        body(1, jb + 1, std::false_type{});
      }
      if (jb < jb1) body(0, jb, std::false_type{});
    } else {
      auto step = [&](int par, int jb) __attribute__((always_inline)) {
        if (steep_cur)
          body(par, jb, std::true_type{});
        else
          body(par, jb, std::false_type{});
      };
      int jb = jb0;
      for (; jb + 1 < jb1; jb += 2) {
        step(0, jb);
        step(1, jb + 1);
      }
      if (jb < jb1) step(0, jb);
    }
  }
  if constexpr (!kStatesOnly) {
#pragma unroll
    for (int nt = 0; nt < 4; ++nt)
#pragma unroll
      for (int i = 0; i < 16; ++i) Hacc[nt][i] *= pending;
  }

  // ---- write the state out (canonical (p, n) layout, four consecutive n per 16-byte store) ----
  if constexpr (kStatesOnly) {
    // (this pass tiles the state differently, see its loop body: tile 2 pt + nt of wave ph)
    // In the accumulators a lane holds 16-byte pieces of 32 different state rows: stored as they are, every
    // store instruction would touch 32 rows, 32 bytes each (measured: 5 us of the pass at 16384 tokens x 80
    // heads, 6.6 of 17 at 2048 x 24).  The wave turns its tile through a private piece of LDS instead -- the
    // tiles there are dead after the loop's last barrier -- half at a time (32 headdim columns x 64 state
    // columns, rows padded by 16 bytes), and stores four whole 256-byte row segments per instruction.  One
    // wave, one piece of LDS, in-order LDS operations: no barrier.
    if (live) {
      constexpr int kTurnStride = 64 + 4;  // floats
      static_assert(2 * HPW * 32 * kTurnStride * sizeof(float) <= L::kXmBufs * HPW * L::kXmElems * sizeof(uint16_t),
                    "the waves' turning tiles fit where Xm^T was");
      float *const turn = reinterpret_cast<float *>(&sXm[0][0]) + wave * (32 * kTurnStride);
      float *slot = p.seg_state + (slot0 + sg + 1) * (kP * kN);
#pragma unroll
      for (int pt = 0; pt < 2; ++pt) {
#pragma unroll
        for (int nt = 0; nt < 2; ++nt)
#pragma unroll
          for (int i4 = 0; i4 < 4; ++i4) {
            const f32x16 &t = Hacc[2 * pt + nt];
            *reinterpret_cast<f32x4 *>(turn + pi_of_row(r) * kTurnStride + 32 * nt + 8 * i4 + 4 * kg) =
                f32x4{t[4 * i4 + 0], t[4 * i4 + 1], t[4 * i4 + 2], t[4 * i4 + 3]};
          }
#pragma unroll
        for (int k = 0; k < 8; ++k) {
          const int row = 4 * k + (lane >> 4), piece = lane & 15;
          *reinterpret_cast<f32x4 *>(slot + static_cast<size_t>(32 * pt + row) * kN + 64 * ph + 4 * piece) =
              *reinterpret_cast<const f32x4 *>(turn + row * kTurnStride + 4 * piece);
        }
      }
      if (lane == 0 && ph == 0) p.seg_decay[slot0 + sg] = seg_total;
    }
  } else if (sg == sv.S - 1 && live) {
    // The same turn for the final state of the full kernel (a wave owns 32 headdim columns x 128 state
    // columns there: two halves of 64 state columns).  Waves 0-3 turn their tiles in what was the B^T
    // buffers, waves 4-7 in the C buffers; every wave is past the loop's last barrier.
    constexpr int kTurnStride = 64 + 4;  // floats
    static_assert(4 * 32 * kTurnStride * sizeof(float) <= 2 * L::kBtElems * sizeof(uint16_t) &&
                      4 * 32 * kTurnStride * sizeof(float) <= L::kCBufs * L::kCElems * sizeof(uint16_t),
                  "four turning tiles fit in either buffer pair");
    float *const turn = reinterpret_cast<float *>(wave < 4 ? &sBt[0][0] : &sC[0][0]) + (wave & 3) * (32 * kTurnStride);
    float *const rows = p.final_state + (bh * kP + 32 * ph) * p.ns.width + p.ns.off;
    const int valid = p.ns.valid;
#pragma unroll
    for (int half = 0; half < 2; ++half) {
#pragma unroll
      for (int nt = 0; nt < 2; ++nt)
#pragma unroll
        for (int i4 = 0; i4 < 4; ++i4) {
          const f32x16 &t = Hacc[2 * half + nt];
          *reinterpret_cast<f32x4 *>(turn + pi_of_row(r) * kTurnStride + 32 * nt + 8 * i4 + 4 * kg) =
              f32x4{t[4 * i4 + 0], t[4 * i4 + 1], t[4 * i4 + 2], t[4 * i4 + 3]};
        }
#pragma unroll
      for (int k = 0; k < 8; ++k) {
        const int row = 4 * k + (lane >> 4), n0 = 64 * half + 4 * (lane & 15);
        if (n0 < valid)
          *reinterpret_cast<f32x4 *>(rows + static_cast<size_t>(row) * p.ns.width + n0) =
              *reinterpret_cast<const f32x4 *>(turn + row * kTurnStride + 4 * (lane & 15));
      }
    }
  }
}

// The mixed walk as a function of its own: it is compiled, and its registers are allocated, apart from
// the kernel around the call, so what the rare steep form needs (it spills) costs the common walk nothing.
// (Arguments by value: a reference would make the kernel keep its own copy in private memory, where
// nothing counts as uniform any more.)
template <int HPW, int kYMode>
__device__ __attribute__((noinline)) void scan_walk_mixed(const ScanParams p, const SeqView sv, const LdsTiles lds) {
  scan_walk<false, HPW, kYMode, true>(p, sv, lds);
}

// Whether the blocks this wave walks in the full scan include a steep one: one lane per block reads the
// marker of its record.
template <int HPW>
__device__ __forceinline__ bool walk_meets_steep_block(const ScanParams &p, const SeqView &sv) {
  const int lane = threadIdx.x & 63;
  const int slot = (sv.col % p.cpg) * HPW + (static_cast<int>(threadIdx.x) >> 7);
  const int h = (sv.col / p.cpg) * p.hpg + min(slot, p.hpg - 1);
  const int hrec = h / p.pdiv;
  const bool plain = p.vp.tok0 == nullptr;
  const size_t rec0 = plain ? (sv.blk0 * p.Hrec + static_cast<size_t>(hrec) * sv.blk_stride) : (hrec * sv.blk_stride + sv.blk0);
  const int jb0 = min(sv.nb, sv.sg * p.seg_blocks), jb1 = min(sv.nb, jb0 + p.seg_blocks);
  const float *marks = p.prep + rec0 * kRec + 2 * kBlk + 2;
  float lowest = 1.f;
  for (int j = jb0; j < jb1; j += 64)
    if (j + lane < jb1) lowest = fminf(lowest, marks[static_cast<size_t>(j + lane) * kRec]);
  return __builtin_amdgcn_ballot_w64(lowest < 0.f) != 0;
}

template <bool kStatesOnly, int HPW, int kYMode = kYPlain>
__global__ __launch_bounds__(128 * HPW) __attribute__((amdgpu_waves_per_eu(2, 2)))
void chunk_scan_kernel(const ScanParams p) {
  using L = ScanLds<kStatesOnly, HPW>;
  __shared__ __align__(16) uint16_t sC[L::kCBufs][L::kCElems];
  __shared__ __align__(16) uint16_t sBt[2][L::kBtElems];
  __shared__ __align__(16) uint16_t sG[L::kGBufs][L::kGElems];
  __shared__ __align__(16) uint16_t sXm[L::kXmBufs * HPW][L::kXmElems];
  __shared__ __align__(16) uint16_t sRaw[L::kRawBufs][L::kRawElems];
  SeqView sv;
  if (!wg_coords(p, !kStatesOnly, sv)) return;  // uniform over the workgroup
  const LdsTiles lds = {(lds_u16 *)&sC[0][0], (lds_u16 *)&sBt[0][0], (lds_u16 *)&sG[0][0], (lds_u16 *)&sXm[0][0],
                        (lds_u16 *)&sRaw[0][0]};
  if constexpr (!kStatesOnly) {
    // Waves of one workgroup may take different walks: both stage the same shared tiles and meet at the
    // same barriers, block for block.
    if (walk_meets_steep_block<HPW>(p, sv)) {
      scan_walk_mixed<HPW, kYMode>(p, sv, lds);
      return;
    }
  }
  scan_walk<kStatesOnly, HPW, kYMode, false>(p, sv, lds);
}

// ---- segment_pass: slot[0] = h0; slot[sg] = exp2(decay[sg-1]) * slot[sg-1] + local[sg-1] --------
// grid (P*N/1024, rows <= sequences*H), four consecutive state elements per thread.  seg_state slot sg (sg >= 1)
// holds the local end state of segment sg-1 on entry and the state entering segment sg on exit.
// The chain over segments is serial, but the loads do not depend on it: they are issued eight
// segments at a time (sixteen measured slower) before the chain consumes them, so the kernel pays a few memory round trips
// instead of one per segment.
__global__ __launch_bounds__(kThreads) void segment_pass_kernel(float *__restrict__ seg_state,
                                                                const float *__restrict__ seg_decay,
                                                                const float *__restrict__ h0, int S_plain, int H,
                                                                int rows, const VarPlan vp, const NSlice ns) {
  constexpr int kAhead = 8;
  const int e = (blockIdx.x * kThreads + threadIdx.x) * 4;
  if (vp.tok0 != nullptr && vp.slot0[vp.nseq] == 0) return;  // no sequence has more than one segment
  for (size_t bh = blockIdx.y; bh < static_cast<size_t>(rows); bh += gridDim.y) {  // (sequence, head)
  int S = S_plain;
  size_t slot0 = bh * S_plain;
  if (vp.tok0 != nullptr) {
    const int q = static_cast<int>(bh / H), h = static_cast<int>(bh % H);
    const int first = vp.item0[q];
    S = vp.item0[q + 1] - first;
    slot0 = static_cast<size_t>(h) * vp.slot_cap + vp.slot0[q];
  }
  if (S < 2) continue;  // a single segment starts from h0 itself
  f32x4 run = {0.f, 0.f, 0.f, 0.f};
  if (h0 && e % kN < ns.valid)  // h0 rows hold ns.width columns, of which this launch owns a slice
    run = *reinterpret_cast<const f32x4 *>(h0 + (bh * kP + e / kN) * ns.width + ns.off + e % kN);
  float *sp = seg_state + slot0 * (kP * kN) + e;
  const float *dp = seg_decay + slot0;
  *reinterpret_cast<f32x4 *>(sp) = run;
  for (int s0 = 1; s0 < S; s0 += kAhead) {
    f32x4 v[kAhead];
    float d[kAhead];
#pragma unroll
    for (int k = 0; k < kAhead; ++k) {
      const int sg = min(s0 + k, S - 1);  // clamped: the surplus loads of the last group are not used
      v[k] = *reinterpret_cast<const f32x4 *>(sp + static_cast<size_t>(sg) * kP * kN);
      d[k] = dp[sg - 1];
    }
#pragma unroll
    for (int k = 0; k < kAhead; ++k) {
      if (s0 + k < S) {
        const float f = fast_exp2(d[k]);
        run = f32x4{f * run.x + v[k].x, f * run.y + v[k].y, f * run.z + v[k].z, f * run.w + v[k].w};
        *reinterpret_cast<f32x4 *>(sp + static_cast<size_t>(s0 + k) * kP * kN) = run;
      }
    }
  }
  }
}

// Blocks per segment.  A segment is any whole number of 64-token blocks; the number of segments, and
// with it the workspace, is bounded by max_segments (plain batch) or by one segment per chunk (packed
// batch).  The
// choice minimises a small cost model fitted to measurements on MI355X (microseconds): one workgroup
// per CU is resident, workgroups run in rounds of 256, a workgroup walks its blocks (plus a prologue
// worth about two) at a per-block time that grows with the number of workgroups competing for
// memory, and more than one segment costs the states pass (same structure, cheaper blocks), the
// serial pass over segment states (traffic proportional to segments x sequences) and two launches.
// The constants are a least-squares fit to 31 timed (shape, segment length) points of the three
// bf16 benchmark shapes (residual 5 us rms).
// The test-only knobs (see Knobs) force chunks or blocks per segment, and pieces per segment in the
// states-only pass.
constexpr int kNumCUs = 256;
double rounds_time(long wgs, double blocks, double t_idle, double t_busy) {
  double t = 0.0;
  for (long left = wgs; left > 0; left -= kNumCUs) {
    const double n = static_cast<double>(left < kNumCUs ? left : kNumCUs);
    const double load = n / kNumCUs;
    t += (blocks + 1.9) * (t_idle + (t_busy - t_idle) * load);
  }
  return t;
}
// Most segments a plain batch may be cut into (the workspace holds one state slot per segment and
// head): one per chunk, or -- short prompts, few heads -- one per block as long as that does not
// exceed what fills the chip several times over; and never more than fill the chip four times over
// (at least 64), which keeps the workspace of a very long prompt small: the choice below would not
// take more anyway.
// Workgroups of four head slots per batch row and segment: every B/C group has ceil(slices per group / 4).
int head_groups(const Dims &d) { return d.G * ((d.hpg * (d.P / kP) + kHeadsPerWg - 1) / kHeadsPerWg); }
int max_segments(const Dims &d) {
  const int nblocks = (d.T + kBlk - 1) / kBlk;
  const long groups = static_cast<long>(d.Bt) * head_groups(d);
  long by_fill = (8L * kNumCUs + groups - 1) / groups;
  if (by_fill > 64) by_fill = 64;
  if (by_fill > nblocks) by_fill = nblocks;
  long most = (4L * kNumCUs + groups - 1) / groups;
  if (most < 64) most = 64;
  long s = d.Nc > by_fill ? d.Nc : by_fill;
  if (s > most) s = most;
  return static_cast<int>(s);
}
// Modelled time of the states-only pass plus the chain over state slots when each of the S - 1
// segments it covers is cut into k pieces (see ScanParams::parts); the best k among the divisors of
// the segment length, at most max_slots slots.  max_parts = 1: segments are not cut.
double states_cost(long groups, double seqs, int S, int seg_blocks, int max_slots, int max_parts, int *parts) {
  double best = 0.0;
  *parts = 1;
  for (int k = 1; k <= max_parts && k <= seg_blocks; ++k) {
    if (seg_blocks % k != 0 || (k > 1 && (S - 1) * k + 1 > max_slots)) continue;
    const double cost = rounds_time(groups * (S - 1) * k, seg_blocks / k, 1.16, 1.16) + 0.0261 * ((S - 1) * k + 1) * seqs;
    if (k == 1 || cost < best) {
      best = cost;
      *parts = k;
    }
  }
  return best;
}

// min_blocks: the shortest segment allowed (packed batches size their tables for whole chunks).
constexpr double kColdXBytes = 144.0 * 1024 * 1024;  // x above this does not survive in the memory-side cache
int choose_seg_blocks(const Dims &d, int min_blocks, int max_slots, int max_parts) {
  const int chunk_blocks = d.L / kBlk;
  const int nblocks = (d.T + kBlk - 1) / kBlk;
  if (const int k = knobs().seg_chunks; k >= 1) return (k > d.Nc ? d.Nc : k) * chunk_blocks;
  if (const int k = knobs().seg_blocks; k >= min_blocks && k >= 1) return k;
  const int slices = d.H * (d.P / kP);
  const long groups = static_cast<long>(d.Bt) * head_groups(d);
  const double seqs = static_cast<double>(d.Bt) * slices;
  const int hi = nblocks > min_blocks ? nblocks : min_blocks;
  int best_blocks = hi;
  double best = 0.0;
  bool have = false;
  // The states pass leaves the x it has read -- every segment but the last of each sequence -- in the
  // memory-side cache, where the full scan finds it again; the last segment's x comes from HBM if the
  // tensor is too large to have stayed there from whoever wrote it, at a measured 1.25 times the per-block
  // time.  Segments somewhat longer than the count needs, leaving a shorter last one, even that out (8 x
  // 4096 tokens x 48 heads: 168 us with 32 + 32 blocks, 161 with 36 + 28).
  const double x_bytes = static_cast<double>(d.Bt) * d.T * d.H * d.P * 2.0;
  const double cold = x_bytes > kColdXBytes ? 1.25 : 1.0;
  for (int cand = min_blocks; cand <= hi; ++cand) {
    const long segs = (nblocks + cand - 1) / cand;
    const double last = static_cast<double>(nblocks - (segs - 1) * cand);
    const double walk = segs > 1 && cold * last > cand ? cold * last : cand;  // the longest walk, in warm blocks
    double cost = rounds_time(groups * segs, walk, 2.57, 3.35);
    int parts;
    if (segs > 1) {
      cost += states_cost(groups, seqs, static_cast<int>(segs), cand, max_slots, max_parts, &parts) + 3.1 + 7.0;
      // a short chain over state slots is summed by the full scan itself (see ScanParams::fold): no pass over
      // segment states and its launch, one more trip to memory per slot beyond the first instead (the net
      // saving measured on six shapes of 24 to 384 sequences: 2 to 11 us)
      if ((segs - 1) * parts <= knobs().fold_max_slots) cost -= 1.5 + 0.025 * seqs;
    }
    if (!have || cost < best) {
      have = true;
      best = cost;
      best_blocks = cand;
    }
  }
  return best_blocks;
}

// Workspace.  Plain batch: rows = Bt sequences of NB blocks each.  Variable-length batch: one "row" whose
// NB is the block capacity ceil(total / 64) + nseq (every sequence may end in a partial block), whose
// segment list holds at most NB / (blocks per chunk) + nseq + 1 entries (a segment is at least a
// chunk, and every sequence has at least one segment) and whose state slots -- needed only by
// sequences of several segments, which are longer than a segment and so cannot be many -- number at
// most min(that, 4 ceil(total / 64) / (blocks per chunk) + 4); then the int32 tables of VarPlan.
struct Layout {
  int NB, S_max, items_max;
  size_t off_G, off_Bt, off_prep, off_state, off_decay, off_tables, off_Cpad, total;
};

Layout make_layout(const Dims &d, bool varlen) {
  Layout w;
  const int rows = varlen ? 1 : d.Bt;
  const int nseq = varlen ? d.Bt : 0;
  w.NB = (d.T + kBlk - 1) / kBlk + nseq;
  const int cb = d.L / kBlk;  // a segment is at least one chunk
  w.items_max = varlen ? w.NB / cb + nseq + 1 : max_segments(d);
  w.S_max = w.items_max;      // state slots per head
  if (varlen) {
    const long tight = 4L * ((d.T + kBlk - 1) / kBlk) / cb + 4;
    if (tight < w.S_max) w.S_max = static_cast<int>(tight);
  }
  const size_t BG = static_cast<size_t>(rows) * d.G, BH = static_cast<size_t>(rows) * d.H;
  const size_t BHs = BH * (d.P / kP);  // 64-column slices
  size_t off = 0;
  w.off_G = off;
  off += round_up(BG * w.NB * kBlk * kBlk * sizeof(uint16_t), 256);
  w.off_Bt = off;
  off += round_up(BG * w.NB * kN * kBlk * sizeof(uint16_t), 256);
  w.off_prep = off;
  off += round_up(BH * w.NB * kRec * sizeof(float), 256);
  w.off_state = off;
  off += round_up(BHs * w.S_max * kP * kN * sizeof(float), 256);
  w.off_decay = off;
  off += round_up(BHs * w.S_max * sizeof(float), 256);
  w.off_tables = off;
  if (varlen) off += round_up((5 * (static_cast<size_t>(nseq) + 1) + w.NB + w.items_max) * sizeof(int32_t), 256);
  // dstate other than 128: a 128-column copy of the slice of C in work
  const size_t tokens = static_cast<size_t>(rows) * d.T;
  w.off_Cpad = off;
  if (d.N != kN) off += round_up(tokens * d.G * kN * sizeof(uint16_t), 256);
  w.total = off;
  return w;
}

bool shape_ok(const Dims &d, unsigned long long tokens, unsigned long long nb) {
  // one sequence of x, C and the per-head block records must be addressable with 32-bit byte offsets
  const unsigned long long lim = 0xFFFF0000ull;
  return d.bf16 && d.P % kP == 0 && d.P <= 16 * kP && d.N % 8 == 0 && d.N <= 4 * kN && d.Bt <= 65535 && d.H <= 65535 &&
         tokens * d.H * (static_cast<unsigned long long>(d.P) * 2) <= lim &&
         tokens * d.G * (static_cast<unsigned long long>(d.N > kN ? d.N : kN) * 2) <= lim &&
         nb * (kN * kBlk * 2) <= lim;
}

// Whether the full kernel writes y with non-temporal stores.  The 256 MiB memory-side cache (Infinity Cache)
// holds x when the kernel starts -- the states-only pass has just read it, or the producer (the convolution)
// has just written it -- unless the y written meanwhile pushes it out before it is read.  Once x takes more
// than a quarter of that cache, x and y no longer fit side by side and y is streamed past the caches.
// Measured (prefill alone, back to back; us with ordinary / non-temporal stores): x of 64-96 MiB 80 / 79, 62 / 62,
// 88 / 88 (no difference: below a quarter of the cache the consumer of y is better off finding it cached);
// 128 MiB 122 / 110 (two passes over x) and 109 / 97 (one); 160 MiB 151 / 131; 192 MiB 178 / 171 and 175 / 153;
// 256 MiB 220 / 211; 320 MiB 278 / 281 (nothing left to protect, nothing lost).  With a dstate above 128 the
// later state slices read y back to add to it, but they read x twice more: the first slice streams y all the
// same (dstate 256: 333 -> 307 us).  The y_stream knob overrides (tests, tuning).
constexpr unsigned long long kMemCacheBytes = 256ull << 20;
bool stream_y(const Dims &d, int rows) {
  if (knobs().y_stream >= 0) return knobs().y_stream != 0;
  const unsigned long long x_bytes = 2ull * rows * d.T * d.H * d.P;
  return 4 * x_bytes > kMemCacheBytes;
}

// d: plain batch (cu == nullptr), or Bt = number of sequences and T = total tokens of a packed batch.
// One state slice ns (see NSlice): y and final_state columns of that slice are written.
// How a call is cut up: blocks per segment, segments per sequence (0 for a packed batch, where the
// device-side tables hold them per sequence), pieces per segment of the states-only pass, and whether the
// full scan sums the chain over state slots itself (ScanParams::fold).
SlicePlan plan_slice(const Dims &d, bool varlen, bool h0_aliases_final_state) {
  const Layout w = make_layout(d, varlen);
  Dims one = d;  // the segment length of a packed batch is chosen as for one sequence of all its tokens
  if (varlen) one.Bt = 1;
  SlicePlan pl;
  // shortest segment: a chunk for a packed batch; what the state slots allow for a plain one
  pl.seg_blocks = choose_seg_blocks(one, varlen ? d.L / kBlk : (w.NB + w.S_max - 1) / w.S_max, w.S_max, varlen ? 1 : 8);
  if (!varlen && (w.NB + pl.seg_blocks - 1) / pl.seg_blocks > w.S_max) pl.seg_blocks = (w.NB + w.S_max - 1) / w.S_max;
  pl.segments = varlen ? 0 : (w.NB + pl.seg_blocks - 1) / pl.seg_blocks;
  // pieces per segment for the states-only pass (see ScanParams): the split with the least modelled
  // time of that pass plus the longer chain over state slots, among the divisors of the segment length
  pl.parts = 1;
  if (!varlen && pl.segments > 1) {
    const long groups = static_cast<long>(d.Bt) * head_groups(d);
    const double seqs = static_cast<double>(d.Bt) * d.H * (d.P / kP);
    (void)states_cost(groups, seqs, pl.segments, pl.seg_blocks, w.S_max, 8, &pl.parts);
    if (const int k = knobs().seg_parts; k >= 1 && pl.seg_blocks % k == 0 && (pl.segments - 1) * k + 1 <= w.S_max) pl.parts = k;
  }
  // A short chain over state slots is a sum of few terms (and h0), which the later segments' workgroups form
  // as they load their state -- one launch and one round trip of every state through memory less (8 x 4096
  // tokens x 48 heads: 162 -> 152 us).  Not when h0 and final_state share memory: the last segment might
  // store the final state before the first has read h0.
  pl.fold = !varlen && pl.segments >= 2 && (pl.segments - 1) * pl.parts <= knobs().fold_max_slots && !h0_aliases_final_state ? 1 : 0;
  return pl;
}

hipError_t launch_slice(const Dims &d, const NSlice ns, const int32_t *cu, const void *x, const float *dt,
                        const float *A, const void *B, const void *C, const float *D, const float *h0, void *y,
                        bool add_to_y, float *final_state, void *workspace, hipStream_t stream, KernelTrace *trace) {
  const bool varlen = cu != nullptr;
  const Layout w = make_layout(d, varlen);
  char *ws = static_cast<char *>(workspace);
  uint16_t *Gd = reinterpret_cast<uint16_t *>(ws + w.off_G);
  uint16_t *Btr = reinterpret_cast<uint16_t *>(ws + w.off_Bt);
  float *prep = reinterpret_cast<float *>(ws + w.off_prep);
  float *seg_state = reinterpret_cast<float *>(ws + w.off_state);
  float *seg_decay = reinterpret_cast<float *>(ws + w.off_decay);
  uint16_t *Cpad = d.N != kN ? reinterpret_cast<uint16_t *>(ws + w.off_Cpad) : nullptr;
  const int rows = varlen ? 1 : d.Bt;
  const size_t state_bytes = static_cast<size_t>(d.Bt) * d.H * d.P * ns.width * sizeof(float);
  const bool h0_aliases = h0 != nullptr && final_state != nullptr &&
                          reinterpret_cast<const char *>(h0) < reinterpret_cast<const char *>(final_state) + state_bytes &&
                          reinterpret_cast<const char *>(final_state) < reinterpret_cast<const char *>(h0) + state_bytes;
  const SlicePlan pl = plan_slice(d, varlen, h0_aliases);
  const int seg_blocks = pl.seg_blocks;

  VarPlan vp = {nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, 0, 0, 0};
  int S = (w.NB + seg_blocks - 1) / seg_blocks;  // plain batch: segments per sequence
  int items = S * d.Bt;                          // segments of the whole batch (varlen: upper bound)
  if (varlen) {
    int32_t *t = reinterpret_cast<int32_t *>(ws + w.off_tables);
    const int n1 = d.Bt + 1;
    int32_t *tok0 = t, *len = t + n1, *blk0 = t + 2 * n1, *item0 = t + 3 * n1, *slot0 = t + 4 * n1,
            *blk_seq = t + 5 * n1, *item_seq = blk_seq + w.NB;
    items = w.NB / seg_blocks + d.Bt + 1;
    if (items > w.items_max) items = w.items_max;
    S = 0;  // per sequence, from the tables
    vp = VarPlan{tok0, len, blk0, item0, slot0, blk_seq, item_seq, d.Bt, w.NB, w.S_max};
    if (!add_to_y) {  // (a later state slice finds the tables of the first)
      launch_varlen_tables(cu, d.T, kBlk, seg_blocks, items, vp, stream);
      trace_mark(trace, stream, "varlen_tables");
    }
  }

  const int n_scores = w.NB * rows * d.G;
  // (the decay records depend on dt and A alone: the first state slice has left them in the workspace)
  const int n_cumsum = add_to_y ? 0 : w.NB * ((d.H + kCumHeads - 1) / kCumHeads) * rows;
  hipLaunchKernelGGL(block_prep_kernel, dim3(n_scores + n_cumsum), dim3(kThreads), 0, stream,
                     static_cast<const uint16_t *>(B), static_cast<const uint16_t *>(C), Gd, Btr, dt, A, prep,
                     d.T, d.H, d.G, w.NB, n_scores, vp, ns, Cpad, d.dtx);
  trace_mark(trace, stream, "block_prep");

  ScanParams p;
  p.x = static_cast<const uint8_t *>(x);
  p.C = Cpad != nullptr ? reinterpret_cast<const uint8_t *>(Cpad) : static_cast<const uint8_t *>(C);
  p.D = D;
  p.ns = ns;
  p.Gd = reinterpret_cast<const uint8_t *>(Gd);
  p.Btr = reinterpret_cast<const uint8_t *>(Btr);
  p.prep = prep;
  p.y = static_cast<uint8_t *>(y);
  p.h0 = h0;
  p.Hin = seg_state;
  p.final_state = final_state;
  p.seg_state = seg_state;
  p.seg_decay = seg_decay;
  p.T = d.T;
  const int pdiv = d.P / kP, Hs = d.H * pdiv;
  p.H = Hs;
  p.pdiv = pdiv;
  p.Hrec = d.H;
  p.G = d.G;
  p.hpg = d.hpg * pdiv;
  p.cpg = (p.hpg + kHeadsPerWg - 1) / kHeadsPerWg;
  p.NB = w.NB;
  p.seg_blocks = seg_blocks;
  p.S = S;
  const int parts = pl.parts;
  p.parts = parts;
  p.part_blocks = seg_blocks / parts;
  p.slots = (S - 1) * parts + 1;
  p.vp = vp;
  p.fold = pl.fold;
  if (varlen || S > 1) {
    // (a packed batch always takes this route: whether any sequence has more than one segment is
    // known on the device only; workgroups of last segments leave the states-only pass at once)
    // heads per workgroup of the states-only kernel.  Two, with two workgroups per CU, measured with the current
    // loop: 40.0 against 35.8 us at 16384 tokens x 80 heads, 31.4 against 28.7 at 8 x 4096 x 48, 14.0 against
    // 15.6 at 2048 x 24 -- slower where it matters.
    constexpr int kStatesHeads = kHeadsPerWg;
    p.cols = d.G * p.cpg;
    p.segs = (S - 1) * parts;
    p.total = p.cols * p.segs * d.Bt;
    if (varlen) p.total = p.cols * items;
    p.per_xcd = (p.total + kXcds - 1) / kXcds;
    hipLaunchKernelGGL((chunk_scan_kernel<true, kStatesHeads>), dim3(kXcds * p.per_xcd), dim3(128 * kStatesHeads), 0,
                       stream, p);
    trace_mark(trace, stream, "segment_states");
    const int rows_bh = d.Bt * Hs;  // a packed batch may have many one-segment sequences: rows are looped over
    if (!p.fold)
      hipLaunchKernelGGL(segment_pass_kernel, dim3(kP * kN / (4 * kThreads), rows_bh > (varlen ? 2048 : 65535) ? (varlen ? 2048 : 65535) : rows_bh),
                         dim3(kThreads), 0, stream, seg_state, seg_decay, h0, p.slots, Hs, rows_bh, vp, ns);
    if (!p.fold) trace_mark(trace, stream, "segment_pass");
  }
  p.cols = d.G * p.cpg;
  p.segs = S;
  p.total = p.cols * p.segs * d.Bt;
  if (varlen) p.total = p.cols * items;
  p.per_xcd = (p.total + kXcds - 1) / kXcds;
  if (add_to_y)
    hipLaunchKernelGGL((chunk_scan_kernel<false, kHeadsPerWg, kYAdd>), dim3(kXcds * p.per_xcd), dim3(kScanThreads), 0,
                       stream, p);
  else if (stream_y(d, rows))
    hipLaunchKernelGGL((chunk_scan_kernel<false, kHeadsPerWg, kYStream>), dim3(kXcds * p.per_xcd), dim3(kScanThreads), 0,
                       stream, p);
  else
    hipLaunchKernelGGL((chunk_scan_kernel<false, kHeadsPerWg>), dim3(kXcds * p.per_xcd), dim3(kScanThreads), 0, stream,
                       p);
  trace_mark(trace, stream, "chunk_scan");
  return hipGetLastError();
}

// All state slices: the first writes y (with the skip term D x), every later one adds its output, without the
// skip term, to y where it stores it (the sum is formed in fp32 from the bf16 values and rounded once more:
// y carries up to 1.5 bf16 ulp with two slices instead of 0.5).
hipError_t launch(const Dims &d, const int32_t *cu, const void *x, const float *dt, const float *A, const void *B,
                  const void *C, const float *D, const float *h0, void *y, float *final_state, void *workspace,
                  hipStream_t stream, KernelTrace *trace) {
  for (int off = 0; off < d.N; off += kN) {
    const NSlice ns = {d.N, off, d.N - off < kN ? d.N - off : kN};
    const hipError_t e = launch_slice(d, ns, cu, x, dt, A, B, C, off == 0 ? D : nullptr, h0, y, off > 0, final_state,
                                      workspace, stream, off == 0 ? trace : nullptr);
    if (e != hipSuccess) return e;
  }
  return hipGetLastError();
}

}  // namespace

// Tables of a packed batch for blocks of blk_len tokens (the MFMA kernels: 64; the generic kernels:
// one chunk) and segments of seg_blocks blocks.  vp names the table arrays (device, int32: tok0, len,
// blk0, item0, slot0 of nseq + 1 entries each, blk_seq of nb_cap, item_seq of item_cap entries).
void launch_varlen_tables(const int32_t *cu, int total, int blk_len, int seg_blocks, int item_cap, const VarPlan &vp,
                          hipStream_t stream) {
  hipLaunchKernelGGL(varlen_scan_kernel, dim3(1), dim3(256), 0, stream, cu, vp.nseq, total, blk_len, seg_blocks,
                     const_cast<int32_t *>(vp.tok0), const_cast<int32_t *>(vp.len), const_cast<int32_t *>(vp.blk0),
                     const_cast<int32_t *>(vp.item0), const_cast<int32_t *>(vp.slot0));
  const int cap = vp.nb_cap > item_cap ? vp.nb_cap : item_cap;
  hipLaunchKernelGGL(varlen_fill_kernel, dim3((cap + 255) / 256), dim3(256), 0, stream, vp.blk0, vp.item0, vp.nseq,
                     seg_blocks, const_cast<int32_t *>(vp.blk_seq), const_cast<int32_t *>(vp.item_seq));
}

// The kernels work on 64-token blocks whatever the chunk length is (results do not depend on it); the chunk
// only bounds the number of segments, for which it counts as the next multiple of 64.
static Dims with_block_chunk(const Dims &d_in) {
  Dims d = d_in;
  d.L = (d.L + kBlk - 1) / kBlk * kBlk;
  d.Nc = (d.T + d.L - 1) / d.L;
  return d;
}

bool mfma_supported(const Dims &d) {
  return shape_ok(d, static_cast<unsigned long long>(d.T), (static_cast<unsigned long long>(d.T) + kBlk - 1) / kBlk);
}

size_t mfma_workspace_bytes(const Dims &d) { return make_layout(with_block_chunk(d), false).total; }

SlicePlan mfma_plan(const Dims &d, bool h0_aliases_final_state) {
  return plan_slice(with_block_chunk(d), false, h0_aliases_final_state);
}

hipError_t launch_prefill_mfma(const Dims &d, const void *x, const float *dt, const float *A, const void *B,
                               const void *C, const float *D, const float *h0, void *y, float *final_state,
                               void *workspace, hipStream_t stream, KernelTrace *trace) {
  return launch(with_block_chunk(d), nullptr, x, dt, A, B, C, D, h0, y, final_state, workspace, stream, trace);
}

// Packed variable-length batch: d.Bt sequences, d.T tokens in total, boundaries in the device array cu.
bool mfma_varlen_supported(const Dims &d) {
  const unsigned long long nb = (static_cast<unsigned long long>(d.T) + kBlk - 1) / kBlk + d.Bt;
  return shape_ok(d, static_cast<unsigned long long>(d.T), nb) && nb <= 0x7fffffffull / 64;
}

size_t mfma_varlen_workspace_bytes(const Dims &d) { return make_layout(with_block_chunk(d), true).total; }

hipError_t launch_prefill_mfma_varlen(const Dims &d, const int32_t *cu_seqlens, const void *x, const float *dt,
                                      const float *A, const void *B, const void *C, const float *D, const float *h0,
                                      void *y, float *final_state, void *workspace, hipStream_t stream,
                                      KernelTrace *trace) {
  return launch(with_block_chunk(d), cu_seqlens, x, dt, A, B, C, D, h0, y, final_state, workspace, stream, trace);
}

}  // namespace ssd
