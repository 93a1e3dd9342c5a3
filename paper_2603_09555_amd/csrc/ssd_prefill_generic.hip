// Generic fp32 prefill: the chunked SSD algorithm (Alg. 1; Eq. 3) for any shape and either
// io dtype, in plain fp32 vector arithmetic.  It is the path for shapes the MFMA kernels do
// not cover (and for fp32 inputs, whose 1e-4 tolerance bf16 matrix operands cannot meet).
//
// Four kernels, one per step of Alg. 1:
//   1. chunk_cumsum   cs[l] = inclusive prefix sum of dt*A inside each chunk   ("Discretise")
//   2. chunk_states   S_c = sum_s exp(cs_end - cs_s) dt_s x_s (x) B_s           ("State accumulate")
//   3. state_pass     H_{c+1} = exp(cs_end) H_c + S_c, sequential over chunks   ("Inter-chunk scan")
//   4. chunk_output   y = (C B^T o exp(segsum)) (dt o x) + exp(cs) C H_c + D x   ("Intra-chunk", "Combine")
// The decay mask exp(cs_l - cs_s), s <= l, is generated on the fly from the prefix sums and
// never stored; masked entries are set to zero without evaluating exp of a positive number.
#include "ssd_internal.hpp"

namespace ssd {
namespace {

constexpr int kThreads = 256;

// Where a chunk lives.  Plain batch: grid coordinates (chunk c of Nc, bh = b * H + h).  Packed
// variable-length batch (vp.tok0 != nullptr): the first coordinate counts chunks over the whole batch
// (every sequence has whole chunks of its own, the last one short), the second is the head; workspace
// arrays are then indexed (h, batch-wide chunk number) with vp.nb_cap chunks per head.
struct ChunkView {
  bool ok;        // false: the grid position is beyond the last chunk
  int h, len;     // head; tokens in the chunk
  size_t tok;     // first token (row of the (tokens, ...) arrays)
  size_t idx;     // index of the chunk in cs / states
};
__device__ __forceinline__ ChunkView chunk_view(int c, int bh, int T, int H, int L, int Nc, const VarPlan &vp) {
  ChunkView v;
  if (vp.tok0 == nullptr) {
    const int b = bh / H;
    v.ok = true;
    v.h = bh % H;
    v.len = min(L, T - c * L);
    v.tok = static_cast<size_t>(b) * T + static_cast<size_t>(c) * L;
    v.idx = static_cast<size_t>(bh) * Nc + c;
    return v;
  }
  v.ok = c < vp.blk0[vp.nseq];
  v.h = bh;
  v.len = 0;
  v.tok = 0;
  v.idx = 0;
  if (v.ok) {
    const int q = vp.blk_seq[c];
    const int cq = c - vp.blk0[q];
    v.len = min(L, vp.len[q] - cq * L);
    v.tok = static_cast<size_t>(vp.tok0[q]) + static_cast<size_t>(cq) * L;
    v.idx = static_cast<size_t>(bh) * vp.nb_cap + c;
  }
  return v;
}

// ---- 1. per-chunk inclusive prefix sum of dt*A ------------------------------------------------
// grid (Nc, Bt*H), one wave per chunk.  cs layout: (Bt, H, Nc, L).
__global__ __launch_bounds__(64) void chunk_cumsum_kernel(const float *__restrict__ dt,
                                                          const float *__restrict__ A,
                                                          float *__restrict__ cs, int T, int H, int L,
                                                          int Nc, const VarPlan vp) {
  const ChunkView cv = chunk_view(blockIdx.x, blockIdx.y, T, H, L, Nc, vp);
  if (!cv.ok) return;
  const int h = cv.h;
  const int lane = threadIdx.x;
  const float Ah = A[h];
  const int len = cv.len;
  float carry = 0.f;
  float *out = cs + cv.idx * L;
  for (int base = 0; base < len; base += 64) {
    const int l = base + lane;
    float v = 0.f;
    if (l < len) v = dt[(cv.tok + l) * H + h] * Ah;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
      const float up = __shfl_up(v, off, 64);
      if (lane >= off) v += up;
    }
    v += carry;
    if (l < len) out[l] = v;
    carry = __shfl(v, 63, 64);
  }
}

// ---- 2. chunk-end states -------------------------------------------------------------------
// grid (ceil(P/64)*ceil(N/64), Nc, Bt*H); each workgroup owns a 64x64 (p, n) tile, each thread a
// strided 4x4 micro-tile.  states layout: (Bt, H, Nc, P, N).
template <typename Io>
__global__ __launch_bounds__(kThreads) void chunk_states_kernel(
    const void *__restrict__ x, const float *__restrict__ dt, const void *__restrict__ B,
    const float *__restrict__ cs, float *__restrict__ states, int T, int H, int P, int N, int G,
    int hpg, int L, int Nc, const VarPlan vp) {
  __shared__ float Xs[32][64 + 1];
  __shared__ float Bs[32][64 + 1];
  const int ntn = (N + 63) / 64;
  const int p_base = (blockIdx.x / ntn) * 64;
  const int n_base = (blockIdx.x % ntn) * 64;
  const ChunkView cv = chunk_view(blockIdx.y, blockIdx.z, T, H, L, Nc, vp);
  if (!cv.ok) return;  // uniform over the workgroup
  const int h = cv.h, g = h / hpg;
  const int len = cv.len;
  const float *csc = cs + cv.idx * L;
  const float cs_end = csc[len - 1];
  const int tp = threadIdx.x / 16, tn = threadIdx.x % 16;
  float acc[4][4] = {};
  for (int s0 = 0; s0 < len; s0 += 32) {
    for (int i = threadIdx.x; i < 32 * 64; i += kThreads) {
      const int s = s0 + i / 64, col = i % 64;
      float xv = 0.f, bv = 0.f;
      if (s < len) {
        const size_t t = cv.tok + s;
        if (p_base + col < P) {
          const float w = expf(cs_end - csc[s]) * dt[t * H + h];
          xv = w * Io::load(x, (t * H + h) * P + p_base + col);
        }
        if (n_base + col < N) bv = Io::load(B, (t * G + g) * N + n_base + col);
      }
      Xs[i / 64][col] = xv;
      Bs[i / 64][col] = bv;
    }
    __syncthreads();
#pragma unroll 4
    for (int s = 0; s < 32; ++s) {
      float xv[4], bv[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        xv[i] = Xs[s][tp + 16 * i];
        bv[i] = Bs[s][tn + 16 * i];
      }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] += xv[i] * bv[j];
    }
    __syncthreads();
  }
  float *out = states + cv.idx * P * N;
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int p = p_base + tp + 16 * i, n = n_base + tn + 16 * j;
      if (p < P && n < N) out[static_cast<size_t>(p) * N + n] = acc[i][j];
    }
}

// ---- 3. sequential inter-chunk pass ------------------------------------------------------------
// grid (ceil(P*N/256), Bt*H); thread = one state element.  On return states[c] holds the state
// ENTERING chunk c, and final_state the state after the last chunk.
__global__ __launch_bounds__(kThreads) void state_pass_kernel(float *__restrict__ states,
                                                              const float *__restrict__ cs,
                                                              const float *__restrict__ h0,
                                                              float *__restrict__ final_state, int T, int H,
                                                              int PN, int L, int Nc, const VarPlan vp) {
  const int e = blockIdx.x * kThreads + threadIdx.x;
  const int bh = blockIdx.y;  // (sequence, head)
  if (e >= PN) return;
  // chunks of this sequence: count, length of the sequence, index of its first chunk in cs / states
  int nc = Nc, seq_len = T;
  size_t first = static_cast<size_t>(bh) * Nc;
  if (vp.tok0 != nullptr) {
    const int q = bh / H, h = bh % H;
    nc = vp.blk0[q + 1] - vp.blk0[q];
    seq_len = vp.len[q];
    first = static_cast<size_t>(h) * vp.nb_cap + vp.blk0[q];
    if (vp.item0[vp.nseq] == 0) return;  // rejected boundaries: empty tables, nothing is written
  }
  float run = h0 ? h0[static_cast<size_t>(bh) * PN + e] : 0.f;
  for (int c = 0; c < nc; ++c) {
    const int len = min(L, seq_len - c * L);
    const float decay = expf(cs[(first + c) * L + len - 1]);
    float *sp = states + (first + c) * PN + e;
    const float s = *sp;
    *sp = run;
    run = decay * run + s;
  }
  final_state[static_cast<size_t>(bh) * PN + e] = run;
}

// ---- 4. chunk output -------------------------------------------------------------------------
// grid (ceil(L/32)*ceil(P/64), Nc, Bt*H); each workgroup owns 32 rows l x 64 columns p of one
// head-chunk; each thread a strided 2x4 micro-tile.
template <typename Io>
__global__ __launch_bounds__(kThreads) void chunk_output_kernel(
    const void *__restrict__ x, const float *__restrict__ dt, const void *__restrict__ B,
    const void *__restrict__ C, const float *__restrict__ D, const float *__restrict__ cs,
    const float *__restrict__ states, void *__restrict__ y, int T, int H, int P, int N, int G, int hpg,
    int L, int Nc, const VarPlan vp) {
  __shared__ float Cs[32][32 + 1];   // C[l][n] tile
  __shared__ float Ts[64][32 + 1];   // H_c[p][n] tile, or B[s][n] tile (first 32 rows)
  __shared__ float Ms[32][32 + 1];   // masked, decayed scores M[l][s]
  __shared__ float Xs[32][64 + 1];   // x[s][p] tile
  __shared__ float cs_l[32], cs_s[32], dt_s[32];

  const int ntp = (P + 63) / 64;
  const int l_base = (blockIdx.x / ntp) * 32;
  const int p_base = (blockIdx.x % ntp) * 64;
  const ChunkView cv = chunk_view(blockIdx.y, blockIdx.z, T, H, L, Nc, vp);
  if (!cv.ok) return;  // uniform over the workgroup
  const int h = cv.h, g = h / hpg;
  const int len = cv.len;
  if (l_base >= len) return;
  const float *csc = cs + cv.idx * L;
  const size_t t0 = cv.tok;
  const int tl = threadIdx.x / 16, tp = threadIdx.x % 16;  // rows tl, tl+16; cols tp+16j

  if (threadIdx.x < 32) cs_l[threadIdx.x] = (l_base + threadIdx.x < len) ? csc[l_base + threadIdx.x] : 0.f;

  // ---- state -> output: acc = C[l,:] . H_c[p,:], then scaled by exp(cs_l) ----
  float acc[2][4] = {};
  const float *Hc = states + cv.idx * P * N;
  for (int n0 = 0; n0 < N; n0 += 32) {
    for (int i = threadIdx.x; i < 32 * 32; i += kThreads) {
      const int r = i / 32, n = n0 + i % 32;
      float v = 0.f;
      if (l_base + r < len && n < N) v = Io::load(C, ((t0 + l_base + r) * G + g) * N + n);
      Cs[r][i % 32] = v;
    }
    for (int i = threadIdx.x; i < 64 * 32; i += kThreads) {
      const int r = i / 32, n = n0 + i % 32;
      float v = 0.f;
      if (p_base + r < P && n < N) v = Hc[static_cast<size_t>(p_base + r) * N + n];
      Ts[r][i % 32] = v;
    }
    __syncthreads();
#pragma unroll 8
    for (int n = 0; n < 32; ++n) {
      const float c0 = Cs[tl][n], c1 = Cs[tl + 16][n];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const float hv = Ts[tp + 16 * j][n];
        acc[0][j] += c0 * hv;
        acc[1][j] += c1 * hv;
      }
    }
    __syncthreads();
  }
  {
    const float e0 = expf(cs_l[tl]), e1 = expf(cs_l[tl + 16]);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      acc[0][j] *= e0;
      acc[1][j] *= e1;
    }
  }

  // ---- intra-chunk: acc += sum_{s<=l} (C_l.B_s) exp(cs_l - cs_s) dt_s x[s,p] ----
  const int s_end = min(len, l_base + 32);  // causal: no column beyond the last row of this tile
  const int ml = threadIdx.x / 8, ms = (threadIdx.x % 8) * 4;  // score micro-tile: row ml, cols ms..ms+3
  for (int s0 = 0; s0 < s_end; s0 += 32) {
    if (threadIdx.x < 32) {
      const int s = s0 + threadIdx.x;
      cs_s[threadIdx.x] = (s < len) ? csc[s] : 0.f;
      dt_s[threadIdx.x] = (s < len) ? dt[(t0 + s) * H + h] : 0.f;
    }
    float sc[4] = {0.f, 0.f, 0.f, 0.f};
    for (int n0 = 0; n0 < N; n0 += 32) {
      for (int i = threadIdx.x; i < 32 * 32; i += kThreads) {
        const int r = i / 32, n = n0 + i % 32;
        float cv = 0.f, bv = 0.f;
        if (n < N) {
          if (l_base + r < len) cv = Io::load(C, ((t0 + l_base + r) * G + g) * N + n);
          if (s0 + r < len) bv = Io::load(B, ((t0 + s0 + r) * G + g) * N + n);
        }
        Cs[r][i % 32] = cv;
        Ts[r][i % 32] = bv;
      }
      __syncthreads();
#pragma unroll 8
      for (int n = 0; n < 32; ++n) {
        const float cv = Cs[ml][n];
#pragma unroll
        for (int j = 0; j < 4; ++j) sc[j] += cv * Ts[ms + j][n];
      }
      __syncthreads();
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int l = l_base + ml, s = s0 + ms + j;
      float m = 0.f;
      if (s <= l && l < len) m = sc[j] * expf(cs_l[ml] - cs_s[ms + j]) * dt_s[ms + j];
      Ms[ml][ms + j] = m;
    }
    for (int i = threadIdx.x; i < 32 * 64; i += kThreads) {
      const int r = i / 64, col = i % 64;
      float v = 0.f;
      if (s0 + r < len && p_base + col < P) v = Io::load(x, ((t0 + s0 + r) * H + h) * P + p_base + col);
      Xs[r][col] = v;
    }
    __syncthreads();
#pragma unroll 8
    for (int s = 0; s < 32; ++s) {
      const float m0 = Ms[tl][s], m1 = Ms[tl + 16][s];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const float xv = Xs[s][tp + 16 * j];
        acc[0][j] += m0 * xv;
        acc[1][j] += m1 * xv;
      }
    }
    __syncthreads();
  }

  // ---- skip connection and store ----
  const float Dh = D[h];
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int l = l_base + tl + 16 * i;
    if (l >= len) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int p = p_base + tp + 16 * j;
      if (p >= P) continue;
      const size_t idx = ((t0 + l) * H + h) * P + p;
      Io::store(y, idx, acc[i][j] + Dh * Io::load(x, idx));
    }
  }
}

// dt = clamp(softplus(raw + bias), lo, hi), written out once (the generic kernels read dt in three places).
__global__ __launch_bounds__(kThreads) void dt_transform_kernel(const float *__restrict__ raw, float *__restrict__ out,
                                                                size_t n, int H, const DtXform dtx) {
  const size_t i = static_cast<size_t>(blockIdx.x) * kThreads + threadIdx.x;
  if (i < n) out[i] = dt_apply(raw[i], static_cast<int>(i % H), dtx);
}

// A chunk longer than the sequence is one short chunk.
Dims clamp_chunk(Dims d) {
  if (d.L > d.T) d.L = d.T;
  d.Nc = (d.T + d.L - 1) / d.L;
  return d;
}

// rows: independent (sequence, head) pairs of the state pass; chunks: first grid coordinate of the
// per-chunk kernels (chunks per batch row, or the chunk capacity of a packed batch); heads_dim: their
// second coordinate (Bt * H, or H for a packed batch).
template <typename Io>
hipError_t launch_typed(const Dims &d, const VarPlan &vp, const void *x, const float *dt, const float *A, const void *B,
                        const void *C, const float *D, const float *h0, void *y, float *final_state,
                        float *cs, float *states, hipStream_t stream, KernelTrace *trace) {
  const bool varlen = vp.tok0 != nullptr;
  const unsigned rows = static_cast<unsigned>(d.Bt) * d.H;
  const unsigned chunks = varlen ? vp.nb_cap : d.Nc;
  const unsigned heads_dim = varlen ? d.H : rows;
  const int PN = d.P * d.N;

  hipLaunchKernelGGL(chunk_cumsum_kernel, dim3(chunks, heads_dim), dim3(64), 0, stream, dt, A, cs, d.T, d.H, d.L,
                     d.Nc, vp);
  trace_mark(trace, stream, "chunk_cumsum");
  const unsigned tiles_pn = ((d.P + 63) / 64) * ((d.N + 63) / 64);
  hipLaunchKernelGGL((chunk_states_kernel<Io>), dim3(tiles_pn, chunks, heads_dim), dim3(kThreads), 0, stream, x, dt,
                     B, cs, states, d.T, d.H, d.P, d.N, d.G, d.hpg, d.L, d.Nc, vp);
  trace_mark(trace, stream, "chunk_states");
  hipLaunchKernelGGL(state_pass_kernel, dim3((PN + kThreads - 1) / kThreads, rows), dim3(kThreads), 0, stream,
                     states, cs, h0, final_state, d.T, d.H, PN, d.L, d.Nc, vp);
  trace_mark(trace, stream, "state_pass");
  const unsigned tiles_lp = ((d.L + 31) / 32) * ((d.P + 63) / 64);
  hipLaunchKernelGGL((chunk_output_kernel<Io>), dim3(tiles_lp, chunks, heads_dim), dim3(kThreads), 0, stream, x, dt,
                     B, C, D, cs, states, y, d.T, d.H, d.P, d.N, d.G, d.hpg, d.L, d.Nc, vp);
  trace_mark(trace, stream, "chunk_output");
  return hipGetLastError();
}

// Workspace: cs (heads x chunks x L), chunk states (heads x chunks x P x N), a transformed copy of dt,
// and for a packed batch its int32 tables.  chunks = Nc per batch row, or ceil(T / L) + nseq.
struct GenLayout {
  size_t chunks, off_states, off_dt, off_tables, total;  // offsets in floats, total in bytes
};
GenLayout gen_layout(const Dims &d, bool varlen) {
  GenLayout w;
  const size_t heads = varlen ? d.H : static_cast<size_t>(d.Bt) * d.H;
  w.chunks = varlen ? static_cast<size_t>(d.Nc) + d.Bt : d.Nc;
  w.off_states = round_up(heads * w.chunks * d.L, 64);
  w.off_dt = w.off_states + heads * w.chunks * d.P * d.N;
  w.off_tables = w.off_dt + round_up((varlen ? 1 : static_cast<size_t>(d.Bt)) * d.T * d.H, 64);
  size_t fl = w.off_tables;
  if (varlen) fl += round_up(5 * (static_cast<size_t>(d.Bt) + 1) + 2 * w.chunks + d.Bt + 1, 64);
  w.total = round_up(fl * sizeof(float), 256);
  return w;
}

// dt through the optional transform, into the workspace copy.
const float *prepared_dt(const Dims &d, const GenLayout &w, size_t n, const float *dt, void *workspace,
                         hipStream_t stream) {
  if (d.dtx.identity()) return dt;
  float *copy = static_cast<float *>(workspace) + w.off_dt;
  hipLaunchKernelGGL(dt_transform_kernel, dim3(static_cast<unsigned>((n + kThreads - 1) / kThreads)), dim3(kThreads),
                     0, stream, dt, copy, n, d.H, d.dtx);
  return copy;
}

}  // namespace

size_t generic_workspace_bytes(const Dims &d_in) { return gen_layout(clamp_chunk(d_in), false).total; }

hipError_t launch_prefill_generic(const Dims &d_in, const void *x, const float *dt, const float *A,
                                  const void *B, const void *C, const float *D, const float *h0, void *y,
                                  float *final_state, void *workspace, hipStream_t stream,
                                  KernelTrace *trace) {
  const Dims d = clamp_chunk(d_in);
  const GenLayout w = gen_layout(d, false);
  dt = prepared_dt(d, w, static_cast<size_t>(d.Bt) * d.T * d.H, dt, workspace, stream);
  float *cs = static_cast<float *>(workspace), *states = cs + w.off_states;
  const VarPlan none = {nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, 0, 0, 0};
  return d.bf16 ? launch_typed<IoBf16>(d, none, x, dt, A, B, C, D, h0, y, final_state, cs, states, stream, trace)
                : launch_typed<IoF32>(d, none, x, dt, A, B, C, D, h0, y, final_state, cs, states, stream, trace);
}

// Packed variable-length batch: d.Bt sequences, d.T tokens in total.
size_t generic_varlen_workspace_bytes(const Dims &d_in) { return gen_layout(clamp_chunk(d_in), true).total; }

hipError_t launch_prefill_generic_varlen(const Dims &d_in, const int32_t *cu, const void *x, const float *dt,
                                         const float *A, const void *B, const void *C, const float *D,
                                         const float *h0, void *y, float *final_state, void *workspace,
                                         hipStream_t stream) {
  const Dims d = clamp_chunk(d_in);
  const GenLayout w = gen_layout(d, true);
  dt = prepared_dt(d, w, static_cast<size_t>(d.T) * d.H, dt, workspace, stream);
  float *cs = static_cast<float *>(workspace), *states = cs + w.off_states;
  int32_t *t = reinterpret_cast<int32_t *>(cs + w.off_tables);
  const int n1 = d.Bt + 1, cap = static_cast<int>(w.chunks);
  // blocks of the tables = chunks; "segments" of one chunk each (only their total is used: zero
  // marks rejected boundaries)
  const VarPlan vp = {t, t + n1, t + 2 * n1, t + 3 * n1, t + 4 * n1, t + 5 * n1, t + 5 * n1 + cap, d.Bt, cap, 0};
  launch_varlen_tables(cu, d.T, d.L, 1, cap + d.Bt + 1, vp, stream);
  return d.bf16 ? launch_typed<IoBf16>(d, vp, x, dt, A, B, C, D, h0, y, final_state, cs, states, stream, nullptr)
                : launch_typed<IoF32>(d, vp, x, dt, A, B, C, D, h0, y, final_state, cs, states, stream, nullptr);
}

}  // namespace ssd
