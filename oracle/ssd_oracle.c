/*
 * fp64 CPU oracle for the Mamba-2 SSD layer core.  TEST INFRASTRUCTURE ONLY.
 *
 * This file is the reference the GPU library is checked against.  It is plain,
 * slow and sequential on purpose: it evaluates the discrete state-space
 * recurrence of the paper (Eq. 2 in "State-space duality", specialised by the
 * Mamba-2 restriction stated right after it: one scalar A per head, B, C and
 * the step size dt depend on the token) one token at a time.  It never forms
 * chunks, prefix sums, decay matrices or masks, so it shares no structure and
 * no code with the chunked GPU path; the chunked method reaches the same
 * result up to rounding order, which is why the definition itself can serve
 * as the oracle.
 *
 * Only tests, the smoke check and the cpu_baseline leg of the benchmark may
 * call into this library.  The product path never does.
 *
 * Per token (Alg. 2 "Discretise" and "SSM step" lines, Eq. 2 for the output;
 * the sign convention -- A is the already negative per-head scalar -- and the
 * Euler form dt*B for the input matrix are readings listed in the design
 * notes):
 *     dA      = exp(dt_t * A)
 *     h[p][n] = dA * h[p][n] + (dt_t * x_t[p]) * B_t[n]
 *     y_t[p]  = sum_n C_t[n] * h[p][n]  +  D * x_t[p]       (updated h)
 *
 * Data model: the caller passes "pairs".  A pair is one (batch row, head)
 * sequence; pairs are independent (per-head scalar A, per-head state).  The
 * Python wrapper next to this file gathers pairs out of the tensor layouts
 * and maps each head to its B/C group.
 *
 * All arithmetic is IEEE double.  Build: gcc -O2 -fopenmp -shared -fPIC
 * (no -ffast-math: the summation order below is the documented one).
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

/* One token of one pair: the body shared by prefill and decode, so that a
 * decode step is literally one iteration of the prefill loop. */
static void ssd_token_step(int P, int N, double A, double D, double dt,
                           const double *x, /* [P]  */
                           const double *B, /* [N]  */
                           const double *C, /* [N]  */
                           double *h,       /* [P][N], updated in place */
                           double *y)       /* [P]  */
{
    const double dA = exp(dt * A);
    for (int p = 0; p < P; ++p) {
        const double u = dt * x[p];
        double *hp = h + (size_t)p * N;
        double acc = 0.0;
        for (int n = 0; n < N; ++n) {
            hp[n] = dA * hp[n] + u * B[n];
            acc += C[n] * hp[n];
        }
        y[p] = acc + D * x[p];
    }
}

/*
 * Sequential scan over T tokens for npairs independent sequences.
 *   x        [npairs][T][P]
 *   dt       [npairs][T]
 *   A, D     [npairs]
 *   bc_index [npairs]          row of B / C this pair reads
 *   B, C     [nbc][T][N]
 *   h0       [npairs][P][N] or NULL (zero initial state)
 *   y        [npairs][T][P]    (out)
 *   state    [npairs][P][N]    (out: state after the last token; == h0 if T==0)
 * Returns 0, or -1 on a null/negative argument.
 */
int ssd_oracle_scan(int npairs, int T, int P, int N, int nbc,
                    const double *x, const double *dt, const double *A,
                    const int32_t *bc_index, const double *B, const double *C,
                    const double *D, const double *h0, double *y, double *state,
                    int nthreads)
{
    if (npairs < 0 || T < 0 || P < 1 || N < 1 || nbc < 1) return -1;
    if (!A || !bc_index || !D || !state) return -1;
    if (T > 0 && (!x || !dt || !B || !C || !y)) return -1;
    for (int i = 0; i < npairs; ++i)
        if (bc_index[i] < 0 || bc_index[i] >= nbc) return -1;
#ifdef _OPENMP
    if (nthreads < 1) nthreads = omp_get_max_threads();
#else
    (void)nthreads;
#endif
#pragma omp parallel for schedule(dynamic, 1) num_threads(nthreads)
    for (int i = 0; i < npairs; ++i) {
        double *h = state + (size_t)i * P * N;
        if (h0)
            memcpy(h, h0 + (size_t)i * P * N, sizeof(double) * (size_t)P * N);
        else
            memset(h, 0, sizeof(double) * (size_t)P * N);
        const double *Bi = B + (size_t)bc_index[i] * T * N;
        const double *Ci = C + (size_t)bc_index[i] * T * N;
        for (int t = 0; t < T; ++t) {
            ssd_token_step(P, N, A[i], D[i], dt[(size_t)i * T + t],
                           x + ((size_t)i * T + t) * P, Bi + (size_t)t * N,
                           Ci + (size_t)t * N, h, y + ((size_t)i * T + t) * P);
        }
    }
    return 0;
}

/*
 * One cached decode step for npairs independent sequences: exactly one
 * iteration of the loop above on the caller's state.
 *   state [npairs][P][N] in/out;  x, y [npairs][P];  dt, A, D [npairs];
 *   B, C [nbc][N] indexed through bc_index.
 */
int ssd_oracle_step(int npairs, int P, int N, int nbc, double *state,
                    const double *x, const double *dt, const double *A,
                    const int32_t *bc_index, const double *B, const double *C,
                    const double *D, double *y, int nthreads)
{
    if (npairs < 0 || P < 1 || N < 1 || nbc < 1) return -1;
    if (!state || !x || !dt || !A || !bc_index || !B || !C || !D || !y) return -1;
    for (int i = 0; i < npairs; ++i)
        if (bc_index[i] < 0 || bc_index[i] >= nbc) return -1;
#ifdef _OPENMP
    if (nthreads < 1) nthreads = omp_get_max_threads();
#else
    (void)nthreads;
#endif
#pragma omp parallel for schedule(static) num_threads(nthreads)
    for (int i = 0; i < npairs; ++i) {
        ssd_token_step(P, N, A[i], D[i], dt[i], x + (size_t)i * P,
                       B + (size_t)bc_index[i] * N, C + (size_t)bc_index[i] * N,
                       state + (size_t)i * P * N, y + (size_t)i * P);
    }
    return 0;
}

/* Number of threads a call with nthreads<1 would use (for the benchmark's
 * "cores" field). */
int ssd_oracle_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
