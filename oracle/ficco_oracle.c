/*
 * CPU oracle for the all-gather -> GEMM pair (and the data-movement half of GEMM -> reduce-scatter).
 *
 * TEST INFRASTRUCTURE ONLY. Nothing in the product path may call this file; it shares no code,
 * header or table with the HIP library. It is deliberately plain and slow.
 *
 * What it computes (paper, Sec. II-B and Fig. 3(a)-(b): every GPU holds a row-slice I_j of the
 * activation and a column-slice W of the weight; the all-gather makes every I_j available, and the
 * GEMM multiplies the gathered activation by W). Decomposition and schedule (Sec. IV, Sec. V-B)
 * change *when* rows are computed, never the result, so the oracle is the definition itself:
 *
 *     A        = [I_0 ; I_1 ; ... ; I_{G-1}]                (row concatenation, shard order)
 *     ref[i,j] = sum_{k=0}^{K-1} (double)A[i,k] * (double)W[k,j]      (fp64, k ascending)
 *
 * Inputs are bf16 bit patterns (1 sign, 8 exponent, 7 mantissa bits); each is widened exactly to
 * fp64. A product of two bf16 values has at most 16 significant bits and is exact in fp64.
 *
 * Build: gcc -O2 -fopenmp -shared -fPIC ficco_oracle.c -o libficco_oracle.so
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* bf16 bits -> fp64, exactly: the 16 bits are the high half of an IEEE fp32. */
static double widen_bf16(uint16_t bits)
{
    uint32_t u = ((uint32_t)bits) << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

/* Row i of the gathered activation: shard i / ms, local row i % ms (Fig. 3(a)). */
static const uint16_t *gathered_row(const uint16_t *const *shards, int64_t ms, int64_t K, int64_t i)
{
    return shards[i / ms] + (i % ms) * K;
}

/*
 * ref = [I_0;...;I_{G-1}] * W.
 *   shards : G host pointers, each [ms, K] bf16 bits, row-major
 *   W      : [K, N] bf16 bits, row-major
 *   ref    : [G*ms, N] fp64, row-major (written)
 * Returns 0, or -1 on a bad argument / allocation failure.
 */
int oracle_ag_gemm_f64(const uint16_t *const *shards, int G, int64_t ms, int64_t K,
                       const uint16_t *W, int64_t N, double *ref)
{
    if (!shards || !W || !ref || G <= 0 || ms < 0 || K < 0 || N < 0) return -1;
    int64_t M = (int64_t)G * ms;
    double *Wd = (double *)malloc(sizeof(double) * (size_t)(K * N ? K * N : 1));
    if (!Wd) return -1;
    for (int64_t t = 0; t < K * N; ++t) Wd[t] = widen_bf16(W[t]);

#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < M; ++i) {
        const uint16_t *a = gathered_row(shards, ms, K, i);
        double *c = ref + i * N;
        for (int64_t j = 0; j < N; ++j) c[j] = 0.0;
        for (int64_t k = 0; k < K; ++k) {
            double aik = widen_bf16(a[k]);
            const double *w = Wd + k * N;
            for (int64_t j = 0; j < N; ++j) c[j] += aik * w[j];
        }
    }
    free(Wd);
    return 0;
}

/*
 * The same definition for a list of rows only (sampling at sizes where the full product would
 * take minutes): out[r, :] = ref[rows[r], :].
 */
int oracle_ag_gemm_rows_f64(const uint16_t *const *shards, int G, int64_t ms, int64_t K,
                            const uint16_t *W, int64_t N, const int64_t *rows, int64_t nrows,
                            double *out)
{
    if (!shards || !W || !out || (!rows && nrows) || G <= 0 || ms <= 0 || K < 0 || N < 0) return -1;
    int64_t M = (int64_t)G * ms;
    for (int64_t r = 0; r < nrows; ++r)
        if (rows[r] < 0 || rows[r] >= M) return -1;

#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < nrows; ++r) {
        const uint16_t *a = gathered_row(shards, ms, K, rows[r]);
        double *c = out + r * N;
        for (int64_t j = 0; j < N; ++j) c[j] = 0.0;
        for (int64_t k = 0; k < K; ++k) {
            double aik = widen_bf16(a[k]);
            const uint16_t *w = W + k * N;
            for (int64_t j = 0; j < N; ++j) c[j] += aik * widen_bf16(w[j]);
        }
    }
    return 0;
}

/* Threads the parallel loops above will use (reported next to the oracle's timing). */
int oracle_num_threads(void)
{
    int n = 1;
#ifdef _OPENMP
    extern int omp_get_max_threads(void);
    n = omp_get_max_threads();
#endif
    return n;
}
