/*
 * CPU oracle for quantized vector-sparse SpMM / SDDMM.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition of what the
 * GPU library must compute.  It shares no code with the HIP path and is used only
 * by the tests, the smoke check and the benchmark's cpu_baseline leg.
 *
 * The sparse operand is handed over as an ordinary dense integer matrix with its
 * zeros materialised, plus one flag per (row panel, column) that says whether that
 * V x 1 column vector is stored.  A "row panel" is V consecutive rows (the
 * "row of vectors" of Section 4.1 of the paper).
 *
 * Every sum is accumulated in int64.  A function returns 0 on success and 1 if any
 * exact result does not fit in int32 (the outputs are then still written, truncated).
 * Parallelism: OpenMP over rows / panels only; no blocking, no reordering of a sum.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int mco_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void mco_set_num_threads(int n)
{
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

/*
 * SpMM (Section 4.2, problem statement: sparse LHS with 1-D vector blocks times a
 * dense row-major RHS):
 *     C[i][j] = sum_k  stored[i / V][k] * A[i][k] * B[k][j]
 * A: M x K, stored: (M/V) x K flags, B: K x N, C: M x N, all row-major.
 */
int mco_spmm(int M, int K, int N, int V,
             const int32_t *A, const uint8_t *stored, const int32_t *B, int32_t *C)
{
    int overflow = 0;
#pragma omp parallel for schedule(dynamic, 8) reduction(| : overflow)
    for (int i = 0; i < M; ++i) {
        int64_t *acc = (int64_t *)calloc((size_t)(N > 0 ? N : 1), sizeof(int64_t));
        const uint8_t *flag = stored + (size_t)(i / V) * K;
        for (int k = 0; k < K; ++k) {
            if (!flag[k]) continue;
            const int64_t a = A[(size_t)i * K + k];
            const int32_t *brow = B + (size_t)k * N;
            for (int j = 0; j < N; ++j) acc[j] += a * (int64_t)brow[j];
        }
        for (int j = 0; j < N; ++j) {
            if (acc[j] > INT32_MAX || acc[j] < INT32_MIN) overflow = 1;
            C[(size_t)i * N + j] = (int32_t)acc[j];
        }
        free(acc);
    }
    return overflow;
}

/*
 * SDDMM (Section 4.3): the product Q * Kmat^T read at the stored vectors of the mask.
 * Q: M x Kd row-major.  Kmat: Nc x Kd row-major (this is the column-major RHS of the
 * paper: one contiguous Kd-long column per output column).  stored: (M/V) x Nc flags.
 * Output S: for panel p ascending, for column c ascending with stored[p][c], the V
 * values  S = sum_k Q[p*V + v][k] * Kmat[c][k],  v = 0..V-1, written consecutively
 * (vector-major; the plain BCRS value order of Section 4.1).
 * S must have room for V * (number of set flags) entries.
 */
int mco_sddmm(int M, int Kd, int Nc, int V,
              const int32_t *Q, const int32_t *Kmat, const uint8_t *stored, int32_t *S)
{
    const int P = M / V;
    int64_t *first = (int64_t *)malloc(sizeof(int64_t) * (size_t)(P + 1));
    first[0] = 0;
    for (int p = 0; p < P; ++p) {
        int64_t cnt = 0;
        for (int c = 0; c < Nc; ++c) cnt += stored[(size_t)p * Nc + c] ? 1 : 0;
        first[p + 1] = first[p] + cnt;
    }
    int overflow = 0;
#pragma omp parallel for schedule(dynamic, 1) reduction(| : overflow)
    for (int p = 0; p < P; ++p) {
        int64_t slot = first[p];
        for (int c = 0; c < Nc; ++c) {
            if (!stored[(size_t)p * Nc + c]) continue;
            for (int v = 0; v < V; ++v) {
                int64_t acc = 0;
                const int32_t *q = Q + (size_t)(p * V + v) * Kd;
                const int32_t *kr = Kmat + (size_t)c * Kd;
                for (int k = 0; k < Kd; ++k) acc += (int64_t)q[k] * (int64_t)kr[k];
                if (acc > INT32_MAX || acc < INT32_MIN) overflow = 1;
                S[slot * V + v] = (int32_t)acc;
            }
            ++slot;
        }
    }
    free(first);
    return overflow;
}
