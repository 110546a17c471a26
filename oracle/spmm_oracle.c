/*
 * ORACLE -- TEST INFRASTRUCTURE ONLY.  Not part of the product path.
 *
 * Plain, serial, obviously-correct CPU evaluation of the sparse-times-dense
 * product the paper's transformation must preserve.  Only tests, the smoke
 * check and the benchmark's cpu_baseline leg may load this file's library; the
 * HIP path shares no code, header, table or helper with it.
 *
 * What is computed (paper, Section 3.1, Listing 1 "Input code"): the loop nest
 *     for i, for k, for j:  if (A[i][k])  C[i][j] += A[i][k] * B[k][j]
 * with A of size M x K sparse, B of size K x N dense row-major and C of size
 * M x N dense row-major (Section 2, first paragraph, gives the shapes).  The
 * zero test is realised by compressed-sparse-row storage (Section 1, third
 * paragraph): only stored entries contribute, in the order they are stored.
 * The method under test is a re-scheduling and re-storage of exactly this
 * sum (Section 3.4 "Safety": the only hazards are write-after-write), so the
 * oracle is the definition itself, written out:
 *
 *     C[i][j] = sum_{p = row_ptr[i]}^{row_ptr[i+1]-1}
 *                   (double)vals[p] * (double)B[col_idx[p]][j]
 *
 * accumulated serially in stored order, in double.  C starts from zero
 * (overwrite semantics, the paper's title equation C = A x B).  Alongside it
 * the normaliser S[i][j] = sum_p |vals[p]| * |B[col_idx[p]][j]| used by the
 * parity metric is produced on request.
 *
 * Parity pins (tests/test_oracle_pins.py): dense triple loop on tiny inputs,
 * a hand-worked example (tests/golden/worked_example.txt), identity /
 * empty-row / linearity / permutation / power-of-two-scaling invariants,
 * numpy and scipy float64 products, the N = 1 sparse matrix-vector case.
 *
 * A row-parallel OpenMP build of this same source (rows are independent, the
 * per-row arithmetic and its order are unchanged, so results are bit-identical)
 * exists for timing only.
 */
#include <stdint.h>
#include <stddef.h>
#include <math.h>

#ifdef _OPENMP
#include <omp.h>
#endif

/* Returns 0 on success, a positive code on malformed input (nothing written
 * beyond what was already computed).  All pointers are host pointers.
 *   row_ptr[M+1], col_idx[nnz], vals[nnz]   CSR of A (int32 indices, fp32)
 *   B[K*N]   row-major, leading dimension N
 *   C[M*N]   row-major double, overwritten
 *   S[M*N]   row-major double, overwritten; may be NULL
 */
int spmm_oracle_f64(int64_t M, int64_t K, int64_t N,
                    const int32_t *row_ptr, const int32_t *col_idx,
                    const float *vals, const float *B,
                    double *C, double *S)
{
    if (M < 0 || K < 0 || N < 0) return 1;
    if (M > 0 && row_ptr == NULL) return 1;
    if (M > 0 && row_ptr[0] != 0) return 2;
    for (int64_t i = 0; i < M; ++i)
        if (row_ptr[i + 1] < row_ptr[i]) return 2;
    if (M > 0) {
        const int64_t nnz = row_ptr[M];
        for (int64_t p = 0; p < nnz; ++p)
            if (col_idx[p] < 0 || (int64_t)col_idx[p] >= K) return 3;
    }

#ifdef _OPENMP
#pragma omp parallel for schedule(dynamic, 16)
#endif
    for (int64_t i = 0; i < M; ++i) {
        double *c_row = C + (size_t)i * (size_t)N;
        double *s_row = S ? S + (size_t)i * (size_t)N : NULL;
        for (int64_t j = 0; j < N; ++j) {
            c_row[j] = 0.0;
            if (s_row) s_row[j] = 0.0;
        }
        /* Stored order over p; every element (i, j) therefore receives its
         * terms one after another in that same order. */
        for (int64_t p = row_ptr[i]; p < row_ptr[i + 1]; ++p) {
            const double a = (double)vals[p];
            const float *b_row = B + (size_t)col_idx[p] * (size_t)N;
            for (int64_t j = 0; j < N; ++j) {
                const double b = (double)b_row[j];
                c_row[j] += a * b;
                if (s_row) s_row[j] += fabs(a) * fabs(b);
            }
        }
    }
    return 0;
}

/* Number of threads the row loop will use (1 in the serial build). */
int spmm_oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
