/*
 * CPU oracle for CSR SpMM.  TEST INFRASTRUCTURE ONLY: nothing in the product path may
 * call, link or load this file; it exists so that tests, the smoke check and the
 * benchmark's cpu_baseline leg have an independent statement of the result.
 *
 * Definition followed (paper, Section 4.1/4.2 and the caption of the SpMM tiling figure):
 *     C_ik = sum_j A_ij * B_jk
 * with A stored in CSR -- rows in a dense level, the columns of each row in a compressed
 * level addressed through row pointers (Appendix C, "Tensor Formats") -- and B, C dense
 * (a sparse-times-dense product is inferred to be a dense array, Appendix C).
 *
 * The sum runs over the *stored* entries of row i, in stored order, in double precision,
 * starting from +0.0.  Each float*float product is exact in double, so the only rounding
 * is in the additions.  No blocking, no reordering, no vector intrinsics, no threads.
 *
 * Pins: tests/test_oracle_pins.py (dense brute force, identity / permutation, row-sum
 * invariant, int64 arithmetic, linearity, all-ones closed form, hand-worked fixture).
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>

/*
 * rows == NULL : compute all m rows; output row r is matrix row r.
 * rows != NULL : compute only the nrows listed matrix rows; output row r is matrix row rows[r].
 * C (and T when not NULL) are row-major double arrays with row stride n.
 * T_ik = sum_j |A_ij| * |B_jk| is the magnitude sum the parity tolerance is scaled by.
 * Returns 0, or -1 on a negative row length / row id out of range.
 */
int spmm_csr_oracle(int64_t m, int64_t n,
                    const int32_t *rowptr, const int32_t *colidx, const float *vals,
                    const float *B, int64_t ldb,
                    const int64_t *rows, int64_t nrows,
                    double *C, double *T)
{
    int64_t count = rows ? nrows : m;
    for (int64_t r = 0; r < count; ++r) {
        int64_t i = rows ? rows[r] : r;
        if (i < 0 || i >= m) return -1;
        double *c_row = C + (size_t)r * (size_t)n;
        double *t_row = T ? T + (size_t)r * (size_t)n : NULL;
        for (int64_t c = 0; c < n; ++c) c_row[c] = 0.0;
        if (t_row) for (int64_t c = 0; c < n; ++c) t_row[c] = 0.0;
        int64_t p0 = rowptr[i], p1 = rowptr[i + 1];
        if (p1 < p0) return -1;
        for (int64_t p = p0; p < p1; ++p) {
            double a = (double)vals[p];
            const float *b_row = B + (size_t)colidx[p] * (size_t)ldb;
            for (int64_t c = 0; c < n; ++c) {
                double b = (double)b_row[c];
                c_row[c] += a * b;
                if (t_row) t_row[c] += fabs(a) * fabs(b);
            }
        }
    }
    return 0;
}
