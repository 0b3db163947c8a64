/*
 * CPU oracle for SDDMM on a CSR pattern.  TEST INFRASTRUCTURE ONLY (see spmm_oracle.c).
 *
 * Definition followed (paper, Section 3.1, first example of the programming-model figure, and
 * Section 5.4): D = A (.) (B C) -- the sparse matrix D is the element-wise product of the sparse
 * matrix A with the dense product B C, computed only where A stores an entry:
 *     D_ij = A_ij * sum_t B_it * C_tj          for every stored (i, j)
 * D has the sparsity pattern (rowptr, colidx) of A, so only its value array is produced.
 * Reading of the layout (the paper fixes none): B is m x d row-major; the second factor is passed
 * transposed, Ct = C^T, k x d row-major, so that column j of C is row j of Ct.
 *
 * The inner sum runs over t = 0..d-1 in order, in double precision, starting from +0.0; the result
 * is then multiplied by A_ij.  T_p = |A_ij| * sum_t |B_it| |C_tj| scales the parity tolerance.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>

int sddmm_csr_oracle(int64_t m, int64_t d,
                     const int32_t *rowptr, const int32_t *colidx, const float *vals,
                     const float *B, int64_t ldb, const float *Ct, int64_t ldc,
                     double *D, double *T)
{
    for (int64_t i = 0; i < m; ++i) {
        int64_t p0 = rowptr[i], p1 = rowptr[i + 1];
        if (p1 < p0) return -1;
        const float *b_row = B + (size_t)i * (size_t)ldb;
        for (int64_t p = p0; p < p1; ++p) {
            const float *c_row = Ct + (size_t)colidx[p] * (size_t)ldc;
            double s = 0.0, t = 0.0;
            for (int64_t q = 0; q < d; ++q) {
                double x = (double)b_row[q], y = (double)c_row[q];
                s += x * y;
                t += fabs(x) * fabs(y);
            }
            D[p] = (double)vals[p] * s;
            if (T) T[p] = fabs((double)vals[p]) * t;
        }
    }
    return 0;
}
