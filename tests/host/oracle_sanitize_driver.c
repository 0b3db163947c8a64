/*
 * Runs the C oracles (oracle/spmm_oracle.c, oracle/sddmm_oracle.c) on a problem read from a text file, with every
 * array in a heap block of exactly its size, so that a build with -fsanitize=address,undefined reports any read or
 * write outside an operand and any undefined arithmetic.  Test infrastructure only.
 *
 * Input:  m k n ldb nnz  nrows d, then rowptr[m+1], colidx[nnz], vals[nnz], B[k*ldb], rows[nrows], X[m*d]
 *         (nrows = 0: all rows; d = 0: no SDDMM; X is the first SDDMM factor, B[:, :d] serves as the transposed second).
 * Output: the SpMM result C and the magnitude sums T (count*n values each), then, if d > 0, D and its magnitude sums
 *         (nnz values each), printed with 17 significant digits.
 */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

int spmm_csr_oracle(int64_t m, int64_t n, const int32_t *rowptr, const int32_t *colidx, const float *vals,
                    const float *B, int64_t ldb, const int64_t *rows, int64_t nrows, double *C, double *T);
int sddmm_csr_oracle(int64_t m, int64_t d, const int32_t *rowptr, const int32_t *colidx, const float *vals,
                     const float *B, int64_t ldb, const float *Ct, int64_t ldc, double *D, double *T);

static void *exact(size_t count, size_t size) {
    const size_t bytes = count * size;
    void *p = malloc(bytes > 0 ? bytes : 1);
    if (!p) exit(3);
    return p;
}

int main(int argc, char **argv) {
    if (argc != 2) return 2;
    FILE *f = fopen(argv[1], "r");
    if (!f) return 2;
    long long m, k, n, ldb, nnz, nrows, d;
    if (fscanf(f, "%lld %lld %lld %lld %lld %lld %lld", &m, &k, &n, &ldb, &nnz, &nrows, &d) != 7) return 2;
    int32_t *rowptr = exact((size_t)m + 1, 4), *colidx = exact((size_t)nnz, 4);
    float *vals = exact((size_t)nnz, 4), *B = exact((size_t)(k * ldb), 4), *X = exact((size_t)(m * d), 4);
    int64_t *rows = exact((size_t)nrows, 8);
    long long v;
    double x;
    for (long long i = 0; i <= m; ++i) { if (fscanf(f, "%lld", &v) != 1) return 2; rowptr[i] = (int32_t)v; }
    for (long long i = 0; i < nnz; ++i) { if (fscanf(f, "%lld", &v) != 1) return 2; colidx[i] = (int32_t)v; }
    for (long long i = 0; i < nnz; ++i) { if (fscanf(f, "%lf", &x) != 1) return 2; vals[i] = (float)x; }
    for (long long i = 0; i < k * ldb; ++i) { if (fscanf(f, "%lf", &x) != 1) return 2; B[i] = (float)x; }
    for (long long i = 0; i < nrows; ++i) { if (fscanf(f, "%lld", &v) != 1) return 2; rows[i] = v; }
    for (long long i = 0; i < m * d; ++i) { if (fscanf(f, "%lf", &x) != 1) return 2; X[i] = (float)x; }
    fclose(f);
    const long long count = nrows ? nrows : m;
    double *C = exact((size_t)(count * n), 8), *T = exact((size_t)(count * n), 8);
    if (spmm_csr_oracle(m, n, rowptr, colidx, vals, B, ldb, nrows ? rows : NULL, nrows, C, T) != 0) return 4;
    for (long long i = 0; i < count * n; ++i) printf("%.17g\n", C[i]);
    for (long long i = 0; i < count * n; ++i) printf("%.17g\n", T[i]);
    if (d > 0) {
        double *D = exact((size_t)nnz, 8), *TD = exact((size_t)nnz, 8);
        if (sddmm_csr_oracle(m, d, rowptr, colidx, vals, X, d, B, ldb, D, TD) != 0) return 4;
        for (long long i = 0; i < nnz; ++i) printf("%.17g\n", D[i]);
        for (long long i = 0; i < nnz; ++i) printf("%.17g\n", TD[i]);
        free(D);
        free(TD);
    }
    free(rowptr); free(colidx); free(vals); free(B); free(X); free(rows); free(C); free(T);
    return 0;
}
