/*
 * scorch_spmm.h -- C ABI of the MI355X (gfx950) CSR SpMM library.
 *
 * Operation (paper, Section 4.2, SpMM example, and the caption of the SpMM tiling figure):
 *
 *        C_ik = sum_j A_ij * B_jk
 *
 * A is m x k, sparse, stored in CSR: a dense row level and a compressed column level reached
 * through row pointers (paper, Appendix C "Tensor Formats").  B (k x n) and C (m x n) are dense:
 * the product of a sparse and a dense matrix is a dense array (paper, Appendix C, format
 * inference).  The loop order is rows -> stored entries -> dense columns, and only the dense
 * column loop is tiled (paper, Sections 4.1 and 4.2); here the column loop is spread over the
 * lanes of a wavefront.
 *
 * Conventions shared by every call
 *   - All array arguments are DEVICE pointers (HIP global memory of the current device) owned by
 *     the caller; the library never allocates or frees device memory and keeps no reference to
 *     an argument after the enqueued work has finished, except the plan workspace (below).
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Work is enqueued
 *     on it and the call returns without waiting, unless stated otherwise.
 *   - rowptr: int32[m+1], rowptr[0] = 0, non-decreasing, rowptr[m] = nnz < 2^31.
 *     colidx: int32[nnz], each in [0, k) (not checked on the device: an index outside [0, k) reads
 *     outside B).  Entries of a row may be in any order and may repeat;
 *     every stored entry contributes one term.  vals: float[nnz].
 *   - B: float, row-major, row stride ldb >= n (elements).  C: float, row-major, row stride
 *     ldc >= n.  C is overwritten (no alpha/beta); a row without stored entries becomes +0.0;
 *     columns n..ldc-1 of C and n..ldb-1 of B are never touched.  B and C must not overlap.
 *   - Arithmetic: fp32 products and fp32 accumulation (fused multiply-add), summation order
 *     fixed by the plan, so repeated calls give bit-identical results.
 *   - Return value: SCORCH_OK or a negative status; nothing throws across this boundary.
 *     On error nothing has been enqueued unless the status is SCORCH_ERR_HIP.
 *     scorch_last_error() gives a thread-local description of the last failure.
 *   - m == 0 or n == 0 is valid and does no work.
 */
#ifndef SCORCH_SPMM_H
#define SCORCH_SPMM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef int32_t scorch_status_t;
enum {
    SCORCH_OK = 0,
    SCORCH_ERR_INVALID_ARG = -1,         /* null pointer, negative size, ldb/ldc < n, ... */
    SCORCH_ERR_UNSUPPORTED = -2,         /* nnz >= 2^31, or a plan used with other dimensions */
    SCORCH_ERR_WORKSPACE_TOO_SMALL = -3, /* plan workspace smaller than the stated bound */
    SCORCH_ERR_HIP = -4                  /* a HIP runtime call failed */
};

typedef struct scorch_spmm_plan_s scorch_spmm_plan_t; /* small host-side handle */

/*
 * Plan-free SpMM: C = A.B in natural row order.  A wavefront takes a short run of consecutive rows
 * (up to 4, up to 16 for small n), walks the short ones (up to 32 entries) side by side and streams the longer ones; the
 * four wavefronts of a workgroup work together on rows with more than 2048 entries (more than 256
 * where such rows are rare).  With B of 8 MB or more and n a multiple of 64 (128) the columns are walked in slices of
 * 64 (128) that are dealt over the accelerator dies, so that each die gathers from a part of B its L2 can keep.
 * Always available and correct for any valid input; no load balancing
 * beyond that, so a row with very many entries still runs on a single workgroup.  (Definition: see
 * the top of this file.)
 */
scorch_status_t scorch_spmm_csr(int32_t m, int32_t k, int32_t n,
                                const int32_t *rowptr, const int32_t *colidx, const float *vals,
                                const float *B, int32_t ldb,
                                float *C, int32_t ldc,
                                void *stream);

/*
 * (Plumbing of this library; the paper has no counterpart: its kernels are generated per call on the CPU.)
 * Size, in bytes, of the device workspace a plan for an m x k matrix with nnz stored entries and
 * n dense columns needs (row lists, partial rows, and for some shapes a repacked copy of B).
 * It depends on the tuning read from the environment (see scorch_spmm_plan); call both with
 * the same environment.  Host-only; touches no device.
 */
scorch_status_t scorch_spmm_plan_workspace_bytes(int32_t m, int32_t k, int32_t n, int64_t nnz, size_t *bytes_out);

/*
 * One-time analysis of a sparsity pattern (the paper names load balance and irregular access
 * as the SpMM problems, related-work section; its own remedy is CPU-side loop tiling).  Rows
 * are classed by their stored length:
 *     short  (len <= LW)        packed into windows of consecutive rows along the merge path
 *                               key_i = rowptr[i] + ALPHA*i, BN key units per window
 *     wave   (LW < len <= CH)   one wavefront per row
 *     block  (len > CH)         cut into pieces of at most BCH entries, one workgroup per piece;
 *                               rows with several pieces are summed from partial rows in a
 *                               fixed order (no floating-point atomics)
 * `workspace` (device, 256-byte aligned, at least the bound above) receives the row lists and
 * holds the partial rows at execution; it must stay allocated and unmodified while the plan
 * lives.  `colidx` may be NULL; when given (device, nnz entries) it is only inspected to see whether
 * every row stores its columns in strictly increasing order, which is what the panel kernel for
 * dense-ish matrices needs (with NULL, or with unsorted or repeated columns in a row, the gather
 * kernels are used).  The
 * call enqueues on `stream` and WAITS for it (it reads nnz and the list sizes back).  The plan is valid for exactly this rowptr content
 * and this n, on the device that was current.
 * When B is more than three times the 256 MB memory-side cache, n >= 96 and colidx is given, the plan also counts how often
 * each column occurs and marks the most referenced columns (up to 64 MB of rows of B) as hot; execution then
 * reads only those rows of B with the default cache policy and the others with the streaming policy.
 * This changes no result bit.
 * Optional environment variable SCORCH_SPMM_TUNE="bn=..,alpha=..,lw=..,ch=..,bch=..,u=..,nt=..,sliced=..,pack=..,panel=..,hot=<KB>,sdblk=..,fix=..,cold=.."
 * overrides the built-in parameter choice (for experiments; sliced = 0, 1 (= 32), 32, 64 or 128 columns of B per
 * accelerator-die slice, panel = 0, 1 or 2; sdblk = blocks of columns of A per accelerator die in the planned
 * SDDMM, 0 = row-wise kernel; fix = 1: partial rows are added inside the fused launch, by the piece that finishes last, instead
 * of by a second launch; cold = 1, 2, 3: cache-policy bits of the loads of the rows of B outside the hot set).
 * The variable is read when a plan is made (and by scorch_spmm_plan_workspace_bytes), never by an execution call.
 */
scorch_status_t scorch_spmm_plan(int32_t m, int32_t k, int32_t n,
                                 const int32_t *rowptr, const int32_t *colidx,
                                 void *workspace, size_t workspace_bytes,
                                 void *stream,
                                 scorch_spmm_plan_t **plan_out);

/*
 * Planned SpMM: the operation at the top of this file (paper, Section 4.2), i.e. the same result contract as
 * scorch_spmm_csr, executed through the plan's row lists (the plan itself has no counterpart in the paper):
 * one fused launch, plus one small fix-up launch when rows were split across workgroups (the pieces
 * leave partial rows in the workspace, which are added in piece order); for wide
 * B with few rows a pre-pass first copies B into column-slice-major order so that each accelerator
 * die keeps its slice of B in its own L2; matrices with a few percent of their entries stored and
 * strictly increasing columns in every row go to a kernel that streams B through LDS, panel by panel,
 * instead of gathering (straight from the caller's B; pack=1 in the tuning text: from a tile-major copy).
 * Never waits, never allocates.  The partial rows and the copy of B live in the plan workspace, so
 * two executions of one plan must not overlap in time (same stream, or synchronise).
 */
scorch_status_t scorch_spmm_csr_planned(const scorch_spmm_plan_t *plan,
                                        const int32_t *rowptr, const int32_t *colidx, const float *vals,
                                        const float *B, int32_t ldb,
                                        float *C, int32_t ldc,
                                        void *stream);

/*
 * Planned SpMM with the epilogue of a GCN-style layer fused into the store of C (paper, Section 5.1:
 * H' = sigma(A^ H W); evaluated as sigma(A^ (H W) + b), the aggregation comes last and its result is
 * activated on the way out instead of in a second pass over C):
 *
 *        C_ik = act( sum_j A_ij * B_jk + bias_k )
 *
 * bias: float[n] on the device, or NULL for no bias.  activation: SCORCH_ACT_IDENTITY or
 * SCORCH_ACT_RELU.  Everything else as scorch_spmm_csr_planned; with bias == NULL and the identity it
 * gives bit-identical results to it.  Rows split across workgroups get bias and activation after their
 * pieces have been added.
 */
enum { SCORCH_ACT_IDENTITY = 0, SCORCH_ACT_RELU = 1 };
scorch_status_t scorch_spmm_csr_planned_epilogue(const scorch_spmm_plan_t *plan,
                                                 const int32_t *rowptr, const int32_t *colidx, const float *vals,
                                                 const float *B, int32_t ldb,
                                                 const float *bias, int32_t activation,
                                                 float *C, int32_t ldc,
                                                 void *stream);

/*
 * Planned SpMM for callers that cannot allocate device memory: code that may not call hipMalloc (tight serving
 * loops, harnesses that forbid it) and therefore cannot hand scorch_spmm_plan a workspace.  Same operation, same
 * arguments and same result bits as scorch_spmm_plan(m, k, n, rowptr, colidx, ...) followed by
 * scorch_spmm_csr_planned on the same operands; the plan's row lists, partial rows and (for some shapes) repacked copy
 * of B live in a static device array of SCORCH_STATIC_SCRATCH_BYTES that each GPU the library runs on holds until the
 * process ends.  The call allocates nothing on the device (no hipMalloc, hipFree or allocating library routine).
 *   - A problem whose plan needs more than SCORCH_STATIC_SCRATCH_BYTES (see scorch_spmm_plan_workspace_bytes) is
 *     refused with SCORCH_ERR_UNSUPPORTED and a message naming both sizes; nothing is enqueued then.
 *   - The pattern is analysed at every call (one wait on `stream` while the list sizes come back), then the
 *     execution is enqueued and the call returns without waiting for it.
 *   - All calls on one GPU share that GPU's array: calls that overlap in time on one GPU (two streams, two host
 *     threads) race on it and give undefined results; calls on one stream are ordered and safe.  Nothing the previous
 *     call left in the array is relied upon.
 */
#define SCORCH_STATIC_SCRATCH_BYTES ((size_t)16 << 20)
scorch_status_t scorch_spmm_csr_static(int32_t m, int32_t k, int32_t n,
                                       const int32_t *rowptr, const int32_t *colidx, const float *vals,
                                       const float *B, int32_t ldb,
                                       float *C, int32_t ldc,
                                       void *stream);

/* (Plumbing; no counterpart in the paper.)  Frees the host handle only (the workspace belongs to the caller).  NULL is
 * accepted. */
scorch_status_t scorch_spmm_plan_destroy(scorch_spmm_plan_t *plan);

/*
 * (Plumbing; no counterpart in the paper.)  What a plan contains, for tests and tools.  Offsets are byte offsets into the
 * caller's workspace:
 *   win_row_start  int32[n_windows + 1]
 *   win_stage      int32[n_windows][2]         entries a window stages (see off_win_stage)
 *   wave_rows      int32[n_wave_rows]          ascending row ids
 *   wave_span      int32[n_wave_rows][2]       their entry ranges (rowptr[row], rowptr[row + 1])
 *   items          int32[n_items][4]           (row, p_begin, p_end, partial slot or -1)
 *   split          int32[n_split_rows][4]      (row, first slot, pieces, 0)
 *   partials       float[n_partial_slots][partial_stride]
 */
typedef struct scorch_spmm_plan_info {
    int32_t m, k, n;
    int64_t nnz;
    int32_t BN, ALPHA, LW, CH, BCH;
    int32_t n_windows, n_short_rows, n_wave_rows, n_items, n_split_rows, n_partial_slots;
    int32_t partial_stride;
    int32_t mode; /* 0 gather kernel, 1 gather kernel with XCD-sliced columns, 2 panel kernel */
    uint64_t off_win_row_start, off_wave_rows, off_items, off_split, off_partials;
    uint64_t workspace_bytes_used;
    int32_t n_hot_columns; /* columns whose rows of B keep the default cache policy (0: no hot/cold split) */
    float hot_share;       /* share of the stored entries that point at those columns (beyond 2^24 entries:
                              of an evenly spread sample of 2^23..2^24 of them, which is what ranks the columns) */
    uint64_t off_wave_span; /* int32[n_wave_rows][2]: entry range [p0, p1) of every wave row, in the order of wave_rows */
    uint64_t off_win_stage; /* int32[n_windows][2]: (first entry, number of entries) between the first and the last
                               short row of the window, capped at 320 entries; (0, -1) for a window without short rows */
} scorch_spmm_plan_info_t;

scorch_status_t scorch_spmm_plan_info(const scorch_spmm_plan_t *plan, scorch_spmm_plan_info_t *out);

/*
 * SDDMM on the pattern of A (paper, Section 3.1, SDDMM example; Section 5.4):
 *
 *        D = A (.) (B C),      D_ij = A_ij * sum_t B_it * C_tj     for every stored (i, j)
 *
 * D has the sparsity pattern of A, so only its values are produced: out_vals[p] for the p-th stored
 * entry (row i, column colidx[p]).  B is m x d (row stride ldb >= d).  The second factor is passed
 * TRANSPOSED: Ct = C^T is k x d (row stride ldct >= d), so that column j of C is the contiguous row j
 * of Ct.  d must not exceed 1024 (any alignment of B and Ct); larger d gives SCORCH_ERR_UNSUPPORTED.  out_vals (float[nnz], device) may be the same array as vals
 * (in place) and must otherwise not overlap any input.  fp32 products, fp32 accumulation, fixed
 * summation order.  The planned variant reuses a plan made by scorch_spmm_plan for the same rowptr
 * (any n); the plan-free variant walks the rows in natural order like scorch_spmm_csr (short runs
 * of rows per wavefront, very long rows shared by the four wavefronts of a workgroup).
 */
scorch_status_t scorch_sddmm_csr(int32_t m, int32_t k, int32_t d,
                                 const int32_t *rowptr, const int32_t *colidx, const float *vals,
                                 const float *B, int32_t ldb, const float *Ct, int32_t ldct,
                                 float *out_vals, void *stream);

scorch_status_t scorch_sddmm_csr_planned(const scorch_spmm_plan_t *plan, int32_t d,
                                         const int32_t *rowptr, const int32_t *colidx, const float *vals,
                                         const float *B, int32_t ldb, const float *Ct, int32_t ldct,
                                         float *out_vals, void *stream);

/*
 * Row pointers for a row-major coordinate list (paper, Appendix C: sparse tensors default to the coordinate
 * format; a COO matrix lists (row, column, value) triples).  Given the row coordinates of nnz entries sorted by
 * row (non-decreasing), writes rowptr_out[0..m] such that the entries of row i are [rowptr_out[i], rowptr_out[i+1]);
 * the column and value arrays of the list then serve unchanged as colidx and vals of the CSR calls above.
 * row_idx: int32[nnz], device, each in [0, m).  rowptr_out: int32[m+1], device.  bad_flag: int32[1], device, or
 * NULL; it is set to 1 when the list is not sorted by row or holds a row outside [0, m) (rowptr_out is then
 * unspecified) and left untouched otherwise -- clear it before the call.  Enqueues one kernel, never waits.
 */
scorch_status_t scorch_coo_to_csr_rowptr(int32_t m, int64_t nnz, const int32_t *row_idx, int32_t *rowptr_out,
                                         int32_t *bad_flag, void *stream);

/*
 * Row pointers for a doubly compressed (DCSR) matrix (paper, Appendix C: both dimensions stored compressed, i.e.
 * only the rows that hold entries are listed).  row_ids: int32[n_stored_rows], device, strictly increasing, each
 * in [0, m): the ids of the stored rows.  row_pos: int32[n_stored_rows + 1], device: entries of row row_ids[r] are
 * [row_pos[r], row_pos[r+1]), row_pos[n_stored_rows] = nnz.  Writes the CSR row pointers rowptr_out[0..m] (rows that
 * are not listed come out empty); colidx and vals of the DCSR matrix serve unchanged.  bad_flag as for
 * scorch_coo_to_csr_rowptr.  Enqueues one kernel, never waits.
 */
scorch_status_t scorch_dcsr_to_csr_rowptr(int32_t m, int32_t n_stored_rows, const int32_t *row_ids,
                                          const int32_t *row_pos, int32_t *rowptr_out, int32_t *bad_flag,
                                          void *stream);

/* (Plumbing; no counterpart in the paper.)  Static text for a status code. */
const char *scorch_status_string(scorch_status_t status);

/* (Plumbing; no counterpart in the paper.)  Thread-local description of the most recent failure in this thread ("" if
 * none). */
const char *scorch_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* SCORCH_SPMM_H */
