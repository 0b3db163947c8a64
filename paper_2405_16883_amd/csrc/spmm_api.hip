// extern "C" entry points: argument checks, plan life cycle, status text.
#include "spmm_internal.h"

#include <cstdarg>
#include <cstdio>
#include <new>

namespace scorch {

static thread_local char g_err[512] = "";

void set_error(const char *fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    std::vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
}

scorch_status_t hip_fail(hipError_t e, const char *what) {
    set_error("%s: %s", what, hipGetErrorString(e));
    return SCORCH_ERR_HIP;
}

static scorch_status_t check_operands(int32_t m, int32_t k, int32_t n, const void *rowptr, const void *colidx,
                                      const void *vals, const void *B, int64_t ldb, const void *C, int64_t ldc) {
    if (m < 0 || k < 0 || n < 0) {
        set_error("negative dimension (m=%d k=%d n=%d)", m, k, n);
        return SCORCH_ERR_INVALID_ARG;
    }
    if (m == 0 || n == 0) return SCORCH_OK;
    if (!rowptr || !C) {
        set_error("rowptr and C must not be NULL");
        return SCORCH_ERR_INVALID_ARG;
    }
    if (ldb < n || ldc < n) {
        set_error("leading dimension smaller than n (ldb=%lld ldc=%lld n=%d)", (long long)ldb, (long long)ldc, n);
        return SCORCH_ERR_INVALID_ARG;
    }
    (void)colidx; (void)vals; (void)B;  // may be NULL only when no entry is stored; never dereferenced then
    return SCORCH_OK;
}

// A plan's row lists and partial rows live in memory of the device that was current when it was made.
static scorch_status_t check_plan_device(const scorch_spmm_plan_t *plan) {
    int dev = -1;
    if (hipGetDevice(&dev) == hipSuccess && plan->device >= 0 && dev != plan->device) {
        set_error("plan was made on device %d but device %d is current", plan->device, dev);
        return SCORCH_ERR_INVALID_ARG;
    }
    return SCORCH_OK;
}

}  // namespace scorch

using namespace scorch;

extern "C" {

scorch_status_t scorch_spmm_csr(int32_t m, int32_t k, int32_t n, const int32_t *rowptr, const int32_t *colidx,
                                const float *vals, const float *B, int32_t ldb, float *C, int32_t ldc,
                                void *stream) {
    scorch_status_t st = check_operands(m, k, n, rowptr, colidx, vals, B, ldb, C, ldc);
    if (st != SCORCH_OK || m == 0 || n == 0) return st;
    return launch_natural(m, k, n, rowptr, colidx, vals, B, ldb, C, ldc, static_cast<hipStream_t>(stream));
}

scorch_status_t scorch_spmm_plan_workspace_bytes(int32_t m, int32_t k, int32_t n, int64_t nnz, size_t *bytes_out) {
    if (!bytes_out || m < 0 || k < 0 || n < 0 || nnz < 0) {
        set_error("workspace_bytes: bad argument");
        return SCORCH_ERR_INVALID_ARG;
    }
    if (nnz >= (int64_t)1 << 31) {
        set_error("nnz = %lld does not fit int32 indices", (long long)nnz);
        return SCORCH_ERR_UNSUPPORTED;
    }
    const PlanParams p = choose_params(m, k, nnz, n, read_tuning_from_env());
    *bytes_out = (size_t)layout_workspace(m, k, nnz, n, p).total;
    return SCORCH_OK;
}

scorch_status_t scorch_spmm_plan(int32_t m, int32_t k, int32_t n, const int32_t *rowptr, const int32_t *colidx,
                                 void *workspace, size_t workspace_bytes, void *stream,
                                 scorch_spmm_plan_t **plan_out) {
    if (!plan_out) {
        set_error("plan_out must not be NULL");
        return SCORCH_ERR_INVALID_ARG;
    }
    *plan_out = nullptr;
    if (m < 0 || k < 0 || n < 0 || (m > 0 && !rowptr)) {
        set_error("plan: bad dimensions or NULL rowptr");
        return SCORCH_ERR_INVALID_ARG;
    }
    if (!workspace || reinterpret_cast<uintptr_t>(workspace) % 256 != 0) {
        set_error("plan: workspace must be a 256-byte aligned device pointer");
        return SCORCH_ERR_INVALID_ARG;
    }
    hipStream_t s = static_cast<hipStream_t>(stream);
    int32_t nnz32 = 0;
    if (m > 0) {
        hipError_t e = hipMemcpyAsync(&nnz32, rowptr + m, sizeof(int32_t), hipMemcpyDeviceToHost, s);
        if (e != hipSuccess) return hip_fail(e, "read nnz from rowptr[m]");
        e = hipStreamSynchronize(s);
        if (e != hipSuccess) return hip_fail(e, "wait for nnz");
        if (nnz32 < 0) {
            set_error("rowptr[m] = %d is negative", nnz32);
            return SCORCH_ERR_INVALID_ARG;
        }
    }
    scorch_spmm_plan_t *plan = new (std::nothrow) scorch_spmm_plan_t();
    if (!plan) {
        set_error("out of host memory");
        return SCORCH_ERR_INVALID_ARG;
    }
    plan->m = m;
    plan->k = k;
    plan->n = n;
    plan->nnz = nnz32;
    plan->tuning = read_tuning_from_env();
    plan->params = choose_params(m, k, nnz32, n, plan->tuning);
    plan->layout = layout_workspace(m, k, nnz32, n, plan->params);
    plan->workspace = static_cast<char *>(workspace);
    if (hipGetDevice(&plan->device) != hipSuccess) plan->device = -1;
    if (workspace_bytes < plan->layout.total) {
        set_error("workspace of %zu bytes is smaller than the %llu needed", workspace_bytes,
                  (unsigned long long)plan->layout.total);
        delete plan;
        return SCORCH_ERR_WORKSPACE_TOO_SMALL;
    }
    scorch_status_t st = build_plan(plan, rowptr, colidx, s);
    if (st != SCORCH_OK) {
        delete plan;
        return st;
    }
    *plan_out = plan;
    return SCORCH_OK;
}

scorch_status_t scorch_spmm_csr_planned(const scorch_spmm_plan_t *plan, const int32_t *rowptr,
                                        const int32_t *colidx, const float *vals, const float *B, int32_t ldb,
                                        float *C, int32_t ldc, void *stream) {
    if (!plan) {
        set_error("plan must not be NULL");
        return SCORCH_ERR_INVALID_ARG;
    }
    scorch_status_t st = check_operands(plan->m, plan->k, plan->n, rowptr, colidx, vals, B, ldb, C, ldc);
    if (st != SCORCH_OK || plan->m == 0 || plan->n == 0) return st;
    if (plan->nnz > 0 && (!colidx || !vals || !B)) {
        set_error("colidx, vals and B must not be NULL when nnz > 0");
        return SCORCH_ERR_INVALID_ARG;
    }
    if ((st = check_plan_device(plan)) != SCORCH_OK) return st;
    return launch_planned(plan, rowptr, colidx, vals, B, ldb, C, ldc, nullptr, 0, static_cast<hipStream_t>(stream));
}

scorch_status_t scorch_spmm_csr_planned_epilogue(const scorch_spmm_plan_t *plan, const int32_t *rowptr,
                                                 const int32_t *colidx, const float *vals, const float *B,
                                                 int32_t ldb, const float *bias, int32_t activation, float *C,
                                                 int32_t ldc, void *stream) {
    if (!plan) {
        set_error("plan must not be NULL");
        return SCORCH_ERR_INVALID_ARG;
    }
    if (activation != SCORCH_ACT_IDENTITY && activation != SCORCH_ACT_RELU) {
        set_error("unknown activation %d", activation);
        return SCORCH_ERR_INVALID_ARG;
    }
    scorch_status_t st = check_operands(plan->m, plan->k, plan->n, rowptr, colidx, vals, B, ldb, C, ldc);
    if (st != SCORCH_OK || plan->m == 0 || plan->n == 0) return st;
    if (plan->nnz > 0 && (!colidx || !vals || !B)) {
        set_error("colidx, vals and B must not be NULL when nnz > 0");
        return SCORCH_ERR_INVALID_ARG;
    }
    if ((st = check_plan_device(plan)) != SCORCH_OK) return st;
    return launch_planned(plan, rowptr, colidx, vals, B, ldb, C, ldc, bias, activation,
                          static_cast<hipStream_t>(stream));
}

static scorch_status_t check_sddmm(int32_t m, int32_t k, int32_t d, const void *rowptr, const void *B, int64_t ldb,
                                   const void *Ct, int64_t ldct, const void *out) {
    if (m < 0 || k < 0 || d < 0) {
        set_error("sddmm: negative dimension (m=%d k=%d d=%d)", m, k, d);
        return SCORCH_ERR_INVALID_ARG;
    }
    if (m == 0) return SCORCH_OK;
    if (!rowptr) {
        set_error("sddmm: rowptr must not be NULL");
        return SCORCH_ERR_INVALID_ARG;
    }
    if (ldb < d || ldct < d) {
        set_error("sddmm: leading dimension smaller than d (ldb=%lld ldct=%lld d=%d)", (long long)ldb, (long long)ldct, d);
        return SCORCH_ERR_INVALID_ARG;
    }
    if (d > 0 && (!B || (k > 0 && !Ct))) {
        set_error("sddmm: B and Ct must not be NULL");
        return SCORCH_ERR_INVALID_ARG;
    }
    (void)out;  // may be NULL only when no entry is stored
    return SCORCH_OK;
}

scorch_status_t scorch_sddmm_csr(int32_t m, int32_t k, int32_t d, const int32_t *rowptr, const int32_t *colidx,
                                 const float *vals, const float *B, int32_t ldb, const float *Ct, int32_t ldct,
                                 float *out_vals, void *stream) {
    scorch_status_t st = check_sddmm(m, k, d, rowptr, B, ldb, Ct, ldct, out_vals);
    if (st != SCORCH_OK || m == 0) return st;
    return launch_sddmm(nullptr, m, d, rowptr, colidx, vals, B, ldb, Ct, ldct, out_vals,
                        static_cast<hipStream_t>(stream));
}

scorch_status_t scorch_sddmm_csr_planned(const scorch_spmm_plan_t *plan, int32_t d, const int32_t *rowptr,
                                         const int32_t *colidx, const float *vals, const float *B, int32_t ldb,
                                         const float *Ct, int32_t ldct, float *out_vals, void *stream) {
    if (!plan) {
        set_error("plan must not be NULL");
        return SCORCH_ERR_INVALID_ARG;
    }
    scorch_status_t st = check_sddmm(plan->m, plan->k, d, rowptr, B, ldb, Ct, ldct, out_vals);
    if (st != SCORCH_OK || plan->m == 0 || plan->nnz == 0) return st;
    if (!colidx || !vals || !out_vals) {
        set_error("sddmm: colidx, vals and out_vals must not be NULL when nnz > 0");
        return SCORCH_ERR_INVALID_ARG;
    }
    if ((st = check_plan_device(plan)) != SCORCH_OK) return st;
    return launch_sddmm(plan, plan->m, d, rowptr, colidx, vals, B, ldb, Ct, ldct, out_vals,
                        static_cast<hipStream_t>(stream));
}

scorch_status_t scorch_coo_to_csr_rowptr(int32_t m, int64_t nnz, const int32_t *row_idx, int32_t *rowptr_out,
                                         int32_t *bad_flag, void *stream) {
    if (m < 0 || nnz < 0 || !rowptr_out || (nnz > 0 && !row_idx)) {
        set_error("coo_to_csr_rowptr: bad argument");
        return SCORCH_ERR_INVALID_ARG;
    }
    if (nnz >= (int64_t)1 << 31) {
        set_error("nnz = %lld does not fit int32 row pointers", (long long)nnz);
        return SCORCH_ERR_UNSUPPORTED;
    }
    return launch_rowptr_from_keys(m, nnz, row_idx, nullptr, false, rowptr_out, bad_flag,
                                   static_cast<hipStream_t>(stream));
}

scorch_status_t scorch_dcsr_to_csr_rowptr(int32_t m, int32_t n_stored_rows, const int32_t *row_ids,
                                          const int32_t *row_pos, int32_t *rowptr_out, int32_t *bad_flag,
                                          void *stream) {
    if (m < 0 || n_stored_rows < 0 || n_stored_rows > m || !rowptr_out || !row_pos || (n_stored_rows > 0 && !row_ids)) {
        set_error("dcsr_to_csr_rowptr: bad argument");
        return SCORCH_ERR_INVALID_ARG;
    }
    return launch_rowptr_from_keys(m, n_stored_rows, row_ids, row_pos, true, rowptr_out, bad_flag,
                                   static_cast<hipStream_t>(stream));
}

scorch_status_t scorch_spmm_plan_destroy(scorch_spmm_plan_t *plan) {
    delete plan;
    return SCORCH_OK;
}

scorch_status_t scorch_spmm_plan_info(const scorch_spmm_plan_t *plan, scorch_spmm_plan_info_t *out) {
    if (!plan || !out) {
        set_error("plan_info: NULL argument");
        return SCORCH_ERR_INVALID_ARG;
    }
    out->m = plan->m;
    out->k = plan->k;
    out->n = plan->n;
    out->nnz = plan->nnz;
    out->BN = plan->params.BN;
    out->ALPHA = plan->params.ALPHA;
    out->LW = plan->params.LW;
    out->CH = plan->params.CH;
    out->BCH = plan->params.BCH;
    out->n_windows = (int32_t)plan->layout.n_windows;
    out->n_short_rows = plan->n_short;
    out->n_wave_rows = plan->n_wave;
    out->n_items = plan->n_items;
    out->n_split_rows = plan->n_split;
    out->n_partial_slots = plan->n_slots;
    out->partial_stride = plan->layout.partial_stride;
    out->mode = plan->params.PANEL ? 2 : (plan->params.SLICED ? 1 : 0);
    out->off_win_row_start = plan->layout.off_win;
    out->off_win_stage = plan->layout.off_stage;
    out->off_wave_span = plan->layout.off_wave_span;
    out->off_wave_rows = plan->layout.off_wave;
    out->off_items = plan->layout.off_items;
    out->off_split = plan->layout.off_split;
    out->off_partials = plan->layout.off_partials;
    out->workspace_bytes_used = plan->layout.total;
    out->n_hot_columns = plan->n_hot;
    out->hot_share = plan->hot_share;
    return SCORCH_OK;
}

const char *scorch_status_string(scorch_status_t status) {
    switch (status) {
        case SCORCH_OK: return "ok";
        case SCORCH_ERR_INVALID_ARG: return "invalid argument";
        case SCORCH_ERR_UNSUPPORTED: return "unsupported size";
        case SCORCH_ERR_WORKSPACE_TOO_SMALL: return "workspace too small";
        case SCORCH_ERR_HIP: return "HIP runtime error";
        default: return "unknown status";
    }
}

const char *scorch_last_error(void) { return scorch::g_err; }

}  // extern "C"
