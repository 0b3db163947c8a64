// scorch_spmm_csr_static: planned SpMM for callers that cannot allocate device memory.
//
// The planned path keeps its row lists, the partial rows of split rows and (for some shapes) a repacked copy of B in
// a device workspace that the caller of scorch_spmm_plan has to allocate.  This entry point brings its own: a
// file-scope device array of kStaticScratchBytes that every GPU the library runs on holds until the process ends.
// It analyses the pattern into that array and executes through the same kernels, so the result is bit-identical to
// scorch_spmm_plan + scorch_spmm_csr_planned on the same operands.  No hipMalloc, no hipFree, no allocating library
// call; the plan handle lives on the host stack.
//
// In host code the array's name is only a stand-in for the symbol, not a device address.  The address is looked up
// once per device with hipGetSymbolAddress (each GPU holds its own copy at its own address) and only that pointer is
// handed to kernels, memsets and copies.
#include "spmm_internal.h"

#include <mutex>

namespace scorch {

constexpr size_t kStaticScratchBytes = SCORCH_STATIC_SCRATCH_BYTES;
constexpr int kMaxDevices = 64;

static __device__ __align__(256) __attribute__((used)) unsigned char scratch[kStaticScratchBytes];

static std::mutex g_scratch_mutex;
static void *g_scratch_ptr[kMaxDevices];  // per device: address of that device's copy of `scratch` (nullptr: not looked up yet)

// Device address of the current device's scratch array (looked up at the first call on that device).
static scorch_status_t scratch_of_current_device(char **out) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_fail(e, "hipGetDevice");
    if (dev < 0 || dev >= kMaxDevices) {
        set_error("device ordinal %d is outside the %d the static scratch table holds", dev, kMaxDevices);
        return SCORCH_ERR_UNSUPPORTED;
    }
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return hip_fail(e, "hipGetSymbolAddress(scratch)");
        if (!p || reinterpret_cast<uintptr_t>(p) % 256 != 0) {
            set_error("static scratch array has no usable device address");
            return SCORCH_ERR_HIP;
        }
        g_scratch_ptr[dev] = p;
    }
    *out = static_cast<char *>(g_scratch_ptr[dev]);
    return SCORCH_OK;
}

}  // namespace scorch

using namespace scorch;

extern "C" scorch_status_t scorch_spmm_csr_static(int32_t m, int32_t k, int32_t n, const int32_t *rowptr,
                                                  const int32_t *colidx, const float *vals, const float *B,
                                                  int32_t ldb, float *C, int32_t ldc, void *stream) {
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
        set_error("leading dimension smaller than n (ldb=%d ldc=%d n=%d)", ldb, ldc, n);
        return SCORCH_ERR_INVALID_ARG;
    }
    hipStream_t s = static_cast<hipStream_t>(stream);
    char *ws = nullptr;
    scorch_status_t st = scratch_of_current_device(&ws);
    if (st != SCORCH_OK) return st;
    int32_t nnz32 = 0;
    hipError_t e = hipMemcpyAsync(&nnz32, rowptr + m, sizeof(int32_t), hipMemcpyDeviceToHost, s);
    if (e == hipSuccess) e = hipStreamSynchronize(s);
    if (e != hipSuccess) return hip_fail(e, "read nnz from rowptr[m]");
    if (nnz32 < 0) {
        set_error("rowptr[m] = %d is negative", nnz32);
        return SCORCH_ERR_INVALID_ARG;
    }
    if (nnz32 > 0 && (!colidx || !vals || !B)) {
        set_error("colidx, vals and B must not be NULL when nnz > 0");
        return SCORCH_ERR_INVALID_ARG;
    }
    scorch_spmm_plan_t plan{};  // on the host stack: nothing is allocated, nothing outlives the call but the enqueued work
    plan.m = m;
    plan.k = k;
    plan.n = n;
    plan.nnz = nnz32;
    plan.tuning = read_tuning_from_env();
    plan.params = choose_params(m, k, nnz32, n, plan.tuning);
    plan.layout = layout_workspace(m, k, nnz32, n, plan.params);
    plan.workspace = ws;
    if (hipGetDevice(&plan.device) != hipSuccess) plan.device = -1;
    if (plan.layout.total > kStaticScratchBytes) {
        set_error("this problem needs %llu bytes of plan workspace, the static scratch array holds %zu: "
                  "use scorch_spmm_plan with a workspace of your own",
                  (unsigned long long)plan.layout.total, kStaticScratchBytes);
        return SCORCH_ERR_UNSUPPORTED;
    }
    // The array keeps what the previous call left.  Everything execution reads is rewritten by build_plan (it clears
    // its own flags and counters and writes every list up to the counts it returns); the partial rows are written
    // by the pieces of a split row before the same launch order reads them.
    st = build_plan(&plan, rowptr, colidx, s);  // waits for the stream: the list sizes come back to the host
    if (st != SCORCH_OK) return st;
    return launch_planned(&plan, rowptr, colidx, vals, B, ldb, C, ldc, nullptr, 0, s);
}
