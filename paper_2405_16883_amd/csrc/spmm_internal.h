// Internal declarations shared by the planner, the execution kernels and the C entry points.
// gfx950 only: 64-wide wavefronts, 256-thread workgroups (4 wavefronts).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "scorch_spmm.h"
#include "tuning.h"
#include "xcd_map.h"

namespace scorch {

constexpr int kWave = 64;
constexpr int kWavesPerBlock = 4;
constexpr int kBlock = kWave * kWavesPerBlock;
// A window stages at most BN + LW entries per wavefront in LDS.
constexpr int kBNMax = 256;
constexpr int kLWMax = 64;
constexpr int kStageMax = kBNMax + kLWMax;
constexpr int kWindowRowsMax = 64;  // one lane per row when reading rowptr
constexpr int kPanelCols = 256; // panel kernel: one wavefront covers 256 columns (64 lanes x float4)
constexpr int kSliceCols = 32;  // XCD-sliced mode: 32 fp32 columns = one 128-byte line of a B row
constexpr int64_t kL2SliceBudget = 2560 * 1024;  // bytes of B an XCD's 4 MB L2 is trusted to keep resident
constexpr int64_t kMallBytes = 256ll << 20;      // memory-side cache shared by all XCDs
constexpr int kDegBins = 32 * 16 + 1;            // column-degree histogram: 16 bins per power of two
constexpr int64_t kHotSampleMax = 1 << 24;  // stored entries counted at most when the columns are ranked by degree

// Parameters that decide how rows are classed and cut (paper has none of this; see the header).
struct PlanParams {
    int32_t BN;     // merge-path key units per window
    int32_t ALPHA;  // key weight of one row: key_i = rowptr[i] + ALPHA*i
    int32_t LW;     // short rows: len <= LW
    int32_t CH;     // wave rows:  LW < len <= CH
    int32_t BCH;    // block rows: pieces of at most BCH entries
    int32_t U;      // gathers in flight per lane group (4 or 8)
    int32_t NT;     // bit 0: streaming (non-temporal) stores for C
    int32_t SLICED; // >0: XCD-sliced execution with this many columns of B per slice (32, 64 or 128; see want_sliced)
    int32_t PACK;   // 1: sliced execution gathers from a slice-major copy of B made at every call
    int32_t PANEL;  // dense-ish sorted rows: stream B through LDS in k-panels (spmm_panel.hip); 1: 256-column tiles, 2: 512
    int32_t PDIRECT; // panel kernel: 1 = fetch the panels from the caller's row-major B instead of a tile-major copy
    int32_t HOT;    // >0: budget in KB for the most referenced rows of B, which alone keep the default cache policy
};

// SCORCH_SPMM_TUNE, parsed (only scorch_spmm_plan and scorch_spmm_plan_workspace_bytes call this)
Tuning read_tuning_from_env();
PlanParams choose_params(int32_t m, int32_t k, int64_t nnz, int32_t n, const Tuning &t);

struct WorkspaceLayout {
    uint64_t off_counts, off_totals, off_win, off_stage, off_wave, off_wave_span, off_items, off_split, off_partials, off_tickets, off_bpack,
        off_coldeg, off_hotmask, off_degbins, total;
    int64_t ticket_tiles;  // arrival counters per split row: one for every column tile a launch may use
    int64_t n_windows, nblk;
    int64_t cap_wave, cap_items, cap_split, cap_slots;
    int32_t partial_stride;
};
WorkspaceLayout layout_workspace(int32_t m, int32_t k, int64_t nnz, int32_t n, const PlanParams &p);

// Everything the execution kernels need, passed by value.
struct ExecArgs {
    const int32_t *rowptr;
    const int32_t *colidx;
    const float *vals;
    const float *B;
    float *C;
    int64_t ldb, ldc;
    int32_t m, n;
    const int32_t *win_row_start;
    const int2 *win_stage;  // per window: (first staged entry, number of staged entries) of its short rows; y < 0: no short row
    const int32_t *wave_rows;
    const int2 *wave_span;  // [p0, p1) of every wave row: spares the wavefront the row-pointer read
    const int4 *items;
    float *partials;
    int32_t *tickets;  // arrival counters of the split rows (nullptr: partial rows are added by the fix-up launch)
    int32_t BCH;       // entries per piece of a long row
    int32_t n_windows, n_wave_rows, n_items;
    int32_t nb_items, nb_wave, nb_win;  // workgroups per path, per column tile
    int32_t partial_stride;
    int32_t LW;
    int32_t ncoltiles;
    int32_t xcd_slices;  // 0 = tile-major grid, else XCD-sliced (see tile_of_workgroup)
    int64_t b_tile_stride;  // 0: B is the caller's row-major matrix; else B is slice-major, floats per slice
    const float *bias;      // epilogue: n floats added to every row of C, or nullptr
    int32_t act;            // epilogue: 0 identity, 1 ReLU
    const uint32_t *hotmask;  // one bit per column of A, set for the most referenced rows of B (hot/cold variants only)
    int32_t rows_per_wave;    // plan-free kernel only: consecutive rows taken by one wavefront
    int64_t b_bytes;          // size of B in bytes (cache-policy experiments of the hot/cold variants only)
};

struct PanelArgs {
    const int32_t *rowptr;
    const int32_t *colidx;
    const float *vals;
    const float *Bp;  // tile-major copy of B (tile t is a dense k x 256 or k x 512 block), or the caller's row-major B
    float *C;
    int64_t ldb;      // row stride of Bp when it is the caller's B
    int64_t ldc;
    int32_t m, k, n;
    int32_t nrb;     // row blocks of 4*RW rows
    int32_t ntiles;  // 256-column tiles
    int32_t xcd_slices;
    const float *bias;
    int32_t act;
};

struct FixupArgs {
    const int4 *split;
    const float *partials;
    float *C;
    int64_t ldc;
    int32_t n, n_split, partial_stride;
    const float *bias;
    int32_t act;
};

#if defined(__HIPCC__)
__device__ __forceinline__ bool tile_of_workgroup(int32_t xcd_slices, int32_t ncoltiles, uint32_t per_tile, uint32_t &ct,
                                                  uint32_t &b) {
    return tile_of_index(blockIdx.x, xcd_slices, ncoltiles, per_tile, ct, b);
}
#endif

}  // namespace scorch

struct scorch_spmm_plan_s {
    int32_t m, k, n;
    int64_t nnz;
    int device;
    scorch::Tuning tuning;  // the environment overrides as they stood when the plan was made
    scorch::PlanParams params;
    scorch::WorkspaceLayout layout;
    char *workspace;
    int32_t n_short, n_wave, n_items, n_split, n_slots;
    int32_t n_hot;    // columns marked hot (0: every gather uses the default cache policy)
    float hot_share;  // share of the stored entries that point at a hot column
};

namespace scorch {

void set_error(const char *fmt, ...);
scorch_status_t hip_fail(hipError_t e, const char *what);

// spmm_plan.hip
scorch_status_t build_plan(scorch_spmm_plan_t *plan, const int32_t *rowptr, const int32_t *colidx,
                           hipStream_t stream);

scorch_status_t launch_rowptr_from_keys(int32_t m, int64_t count, const int32_t *keys, const int32_t *pos,
                                        bool strictly_increasing, int32_t *rowptr, int32_t *bad_flag,
                                        hipStream_t stream);

// spmm_exec.hip
scorch_status_t launch_planned(const scorch_spmm_plan_t *plan, const int32_t *rowptr, const int32_t *colidx,
                               const float *vals, const float *B, int64_t ldb, float *C, int64_t ldc,
                               const float *bias, int32_t act, hipStream_t stream);
scorch_status_t launch_pack_b(const float *B, int64_t ldb, int32_t k, int32_t n, int32_t W, float *Bp,
                              hipStream_t stream);

// spmm_panel.hip
bool panel_operands_ok(int32_t n, const float *B, int64_t ldb, const float *C, int64_t ldc);
scorch_status_t launch_panel(const scorch_spmm_plan_t *plan, const int32_t *rowptr, const int32_t *colidx,
                             const float *vals, const float *B, int64_t ldb, float *C, int64_t ldc,
                             const float *bias, int32_t act, hipStream_t stream);

// sddmm_exec.hip (plan == nullptr: plan-free, one wavefront per row)
scorch_status_t launch_sddmm(const scorch_spmm_plan_t *plan, int32_t m, int32_t d, const int32_t *rowptr,
                             const int32_t *colidx, const float *vals, const float *B, int64_t ldb, const float *Ct,
                             int64_t ldct, float *out, hipStream_t stream);

scorch_status_t launch_natural(int32_t m, int32_t k, int32_t n, const int32_t *rowptr, const int32_t *colidx,
                               const float *vals, const float *B, int64_t ldb, float *C, int64_t ldc,
                               hipStream_t stream);

}  // namespace scorch
