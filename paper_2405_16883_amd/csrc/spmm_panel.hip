// Panel kernel: CSR SpMM for dense-ish matrices (a few percent of the entries stored, e.g. an
// unstructured-pruned weight), C_ik = sum_j A_ij * B_jk (paper, Section 4.2).
//
// The gather kernels fetch one B row per stored entry from L2; at ~10 % density every B row is wanted
// by ~10 % of the rows of A, so it is cheaper to stream B through LDS once per block of rows and let
// every row pick its entries out of LDS.  The loop order of the paper (rows, stored entries, dense
// columns innermost and tiled) is kept per wavefront; what is added is a tiling of the *sparse* index j
// into panels of 64 B rows -- which the paper avoids on CPUs because it needs a search in the sparse
// level (Section 4.2).  Here the search is free: columns inside a row are sorted (checked by the
// planner), every wavefront keeps a 64-entry register window of each of its rows (one entry per lane),
// and the entries that fall into the current panel are the next few lanes of that window, found with
// one ballot.  Entries reach the ALU by v_readlane (scalar broadcast), B values by ds_read_b128.
//
//   workgroup = 16 wavefronts = 64 rows x one 256-column tile of C
//   wavefront = 4 rows, lane l owns columns 4l..4l+3 of the tile, accumulators stay in registers
//   panel     = 64 rows x 256 columns of B (64 KB of LDS), read from a tile-major copy of B
// Column tiles are dealt to the XCDs (tile_of_workgroup) so that the workgroups that walk the same
// tile of B run on the same die, start together and find the panels in that die's L2.
#include "spmm_internal.h"

#include <climits>

namespace scorch {

typedef float f4 __attribute__((ext_vector_type(4)));

// RW rows per wavefront, WPB wavefronts per workgroup, kBatch LDS reads in flight per row and panel,
// Q float4 per lane: the tile is 256*Q columns wide and a panel holds 64/Q rows of B (64 KB of LDS).
template <int RW, int WPB, int kBatch, int Q>
__global__ __launch_bounds__(WPB * kWave) void spmm_panel_kernel(const PanelArgs a) {
    constexpr int kRowQuads = Q * (kPanelCols / 4);  // float4 per LDS row
    constexpr int kRows = kPanelRows / Q;            // B rows per panel
    __shared__ f4 s_b[kRows * kRowQuads];
    const int tid = threadIdx.x;
    const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform: keeps the row state in SGPRs
    const int lane = tid & 63;
    uint32_t ct, rb;
    if (!tile_of_workgroup(a.xcd_slices, a.ntiles, (uint32_t)a.nrb, ct, rb)) return;
    const int c0 = (int)ct * (Q * kPanelCols) + lane * 4;  // lane owns columns c0 + 256 q .. +3, q < Q
    const f4 *Bt = reinterpret_cast<const f4 *>(a.Bp + (int64_t)ct * a.k * (Q * kPanelCols));
    const int64_t row_base = (int64_t)rb * (WPB * RW) + wv * RW;

    int pend[RW], wbase[RW], pos[RW], colreg[RW];
    float valreg[RW];
    f4 acc[RW][Q];
#pragma unroll
    for (int r = 0; r < RW; ++r) {
        const int64_t row = row_base + r;
        int p0 = 0, p1 = 0;
        if (row < a.m) {
            p0 = a.rowptr[row];
            p1 = a.rowptr[row + 1];
        }
        wbase[r] = p0;
        pend[r] = p1;
        pos[r] = 0;
        const int p = p0 + lane;
        colreg[r] = p < p1 ? a.colidx[p] : INT_MAX;
        valreg[r] = p < p1 ? a.vals[p] : 0.f;
#pragma unroll
        for (int q = 0; q < Q; ++q) acc[r][q] = f4{0.f, 0.f, 0.f, 0.f};
    }

    for (int k0 = 0; k0 < a.k; k0 += kRows) {
        __syncthreads();  // everyone is done with the previous panel
        const int quads = min(kRows, a.k - k0) * kRowQuads;
        const f4 *src = Bt + (int64_t)k0 * kRowQuads;
        for (int i = tid; i < quads; i += WPB * kWave) s_b[i] = src[i];
        __syncthreads();
        const int kend = k0 + kRows;
#pragma unroll
        for (int r = 0; r < RW; ++r) {
            while (true) {
                // columns are sorted: the entries of this window below kend are its first `lim` lanes
                const int lim = __builtin_popcountll(__ballot(colreg[r] < kend));
                for (int j = pos[r]; j < lim; j += kBatch) {
                    // issue the LDS reads of a whole batch first, then the multiply-adds; all branches are
                    // wave-uniform (scalar), entries past `lim` are skipped
                    f4 x[kBatch][Q];
#pragma unroll
                    for (int u = 0; u < kBatch; ++u) {
                        if (j + u < lim) {
                            const int c = __builtin_amdgcn_readlane(colreg[r], j + u);
#pragma unroll
                            for (int q = 0; q < Q; ++q) x[u][q] = s_b[(c - k0) * kRowQuads + q * (kPanelCols / 4) + lane];
                        }
                    }
#pragma unroll
                    for (int u = 0; u < kBatch; ++u) {
                        if (j + u < lim) {
                            const float v = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(valreg[r]), j + u));
#pragma unroll
                            for (int q = 0; q < Q; ++q)
#pragma unroll
                                for (int i = 0; i < 4; ++i) acc[r][q][i] = __builtin_fmaf(v, x[u][q][i], acc[r][q][i]);
                        }
                    }
                }
                pos[r] = lim;
                if (lim == kWave && wbase[r] + kWave < pend[r]) {
                    // window used up and the row goes on: slide it
                    wbase[r] += kWave;
                    const int p = wbase[r] + lane;
                    colreg[r] = p < pend[r] ? a.colidx[p] : INT_MAX;
                    valreg[r] = p < pend[r] ? a.vals[p] : 0.f;
                    pos[r] = 0;
                } else {
                    break;
                }
            }
        }
    }
#pragma unroll
    for (int r = 0; r < RW; ++r) {
        const int64_t row = row_base + r;
#pragma unroll
        for (int q = 0; q < Q; ++q) {
            const int c = c0 + q * kPanelCols;
            if (row < a.m && c < a.n) {
                f4 v = acc[r][q];
                if (a.bias)
#pragma unroll
                    for (int i = 0; i < 4; ++i) v[i] += a.bias[c + i];
                if (a.act == 1)
#pragma unroll
                    for (int i = 0; i < 4; ++i) v[i] = fmaxf(v[i], 0.f);
                __builtin_nontemporal_store(v, reinterpret_cast<f4 *>(a.C + row * a.ldc + c));
            }
        }
    }
}

bool panel_operands_ok(int32_t n, const float *B, int64_t ldb, const float *C, int64_t ldc) {
    const uintptr_t pb = reinterpret_cast<uintptr_t>(B), pc = reinterpret_cast<uintptr_t>(C);
    return n % 4 == 0 && ldb % 4 == 0 && ldc % 4 == 0 && pb % 16 == 0 && pc % 16 == 0;
}

scorch_status_t launch_panel(const scorch_spmm_plan_t *plan, const int32_t *rowptr, const int32_t *colidx,
                             const float *vals, const float *B, int64_t ldb, float *C, int64_t ldc,
                             const float *bias, int32_t act, hipStream_t stream) {
    // Shapes (rows per wavefront / wavefronts per workgroup / float4 per lane).  Both keep 8 wavefronts per SIMD
    // resident (<= 64 VGPRs, two 1024-thread workgroups per CU), which is what hides the LDS and scalar latencies:
    // a 4-wavefront, 16-rows-per-wavefront shape of the same kernel ran 2.1x slower.
    const int variant = plan->params.PANEL;
    struct Shape { int RW, WPB, Q; };
    const Shape sh = variant == 2 ? Shape{2, 16, 2} : Shape{4, 16, 1};
    const int W = sh.Q * kPanelCols;
    float *Bp = reinterpret_cast<float *>(plan->workspace + plan->layout.off_bpack);
    scorch_status_t st = launch_pack_b(B, ldb, plan->k, plan->n, W, Bp, stream);
    if (st != SCORCH_OK) return st;
    PanelArgs a{};
    a.rowptr = rowptr;
    a.colidx = colidx;
    a.vals = vals;
    a.Bp = Bp;
    a.C = C;
    a.ldc = ldc;
    a.m = plan->m;
    a.k = plan->k;
    a.n = plan->n;
    a.nrb = (plan->m + sh.WPB * sh.RW - 1) / (sh.WPB * sh.RW);
    a.ntiles = (plan->n + W - 1) / W;
    a.xcd_slices = xcd_slots_for(a.ntiles);
    a.bias = bias;
    a.act = act;
    const int64_t grid = xcd_grid_size(a.xcd_slices, a.ntiles, a.nrb);
    if (grid > 0x7fffffffLL) {
        set_error("launch grid of %lld workgroups exceeds the HIP limit", (long long)grid);
        return SCORCH_ERR_UNSUPPORTED;
    }
    const dim3 g((uint32_t)grid), b(sh.WPB * kWave);
    if (variant == 2) hipLaunchKernelGGL((spmm_panel_kernel<2, 16, 2, 2>), g, b, 0, stream, a);
    else hipLaunchKernelGGL((spmm_panel_kernel<4, 16, 4, 1>), g, b, 0, stream, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return hip_fail(e, "launch spmm_panel_kernel");
    return SCORCH_OK;
}

}  // namespace scorch
