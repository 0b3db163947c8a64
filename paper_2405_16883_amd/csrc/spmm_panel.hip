// Panel kernel: CSR SpMM for dense-ish matrices (a few percent of the entries stored, e.g. an
// unstructured-pruned weight), C_ik = sum_j A_ij * B_jk (paper, Section 4.2).
//
// The gather kernels fetch one B row per stored entry from L2; at ~10 % density every B row is wanted
// by ~10 % of the rows of A, so it is cheaper to stream B through LDS once per block of rows and let
// every row pick its entries out of LDS.  The loop order of the paper (rows, stored entries, dense
// columns innermost and tiled) is kept per wavefront; what is added is a tiling of the *sparse* index j
// into panels of 32 or 64 B rows -- which the paper avoids on CPUs because it needs a search in the
// sparse level (Section 4.2).  Here the search is free: columns inside a row are strictly increasing
// (checked by the planner), every wavefront keeps a 64-entry register window of each of its rows (one
// entry per lane), and the entries that fall into the current panel are the next few lanes of that
// window, found with one ballot.  Entries reach the ALU by v_readlane (scalar broadcast), B values by
// ds_read_b128.
//
//   workgroup = 16 wavefronts = 64 rows x one tile of C (256 or 512 columns), one workgroup per CU
//   wavefront = 4 rows, lane l owns columns 4l..4l+3 (and 256+4l.. for the wide tile), accumulators in registers
//   panel     = 64 rows x 256 columns (64 KB) or 40 rows x 512 columns (80 KB) of a tile-major copy of B, two in LDS
// Column tiles are dealt to the XCDs (tile_of_workgroup) so that the workgroups that walk the same
// tile of B run on the same die, start together and find the panels in that die's L2.
#include "spmm_internal.h"

#include <climits>

namespace scorch {

typedef float f4 __attribute__((ext_vector_type(4)));

// Template parameters: RW rows per wavefront, kBatch entries whose LDS reads are in flight together, Q float4 per
// lane (the tile is 256*Q columns wide), KR rows of B per panel (KR * Q KB of LDS: 64 KB for the narrow tile, where a
// panel may not be taller than a row's 64-entry window, 80 KB for the wide one, which fills the 160 KB of a CU).
//
// The panel is double-buffered: one 1024-thread workgroup per CU holds two panels in LDS.  The next panel is
// fetched straight from global memory into LDS (global_load_lds_dwordx4: no registers, no ds_write) while the
// wavefronts work on the current one, and one barrier per panel both publishes the fetched panel and retires
// the one before it.  A workgroup covers 16*RW rows, so B crosses L2 -> LDS m/(16*RW) times.
template <int Q, int KR, bool DIRECT>
__device__ __forceinline__ void panel_fetch(const f4 *Bt, int k, int k0, f4 *sbuf, int wv, int lane, int64_t row_quads,
                                            int quads_left) {
    constexpr int kRowQuads = Q * (kPanelCols / 4);
    // The panel is KR * Q chunks of 1 KB (64 lanes x 16 bytes), dealt to the 16 wavefronts; a chunk is half a row or a
    // row of B inside the tile, so it lies wholly inside or wholly outside the matrix.  The wavefront-uniform parts
    // (panel base, validity of a chunk) are kept in scalar registers; a lane adds only its 32-bit offset.
    if constexpr (!DIRECT) {
        // tile-major copy of B: the panel is one contiguous range
        const f4 *panel = Bt + (int64_t)k0 * kRowQuads;
#pragma unroll
        for (int c = 0; c < KR * Q / 16; ++c) {
            const int chunk = c * 16 + wv;
            if (k0 + chunk / Q < k) __builtin_amdgcn_global_load_lds(panel + (uint32_t)(chunk * 64 + lane), sbuf + chunk * 64, 16, 0, 0);
        }
    } else {
        // the caller's row-major B: Bt points at the tile's first column of row 0, rows are row_quads vectors apart, and
        // only quads_left vectors of a row lie inside the matrix (ragged last tile: the lanes past the row's end load
        // nothing, and what they leave in LDS only feeds columns that are never stored)
#pragma unroll
        for (int c = 0; c < KR * Q / 16; ++c) {
            const int chunk = c * 16 + wv;
            const int row = chunk / Q, half = chunk % Q;
            if (k0 + row < k && half * 64 + lane < quads_left)
                __builtin_amdgcn_global_load_lds(Bt + (int64_t)(k0 + row) * row_quads + (uint32_t)(half * 64 + lane),
                                                 sbuf + chunk * 64, 16, 0, 0);
        }
    }
}

// Barrier that publishes a fetched panel.  The direct-to-LDS loads are counted by the issuing wavefront's vector-memory
// counter, and a workgroup barrier by itself only orders the LDS instructions a wavefront has issued: without the
// wait, wavefront A could pass the barrier while its chunk of the panel is still in flight and wavefront B would read
// stale LDS.  So every wavefront first drains its own loads (vmcnt(0)), then joins the barrier.  The fetch was issued
// before the previous panel's work, so the wait is normally already satisfied.
__device__ __forceinline__ void panel_publish() {
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
}

template <int RW, int kBatch, int Q>
struct PanelRows {
    int pend[RW], wbase[RW], pos[RW], colreg[RW], colnext[RW];
    float valreg[RW], valnext[RW];
    f4 acc[RW][Q];
};

// NB visits of one row: entries jj .. jj+NB-1 of the row's window (all inside the current panel).  The LDS reads
// of all NB entries are issued before the first multiply-add.
template <int NB, int Q, int KR>
__device__ __forceinline__ void panel_visits(f4 (&acc)[Q], int colreg, float valreg, int jj, const f4 *sbuf, int k0,
                                             int lane) {
    constexpr int kRowQuads = Q * (kPanelCols / 4);
    f4 x[NB][Q];
#pragma unroll
    for (int u = 0; u < NB; ++u) {
        const int c = __builtin_amdgcn_readlane(colreg, jj + u);
#pragma unroll
        for (int q = 0; q < Q; ++q) x[u][q] = sbuf[(c - k0) * kRowQuads + q * (kPanelCols / 4) + lane];
    }
#pragma unroll
    for (int u = 0; u < NB; ++u) {
        const float v = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(valreg), jj + u));
#pragma unroll
        for (int q = 0; q < Q; ++q)
#pragma unroll
            for (int i = 0; i < 4; ++i) acc[q][i] = __builtin_fmaf(v, x[u][q][i], acc[q][i]);
    }
}

// One panel's worth of work for the RW rows of a wavefront.  Columns within a row are strictly increasing
// (checked by the planner), so a panel of kRows rows of B takes at most kRows entries of a row: they are the
// lanes [pos, lim) of the row's 64-entry window.  A window that would be left with fewer than kRows entries is
// replaced: the replacement is requested before the panel's work and installed after it, so that its latency is
// hidden behind the work.  The visits of all RW rows are issued together (LDS reads first, multiply-adds after)
// to give a wavefront several independent reads per wait.
template <int RW, int kBatch, int Q, int KR>
__device__ __forceinline__ void panel_compute(PanelRows<RW, kBatch, Q> &st, const f4 *sbuf, int k0, int lane,
                                              const int32_t *colidx, const float *vals) {
    constexpr int kRows = KR;
    const int kend = k0 + kRows;
    int lim[RW], j[RW];
    bool shift[RW];
#pragma unroll
    for (int r = 0; r < RW; ++r) {
        lim[r] = (int)__builtin_popcountll(__ballot(st.colreg[r] < kend));
        asm("" : "+s"(lim[r]));  // a 32-bit scalar from here on (else the comparisons below are done in 64 bits on the VALU)
        j[r] = st.pos[r];
        shift[r] = lim[r] > kWave - kRows && st.wbase[r] + lim[r] < st.pend[r];
        if (shift[r]) {
            const int p = st.wbase[r] + lim[r] + lane;
            st.colnext[r] = p < st.pend[r] ? colidx[p] : INT_MAX;
            st.valnext[r] = p < st.pend[r] ? vals[p] : 0.f;
        }
    }
#pragma unroll
    for (int r = 0; r < RW; ++r) {
        // Whole batches first, without a test per entry (all branches here are wave-uniform, and the scalar
        // instructions of such tests cost issue slots like vector ones: this loop is bound by instruction issue), then
        // half a batch if that many entries are left, then the remaining entries one at a time.
        int jj = j[r];
        for (; jj + kBatch <= lim[r]; jj += kBatch) panel_visits<kBatch, Q, KR>(st.acc[r], st.colreg[r], st.valreg[r], jj, sbuf, k0, lane);
        if constexpr (kBatch >= 4) {
            if (jj + kBatch / 2 <= lim[r]) {
                panel_visits<kBatch / 2, Q, KR>(st.acc[r], st.colreg[r], st.valreg[r], jj, sbuf, k0, lane);
                jj += kBatch / 2;
            }
        }
        for (; jj < lim[r]; ++jj) panel_visits<1, Q, KR>(st.acc[r], st.colreg[r], st.valreg[r], jj, sbuf, k0, lane);
    }
#pragma unroll
    for (int r = 0; r < RW; ++r) {
        if (shift[r]) {
            st.wbase[r] += lim[r];
            st.colreg[r] = st.colnext[r];
            st.valreg[r] = st.valnext[r];
            st.pos[r] = 0;
        } else {
            st.pos[r] = lim[r];
        }
    }
}

template <int RW, int kBatch, int Q, int KR, bool DIRECT>
__global__ __launch_bounds__(16 * kWave) void spmm_panel_kernel(const PanelArgs a) {
    constexpr int WPB = 16;
    constexpr int kRowQuads = Q * (kPanelCols / 4);
    constexpr int kRows = KR;
    static_assert(KR <= kWave, "a panel must not take more entries of a row than its 64-entry window holds");
    static_assert((KR * Q) % 16 == 0 && 2 * KR * Q <= 160, "two panels of KR*Q KB, dealt to 16 wavefronts, in 160 KB of LDS");
    __shared__ f4 s_b0[kRows * kRowQuads];
    __shared__ f4 s_b1[kRows * kRowQuads];
    const int tid = threadIdx.x;
    const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lane = tid & 63;
    uint32_t ct, rb;
    if (!tile_of_workgroup(a.xcd_slices, a.ntiles, (uint32_t)a.nrb, ct, rb)) return;
    const int c0 = (int)ct * (Q * kPanelCols) + lane * 4;
    // tile-major copy: tile ct is a dense k x (256 Q) block; row-major B: the tile starts at column 256 Q ct of every row
    const f4 *Bt = reinterpret_cast<const f4 *>(DIRECT ? a.Bp + (int64_t)ct * (Q * kPanelCols)
                                                       : a.Bp + (int64_t)ct * a.k * (Q * kPanelCols));
    const int64_t row_quads = a.ldb / 4;
    const int quads_left = (a.n - (int)ct * (Q * kPanelCols)) / 4;
    const int64_t row_base = (int64_t)rb * (WPB * RW) + wv * RW;

    panel_fetch<Q, KR, DIRECT>(Bt, a.k, 0, s_b0, wv, lane, row_quads, quads_left);
    PanelRows<RW, kBatch, Q> st;
#pragma unroll
    for (int r = 0; r < RW; ++r) {
        const int64_t row = row_base + r;
        int p0 = 0, p1 = 0;
        if (row < a.m) {
            p0 = a.rowptr[row];
            p1 = a.rowptr[row + 1];
        }
        st.wbase[r] = p0;
        st.pend[r] = p1;
        st.pos[r] = 0;
        const int p = p0 + lane;
        st.colreg[r] = p < p1 ? a.colidx[p] : INT_MAX;
        st.valreg[r] = p < p1 ? a.vals[p] : 0.f;
        st.colnext[r] = INT_MAX;
        st.valnext[r] = 0.f;
#pragma unroll
        for (int q = 0; q < Q; ++q) st.acc[r][q] = f4{0.f, 0.f, 0.f, 0.f};
    }
    for (int k0 = 0; k0 < a.k; k0 += 2 * kRows) {
        panel_publish();  // panel k0 has landed in s_b0; nobody reads s_b1 any more
        const bool odd = k0 + kRows < a.k;
        if (odd) panel_fetch<Q, KR, DIRECT>(Bt, a.k, k0 + kRows, s_b1, wv, lane, row_quads, quads_left);
        panel_compute<RW, kBatch, Q, KR>(st, s_b0, k0, lane, a.colidx, a.vals);
        if (odd) {
            panel_publish();  // panel k0 + kRows has landed in s_b1; nobody reads s_b0 any more
            if (k0 + 2 * kRows < a.k) panel_fetch<Q, KR, DIRECT>(Bt, a.k, k0 + 2 * kRows, s_b0, wv, lane, row_quads, quads_left);
            panel_compute<RW, kBatch, Q, KR>(st, s_b1, k0 + kRows, lane, a.colidx, a.vals);
        }
    }
#pragma unroll
    for (int r = 0; r < RW; ++r) {
        const int64_t row = row_base + r;
#pragma unroll
        for (int q = 0; q < Q; ++q) {
            const int c = c0 + q * kPanelCols;
            if (row < a.m && c < a.n) {
                f4 v = st.acc[r][q];
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
    // Two shapes: tile of 256 columns with 64-row panels, or tile of 512 columns with 40-row panels (the wide
    // tile halves the per-entry broadcast overhead and is chosen for denser matrices and n >= 512).  Both use
    // 64 rows per workgroup and 128 or 160 KB of LDS, i.e. one workgroup and four wavefronts per SIMD on a CU.
    const int variant = plan->params.PANEL;
    struct Shape { int RW, WPB, Q; };
    const Shape sh = variant == 3 ? Shape{4, 16, 4} : (variant == 2 ? Shape{4, 16, 2} : Shape{4, 16, 1});
    const int W = sh.Q * kPanelCols;
    // The panels are fetched either from a tile-major copy of B made here (one read and one write of B per call) or
    // straight from the caller's row-major B (pack=0 in the tuning text; see want_panel for the measurements).
    const bool direct = plan->params.PDIRECT != 0;
    const float *Bsrc = B;
    if (!direct) {
        float *Bp = reinterpret_cast<float *>(plan->workspace + plan->layout.off_bpack);
        scorch_status_t st = launch_pack_b(B, ldb, plan->k, plan->n, W, Bp, stream);
        if (st != SCORCH_OK) return st;
        Bsrc = Bp;
    }
    PanelArgs a{};
    a.rowptr = rowptr;
    a.colidx = colidx;
    a.vals = vals;
    a.Bp = Bsrc;
    a.ldb = ldb;
    a.C = C;
    a.ldc = ldc;
    a.m = plan->m;
    a.k = plan->k;
    a.n = plan->n;
    a.nrb = (plan->m + sh.WPB * sh.RW - 1) / (sh.WPB * sh.RW);
    a.ntiles = (plan->n + W - 1) / W;
    a.xcd_slices = 1;
    a.bias = bias;
    a.act = act;
    const int64_t grid = xcd_grid_size(a.xcd_slices, a.ntiles, a.nrb);
    if (grid > 0x7fffffffLL) {
        set_error("launch grid of %lld workgroups exceeds the HIP limit", (long long)grid);
        return SCORCH_ERR_UNSUPPORTED;
    }
    const dim3 g((uint32_t)grid), b(sh.WPB * kWave);
    if (variant == 3) {
        // experiment (panel=3 in the tuning text, direct fetch only): 1024-column tiles, 20-row panels
        hipLaunchKernelGGL((spmm_panel_kernel<4, 2, 4, 20, true>), g, b, 0, stream, a);
    } else if (variant == 2) {
        if (direct) hipLaunchKernelGGL((spmm_panel_kernel<4, 2, 2, 40, true>), g, b, 0, stream, a);
        else hipLaunchKernelGGL((spmm_panel_kernel<4, 2, 2, 40, false>), g, b, 0, stream, a);
    } else {
        if (direct) hipLaunchKernelGGL((spmm_panel_kernel<4, 4, 1, 64, true>), g, b, 0, stream, a);
        else hipLaunchKernelGGL((spmm_panel_kernel<4, 4, 1, 64, false>), g, b, 0, stream, a);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return hip_fail(e, "launch spmm_panel_kernel");
    return SCORCH_OK;
}

}  // namespace scorch
