// Planner: one-time analysis of a CSR sparsity pattern on the device.
//
// The paper's remedy for SpMM cost is CPU-side loop ordering and tiling (Sections 4.1, 4.2); it
// names load balance and irregular access as the open problems of sparse kernels (related-work
// section).  On a GPU the skew of row lengths decides everything, so rows are classed by length
// and handed to different execution paths (see spmm_exec.hip):
//   short  len <= LW       -> windows of consecutive rows, cut along the merge path
//                             key_i = rowptr[i] + ALPHA*i every BN key units
//   wave   LW < len <= CH  -> ascending list of row ids, one wavefront each
//   block  len > CH        -> pieces of at most BCH entries; a row with several pieces gets
//                             consecutive partial-row slots and an entry in the split list
// All lists come out in ascending row order (stable compaction), so the plan is a pure function
// of rowptr and the parameters.
#include "spmm_internal.h"
#include "rowptr_keys.h"

#include <algorithm>
#include <cstdlib>

namespace scorch {

constexpr int kQ = 5;  // counted quantities: wave rows, items, split rows, slots, short rows

struct PlanArgs {
    const int32_t *rowptr;
    int32_t m;
    int32_t LW, CH, BCH;
    int64_t nblk;
    int32_t *counts;  // [kQ][nblk], turned into exclusive offsets by the scan
    int32_t *totals;  // [kQ]
    int32_t *wave_rows;
    int2 *wave_span;  // entry range [p0, p1) of every wave row, beside its id
    int4 *items;
    int4 *split;
    int64_t cap_wave, cap_items, cap_split;  // list capacities: writes beyond them are dropped
};

struct RowClass {
    int wave, items, split, slots, is_short;
};

__device__ __forceinline__ RowClass classify(int len, int LW, int CH, int BCH) {
    RowClass r{0, 0, 0, 0, 0};
    if (len <= LW) r.is_short = 1;
    else if (len <= CH) r.wave = 1;
    else {
        r.items = (len + BCH - 1) / BCH;
        if (r.items > 1) {
            r.split = 1;
            r.slots = r.items;
        }
    }
    return r;
}

// Exclusive prefix sum over the 256 threads of a workgroup; `total` is the workgroup sum.
__device__ __forceinline__ int block_exclusive_scan(int v, int &total, int *s_wave /*[4]*/) {
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    int inc = v;
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) {
        const int o = __shfl_up(inc, off, kWave);
        if (lane >= off) inc += o;
    }
    __syncthreads();
    if (lane == kWave - 1) s_wave[wv] = inc;
    __syncthreads();
    int base = 0;
    total = 0;
#pragma unroll
    for (int w = 0; w < kWavesPerBlock; ++w) {
        const int t = s_wave[w];
        if (w < wv) base += t;
        total += t;
    }
    return base + inc - v;
}

__global__ __launch_bounds__(kBlock) void plan_count_kernel(const PlanArgs a) {
    __shared__ int s_wave[kWavesPerBlock];
    const int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    RowClass rc{0, 0, 0, 0, 0};
    if (i < a.m) rc = classify(a.rowptr[i + 1] - a.rowptr[i], a.LW, a.CH, a.BCH);
    const int q[kQ] = {rc.wave, rc.items, rc.split, rc.slots, rc.is_short};
#pragma unroll
    for (int k = 0; k < kQ; ++k) {
        int total;
        (void)block_exclusive_scan(q[k], total, s_wave);
        if (threadIdx.x == 0) a.counts[(int64_t)k * a.nblk + blockIdx.x] = total;
    }
}

// One workgroup of 1024 threads turns each of the kQ count arrays into exclusive offsets and stores the totals:
// every thread sums a contiguous slice, the 1024 slice sums are scanned with wavefront shuffles (16 wavefronts),
// then every thread rewrites its slice.
__global__ __launch_bounds__(1024) void plan_scan_kernel(const PlanArgs a) {
    __shared__ int s_wave[16];
    const int tid = threadIdx.x;
    const int lane = tid & 63, wv = tid >> 6;
    const int64_t per = (a.nblk + 1023) / 1024;
    for (int k = 0; k < kQ; ++k) {
        int32_t *c = a.counts + (int64_t)k * a.nblk;
        const int64_t lo = std::min<int64_t>((int64_t)tid * per, a.nblk);
        const int64_t hi = std::min<int64_t>(lo + per, a.nblk);
        int sum = 0;
        for (int64_t j = lo; j < hi; ++j) sum += c[j];
        int inc = sum;
#pragma unroll
        for (int off = 1; off < kWave; off <<= 1) {
            const int o = __shfl_up(inc, off, kWave);
            if (lane >= off) inc += o;
        }
        __syncthreads();  // s_wave of the previous quantity has been read
        if (lane == kWave - 1) s_wave[wv] = inc;
        __syncthreads();
        int base = 0, total = 0;
#pragma unroll
        for (int w = 0; w < 16; ++w) {
            const int t = s_wave[w];
            if (w < wv) base += t;
            total += t;
        }
        if (tid == 0) a.totals[k] = total;
        int run = base + inc - sum;
        for (int64_t j = lo; j < hi; ++j) {
            const int t = c[j];
            c[j] = run;
            run += t;
        }
    }
}

__global__ __launch_bounds__(kBlock) void plan_scatter_kernel(const PlanArgs a) {
    __shared__ int s_wave[kWavesPerBlock];
    const int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    RowClass rc{0, 0, 0, 0, 0};
    int p0 = 0, p1 = 0;
    if (i < a.m) {
        p0 = a.rowptr[i];
        p1 = a.rowptr[i + 1];
        rc = classify(p1 - p0, a.LW, a.CH, a.BCH);
    }
    int total;
    const int pos_wave = a.counts[0 * a.nblk + blockIdx.x] + block_exclusive_scan(rc.wave, total, s_wave);
    const int pos_item = a.counts[1 * a.nblk + blockIdx.x] + block_exclusive_scan(rc.items, total, s_wave);
    const int pos_split = a.counts[2 * a.nblk + blockIdx.x] + block_exclusive_scan(rc.split, total, s_wave);
    const int pos_slot = a.counts[3 * a.nblk + blockIdx.x] + block_exclusive_scan(rc.slots, total, s_wave);
    // The capacities hold for every valid rowptr; the guards only keep a malformed one in bounds
    // (the host then reports the overflow from the totals).
    if (rc.wave && pos_wave < a.cap_wave) {
        a.wave_rows[pos_wave] = (int)i;
        a.wave_span[pos_wave] = make_int2(p0, p1);
    }
    for (int c = 0; c < rc.items && (int64_t)pos_item + c < a.cap_items; ++c) {
        const int b = p0 + c * a.BCH;
        a.items[pos_item + c] = make_int4((int)i, b, min(p1, b + a.BCH), rc.split ? pos_slot + c : -1);
    }
    if (rc.split && pos_split < a.cap_split) a.split[pos_split] = make_int4((int)i, pos_slot, rc.items, 0);
}

// win_row_start[w] = number of rows whose key rowptr[i] + ALPHA*i is below w*BN.
__global__ __launch_bounds__(kBlock) void plan_window_kernel(const int32_t *rowptr, int32_t m, int32_t BN,
                                                             int32_t ALPHA, int64_t n_windows,
                                                             int32_t *win_row_start) {
    const int64_t w = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (w > n_windows) return;
    if (w == n_windows) {
        win_row_start[w] = m;
        return;
    }
    const int64_t target = w * (int64_t)BN;
    int64_t lo = 0, hi = m;
    while (lo < hi) {
        const int64_t mid = (lo + hi) >> 1;
        const int64_t key = (int64_t)rowptr[mid] + (int64_t)ALPHA * mid;
        if (key < target) lo = mid + 1;
        else hi = mid;
    }
    win_row_start[w] = (int32_t)lo;
}

// What a window's wavefront stages in LDS: the entries from the first to the last short row of the window (rows of
// up to LW entries; the window holds at most 64 rows), at most stage_max of them.  Stored in the plan so that the
// execution kernel can fetch colidx/vals at once instead of waiting for the row pointers first.
// stage[w] = (first entry, number of entries), or (0, -1) for a window without short rows.
__global__ __launch_bounds__(kBlock) void plan_stage_kernel(const int32_t *rowptr, const int32_t *win_row_start,
                                                            int64_t n_windows, int32_t LW, int32_t stage_max,
                                                            int2 *stage) {
    const int64_t w = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (w >= n_windows) return;
    const int r0 = win_row_start[w];
    const int r1 = min(win_row_start[w + 1], r0 + kWindowRowsMax);
    int first = -1, last = -1;
    int prev = r0 < r1 ? rowptr[r0] : 0;
    int sbeg = 0, send = 0;
    for (int r = r0; r < r1; ++r) {
        const int next = rowptr[r + 1];
        if (next - prev <= LW) {
            if (first < 0) {
                first = r;
                sbeg = prev;
            }
            last = r;
            send = next;
        }
        prev = next;
    }
    stage[w] = first < 0 ? make_int2(0, -1) : make_int2(sbeg, min(send - sbeg, stage_max));
    (void)last;
}

// Sets *flag when some row's column indices are not strictly increasing (one wavefront per row).
__global__ __launch_bounds__(kBlock) void plan_sorted_kernel(const int32_t *rowptr, const int32_t *colidx, int32_t m,
                                                             int32_t *flag) {
    const int lane = threadIdx.x & 63;
    for (int64_t row = (int64_t)blockIdx.x * kWavesPerBlock + (threadIdx.x >> 6); row < m;
         row += (int64_t)gridDim.x * kWavesPerBlock) {
        const int p0 = rowptr[row], p1 = rowptr[row + 1];
        bool bad = false;
        for (int p = p0 + 1 + lane; p < p1; p += kWave) bad |= colidx[p] <= colidx[p - 1];
        if (bad) *flag = 1;
    }
}

// ---- hot columns ------------------------------------------------------------------------------------------
// When B is larger than the memory-side cache, the gathers of the rarely referenced rows of B stream through that
// cache and evict the often referenced ones.  The planner therefore counts how often every column of A occurs,
// marks the most referenced columns up to a byte budget as hot (one bit per column), and the kernels read only
// those rows of B with the default cache policy and all others with the streaming (nt) policy, which on this
// hardware leaves the memory-side cache alone.

// deg[c] = number of sampled stored entries with column c.  One entry is taken out of every `stride` consecutive
// ones (stride a power of two; 1 = all entries), at a position that varies from one group of entries to the next:
// a fixed position would always pick the same rank within rows of a regular length, i.e. always low or always high
// columns.  The count only ranks the columns for a cache policy, so a sample serves; the atomic additions (one
// 32-byte memory transaction each) are what the planner spends most of its time on for a large matrix.
__global__ __launch_bounds__(kBlock) void plan_coldeg_kernel(const int32_t *colidx, int64_t nnz, int32_t k,
                                                             int32_t stride, int32_t *deg) {
    const int64_t groups = (nnz + stride - 1) / stride;
    for (int64_t g = (int64_t)blockIdx.x * kBlock + threadIdx.x; g < groups; g += (int64_t)gridDim.x * kBlock) {
        const int64_t p = g * stride + (int64_t)((((uint32_t)g * 2654435761u) >> 16) & (uint32_t)(stride - 1));
        if (p >= nnz) continue;
        const int c = colidx[p];
        if ((uint32_t)c < (uint32_t)k) atomicAdd(&deg[c], 1);
    }
}

// Histogram bin of a degree: 16 bins per power of two, monotone in d; bin 0 holds d = 0.
__host__ __device__ __forceinline__ int degree_bin(int d) {
    if (d <= 0) return 0;
    const int e = 31 - __builtin_clz((unsigned)d);
    const int frac = e >= 4 ? (d >> (e - 4)) & 15 : (d << (4 - e)) & 15;
    return e * 16 + frac + 1;
}

// bins[b] = (number of columns, number of stored entries) whose degree falls into bin b.  Counted per workgroup
// in LDS first: nearly all columns of a graph fall into a handful of bins.
__global__ __launch_bounds__(kBlock) void plan_degbins_kernel(const int32_t *deg, int32_t k, unsigned long long *bins) {
    __shared__ unsigned int s_cnt[kDegBins], s_sum[kDegBins];  // a workgroup sees fewer than 2^31 entries in total
    for (int b = threadIdx.x; b < kDegBins; b += kBlock) {
        s_cnt[b] = 0;
        s_sum[b] = 0;
    }
    __syncthreads();
    for (int64_t c = (int64_t)blockIdx.x * kBlock + threadIdx.x; c < k; c += (int64_t)gridDim.x * kBlock) {
        const int d = deg[c];
        const int b = degree_bin(d);
        atomicAdd(&s_cnt[b], 1u);
        atomicAdd(&s_sum[b], (unsigned int)d);
    }
    __syncthreads();
    for (int b = threadIdx.x; b < kDegBins; b += kBlock) {
        if (s_cnt[b]) {
            atomicAdd(&bins[2 * b], (unsigned long long)s_cnt[b]);
            atomicAdd(&bins[2 * b + 1], (unsigned long long)s_sum[b]);
        }
    }
}

// mask word w holds the hot bits of columns 32w .. 32w+31: hot = degree bin >= min_bin.
__global__ __launch_bounds__(kBlock) void plan_hotmask_kernel(const int32_t *deg, int32_t k, int min_bin, int64_t nwords,
                                                              uint32_t *mask) {
    for (int64_t w = (int64_t)blockIdx.x * kBlock + threadIdx.x; w < nwords; w += (int64_t)gridDim.x * kBlock) {
        uint32_t bits = 0;
        for (int i = 0; i < 32; ++i) {
            const int64_t c = w * 32 + i;
            if (c < k && degree_bin(deg[c]) >= min_bin) bits |= 1u << i;
        }
        mask[w] = bits;
    }
}

static scorch_status_t mark_hot_columns(scorch_spmm_plan_t *plan, const int32_t *colidx, bool forced, hipStream_t stream) {
    const WorkspaceLayout &L = plan->layout;
    char *ws = plan->workspace;
    int32_t *deg = reinterpret_cast<int32_t *>(ws + L.off_coldeg);
    uint32_t *mask = reinterpret_cast<uint32_t *>(ws + L.off_hotmask);
    unsigned long long *bins = reinterpret_cast<unsigned long long *>(ws + L.off_degbins);
    hipError_t e = hipMemsetAsync(deg, 0, (size_t)plan->k * 4, stream);
    if (e == hipSuccess) e = hipMemsetAsync(bins, 0, (size_t)kDegBins * 16, stream);
    if (e != hipSuccess) return hip_fail(e, "clear column degrees");
    // every entry up to 2^24 of them, beyond that every 2nd, 4th, ... so that at most 2^24 are counted
    int32_t stride = 1;
    while ((plan->nnz + stride - 1) / stride > kHotSampleMax) stride *= 2;
    const int64_t groups = (plan->nnz + stride - 1) / stride;
    const uint32_t g1 = (uint32_t)std::min<int64_t>((groups + kBlock - 1) / kBlock, 256 * 64);
    const uint32_t g2 = (uint32_t)std::min<int64_t>(((int64_t)plan->k + kBlock - 1) / kBlock, 256 * 4);
    hipLaunchKernelGGL(plan_coldeg_kernel, dim3(g1), dim3(kBlock), 0, stream, colidx, plan->nnz, plan->k, stride, deg);
    hipLaunchKernelGGL(plan_degbins_kernel, dim3(g2), dim3(kBlock), 0, stream, deg, plan->k, bins);
    e = hipGetLastError();
    if (e != hipSuccess) return hip_fail(e, "launch column-degree kernels");
    static_assert(sizeof(unsigned long long) == 8, "bin layout");
    unsigned long long host_bins[2 * kDegBins];
    e = hipMemcpyAsync(host_bins, bins, sizeof(host_bins), hipMemcpyDeviceToHost, stream);
    if (e == hipSuccess) e = hipStreamSynchronize(stream);
    if (e != hipSuccess) return hip_fail(e, "read the column-degree histogram");
    // a row of B occupies whole 128-byte lines in the caches
    const int64_t row_bytes = ((int64_t)plan->n * 4 + 127) / 128 * 128;
    const int64_t max_rows = std::max<int64_t>(1, (int64_t)plan->params.HOT * 1024 / row_bytes);
    int64_t rows = 0, entries = 0;
    int min_bin = kDegBins;
    for (int b = kDegBins - 1; b >= 1; --b) {  // bin 0: columns that never occur
        if (rows + (int64_t)host_bins[2 * b] > max_rows) break;
        rows += (int64_t)host_bins[2 * b];
        entries += (int64_t)host_bins[2 * b + 1];
        min_bin = b;
    }
    plan->n_hot = 0;
    plan->hot_share = groups > 0 ? (float)std::min(1.0, (double)entries / (double)groups) : 0.f;  // of the sampled entries
    // Worth it only when a small part of B takes a large part of the gathers (measured on the large power-law
    // workload: 5 % of the rows of B, 54 % of the gathers, 6.5 % less time).
    if (rows == 0 || (!forced && plan->hot_share < 0.25f)) return SCORCH_OK;
    const int64_t nwords = (int64_t)plan->k / 32 + 1;
    const uint32_t g3 = (uint32_t)std::min<int64_t>((nwords + kBlock - 1) / kBlock, 256 * 16);
    hipLaunchKernelGGL(plan_hotmask_kernel, dim3(g3), dim3(kBlock), 0, stream, deg, plan->k, min_bin, nwords, mask);
    e = hipGetLastError();
    if (e != hipSuccess) return hip_fail(e, "launch plan_hotmask_kernel");
    plan->n_hot = (int32_t)std::min<int64_t>(rows, 0x7fffffff);
    return SCORCH_OK;
}

// Row pointers from a sorted list of row keys.  Coordinate list: keys are the row coordinates of the entries and
// position p itself is the pointer (pos == nullptr).  Doubly compressed rows: keys are the ids of the stored rows
// and pos[p] is where row keys[p] starts (pos[count] = nnz).  Key p closes the rows between its predecessor and
// itself: rowptr[r] = pos[p] for keys[p-1] < r <= keys[p]; the sentinel p = count closes the rows up to m.
__global__ __launch_bounds__(kBlock) void rowptr_from_keys_kernel(const int32_t *keys, const int32_t *pos, int64_t count,
                                                                  int32_t m, bool strictly_increasing, int32_t *rowptr,
                                                                  int32_t *bad_flag) {
    for (int64_t p = (int64_t)blockIdx.x * kBlock + threadIdx.x; p <= count; p += (int64_t)gridDim.x * kBlock) {
        const int prev = p > 0 ? keys[p - 1] : -1;
        const int cur = p < count ? keys[p] : m;
        int32_t lo, hi;
        if (!rowptr_fill_range(p, count, prev, cur, m, strictly_increasing, lo, hi)) {
            if (bad_flag) *bad_flag = 1;
            continue;
        }
        const int32_t value = pos ? pos[p] : (int32_t)p;
        for (int r = lo; r <= hi; ++r) rowptr[r] = value;  // 0 <= lo, hi <= m
    }
}

scorch_status_t launch_rowptr_from_keys(int32_t m, int64_t count, const int32_t *keys, const int32_t *pos,
                                        bool strictly_increasing, int32_t *rowptr, int32_t *bad_flag,
                                        hipStream_t stream) {
    const uint32_t grid = (uint32_t)std::min<int64_t>((count + 1 + kBlock - 1) / kBlock, 256 * 32);
    hipLaunchKernelGGL(rowptr_from_keys_kernel, dim3(grid), dim3(kBlock), 0, stream, keys, pos, count, m,
                       strictly_increasing, rowptr, bad_flag);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return hip_fail(e, "launch rowptr_from_keys_kernel");
    return SCORCH_OK;
}

// ------------------------------------------------------------------------------------------
// host side
// ------------------------------------------------------------------------------------------
Tuning read_tuning_from_env() { return parse_tuning(std::getenv("SCORCH_SPMM_TUNE")); }

static int32_t pow2_floor(int64_t x) {
    int32_t p = 1;
    while ((int64_t)p * 2 <= x) p *= 2;
    return p;
}

// XCD-sliced execution pays when B as a whole overflows an XCD's 4 MB L2 at least twice over but a 128-byte-wide
// column slice of it fits, and rows are long enough that re-reading colidx/vals and walking the row once per slice
// is cheap next to the gathers (8 bytes of A against 128 bytes of B per entry and slice).  Measured on uniform random
// patterns: 164 entries per row, B 8-32 MB: 1.3-2.1x faster than the plain gather; 82 entries, B 8-33 MB: 1.0-1.5x;
// 65 entries: even; 33-41 entries: 1.2-1.4x slower; B of 4 MB (mostly L2-resident anyway): 1.1-1.3x slower.
// Beyond that: the 128-byte slices still win over whole rows when a slice is a few times larger than an XCD's L2
// (uniform patterns and a power-law graph with 100-164 entries per row, slices of 4-13 MB: 1.1-2.3x faster; a
// 17 MB slice: 1.1x slower), and with shorter rows 256-byte slices do (an XCD's L2 then keeps twice to sixteen times
// as many rows of B as with whole rows, and a wavefront has 4 rows of B in flight per load): power-law graphs of
// 50 k to 1 M nodes, 5 to 100 entries per row, n = 128 to 1024 in multiples of 64: 5-30 % less time than whole rows
// (one case of 21: 1 %); uniform and pruned patterns outside the 128-byte rule: 0-43 % less; n = 160: 0-16 % less;
// n = 96, 100, 132: 4-30 % more, hence the multiple of 64.  Returns the columns per slice (0 = whole rows).
static int32_t want_sliced(int32_t m, int32_t k, int64_t nnz, int32_t n, bool hot_candidate) {
    if (m <= 0 || n % 4 != 0 || n < 2 * kSliceCols) return 0;
    const int64_t slice_bytes = (int64_t)k * kSliceCols * 4;
    const int64_t b_bytes = (int64_t)k * n * 4;
    const bool long_rows = nnz / m >= 64 && b_bytes >= 8ll << 20;
    if (long_rows && slice_bytes <= kL2SliceBudget) return kSliceCols;
    if (hot_candidate) return 0;  // the hot/cold split needs whole rows
    if (long_rows && slice_bytes <= 13ll << 20 && n >= 128) return kSliceCols;  // n = 64 with a 13 MB slice: 2-6 % more time
    // B of 6 MB (1.5 L2s), 410 entries per row, n = 384: 19 % less time with 256-byte slices; B of 4 MB: 23 % more
    return (n >= 128 && n % 64 == 0 && b_bytes >= 6ll << 20) ? 64 : 0;
}

// The panel kernel (spmm_panel.hip) streams all of B through LDS once per block of 64 rows of A, a cost that does
// not depend on nnz, and then pays per entry less than the gather kernels.  It needs a workgroup (64 rows x 512 or
// 256 columns) for every CU.  From sweeps over unstructured-pruned shapes (4096..65536 rows, k 2048..16384):
//   wide tiles (n >= 512): ahead of the gather kernels from 3 % stored entries upwards (3 %: 0.70 against 0.73 ms,
//     4 %: 0.39 against 0.47, 6 %: 0.48 against 0.70, 10 %: 0.65 against 1.12), behind with fewer than 256 workgroups;
//   narrow tiles: about even with the gather kernels at 10 % (0.50 against 0.52 ms, 0.54 against 0.62), behind at
//     4-8 %; used from 10 % upwards when only they give 256 workgroups.
// Returns the kernel shape (0 = do not use, 1 = 256-column tiles, 2 = 512-column tiles).
static int32_t want_panel(int32_t m, int32_t k, int64_t nnz, int32_t n) {
    if (m <= 0 || k < 1024 || n % 4 != 0 || n < kPanelCols || nnz / m < 128) return 0;
    const double density = (double)nnz / ((double)m * (double)k);
    const int64_t row_blocks = ((int64_t)m + 63) / 64;
    if (n >= 2 * kPanelCols && density >= 0.03 && row_blocks * ((n + 2 * kPanelCols - 1) / (2 * kPanelCols)) >= 256) return 2;
    // 256-column tiles: from 7.5 % stored entries upwards, counted per tile column actually used (a last tile that is
    // half empty costs as much as a full one).  Measured on pruned-weight shapes with n = 256, 384, 4096: at 8 % the
    // panel kernel is 0-23 % faster than the gathers, at 10 % 0-30 %, at 6 % between 10 % faster and 20 % slower.
    const int64_t tiles1 = (n + kPanelCols - 1) / kPanelCols;
    if (density * (double)n / (double)(tiles1 * kPanelCols) >= 0.075 && row_blocks * tiles1 >= 256) return 1;
    return 0;
}

PlanParams choose_params(int32_t m, int32_t k, int64_t nnz, int32_t n, const Tuning &t) {
    PlanParams p;
    p.ALPHA = 4;
    // Windows of 128 key units, but small problems get smaller windows so that there are a few thousand
    // wavefronts' worth of them (a lane group walks its rows one after the other, each a full memory latency).
    // Narrow B (n <= 32) means 8 or more lane groups per wavefront, each walking one row of the window (for n <= 4
    // the lanes split the window's entries): larger windows keep more of them busy.
    const int32_t bn_cap = n <= 32 ? kBNMax : 128;
    p.BN = std::min<int32_t>(bn_cap, std::max<int32_t>(16, pow2_floor(std::max<int64_t>(1, (nnz + (int64_t)p.ALPHA * m) / 4096))));
    p.LW = 32;
    // B several times larger than the memory-side cache: see build_plan (hot columns).
    const bool hot_candidate = (int64_t)k * n * 4 > 3 * kMallBytes && n >= 96 && nnz >= 4 * (int64_t)k;
    p.SLICED = want_sliced(m, k, nnz, n, hot_candidate);
    if (t.sliced >= 0) {  // 0: off, 1: the default width, 32 / 64 / 128: that many columns per slice
        const int32_t cols = t.sliced == 1 ? kSliceCols : t.sliced;
        p.SLICED = ((cols == 32 || cols == 64 || cols == 128) && n % 4 == 0) ? cols : 0;
    }
    // A row stride of B above 512 bytes scatters a 128-byte column slice over few L2 sets; gather from a
    // dense slice-major copy instead (costs one read and one write of B per call).
    p.PACK = (p.SLICED == kSliceCols && n > 128) ? 1 : 0;
    if (t.pack >= 0) p.PACK = (p.SLICED == kSliceCols && t.pack != 0) ? 1 : 0;
    p.PANEL = want_panel(m, k, nnz, n);
    if (t.panel >= 0) p.PANEL = (t.panel > 0 && t.panel <= 3 && n % 4 == 0 && k > 0) ? t.panel : 0;
    // The panel kernel fetches its panels straight from the caller's row-major B (pruned-FFN workload, row stride 8 KB:
    // 1.10 against 1.13 ms with a tile-major copy made at every call, which costs one read and one write of B; the
    // workgroups of a tile column walk the same panels at the same time, so only a few panels per die have to stay in
    // L2 and the set conflicts of a power-of-two stride do not matter); pack=1 brings the copy back.
    p.PDIRECT = (p.PANEL && (t.pack != 1 || p.PANEL == 3)) ? 1 : 0;
    // Enough independent wavefront tasks to fill 256 CUs several times over, but pieces long
    // enough that the per-piece overhead stays small.
    const int64_t coltiles = p.SLICED ? (n + p.SLICED - 1) / p.SLICED : std::max<int64_t>(1, (n + 511) / 512);
    const int32_t ch_cap = p.SLICED ? 4096 : 1024;
    p.CH = std::min<int32_t>(ch_cap, std::max<int32_t>(256, pow2_floor(std::max<int64_t>(1, nnz * coltiles / 32768))));
    p.U = 8;
    p.NT = 1;
    // B several times larger than the memory-side cache: see build_plan (hot columns).  Budget: a quarter of that
    // cache.  Measured on the large power-law pattern: B 3.8x / 4.9x / 9.8x the cache: 5-6 % less time; 2.4x: 4 % more;
    // 1.2x: 57 % more (the cache then holds most of B anyway and the streaming policy forfeits that).
    // Rows of B narrower than three cache lines lose with it on every pattern tried (n = 64: 4-18 % more time).
    p.HOT = (hot_candidate && p.SLICED == 0) ? (int32_t)(kMallBytes / 4 / 1024) : 0;
    if (t.hot >= 0) p.HOT = t.hot;
    if (t.bn > 0) p.BN = t.bn;
    if (t.alpha > 0) p.ALPHA = t.alpha;
    if (t.lw > 0) p.LW = t.lw;
    if (t.ch > 0) p.CH = t.ch;
    // One-lane groups (n <= 4): a workgroup takes 256 entries per step, so much longer pieces are still short chains,
    // and rows that are not cut need no second launch (mid-size graph pattern, n = 1: 21.2 -> 18.1 us).
    p.BCH = (n <= 4 ? 64 : 4) * p.CH;
    if (t.bch > 0) p.BCH = t.bch;
    if (t.u > 0) p.U = t.u;
    if (t.nt >= 0) p.NT = t.nt;
    // Hard limits the kernels rely on.
    p.BN = std::min(std::max(p.BN, 16), kBNMax);
    p.LW = std::min(std::max(p.LW, 0), kLWMax);
    p.ALPHA = std::max(p.ALPHA, (p.BN + kWindowRowsMax - 1) / kWindowRowsMax);  // <= 64 rows per window
    p.CH = std::max(p.CH, p.LW);
    p.BCH = std::max(p.BCH, 64);
    p.U = p.U >= 8 ? 8 : 4;
    p.NT &= 1;
    return p;
}

static uint64_t align_up(uint64_t x, uint64_t a) { return (x + a - 1) / a * a; }

WorkspaceLayout layout_workspace(int32_t m, int32_t k, int64_t nnz, int32_t n, const PlanParams &p) {
    WorkspaceLayout L{};
    L.nblk = ((int64_t)m + kBlock - 1) / kBlock;
    L.n_windows = (nnz + (int64_t)p.ALPHA * m) / p.BN + 1;
    L.cap_wave = std::min<int64_t>(m, nnz / (p.LW + 1));
    const int64_t long_rows = std::min<int64_t>(m, nnz / ((int64_t)p.CH + 1));
    L.cap_items = nnz / p.BCH + long_rows;
    L.cap_split = std::min<int64_t>(m, nnz / ((int64_t)p.BCH + 1));
    L.cap_slots = nnz / p.BCH + L.cap_split;
    L.partial_stride = (n + 3) / 4 * 4;
    uint64_t off = 0;
    L.off_counts = off;
    off = align_up(off + (uint64_t)kQ * L.nblk * 4, 256);
    L.off_totals = off;
    off = align_up(off + kQ * 4, 256);
    L.off_win = off;
    off = align_up(off + (uint64_t)(L.n_windows + 1) * 4, 256);
    L.off_stage = off;
    off = align_up(off + (uint64_t)L.n_windows * 8, 256);
    L.off_wave = off;
    off = align_up(off + (uint64_t)L.cap_wave * 4, 256);
    L.off_wave_span = off;
    off = align_up(off + (uint64_t)L.cap_wave * 8, 256);
    L.off_items = off;
    off = align_up(off + (uint64_t)L.cap_items * 16, 256);
    L.off_split = off;
    off = align_up(off + (uint64_t)L.cap_split * 16, 256);
    L.off_partials = off;
    off = align_up(off + (uint64_t)L.cap_slots * L.partial_stride * 4, 256);
    // arrival counters: a split row has one per column tile of the launch; the narrowest tile any mapping uses is 16 columns
    L.ticket_tiles = std::max<int64_t>(1, ((int64_t)n + 15) / 16);
    L.off_tickets = off;
    off = align_up(off + (uint64_t)L.cap_slots * L.ticket_tiles * 4, 256);  // indexed by a split row's first slot
    L.off_bpack = off;
    if (p.PACK || (p.PANEL && !p.PDIRECT)) off = align_up(off + (uint64_t)k * ((n + 2 * kPanelCols - 1) / (2 * kPanelCols)) * (2 * kPanelCols) * 4, 256);
    L.off_coldeg = off;
    if (p.HOT) off = align_up(off + (uint64_t)k * 4, 256);
    L.off_hotmask = off;
    if (p.HOT) off = align_up(off + ((uint64_t)k / 32 + 2) * 4, 256);
    L.off_degbins = off;
    if (p.HOT) off = align_up(off + (uint64_t)kDegBins * 16, 256);
    L.total = std::max<uint64_t>(off, 256);
    return L;
}

scorch_status_t build_plan(scorch_spmm_plan_t *plan, const int32_t *rowptr, const int32_t *colidx,
                           hipStream_t stream) {
    const WorkspaceLayout &L = plan->layout;
    char *ws = plan->workspace;
    int32_t totals[kQ] = {0, 0, 0, 0, 0};
    int32_t unsorted = 0;
    // The panel kernel needs every row's columns in strictly increasing order; without colidx this cannot be
    // verified, so the mode is dropped.
    if (plan->params.PANEL && (!colidx || plan->m == 0 || plan->nnz == 0)) plan->params.PANEL = 0;
    if (plan->params.PANEL) {
        int32_t *flag = reinterpret_cast<int32_t *>(ws + L.off_totals) + 8;
        hipError_t e = hipMemsetAsync(flag, 0, sizeof(int32_t), stream);
        if (e != hipSuccess) return hip_fail(e, "clear sortedness flag");
        const uint32_t g = (uint32_t)std::min<int64_t>(((int64_t)plan->m + kWavesPerBlock - 1) / kWavesPerBlock, 256 * 16);
        hipLaunchKernelGGL(plan_sorted_kernel, dim3(g), dim3(kBlock), 0, stream, rowptr, colidx, plan->m, flag);
        e = hipMemcpyAsync(&unsorted, flag, sizeof(int32_t), hipMemcpyDeviceToHost, stream);
        if (e != hipSuccess) return hip_fail(e, "copy sortedness flag");
    }
    plan->n_hot = 0;
    plan->hot_share = 0.f;
    if (plan->params.HOT && colidx && plan->nnz > 0 && plan->k > 0) {
        scorch_status_t st = mark_hot_columns(plan, colidx, plan->tuning.hot > 0, stream);
        if (st != SCORCH_OK) return st;
    }
    if (plan->m > 0) {
        PlanArgs a{};
        a.rowptr = rowptr;
        a.m = plan->m;
        a.LW = plan->params.LW;
        a.CH = plan->params.CH;
        a.BCH = plan->params.BCH;
        a.nblk = L.nblk;
        a.counts = reinterpret_cast<int32_t *>(ws + L.off_counts);
        a.totals = reinterpret_cast<int32_t *>(ws + L.off_totals);
        a.wave_rows = reinterpret_cast<int32_t *>(ws + L.off_wave);
        a.wave_span = reinterpret_cast<int2 *>(ws + L.off_wave_span);
        a.items = reinterpret_cast<int4 *>(ws + L.off_items);
        a.split = reinterpret_cast<int4 *>(ws + L.off_split);
        a.cap_wave = L.cap_wave;
        a.cap_items = L.cap_items;
        a.cap_split = L.cap_split;
        hipLaunchKernelGGL(plan_count_kernel, dim3((uint32_t)L.nblk), dim3(kBlock), 0, stream, a);
        hipLaunchKernelGGL(plan_scan_kernel, dim3(1), dim3(1024), 0, stream, a);
        hipLaunchKernelGGL(plan_scatter_kernel, dim3((uint32_t)L.nblk), dim3(kBlock), 0, stream, a);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return hip_fail(e, "launch plan kernels");
        e = hipMemcpyAsync(totals, a.totals, sizeof(totals), hipMemcpyDeviceToHost, stream);
        if (e != hipSuccess) return hip_fail(e, "copy plan totals");
    }
    {
        // also for m == 0: the window table then reads [0, 0]
        const int64_t wblocks = (L.n_windows + 1 + kBlock - 1) / kBlock;
        hipLaunchKernelGGL(plan_window_kernel, dim3((uint32_t)wblocks), dim3(kBlock), 0, stream, rowptr, plan->m,
                           plan->params.BN, plan->params.ALPHA, L.n_windows,
                           reinterpret_cast<int32_t *>(ws + L.off_win));
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return hip_fail(e, "launch plan_window_kernel");
        hipLaunchKernelGGL(plan_stage_kernel, dim3((uint32_t)wblocks), dim3(kBlock), 0, stream, rowptr,
                           reinterpret_cast<const int32_t *>(ws + L.off_win), L.n_windows, plan->params.LW, kStageMax,
                           reinterpret_cast<int2 *>(ws + L.off_stage));
        e = hipGetLastError();
        if (e != hipSuccess) return hip_fail(e, "launch plan_stage_kernel");
        // the arrival counters of split rows start at zero; every launch leaves them at zero again
        if (L.cap_slots > 0) {
            e = hipMemsetAsync(ws + L.off_tickets, 0, (size_t)L.cap_slots * L.ticket_tiles * 4, stream);
            if (e != hipSuccess) return hip_fail(e, "clear arrival counters");
        }
        e = hipStreamSynchronize(stream);
        if (e != hipSuccess) return hip_fail(e, "wait for plan kernels");
    }
    if (unsorted) plan->params.PANEL = 0;
    plan->n_wave = totals[0];
    plan->n_items = totals[1];
    plan->n_split = totals[2];
    plan->n_slots = totals[3];
    plan->n_short = totals[4];
    if (plan->n_wave > L.cap_wave || plan->n_items > L.cap_items || plan->n_split > L.cap_split ||
        plan->n_slots > L.cap_slots) {
        set_error("plan lists exceed the workspace bound (rowptr changed or is not non-decreasing?)");
        return SCORCH_ERR_INVALID_ARG;
    }
    return SCORCH_OK;
}

}  // namespace scorch
