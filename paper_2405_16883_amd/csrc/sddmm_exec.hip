// SDDMM on a CSR pattern for gfx950:  D = A (.) (B C),  D_ij = A_ij * sum_t B_it C_tj  on the stored entries
// of A (paper, Section 3.1, first example of the programming-model figure; Section 5.4).  The paper's point
// is fusion: the dense product is never formed, only the sampled dot products are.  Here that is one kernel
// that, per stored entry, gathers row j of Ct = C^T, multiplies it with the row i of B held in registers and
// reduces over the lanes.  The row classes, windows and pieces of the SpMM plan are reused unchanged; as no
// sum runs over the entries of a row, pieces of a long row need no partial rows and no fix-up.
//
// Lane mapping as in the SpMM kernels: a group of G lanes covers the d columns (V floats per load, T loads per
// lane), a wavefront holds S = 64/G groups.  Eight entries are processed per group and step; their eight
// per-lane partial dot products are reduced with a halving butterfly (4 + 2 + 1 exchanges over lane distances
// 1, 2, 4 -- DPP and ds_swizzle -- then one exchange per remaining distance), i.e. about one cross-lane
// operation per entry instead of log2(G).  Rows of B and Ct that are not 16-byte aligned, or d not a multiple
// of 4, use four-float loads at float alignment (template flag UA); the vector that would run past column d is
// moved back to end at d and the elements it shares with its neighbour are zeroed in both operands, so every
// column enters the dot product once.
#include "device_util.h"
#include "spmm_internal.h"

#include <algorithm>

namespace scorch {

constexpr int kSddmmBatch = 8;

struct SddmmArgs {
    const int32_t *rowptr;
    const int32_t *colidx;
    const float *vals;
    const float *B;   // m x d, row stride ldb
    const float *Ct;  // k x d, row stride ldct
    float *out;       // nnz
    int64_t ldb, ldct;
    int32_t m, d;
    const int32_t *win_row_start;
    const int2 *win_stage;  // per window: (first staged entry, number of staged entries); y < 0: no short row
    const int32_t *wave_rows;
    const int2 *wave_span;  // [p0, p1) of every wave row
    const int4 *items;
    int32_t n_windows, n_wave_rows, n_items;
    int32_t nb_items, nb_wave, nb_win;
    int32_t LW;
    int32_t rows_per_wave;  // plan-free path only: consecutive rows taken by one wavefront
    int32_t k;              // column-block kernel: rows of Ct
    int32_t block_rows;     // column-block kernel: rows of Ct per block
    int32_t rounds;         // column-block kernel: blocks per XCD (block = round * 8 + XCD)
};

// Plan-free path: row lengths up to which a lane group walks a row alone / a wavefront streams a row alone (the larger
// limit when the workgroup has more than two rows beyond the smaller one), and the longest run of rows per wavefront.
constexpr int kSddmmShort = 32;
constexpr int kSddmmMid = 256;
constexpr int kSddmmLong = 2048;
constexpr int kSddmmRowsMax = 16;

// Sums r[0..7] over the G lanes of a group.  Returns, in every lane, the total of entry
// u = 4*bit0(lig) + 2*bit1(lig) + bit2(lig) of the batch.
template <int G> __device__ __forceinline__ float group_reduce8(float (&r)[kSddmmBatch], int lig) {
    static_assert(G >= 8, "a group must have at least 8 lanes");
    const bool h1 = (lig & 1) != 0;
#pragma unroll
    for (int h = 0; h < 4; ++h) {
        const float send = h1 ? r[h] : r[h + 4];
        const float keep = h1 ? r[h + 4] : r[h];
        r[h] = keep + lane_xor<1>(send);
    }
    const bool h2 = (lig & 2) != 0;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const float send = h2 ? r[h] : r[h + 2];
        const float keep = h2 ? r[h + 2] : r[h];
        r[h] = keep + lane_xor<2>(send);
    }
    const bool h4 = (lig & 4) != 0;
    float s = (h4 ? r[1] : r[0]) + lane_xor<4>(h4 ? r[0] : r[1]);
    if constexpr (G > 8) s += lane_xor<8>(s);
    if constexpr (G > 16) s += lane_xor<16>(s);
    if constexpr (G > 32) s += lane_xor<32>(s);
    return s;
}

// Zeroes the first nm (0..V-1) elements of a vector.
template <int V> __device__ __forceinline__ void zero_head(typename Vec<V>::type &v, int nm) {
    if constexpr (V > 1) {
#pragma unroll
        for (int i = 0; i < V - 1; ++i)
            if (i < nm) v[i] = 0.f;
    }
}

// One lane group computes the staged entries e0, e0+es, ... (< e_end) of a row whose B row is in x:
//   out_base[e] = val[e] * <x, Ct[col[e], :]>
// With lidx, staged entry e is written to out_base[lidx[e]] (entries picked out of a row, see the column-block kernel).
template <int V, int G, int T, bool UA>
__device__ __forceinline__ void sddmm_entries(const typename Vec<V>::type (&x)[T], const int *lcol, const float *lval,
                                              int e0, int e_end, int es, const float *Yc, int64_t ldct,
                                              const bool (&colok)[T], const int (&coff)[T], const int (&nmask)[T],
                                              int lig, float *out_base, const int *lidx = nullptr) {
    using vec = typename Vec<V>::type;
    const int my_u = ((lig & 1) << 2) | (lig & 2) | ((lig & 4) >> 2);
    for (int e = e0; e < e_end; e += es * kSddmmBatch) {
        vec y[kSddmmBatch][T];
#pragma unroll
        for (int u = 0; u < kSddmmBatch; ++u) {
            const int ee = e + u * es;
            const bool ok = ee < e_end;
            const int c = lcol[ok ? ee : e0];
            const float *yp = Yc + (int64_t)c * ldct;
#pragma unroll
            for (int t = 0; t < T; ++t) {
                y[u][t] = (ok && colok[t]) ? vload<V, UA>(yp + coff[t]) : vzero<V>();
                if constexpr (UA) zero_head<V>(y[u][t], nmask[t]);
            }
        }
        float r[kSddmmBatch];
#pragma unroll
        for (int u = 0; u < kSddmmBatch; ++u) {
            float s = 0.f;
#pragma unroll
            for (int t = 0; t < T; ++t) {
                if constexpr (V == 1) s = __builtin_fmaf(x[t], y[u][t], s);
                else
#pragma unroll
                    for (int i = 0; i < V; ++i) s = __builtin_fmaf(x[t][i], y[u][t][i], s);
            }
            r[u] = s;
        }
        const float total = group_reduce8<G>(r, lig);
        const int ee = e + my_u * es;
        if (lig < kSddmmBatch && ee < e_end) out_base[lidx ? lidx[ee] : ee] = lval[ee] * total;
    }
}

// A wavefront walks the entries [pfirst, p1) of one row in chunks of 64 that are `stride` apart.
template <int V, int G, int T, bool NTA, bool UA>
__device__ __forceinline__ void sddmm_row(const typename Vec<V>::type (&x)[T], int *lcol, float *lval, int lane, int grp,
                                          int lig, int pfirst, int p1, int stride, const SddmmArgs &a, const float *Yc,
                                          const bool (&colok)[T], const int (&coff)[T], const int (&nmask)[T]) {
    constexpr int S = kWave / G;
    int pc = pfirst + lane;
    int cn = 0;
    float vn = 0.f;
    if (pc < p1) {
        cn = ld_idx<NTA>(a.colidx + pc);
        vn = ld_val<NTA>(a.vals + pc);
    }
    for (int base = pfirst; base < p1; base += stride) {
        lcol[lane] = cn;
        lval[lane] = vn;
        pc = base + stride + lane;
        if (pc < p1) {
            cn = ld_idx<NTA>(a.colidx + pc);
            vn = ld_val<NTA>(a.vals + pc);
        }
        wave_lds_sync();
        const int cnt = min(kWave, p1 - base);
        sddmm_entries<V, G, T, UA>(x, lcol, lval, grp, cnt, S, Yc, a.ldct, colok, coff, nmask, lig, a.out + base);
        wave_lds_sync();
    }
}

template <int V, int T, bool UA>
__device__ __forceinline__ void load_x(typename Vec<V>::type (&x)[T], const float *Brow, const bool (&colok)[T],
                                       const int (&coff)[T], const int (&nmask)[T]) {
#pragma unroll
    for (int t = 0; t < T; ++t) {
        x[t] = colok[t] ? vload<V, UA>(Brow + coff[t]) : vzero<V>();
        if constexpr (UA) zero_head<V>(x[t], nmask[t]);
    }
}

constexpr int sddmm_smem_ints_per_wave() { return 2 * kStageMax + kWindowRowsMax + 2; }

template <int V, int G, int T, bool PLANNED, bool UA>
__global__ __launch_bounds__(kBlock) void sddmm_kernel(const SddmmArgs a) {
    using vec = typename Vec<V>::type;
    constexpr int S = kWave / G;
    constexpr int GV = G * V;
    __shared__ int s_raw[kWavesPerBlock * sddmm_smem_ints_per_wave()];
    const int tid = threadIdx.x;
    const int wv = tid >> 6;
    const int lane = tid & 63;
    const int grp = lane / G;
    const int lig = lane % G;
    const int c0 = lig * V;
    bool colok[T];
    int coff[T], nmask[T];  // first column of the lane's t-th vector; leading elements shared with the neighbour
#pragma unroll
    for (int t = 0; t < T; ++t) {
        colok[t] = (c0 + t * GV) < a.d;
        coff[t] = UA ? min(c0 + t * GV, a.d - V) : c0 + t * GV;
        nmask[t] = c0 + t * GV - coff[t];
    }
    const float *Yc = a.Ct;
    int *lcol = s_raw + wv * sddmm_smem_ints_per_wave();
    float *lval = reinterpret_cast<float *>(lcol + kStageMax);
    int *lrp = lcol + 2 * kStageMax;
    vec x[T];
    const uint32_t b = blockIdx.x;

    if constexpr (!PLANNED) {
        // Plan-free: rows in natural order, a run of consecutive rows per wavefront.  The wavefront reads the run's row
        // pointers once and proceeds greedily: the next rows that are short and fit the LDS stage together are staged
        // and walked one row per lane group; a longer row is streamed by the whole wavefront; a row beyond kSddmmLong
        // entries (kSddmmMid when such rows are rare in the workgroup, i.e. the outliers of a graph) is left to the
        // end, where the 4 wavefronts split its entries (entries are independent: nothing to combine).
        __shared__ int s_long[kWavesPerBlock * kSddmmRowsMax];
        __shared__ int s_nlong, s_nmid;
        const int NR = a.rows_per_wave;
        const int64_t r0 = ((int64_t)b * kWavesPerBlock + wv) * NR;
        const int nr = (int)max((int64_t)0, min((int64_t)NR, (int64_t)a.m - r0));
        if (tid == 0) {
            s_nlong = 0;
            s_nmid = 0;
        }
        __syncthreads();
        const int rpv = nr > 0 ? a.rowptr[r0 + min(lane, nr)] : 0;
        const int rnext = __shfl_down(rpv, 1, kWave);  // lanes past the run hold the last pointer; lane 63 is never a row
        const int nmid = (int)__builtin_popcountll(__ballot(lane < nr && rnext - rpv > kSddmmMid));
        if (lane == 0 && nmid > 0) atomicAdd(&s_nmid, nmid);
        __syncthreads();
        const int long_limit = s_nmid <= 2 ? kSddmmMid : kSddmmLong;
        if (nr > 0) {
            lrp[lane] = rpv;
            wave_lds_sync();
            int i = 0;
            while (i < nr) {
                const int base = lrp[i];
                // rows i .. j-1: the longest run of short rows that fits the stage
                const bool stops = lane >= i && (lane >= nr || rnext - rpv > kSddmmShort || rnext - base > kStageMax);
                const int j = __builtin_ctzll(__ballot(stops));  // lane nr always stops
                if (j == i) {
                    const int p1 = lrp[i + 1];
                    if (p1 - base <= long_limit) {
                        load_x<V, T, UA>(x, a.B + (r0 + i) * a.ldb, colok, coff, nmask);
                        sddmm_row<V, G, T, false, UA>(x, lcol, lval, lane, grp, lig, base, p1, kWave, a, Yc, colok, coff, nmask);
                    } else if (lane == 0) {
                        s_long[atomicAdd(&s_nlong, 1)] = (int)(r0 + i);
                    }
                    ++i;
                    continue;
                }
                const int cnt = min(lrp[j] - base, kStageMax);
                for (int e = lane; e < cnt; e += kWave) {
                    lcol[e] = a.colidx[base + e];
                    lval[e] = a.vals[base + e];
                }
                wave_lds_sync();
                for (int ri = i + grp; ri < j; ri += S) {
                    const int q0 = lrp[ri], q1 = lrp[ri + 1];
                    if (q1 == q0) continue;
                    load_x<V, T, UA>(x, a.B + (r0 + ri) * a.ldb, colok, coff, nmask);
                    sddmm_entries<V, G, T, UA>(x, lcol, lval, q0 - base, q1 - base, 1, Yc, a.ldct, colok, coff, nmask, lig,
                                               a.out + base);
                }
                wave_lds_sync();  // the stage is refilled next
                i = j;
            }
        }
        __syncthreads();
        const int nlong = s_nlong;
        for (int w = 0; w < nlong; ++w) {
            const int64_t row = s_long[w];
            load_x<V, T, UA>(x, a.B + row * a.ldb, colok, coff, nmask);
            sddmm_row<V, G, T, false, UA>(x, lcol, lval, lane, grp, lig, a.rowptr[row] + wv * kWave, a.rowptr[row + 1], kBlock,
                                          a, Yc, colok, coff, nmask);
        }
        return;
    }

    if (b < (uint32_t)a.nb_items) {
        // piece of a long row: the 4 wavefronts take interleaved chunks; entries are independent
        const int4 it = a.items[b];
        load_x<V, T, UA>(x, a.B + (int64_t)it.x * a.ldb, colok, coff, nmask);
        sddmm_row<V, G, T, false, UA>(x, lcol, lval, lane, grp, lig, it.y + wv * kWave, it.z, kBlock, a, Yc, colok, coff,
                                      nmask);
        return;
    }
    if (b < (uint32_t)(a.nb_items + a.nb_wave)) {
        const int idx = (int)(b - a.nb_items) * kWavesPerBlock + wv;
        if (idx >= a.n_wave_rows) return;
        const int row = a.wave_rows[idx];
        const int2 span = a.wave_span[idx];  // the row's entry range, kept in the plan beside its id
        load_x<V, T, UA>(x, a.B + (int64_t)row * a.ldb, colok, coff, nmask);
        sddmm_row<V, G, T, false, UA>(x, lcol, lval, lane, grp, lig, span.x, span.y, kWave, a, Yc, colok, coff, nmask);
        return;
    }
    // window of consecutive short rows: stage the window's entries once, one lane group per row
    const int w = (int)(b - a.nb_items - a.nb_wave) * kWavesPerBlock + wv;
    if (w >= a.n_windows) return;
    const int r0 = a.win_row_start[w];
    const int r1 = a.win_row_start[w + 1];
    // which entries the window stages (first to last short row) is known from the plan, so colidx/vals are requested
    // together with the row pointers instead of after them
    const int2 stg = a.win_stage[w];
    if (stg.y <= 0) return;  // no short row, or only empty ones
    const int nr = min(r1 - r0, kWindowRowsMax);
    const int sbeg = stg.x, cnt = stg.y;
    const int rpv = a.rowptr[r0 + min(lane, nr)];
    const int rlast = a.rowptr[r0 + nr];
    for (int e = lane; e < cnt; e += kWave) {
        lcol[e] = a.colidx[sbeg + e];
        lval[e] = a.vals[sbeg + e];
    }
    lrp[lane] = rpv;
    if (lane == 0) lrp[nr] = rlast;
    wave_lds_sync();
    for (int ri = grp; ri < nr; ri += S) {
        const int q0 = lrp[ri], q1 = lrp[ri + 1];
        if (q1 - q0 > a.LW || q1 == q0) continue;
        load_x<V, T, UA>(x, a.B + (int64_t)(r0 + ri) * a.ldb, colok, coff, nmask);
        sddmm_entries<V, G, T, UA>(x, lcol, lval, q0 - sbeg, q1 - sbeg, 1, Yc, a.ldct, colok, coff, nmask, lig, a.out + sbeg);
    }
}

// Column-block kernel, for matrices whose rows are long and whose second factor overflows an XCD's L2 a few times:
// the rows of Ct (= columns of A) are cut into 8 * rounds blocks, and XCD x takes, for every row of A, only the stored
// entries whose column falls into block round * 8 + x.  Its gathers then stay within a block of Ct that its L2 keeps.
// Entries of an SDDMM are independent, so nothing has to be combined between XCDs (the SpMM cannot do this: it would
// have to add partial rows).  A wavefront scans the row's colidx 64 at a time, compacts the entries of its block into
// the LDS stage together with their positions, and the lane groups then take the staged entries in turn.  Every XCD
// scans every row: 8 * rounds reads of colidx and of the rows of B, against 4 d bytes gathered per entry.
constexpr int kSddmmBlockRowsPerWave = 4;

template <int V, int G, int T, bool UA>
__global__ __launch_bounds__(kBlock) void sddmm_colblock_kernel(const SddmmArgs a) {
    using vec = typename Vec<V>::type;
    constexpr int S = kWave / G;
    constexpr int GV = G * V;
    __shared__ int s_raw[kWavesPerBlock * 3 * kStageMax];
    const int tid = threadIdx.x;
    const int wv = tid >> 6;
    const int lane = tid & 63;
    const int grp = lane / G;
    const int lig = lane % G;
    const int c0 = lig * V;
    bool colok[T];
    int coff[T], nmask[T];
#pragma unroll
    for (int t = 0; t < T; ++t) {
        colok[t] = (c0 + t * GV) < a.d;
        coff[t] = UA ? min(c0 + t * GV, a.d - V) : c0 + t * GV;
        nmask[t] = c0 + t * GV - coff[t];
    }
    int *lcol = s_raw + wv * 3 * kStageMax;
    float *lval = reinterpret_cast<float *>(lcol + kStageMax);
    int *lidx = lcol + 2 * kStageMax;
    // workgroup index = (round * row groups + row group) * 8 + XCD: consecutive workgroups go to different XCDs
    const uint32_t xcd = blockIdx.x & (kXcds - 1);
    const uint32_t q = blockIdx.x / kXcds;
    const uint32_t row_groups = (uint32_t)((a.m + kWavesPerBlock * kSddmmBlockRowsPerWave - 1) / (kWavesPerBlock * kSddmmBlockRowsPerWave));
    const uint32_t round = q / row_groups;
    const uint32_t rg = q - round * row_groups;
    const int64_t lo64 = (int64_t)(round * kXcds + xcd) * a.block_rows;
    if (lo64 >= a.k) return;
    const int lo = (int)lo64;
    const int hi = (int)min((int64_t)a.k, lo64 + a.block_rows);
    const int64_t row0 = ((int64_t)rg * kWavesPerBlock + wv) * kSddmmBlockRowsPerWave;
    vec x[T];
    for (int64_t row = row0; row < min((int64_t)a.m, row0 + kSddmmBlockRowsPerWave); ++row) {
        const int p0 = a.rowptr[row], p1 = a.rowptr[row + 1];
        bool have_x = false;
        int staged = 0;
        for (int base = p0; base < p1; base += kWave) {
            const int p = base + lane;
            const int c = p < p1 ? a.colidx[p] : -1;
            const bool in = c >= lo && c < hi;
            const unsigned long long mask = __ballot(in);
            if (mask != 0ull) {
                const int pos = staged + (int)__builtin_popcountll(mask & ((1ull << lane) - 1ull));
                if (in) {
                    lcol[pos] = c;
                    lval[pos] = a.vals[p];
                    lidx[pos] = p;
                }
                staged += (int)__builtin_popcountll(mask);
            }
            if (staged > kStageMax - kWave || (base + kWave >= p1 && staged > 0)) {
                if (!have_x) {
                    load_x<V, T, UA>(x, a.B + row * a.ldb, colok, coff, nmask);
                    have_x = true;
                }
                wave_lds_sync();
                sddmm_entries<V, G, T, UA>(x, lcol, lval, grp, staged, S, a.Ct, a.ldct, colok, coff, nmask, lig, a.out, lidx);
                wave_lds_sync();
                staged = 0;
            }
        }
    }
}

// ------------------------------------------------------------------------------------------
typedef void (*sddmm_fn)(const SddmmArgs);

// Compiled variants: V = 4 with every group size, aligned or not; V = 2 and V = 1 only occur for d < 4 (G = 8).
template <bool PLANNED> static sddmm_fn pick_sddmm(int V, int G, int T, bool UA) {
#define SCORCH_SD(Vv, Gg, Tt, Uu) return sddmm_kernel<Vv, Gg, Tt, PLANNED, Uu>;
#define SCORCH_SD_G4(Uu)                                  \
    if (T == 4) { SCORCH_SD(4, 64, 4, Uu) }               \
    if (T == 2) { SCORCH_SD(4, 64, 2, Uu) }               \
    switch (G) {                                          \
        case 8: SCORCH_SD(4, 8, 1, Uu)                    \
        case 16: SCORCH_SD(4, 16, 1, Uu)                  \
        case 32: SCORCH_SD(4, 32, 1, Uu)                  \
        default: SCORCH_SD(4, 64, 1, Uu)                  \
    }
    if (V == 4) {
        if (UA) { SCORCH_SD_G4(true) } else { SCORCH_SD_G4(false) }
    }
    if (V == 2) { SCORCH_SD(2, 8, 1, false) }
    SCORCH_SD(1, 8, 1, false)
#undef SCORCH_SD_G4
#undef SCORCH_SD
}

static sddmm_fn pick_sddmm_colblock(int V, int G, int T, bool UA) {
#define SCORCH_SDB(Vv, Gg, Tt, Uu) return sddmm_colblock_kernel<Vv, Gg, Tt, Uu>;
#define SCORCH_SDB_G4(Uu)                                 \
    if (T == 4) { SCORCH_SDB(4, 64, 4, Uu) }              \
    if (T == 2) { SCORCH_SDB(4, 64, 2, Uu) }              \
    switch (G) {                                          \
        case 8: SCORCH_SDB(4, 8, 1, Uu)                   \
        case 16: SCORCH_SDB(4, 16, 1, Uu)                 \
        case 32: SCORCH_SDB(4, 32, 1, Uu)                 \
        default: SCORCH_SDB(4, 64, 1, Uu)                 \
    }
    if (V == 4) {
        if (UA) { SCORCH_SDB_G4(true) } else { SCORCH_SDB_G4(false) }
    }
    if (V == 2) { SCORCH_SDB(2, 8, 1, false) }
    SCORCH_SDB(1, 8, 1, false)
#undef SCORCH_SDB_G4
#undef SCORCH_SDB
}

static bool pick_sddmm_mapping(int32_t d, const float *B, int64_t ldb, const float *Ct, int64_t ldct, int &V, int &G,
                               int &T, bool &UA) {
    const uintptr_t pb = reinterpret_cast<uintptr_t>(B), pc = reinterpret_cast<uintptr_t>(Ct);
    UA = false;
    if (d % 4 == 0 && ldb % 4 == 0 && ldct % 4 == 0 && pb % 16 == 0 && pc % 16 == 0) V = 4;
    else if (d >= 4) {
        V = 4;
        UA = true;
    } else if (d % 2 == 0 && ldb % 2 == 0 && ldct % 2 == 0 && pb % 8 == 0 && pc % 8 == 0) V = 2;
    else V = 1;
    const int lanes = (d + V - 1) / V;
    T = 1;
    if (lanes <= kWave) {
        G = 8;
        while (G < lanes) G <<= 1;
    } else {
        G = kWave;
        T = lanes <= 2 * kWave ? 2 : 4;
        if (lanes > 4 * kWave) return false;
    }
    return true;
}

scorch_status_t launch_sddmm(const scorch_spmm_plan_t *plan, int32_t m, int32_t d, const int32_t *rowptr,
                             const int32_t *colidx, const float *vals, const float *B, int64_t ldb, const float *Ct,
                             int64_t ldct, float *out, hipStream_t stream) {
    int V, G, T;
    bool UA;
    if (!pick_sddmm_mapping(d, B, ldb, Ct, ldct, V, G, T, UA)) {
        set_error("sddmm: d = %d exceeds the %d columns one wavefront covers", d, 4 * kWave * V);
        return SCORCH_ERR_UNSUPPORTED;
    }
    SddmmArgs a{};
    a.rowptr = rowptr;
    a.colidx = colidx;
    a.vals = vals;
    a.B = B;
    a.Ct = Ct;
    a.out = out;
    a.ldb = ldb;
    a.ldct = ldct;
    a.m = m;
    a.d = d;
    int64_t grid;
    sddmm_fn fn;
    // Column blocks over the XCDs (sddmm_colblock_kernel): rows without outliers (none cut by the plan) and a second
    // factor of a few L2s.  Measured against the row-wise kernel on uniform and pruned patterns, k = 4096 ... 65 536,
    // d = 64 ... 1024: Ct of 17-34 MB: 1.3-2.2x faster with one block per XCD (also with 33 entries per row); 67 MB:
    // 1.4-2.2x with two blocks per XCD (one: 1.5x); 8 MB: between 1.27x faster (1638 entries per row) and 1.15x slower
    // (164); 4 MB and less: 1.1-3x slower.  sdblk=<blocks per XCD> in the tuning variable forces it, sdblk=0 turns it off.
    int32_t rounds = 0;
    if (plan && plan->m > 0 && plan->k > 0) {
        const int64_t ct_bytes = (int64_t)plan->k * d * 4;
        const int64_t avg = plan->nnz / plan->m;
        const bool big_enough = (avg >= 1024 && ct_bytes >= (8ll << 20)) || (avg >= 64 && ct_bytes >= (12ll << 20)) ||
                                (avg >= 24 && ct_bytes >= (16ll << 20));
        // one block per XCD and 42 MB of Ct, four at most (Ct of 134 MB: 1.3-1.8x faster with 3-4 blocks per XCD; 268 MB:
        // 1.1-1.4x with 4)
        if (big_enough && plan->n_split == 0 && ct_bytes <= (300ll << 20))
            rounds = (int32_t)std::min<int64_t>(4, (ct_bytes + (42ll << 20) - 1) / (42ll << 20));
        if (plan->tuning.sdblk >= 0) rounds = std::min(plan->tuning.sdblk, 64);  // as it stood when the plan was made
    }
    if (rounds > 0) {
        a.k = plan->k;
        a.rounds = rounds;
        a.block_rows = (int32_t)(((int64_t)plan->k + (int64_t)kXcds * rounds - 1) / ((int64_t)kXcds * rounds));
        const int64_t row_groups = ((int64_t)m + kWavesPerBlock * kSddmmBlockRowsPerWave - 1) / (kWavesPerBlock * kSddmmBlockRowsPerWave);
        grid = row_groups * kXcds * rounds;
        fn = pick_sddmm_colblock(V, G, T, UA);
    } else if (plan) {
        char *ws = plan->workspace;
        a.win_row_start = reinterpret_cast<const int32_t *>(ws + plan->layout.off_win);
        a.win_stage = reinterpret_cast<const int2 *>(ws + plan->layout.off_stage);
        a.wave_rows = reinterpret_cast<const int32_t *>(ws + plan->layout.off_wave);
        a.wave_span = reinterpret_cast<const int2 *>(ws + plan->layout.off_wave_span);
        a.items = reinterpret_cast<const int4 *>(ws + plan->layout.off_items);
        a.n_windows = (int32_t)plan->layout.n_windows;
        a.n_wave_rows = plan->n_wave;
        a.n_items = plan->n_items;
        a.nb_items = plan->n_items;
        a.nb_wave = (plan->n_wave + kWavesPerBlock - 1) / kWavesPerBlock;
        a.nb_win = plan->n_short > 0 ? (int32_t)((plan->layout.n_windows + kWavesPerBlock - 1) / kWavesPerBlock) : 0;
        a.LW = plan->params.LW;
        grid = (int64_t)a.nb_items + a.nb_wave + a.nb_win;
        fn = pick_sddmm<true>(V, G, T, UA);
    } else {
        // rows per wavefront: 4 (up to one per lane group, 16 at most, when the groups are narrow) once that leaves a
        // workgroup for every compute unit
        const int64_t rows_cap = std::max(4, std::min(kSddmmRowsMax, kWave / G));
        a.rows_per_wave = (int32_t)std::min<int64_t>(rows_cap, std::max<int64_t>(1, m / 4096));
        grid = ((int64_t)m + (int64_t)kWavesPerBlock * a.rows_per_wave - 1) / ((int64_t)kWavesPerBlock * a.rows_per_wave);
        fn = pick_sddmm<false>(V, G, T, UA);
    }
    if (grid > 0x7fffffffLL) {
        set_error("launch grid of %lld workgroups exceeds the HIP limit", (long long)grid);
        return SCORCH_ERR_UNSUPPORTED;
    }
    if (grid == 0) return SCORCH_OK;
    hipLaunchKernelGGL(fn, dim3((uint32_t)grid), dim3(kBlock), 0, stream, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return hip_fail(e, "launch sddmm_kernel");
    return SCORCH_OK;
}

}  // namespace scorch
