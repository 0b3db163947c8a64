// Execution kernels for CSR SpMM on gfx950:  C_ik = sum_j A_ij * B_jk  (paper, Section 4.2).
//
// Loop structure kept from the paper (Sections 4.1, 4.2): rows outermost, the stored entries of a
// row next, the dense column index innermost, and only that dense column loop is tiled.  On the
// GPU the column loop is laid across lanes: a group of G lanes covers G*V*T consecutive columns
// (V floats per load, T loads per lane), so every read of a B row and every write of a C row is a
// contiguous, coalesced burst.  A wavefront holds S = 64/G such groups.  V = 4 whenever n >= 4; rows
// that are not 16-byte aligned use the same loads at float alignment (template flag UA), and a row
// whose length is not a multiple of 4 ends with a vector that overlaps its neighbour.
//
// Three paths share one launch; the workgroup index selects the path:
//   items   one workgroup per piece of a long row; 4 wavefronts split the piece, partial sums are
//           combined through LDS and written to C or to a partial row
//   wave    one wavefront per medium row; the S groups take interleaved entries and are combined
//           with cross-lane shuffles
//   window  one wavefront per window of consecutive short rows; the window's colidx/vals are
//           staged in LDS with coalesced loads, then each group walks one row at a time
// No MFMA: the work is a gather, not a dense contraction.  No atomics: summation order is fixed.
#include "spmm_internal.h"
#include "device_util.h"

#include <algorithm>

namespace scorch {

// Address of row c of B as seen by one lane (base = B + the lane's column offset): one 32x32->64-bit multiply
// and one shift-add (c >= 0 and the row stride fit 32 bits).
__device__ __forceinline__ const float *b_row(const float *base, int c, uint32_t ldb) {
    return base + (uint64_t)(uint32_t)c * ldb;
}

// One batch of U staged entries e, e+es, ... of a row:  acc[t] += val * B[col, boff[t] .. +V).  The U gathers
// are issued before the first multiply so that U reads of B rows are in flight per group.  PRED: entries at or
// past e_end are skipped (last batch of a row); otherwise the batch is whole and nothing is tested per entry.
// How the rows of B outside the hot set are read (hot/cold variants only).  0: streaming (non-temporal) loads, the
// default.  1..3: experiments with the other cache-policy bits of gfx950 loads, issued as buffer loads so that the
// bits can be chosen: 1 = device scope (sc1: not kept in the vector L1), 2 = system scope (sc0 sc1), 3 = sc1 + nt.
struct ColdPath {
    __amdgpu_buffer_rsrc_t rsrc;  // covers B (only used when B is smaller than 4 GB)
    uint32_t ldb_bytes;
};
template <int COLD> __device__ __forceinline__ Vec<4>::type cold_load(const ColdPath &cp, uint32_t byte_off) {
    typedef int i4 __attribute__((ext_vector_type(4)));
    constexpr int aux = COLD == 1 ? 16 : (COLD == 2 ? 17 : 18);
    const i4 raw = __builtin_amdgcn_raw_buffer_load_b128(cp.rsrc, (int)byte_off, 0, aux);
    Vec<4>::type x;
#pragma unroll
    for (int i = 0; i < 4; ++i) x[i] = __int_as_float(raw[i]);
    return x;
}

template <int V, int T, int U, bool UA, bool HOT, bool PRED, int COLD = 0>
__device__ __forceinline__ void gather_batch(typename Vec<V>::type (&acc)[T], const int *lcol, const float *lval,
                                             int e, int e_end, int es, const float *const (&bbase)[T],
                                             uint32_t ldb, const ColdPath *cp = nullptr, const int *boffb = nullptr) {
    using vec = typename Vec<V>::type;
    vec x[U][T];
    float v[U];
    int c[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int ee = e + u * es;
        const bool ok = !PRED || ee < e_end;
        c[u] = lcol[ok ? ee : e];
        v[u] = ok ? lval[ee] : 0.f;
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const bool ok = !PRED || e + u * es < e_end;
        const bool hot = !HOT || c[u] < 0;
        const int cu = HOT ? (c[u] & 0x7fffffff) : c[u];
#pragma unroll
        for (int t = 0; t < T; ++t) {
            const float *bp = b_row(bbase[t], cu, ldb);
            if (ok) {
                if (hot) {
                    x[u][t] = vload<V, UA>(bp);
                } else {
                    // the empty statements keep this load from being merged with the one of the other branch
                    // (hoisted above or sunk below the branch, the merged load loses the streaming policy)
                    asm volatile("");
                    if constexpr (COLD == 0 || V != 4) x[u][t] = __builtin_nontemporal_load(reinterpret_cast<const vec *>(bp));
                    else x[u][t] = cold_load<COLD>(*cp, (uint32_t)cu * cp->ldb_bytes + (uint32_t)boffb[t]);
                    asm volatile("");
                }
            } else {
                x[u][t] = vzero<V>();
            }
        }
    }
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
        for (int t = 0; t < T; ++t) vfma<V>(acc[t], v[u], x[u][t]);
}

// One lane group accumulates the staged entries e0, e0+es, ... (< e_end) of a row: whole batches first, then
// one partial batch.  boff[t] is a readable offset in every lane (lanes past column n point at the last
// vector of the row), so the loads carry no column test; `active` is false in the lanes whose first vector lies
// past column n: they skip the row altogether.
template <int V, int T, int U, bool UA, bool HOT = false, int COLD = 0>
__device__ __forceinline__ void gather_fma(typename Vec<V>::type (&acc)[T], const int *lcol, const float *lval,
                                           int e0, int e_end, int es, const float *Bc, uint32_t ldb, bool active,
                                           const int (&boff)[T], const ColdPath *cp = nullptr) {
    if (!active) return;
    const float *bbase[T];
    int boffb[T];
#pragma unroll
    for (int t = 0; t < T; ++t) {
        bbase[t] = Bc + boff[t];
        boffb[t] = boff[t] * 4;
    }
    int e = e0;
    for (; e + (U - 1) * es < e_end; e += U * es)
        gather_batch<V, T, U, UA, HOT, false, COLD>(acc, lcol, lval, e, e_end, es, bbase, ldb, cp, boffb);
    if (e < e_end) gather_batch<V, T, U, UA, HOT, true, COLD>(acc, lcol, lval, e, e_end, es, bbase, ldb, cp, boffb);
}

// Adds up the S = 64/G lane groups of a wavefront (xor butterfly over the lane distances G..32; DPP,
// ds_swizzle or ds_bpermute depending on the distance); every lane ends with the full sum.
template <int V, int G, int T, int OFF = G>
__device__ __forceinline__ void reduce_groups(typename Vec<V>::type (&acc)[T]) {
    if constexpr (OFF < kWave) {
#pragma unroll
        for (int t = 0; t < T; ++t) {
            auto o = vlane_xor<V, OFF>(acc[t]);
            vadd<V>(acc[t], o);
        }
        reduce_groups<V, G, T, OFF * 2>(acc);
    }
}

// A wavefront walks the entries [p0 + first, p1) of one row in chunks of 64 that are `stride`
// apart (stride = 64 for a whole wavefront-row, 256 when 4 wavefronts share a piece).  Each chunk
// is read with one coalesced load per array, parked in LDS, and broadcast from there to the lane
// groups; the next chunk is fetched into registers while the current one is consumed.
__device__ __forceinline__ int mark_hot(int c, const uint32_t *mask) {
    return c | (int)(((mask[c >> 5] >> (c & 31)) & 1u) << 31);
}

template <int V, int G, int T, int U, bool NTA, bool UA, bool HOT = false, int COLD = 0>
__device__ __forceinline__ void row_accumulate(typename Vec<V>::type (&acc)[T], int *lcol, float *lval, int lane,
                                               int grp, int pfirst, int p1, int stride, const int32_t *colidx,
                                               const float *vals, const float *Bc, uint32_t ldb,
                                               bool active, const int (&boff)[T],
                                               const uint32_t *hotmask = nullptr, const ColdPath *cp = nullptr) {
    constexpr int S = kWave / G;
    if constexpr (G == 1 && T == 1 && !HOT) {
        // One-lane groups (n <= 4): every lane owns the entries pfirst + lane + i * stride and needs no broadcast, so
        // the stage is skipped: U index/value pairs are read straight into registers, then U gathers are issued.  A row
        // of up to 64 U entries costs two memory round trips instead of two per 64 entries.  The order in which a lane
        // adds its products is the same as with the stage.
        using vec = typename Vec<V>::type;
        if (!active) return;
        const float *base = Bc + boff[0];
        for (int pb = pfirst + lane; pb - lane < p1; pb += stride * U) {
            int c[U];
            float v[U];
            vec x[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int p = pb + u * stride;
                const bool ok = p < p1;
                c[u] = ok ? ld_idx<NTA>(colidx + p) : 0;
                v[u] = ok ? ld_val<NTA>(vals + p) : 0.f;
            }
#pragma unroll
            for (int u = 0; u < U; ++u) x[u] = pb + u * stride < p1 ? vload<V, UA>(b_row(base, c[u], ldb)) : vzero<V>();
#pragma unroll
            for (int u = 0; u < U; ++u) vfma<V>(acc[0], v[u], x[u]);
        }
        return;
    }
    int pc = pfirst + lane;
    int cn = 0;
    float vn = 0.f;
    if (pc < p1) {
        cn = ld_idx<NTA>(colidx + pc);
        vn = ld_val<NTA>(vals + pc);
        if constexpr (HOT) cn = mark_hot(cn, hotmask);
    }
    for (int base = pfirst; base < p1; base += stride) {
        lcol[lane] = cn;
        lval[lane] = vn;
        pc = base + stride + lane;
        if (pc < p1) {
            cn = ld_idx<NTA>(colidx + pc);
            vn = ld_val<NTA>(vals + pc);
            if constexpr (HOT) cn = mark_hot(cn, hotmask);
        }
        wave_lds_sync();
        const int cnt = min(kWave, p1 - base);
        gather_fma<V, T, U, UA, HOT, COLD>(acc, lcol, lval, grp, cnt, S, Bc, ldb, active, boff, cp);
        wave_lds_sync();
    }
}

constexpr int smem_ints_per_wave() { return 2 * kStageMax + kWindowRowsMax + 2; }

template <int V, int G, int T, int U, int NT, bool UA, bool HOT = false, int COLD = 0>
__global__ __launch_bounds__(kBlock) void spmm_fused_kernel(const ExecArgs a) {
    using vec = typename Vec<V>::type;
    constexpr int S = kWave / G;
    constexpr int GV = G * V;
    constexpr int TW = GV * T;
    constexpr bool NTC = (NT & 1) != 0;  // streaming stores for C
    // colidx/vals are read with plain loads (a streaming hint made no difference), except in the hot/cold variants:
    // there the memory-side cache is reserved for the hot rows of B and the 8 bytes per entry of A would only
    // displace them (workload 4: another 2.7 % less time)
    constexpr bool NTA = HOT;

    __shared__ int s_raw[kWavesPerBlock * smem_ints_per_wave()];
    __shared__ float s_red[kWavesPerBlock * TW];
    // one-lane groups (n <= 4) only: the products of a window's entries, summed per row afterwards
    __shared__ __attribute__((aligned(16))) float s_prod[G == 1 ? kWavesPerBlock * kStageMax * V : 1];
    __shared__ int s_flag;  // piece of a split row: this workgroup drew the row's last ticket

    const int tid = threadIdx.x;
    const int wv = tid >> 6;
    const int lane = tid & 63;
    const int grp = lane / G;
    const int lig = lane % G;

    const uint32_t per_tile = (uint32_t)a.nb_items + (uint32_t)a.nb_wave + (uint32_t)a.nb_win;
    uint32_t ct, b;
    if (!tile_of_workgroup(a.xcd_slices, a.ncoltiles, per_tile, ct, b)) return;

    // coff[t]: first column of the lane's t-th vector.  With unaligned rows (UA) n need not be a multiple of V:
    // the vector that would run past column n is moved back to end at n, so it overlaps its neighbour and both
    // lanes compute and store the same values for the shared columns.  Vectors wholly past column n (colok false)
    // point at the last vector of the row as well: they may be read, and are never stored.
    const int c0 = (int)ct * TW + lig * V;
    bool colok[T];
    int coff[T], boff[T];
#pragma unroll
    for (int t = 0; t < T; ++t) {
        colok[t] = (c0 + t * GV) < a.n;
        coff[t] = min(c0 + t * GV, a.n - V);
        // packed B (XCD-sliced mode with a repacked copy): slice ct is a dense k x 32 block
        boff[t] = a.b_tile_stride ? lig * V + t * GV : coff[t];
    }
    const float *Bc = a.b_tile_stride ? a.B + (int64_t)ct * a.b_tile_stride : a.B;
    const uint32_t ldb = (uint32_t)a.ldb;
    ColdPath cold{};
    if constexpr (COLD != 0) {
        cold.rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(Bc), 0, (uint32_t)a.b_bytes, 0x00020000);
        cold.ldb_bytes = ldb * 4u;
    }
    const ColdPath *cp = COLD != 0 ? &cold : nullptr;

    int *lcol = s_raw + wv * smem_ints_per_wave();
    float *lval = reinterpret_cast<float *>(lcol + kStageMax);
    int *lrp = lcol + 2 * kStageMax;

    vec acc[T];
#pragma unroll
    for (int t = 0; t < T; ++t) acc[t] = vzero<V>();

    if (b < (uint32_t)a.nb_items) {
        // ---- piece of a long row: 4 wavefronts, LDS tree, then C or a partial row ----
        const int4 it = a.items[b];
        row_accumulate<V, G, T, U, NTA, UA, HOT, COLD>(acc, lcol, lval, lane, grp, it.y + wv * kWave, it.z, kBlock, a.colidx,
                                                       a.vals, Bc, ldb, colok[0], boff, a.hotmask, cp);
        reduce_groups<V, G, T>(acc);
        if (grp == 0) {
#pragma unroll
            for (int t = 0; t < T; ++t) {
                if constexpr (V == 1) s_red[wv * TW + t * GV + lig] = acc[t];
                else
#pragma unroll
                    for (int i = 0; i < V; ++i) s_red[wv * TW + t * GV + lig * V + i] = acc[t][i];
            }
        }
        __syncthreads();
        if (wv == 0 && grp == 0) {
            float *dst = it.w < 0 ? a.C + (int64_t)it.x * a.ldc : a.partials + (int64_t)it.w * a.partial_stride;
#pragma unroll
            for (int t = 0; t < T; ++t) {
                if (!colok[t]) continue;
                vec r;
#pragma unroll
                for (int i = 0; i < V; ++i) {
                    const int o = t * GV + lig * V + i;
                    float s = s_red[o];
#pragma unroll
                    for (int w = 1; w < kWavesPerBlock; ++w) s += s_red[w * TW + o];
                    if constexpr (V == 1) r = s;
                    else r[i] = s;
                }
                // a partial row gets its epilogue after the pieces are added
                if (it.w < 0) r = apply_epilogue<V>(r, a.bias ? a.bias + coff[t] : nullptr, a.act);
                if (it.w < 0) vstore<V, NTC, UA>(dst + coff[t], r);
                else vstore<V, false, UA>(dst + coff[t], r);
            }
        }
        if (it.w < 0 || a.tickets == nullptr) return;  // whole row done, or the fix-up launch adds the partial rows
        // ---- piece of a split row: the workgroup that arrives last adds up the row's partial rows ----
        // Every piece publishes its partial row (device-scope release), then takes a ticket of the row (integer
        // atomic); the piece that draws the last ticket knows that all partial rows are visible (device-scope
        // acquire) and adds them in piece order, whichever piece it is: the sum does not depend on the arrival order,
        // and no floating-point atomics are involved.  The counter is left at zero for the next launch.
        const int row_p0 = a.rowptr[it.x], row_p1 = a.rowptr[it.x + 1];
        const int piece = (it.y - row_p0) / a.BCH;
        const int pieces = (row_p1 - row_p0 + a.BCH - 1) / a.BCH;
        const int first = it.w - piece;
        if (wv == 0) {
            __threadfence();  // release: this wavefront's stores of the partial row, device-wide
            if (lane == 0) {
                int32_t *tk = a.tickets + ((int64_t)first * a.ncoltiles + ct);
                const int old = atomicAdd(tk, 1);
                const int is_last = old == pieces - 1;
                if (is_last) atomicExch(tk, 0);
                s_flag = is_last;
            }
        }
        __syncthreads();
        if (!s_flag) return;
        __threadfence();  // acquire: the other pieces' partial rows
        {
            const float *src = a.partials + (int64_t)first * a.partial_stride;
            float *dst = a.C + (int64_t)it.x * a.ldc;
            const int cbeg = (int)ct * TW, cend = min(a.n, cbeg + TW);
            for (int c = cbeg + tid; c < cend; c += kBlock) {
                // read past this die's L2: the other pieces may have run on other dies
                float sum = __hip_atomic_load(src + c, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                for (int i = 1; i < pieces; ++i)
                    sum += __hip_atomic_load(src + (int64_t)i * a.partial_stride + c, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                if (a.bias) sum += a.bias[c];
                if (a.act == 1) sum = fmaxf(sum, 0.f);
                dst[c] = sum;
            }
        }
        return;
    }

    if (b < (uint32_t)(a.nb_items + a.nb_wave)) {
        // ---- medium row: one wavefront, groups interleave entries, shuffle reduction ----
        const int idx = (int)(b - a.nb_items) * kWavesPerBlock + wv;
        if (idx >= a.n_wave_rows) return;
        const int row = a.wave_rows[idx];
        const int2 span = a.wave_span[idx];  // the row's entry range, kept in the plan beside its id
        const int p0 = span.x, p1 = span.y;
        row_accumulate<V, G, T, U, NTA, UA, HOT, COLD>(acc, lcol, lval, lane, grp, p0, p1, kWave, a.colidx, a.vals, Bc, ldb,
                                                       colok[0], boff, a.hotmask, cp);
        reduce_groups<V, G, T>(acc);
        if (grp == 0) {
            float *dst = a.C + (int64_t)row * a.ldc;
#pragma unroll
            for (int t = 0; t < T; ++t)
                if (colok[t]) vstore<V, NTC, UA>(dst + coff[t], apply_epilogue<V>(acc[t], a.bias ? a.bias + coff[t] : nullptr, a.act));
        }
        return;
    }

    // ---- window of consecutive short rows ----
    const int w = (int)(b - a.nb_items - a.nb_wave) * kWavesPerBlock + wv;
    if (w >= a.n_windows) return;
    const int r0 = a.win_row_start[w];
    const int r1 = a.win_row_start[w + 1];
    // which entries the window stages is known from the plan, so colidx/vals are requested together with the row
    // pointers instead of after them
    const int2 stg = a.win_stage[w];
    if (stg.y < 0) return;  // no short row in this window
    const int nr = min(r1 - r0, kWindowRowsMax);
    const int sbeg = stg.x, cnt = stg.y;
    const int rpv = a.rowptr[r0 + min(lane, nr)];
    const int rlast = a.rowptr[r0 + nr];
    int rnext = __shfl_down(rpv, 1, kWave);
    if (lane == kWave - 1) rnext = rlast;
    const bool is_short = lane < nr && (rnext - rpv) <= a.LW;
    if constexpr (G == 1) {
        // SpMV and its neighbours (n <= 4, one lane per entry): a window has far fewer rows than the wavefront has
        // lanes, so the lanes split the window's *entries* instead of its rows: every lane reads its entries
        // (coalesced), gathers the V values of B they point at, and parks the products in LDS; then the lane of
        // each short row adds up that row's products in stored order.
        vec *prod = reinterpret_cast<vec *>(s_prod) + wv * kStageMax;
        constexpr int kSteps = (kStageMax + kWave - 1) / kWave;
        vec x[kSteps];
        float v[kSteps];
#pragma unroll
        for (int i = 0; i < kSteps; ++i) {
            const int e = lane + i * kWave;
            const bool ok = e < cnt;
            const int c = ok ? a.colidx[sbeg + e] : 0;
            v[i] = ok ? a.vals[sbeg + e] : 0.f;
            x[i] = ok ? vload<V, UA>(b_row(Bc, c, ldb) + boff[0]) : vzero<V>();
        }
#pragma unroll
        for (int i = 0; i < kSteps; ++i) {
            const int e = lane + i * kWave;
            if (e < cnt) {
                vec pr = vzero<V>();
                vfma<V>(pr, v[i], x[i]);
                prod[e] = pr;
            }
        }
        wave_lds_sync();
        if (is_short) {
            for (int q = rpv - sbeg; q < rnext - sbeg; ++q) vadd<V>(acc[0], prod[q]);
            vstore<V, NTC, UA>(a.C + (int64_t)(r0 + lane) * a.ldc + coff[0],
                           apply_epilogue<V>(acc[0], a.bias ? a.bias + coff[0] : nullptr, a.act));
        }
        return;
    }
    for (int e = lane; e < cnt; e += kWave) {
        int c = ld_idx<NTA>(a.colidx + sbeg + e);
        if constexpr (HOT) c = mark_hot(c, a.hotmask);
        lcol[e] = c;
        lval[e] = ld_val<NTA>(a.vals + sbeg + e);
    }
    lrp[lane] = rpv;
    if (lane == 0) lrp[nr] = rlast;
    // the lane's bias values are the same for every row of the window: read once
    const bool has_bias = a.bias != nullptr;
    vec bias_r[T];
#pragma unroll
    for (int t = 0; t < T; ++t) bias_r[t] = (has_bias && colok[t]) ? vload<V, UA>(a.bias + coff[t]) : vzero<V>();
    wave_lds_sync();
    for (int ri = grp; ri < nr; ri += S) {
        const int q0 = lrp[ri], q1 = lrp[ri + 1];
        if (q1 - q0 > a.LW) continue;  // medium/long row: handled by another path
#pragma unroll
        for (int t = 0; t < T; ++t) acc[t] = vzero<V>();
        gather_fma<V, T, U, UA, HOT, COLD>(acc, lcol, lval, q0 - sbeg, q1 - sbeg, 1, Bc, ldb, colok[0], boff, cp);
        float *dst = a.C + (int64_t)(r0 + ri) * a.ldc;
#pragma unroll
        for (int t = 0; t < T; ++t)
            if (colok[t]) vstore<V, NTC, UA>(dst + coff[t], apply_epilogue_reg<V>(acc[t], has_bias, bias_r[t], a.act));
    }
}

// Plan-free path: rows in natural order, a run of up to kNaturalRowsMax consecutive rows per wavefront (the host
// picks the run length from m alone, so that the grid still fills the chip; nothing about the row lengths is known
// before the launch).  A wavefront reads the row pointers of its run once (a lane per row) and then proceeds
// greedily: the next rows, as long as they are short (up to kNaturalShort entries) and fit the LDS stage together,
// are staged with coalesced reads and walked one row per lane group, like a window of the planned path; a longer
// row is streamed through the stage by the whole wavefront, the lane groups taking interleaved entries; a row of
// more than kNaturalLong entries (kNaturalMid if such rows are rare in the workgroup) is left to the end, where all 4
// wavefronts of the workgroup take it together (interleaved 64-entry chunks, LDS tree), which shortens the serial
// chain of a heavy row fourfold without any scratch memory.
constexpr int kNaturalLong = 2048;
constexpr int kNaturalMid = 256;
constexpr int kNaturalRowsMax = 16;
constexpr int kNaturalShort = 32;

template <int V, int G, int T, int U, int NT, bool UA>
__global__ __launch_bounds__(kBlock) void spmm_natural_kernel(const ExecArgs a) {
    using vec = typename Vec<V>::type;
    constexpr int S = kWave / G;
    constexpr int GV = G * V;
    constexpr int TW = GV * T;
    constexpr bool NTC = (NT & 1) != 0;
    __shared__ int s_raw[kWavesPerBlock * smem_ints_per_wave()];
    __shared__ float s_red[kWavesPerBlock * TW];
    __shared__ int s_long[kWavesPerBlock * kNaturalRowsMax];  // rows left to the whole workgroup
    __shared__ int s_nlong, s_nmid;
    const int tid = threadIdx.x;
    const int wv = tid >> 6;
    const int lane = tid & 63;
    const int grp = lane / G;
    const int lig = lane % G;
    const uint32_t per_tile = (uint32_t)a.nb_wave;
    uint32_t ct, b;
    if (!tile_of_workgroup(a.xcd_slices, a.ncoltiles, per_tile, ct, b)) return;  // the same for the whole workgroup
    const int NR = a.rows_per_wave;
    const int64_t r0 = ((int64_t)b * kWavesPerBlock + wv) * NR;
    const int nr = (int)max((int64_t)0, min((int64_t)NR, (int64_t)a.m - r0));
    const int c0 = (int)ct * TW + lig * V;
    bool colok[T];
    int coff[T];  // see spmm_fused_kernel
#pragma unroll
    for (int t = 0; t < T; ++t) {
        colok[t] = (c0 + t * GV) < a.n;
        coff[t] = min(c0 + t * GV, a.n - V);
    }
    const uint32_t ldb = (uint32_t)a.ldb;
    int *lcol = s_raw + wv * smem_ints_per_wave();
    float *lval = reinterpret_cast<float *>(lcol + kStageMax);
    int *lrp = lcol + 2 * kStageMax;
    vec acc[T];
    if (tid == 0) {
        s_nlong = 0;
        s_nmid = 0;
    }
    __syncthreads();
    const int rpv = nr > 0 ? a.rowptr[r0 + min(lane, nr)] : 0;
    const int rnext = __shfl_down(rpv, 1, kWave);  // lanes past the run hold the last pointer; lane 63 is never a row
    // Rows of more than kNaturalMid entries: outliers of a graph if the workgroup has one or two of them (then all 4
    // wavefronts take each of them together), the normal case of a matrix with long rows if it has more (then every
    // wavefront keeps its own rows, up to kNaturalLong entries)
    const int nmid = (int)__builtin_popcountll(__ballot(lane < nr && rnext - rpv > kNaturalMid));
    if (lane == 0 && nmid > 0) atomicAdd(&s_nmid, nmid);
    __syncthreads();
    const int long_limit = s_nmid <= 2 ? kNaturalMid : kNaturalLong;
    if (nr > 0) {
        lrp[lane] = rpv;
        wave_lds_sync();
        int i = 0;
        while (i < nr) {
            const int base = lrp[i];
            // rows i .. j-1: the longest run of short rows (one lane group walks a row alone, so only rows of up to
            // kNaturalShort entries qualify) that fits the stage
            const bool stops = lane >= i && (lane >= nr || rnext - rpv > kNaturalShort || rnext - base > kStageMax);
            const int j = __builtin_ctzll(__ballot(stops));  // lane nr always stops
            if (j == i) {
                const int p1 = lrp[i + 1];
                if (p1 - base <= long_limit) {
#pragma unroll
                    for (int t = 0; t < T; ++t) acc[t] = vzero<V>();
                    row_accumulate<V, G, T, U, false, UA>(acc, lcol, lval, lane, grp, base, p1, kWave, a.colidx, a.vals,
                                                          a.B, ldb, colok[0], coff);
                    reduce_groups<V, G, T>(acc);
                    if (grp == 0) {
                        float *dst = a.C + (r0 + i) * a.ldc;
#pragma unroll
                        for (int t = 0; t < T; ++t)
                            if (colok[t])
                                vstore<V, NTC, UA>(dst + coff[t], apply_epilogue<V>(acc[t], a.bias ? a.bias + coff[t] : nullptr, a.act));
                    }
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
#pragma unroll
                for (int t = 0; t < T; ++t) acc[t] = vzero<V>();
                gather_fma<V, T, U, UA>(acc, lcol, lval, lrp[ri] - base, lrp[ri + 1] - base, 1, a.B, ldb, colok[0], coff);
                float *dst = a.C + (r0 + ri) * a.ldc;
#pragma unroll
                for (int t = 0; t < T; ++t)
                    if (colok[t])
                        vstore<V, NTC, UA>(dst + coff[t], apply_epilogue<V>(acc[t], a.bias ? a.bias + coff[t] : nullptr, a.act));
            }
            wave_lds_sync();  // the stage is refilled next
            i = j;
        }
    }
    __syncthreads();
    // long rows of this workgroup, one after the other, all wavefronts on each (the loop is workgroup-uniform; the
    // order of the list varies from run to run, the result of each row does not depend on it)
    const int nlong = s_nlong;
    for (int w = 0; w < nlong; ++w) {
        const int64_t row = s_long[w];
        const int q0 = a.rowptr[row], q1 = a.rowptr[row + 1];
#pragma unroll
        for (int t = 0; t < T; ++t) acc[t] = vzero<V>();
        // twice the gathers in flight: these rows are few, and the longest of them is the serial chain of the launch
        row_accumulate<V, G, T, 2 * U, false, UA>(acc, lcol, lval, lane, grp, q0 + wv * kWave, q1, kBlock, a.colidx,
                                                  a.vals, a.B, ldb, colok[0], coff);
        reduce_groups<V, G, T>(acc);
        __syncthreads();  // s_red of the previous long row has been read
        if (grp == 0) {
#pragma unroll
            for (int t = 0; t < T; ++t) {
                if constexpr (V == 1) s_red[wv * TW + t * GV + lig] = acc[t];
                else
#pragma unroll
                    for (int i = 0; i < V; ++i) s_red[wv * TW + t * GV + lig * V + i] = acc[t][i];
            }
        }
        __syncthreads();
        if (wv == 0 && grp == 0) {
            float *dst = a.C + row * a.ldc;
#pragma unroll
            for (int t = 0; t < T; ++t) {
                if (!colok[t]) continue;
                vec r;
#pragma unroll
                for (int i = 0; i < V; ++i) {
                    const int o = t * GV + lig * V + i;
                    float sum = s_red[o];
#pragma unroll
                    for (int x = 1; x < kWavesPerBlock; ++x) sum += s_red[x * TW + o];
                    if constexpr (V == 1) r = sum;
                    else r[i] = sum;
                }
                vstore<V, NTC, UA>(dst + coff[t], apply_epilogue<V>(r, a.bias ? a.bias + coff[t] : nullptr, a.act));
            }
        }
    }
}

// Copies B (k x n, row stride ldb) into slice-major order: slice s is a dense k x W block holding
// columns [W s, W s + W).  A column slice of a row-major B with a large power-of-two row stride
// lands in few L2 sets; the dense copy makes a slice a contiguous range that an XCD's L2 keeps
// (W = 32, gather kernel) or that streams as whole kilobyte rows into LDS (W = 256, panel kernel).
__global__ __launch_bounds__(kBlock) void spmm_pack_b_kernel(const float *B, int64_t ldb, int32_t k, int32_t n,
                                                             int32_t W, float *Bp) {
    typedef float f4 __attribute__((ext_vector_type(4)));
    const int quads = (n + 3) / 4;  // n % 4 == 0 is guaranteed by the caller
    const int64_t total = (int64_t)k * quads;
    for (int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x; i < total; i += (int64_t)gridDim.x * kBlock) {
        const int64_t r = i / quads;
        const int c = (int)(i - r * quads) * 4;
        const f4 v = *reinterpret_cast<const f4 *>(B + r * ldb + c);
        const int s = c / W;
        *reinterpret_cast<f4 *>(Bp + ((int64_t)s * k + r) * W + (c - s * W)) = v;
    }
}

scorch_status_t launch_pack_b(const float *B, int64_t ldb, int32_t k, int32_t n, int32_t W, float *Bp,
                              hipStream_t stream) {
    const int64_t quads = (int64_t)k * (n / 4);
    if (quads == 0) return SCORCH_OK;
    const uint32_t pgrid = (uint32_t)std::min<int64_t>((quads + kBlock - 1) / kBlock, 256 * 32);
    hipLaunchKernelGGL(spmm_pack_b_kernel, dim3(pgrid), dim3(kBlock), 0, stream, B, ldb, k, n, W, Bp);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return hip_fail(e, "launch spmm_pack_b_kernel");
    return SCORCH_OK;
}

// Rows cut into several pieces: add the partial rows in piece order.
__global__ __launch_bounds__(kBlock) void spmm_fixup_kernel(const FixupArgs a) {
    const int s = blockIdx.x;
    if (s >= a.n_split) return;
    const int4 d = a.split[s];
    const float *src = a.partials + (int64_t)d.y * a.partial_stride;
    float *dst = a.C + (int64_t)d.x * a.ldc;
    for (int c = threadIdx.x; c < a.n; c += kBlock) {
        float sum = src[c];
        for (int i = 1; i < d.z; ++i) sum += src[(int64_t)i * a.partial_stride + c];
        if (a.bias) sum += a.bias[c];
        if (a.act == 1) sum = fmaxf(sum, 0.f);
        dst[c] = sum;
    }
}

// ------------------------------------------------------------------------------------------
// host side: pick the lane mapping from n and the operand alignment, then launch
// ------------------------------------------------------------------------------------------

struct Mapping {
    int V, G, T, ncoltiles;
    bool UA;  // four floats per lane at float alignment, last vector of a row moved back to end at column n
    int xcd_slices;  // 0: tile-major grid; 1: column slices dealt over the XCDs (see tile_of_workgroup)
};

static Mapping pick_mapping(int32_t n, const float *B, int64_t ldb, const float *C, int64_t ldc, int slice_cols) {
    Mapping mp{};
    const uintptr_t pb = reinterpret_cast<uintptr_t>(B), pc = reinterpret_cast<uintptr_t>(C);
    if (n % 4 == 0 && ldb % 4 == 0 && ldc % 4 == 0 && pb % 16 == 0 && pc % 16 == 0) mp.V = 4;
    else if (n >= 4) {
        // rows that are not 16-byte aligned, or n not a multiple of 4: still four floats per lane
        mp.V = 4;
        mp.UA = true;
    } else if (n % 2 == 0 && ldb % 2 == 0 && ldc % 2 == 0 && pb % 8 == 0 && pc % 8 == 0) mp.V = 2;
    else mp.V = 1;
    mp.xcd_slices = 0;
    if (slice_cols > 0 && mp.V == 4 && !mp.UA) {
        // column slices of B (32 columns = one 128-byte line of a row, or 64 or 128), one slice per XCD at a time
        mp.G = slice_cols / 4;
        mp.T = 1;
        mp.ncoltiles = (n + slice_cols - 1) / slice_cols;
        mp.xcd_slices = 1;
        return mp;
    }
    const int lanes = (n + mp.V - 1) / mp.V;
    if (lanes <= kWave) {
        // n <= 4 (SpMV and its neighbours): one lane per group, the 64 lanes of a wavefront take 64 entries
        // of a row (or 64 short rows of a window) per step and are combined by the xor butterfly
        int g = 1;
        while (g < lanes) g <<= 1;
        mp.G = g;
        mp.T = 1;
        mp.ncoltiles = 1;
    } else {
        mp.G = kWave;
        mp.T = 2;
        const int tw = mp.G * mp.V * mp.T;
        mp.ncoltiles = (n + tw - 1) / tw;
    }
    return mp;
}

static int64_t grid_size(const Mapping &mp, int64_t per_tile) {
    return xcd_grid_size(mp.xcd_slices, mp.ncoltiles, per_tile);
}

typedef void (*kernel_fn)(const ExecArgs);

// Compiled variants: V = 4 with every group size, aligned or not; V = 2 and V = 1 only occur for n < 4, i.e. with
// groups of 1, 2 or 4 lanes.
#define SCORCH_PICK_NT(KERNEL, V, G, T, U, UA)                              \
    if (NT & 1) return KERNEL<V, G, T, U, 1, UA>;                           \
    return KERNEL<V, G, T, U, 0, UA>;
#define SCORCH_PICK_U(KERNEL, V, G, T, UA)                                  \
    if (U >= 8) { SCORCH_PICK_NT(KERNEL, V, G, T, 8, UA) } else { SCORCH_PICK_NT(KERNEL, V, G, T, 4, UA) }
#define SCORCH_PICK_G4(KERNEL, UA)                                          \
    if (T == 2) { SCORCH_PICK_U(KERNEL, 4, 64, 2, UA) }                     \
    switch (G) {                                                            \
        case 1: SCORCH_PICK_U(KERNEL, 4, 1, 1, UA)                          \
        case 2: SCORCH_PICK_U(KERNEL, 4, 2, 1, UA)                          \
        case 4: SCORCH_PICK_U(KERNEL, 4, 4, 1, UA)                          \
        case 8: SCORCH_PICK_U(KERNEL, 4, 8, 1, UA)                          \
        case 16: SCORCH_PICK_U(KERNEL, 4, 16, 1, UA)                        \
        case 32: SCORCH_PICK_U(KERNEL, 4, 32, 1, UA)                        \
        default: SCORCH_PICK_U(KERNEL, 4, 64, 1, UA)                        \
    }
#define SCORCH_PICK(KERNEL)                                                 \
    if (V == 4) {                                                           \
        if (UA) { SCORCH_PICK_G4(KERNEL, true) } else { SCORCH_PICK_G4(KERNEL, false) } \
    }                                                                       \
    if (V == 2) { SCORCH_PICK_U(KERNEL, 2, 1, 1, false) }                   \
    switch (G) {                                                            \
        case 1: SCORCH_PICK_U(KERNEL, 1, 1, 1, false)                       \
        case 2: SCORCH_PICK_U(KERNEL, 1, 2, 1, false)                       \
        default: SCORCH_PICK_U(KERNEL, 1, 4, 1, false)                      \
    }

static kernel_fn pick_fused(int V, int G, int T, int U, int NT, bool UA) { SCORCH_PICK(spmm_fused_kernel) }
static kernel_fn pick_fused_hot(int G, int T, int cold) {
    // experiments with the cache policy of the cold rows: whole rows of 97..128 columns only
    if (G == 32 && T == 1 && cold == 1) return spmm_fused_kernel<4, 32, 1, 8, 1, false, true, 1>;
    if (G == 32 && T == 1 && cold == 2) return spmm_fused_kernel<4, 32, 1, 8, 1, false, true, 2>;
    if (G == 32 && T == 1 && cold == 3) return spmm_fused_kernel<4, 32, 1, 8, 1, false, true, 3>;
    if (T == 2) return spmm_fused_kernel<4, 64, 2, 8, 1, false, true>;
    switch (G) {
        case 8: return spmm_fused_kernel<4, 8, 1, 8, 1, false, true>;
        case 16: return spmm_fused_kernel<4, 16, 1, 8, 1, false, true>;
        case 32: return spmm_fused_kernel<4, 32, 1, 8, 1, false, true>;
        default: return spmm_fused_kernel<4, 64, 1, 8, 1, false, true>;
    }
}
// The plan-free path is compiled for one unroll depth (8) and streaming stores only.
#define SCORCH_NATURAL(V, G, T, UA) return spmm_natural_kernel<V, G, T, 8, 1, UA>;
#define SCORCH_NATURAL_G4(UA)                                               \
    if (T == 2) { SCORCH_NATURAL(4, 64, 2, UA) }                            \
    switch (G) {                                                            \
        case 1: SCORCH_NATURAL(4, 1, 1, UA)                                 \
        case 2: SCORCH_NATURAL(4, 2, 1, UA)                                 \
        case 4: SCORCH_NATURAL(4, 4, 1, UA)                                 \
        case 8: SCORCH_NATURAL(4, 8, 1, UA)                                 \
        case 16: SCORCH_NATURAL(4, 16, 1, UA)                               \
        case 32: SCORCH_NATURAL(4, 32, 1, UA)                               \
        default: SCORCH_NATURAL(4, 64, 1, UA)                               \
    }
static kernel_fn pick_natural(int V, int G, int T, bool UA) {
    if (V == 4) {
        if (UA) { SCORCH_NATURAL_G4(true) } else { SCORCH_NATURAL_G4(false) }
    }
    if (V == 2) { SCORCH_NATURAL(2, 1, 1, false) }
    switch (G) {
        case 1: SCORCH_NATURAL(1, 1, 1, false)
        case 2: SCORCH_NATURAL(1, 2, 1, false)
        default: SCORCH_NATURAL(1, 4, 1, false)
    }
}

static inline int64_t ceil_div64(int64_t a, int64_t b) { return (a + b - 1) / b; }

scorch_status_t launch_planned(const scorch_spmm_plan_t *plan, const int32_t *rowptr, const int32_t *colidx,
                               const float *vals, const float *B, int64_t ldb, float *C, int64_t ldc,
                               const float *bias, int32_t act, hipStream_t stream) {
    if (plan->params.PANEL && panel_operands_ok(plan->n, B, ldb, C, ldc))
        return launch_panel(plan, rowptr, colidx, vals, B, ldb, C, ldc, bias, act, stream);
    const Mapping mp = pick_mapping(plan->n, B, ldb, C, ldc, plan->params.SLICED);
    ExecArgs a{};
    a.rowptr = rowptr;
    a.colidx = colidx;
    a.vals = vals;
    a.B = B;
    a.C = C;
    a.ldb = ldb;
    a.ldc = ldc;
    a.m = plan->m;
    a.n = plan->n;
    char *ws = plan->workspace;
    a.win_row_start = reinterpret_cast<const int32_t *>(ws + plan->layout.off_win);
    a.win_stage = reinterpret_cast<const int2 *>(ws + plan->layout.off_stage);
    a.wave_rows = reinterpret_cast<const int32_t *>(ws + plan->layout.off_wave);
    a.wave_span = reinterpret_cast<const int2 *>(ws + plan->layout.off_wave_span);
    a.items = reinterpret_cast<const int4 *>(ws + plan->layout.off_items);
    a.partials = reinterpret_cast<float *>(ws + plan->layout.off_partials);
    // Partial rows of split rows are added by a second, small launch.  Adding them inside the fused launch, by the piece
    // that arrives last, is built and tested but off by default (fix=1 in the tuning text turns it on): with proper
    // device-scope release/acquire fences every piece makes its die write back and invalidate its L2, which cost 90 us
    // on the mid-size graph workload (213 against 123 us).  A variant with written-through atomic stores instead of
    // fences saved 3.5 us there, but the order between the partial row and the ticket then rests on when a
    // written-through store counts as complete, which the language-level memory model does not promise: not kept.
    const bool fold = plan->n_split > 0 && plan->tuning.fix > 0;
    a.tickets = fold ? reinterpret_cast<int32_t *>(ws + plan->layout.off_tickets) : nullptr;
    a.BCH = plan->params.BCH;
    a.n_windows = (int32_t)plan->layout.n_windows;
    a.n_wave_rows = plan->n_wave;
    a.n_items = plan->n_items;
    a.nb_items = plan->n_items;
    a.nb_wave = (int32_t)ceil_div64(plan->n_wave, kWavesPerBlock);
    a.nb_win = plan->n_short > 0 ? (int32_t)ceil_div64(plan->layout.n_windows, kWavesPerBlock) : 0;
    a.partial_stride = plan->layout.partial_stride;
    a.LW = plan->params.LW;
    a.ncoltiles = mp.ncoltiles;
    a.xcd_slices = mp.xcd_slices;
    a.bias = bias;
    a.act = act;
    const int64_t per_tile = (int64_t)a.nb_items + a.nb_wave + a.nb_win;
    const int64_t grid = grid_size(mp, per_tile);
    if (grid > 0x7fffffffLL) {
        set_error("launch grid of %lld workgroups exceeds the HIP limit", (long long)grid);
        return SCORCH_ERR_UNSUPPORTED;
    }
    if (grid > 0 && mp.xcd_slices != 0 && plan->params.PACK && plan->k > 0) {
        float *Bp = reinterpret_cast<float *>(ws + plan->layout.off_bpack);
        scorch_status_t st = launch_pack_b(B, ldb, plan->k, plan->n, kSliceCols, Bp, stream);
        if (st != SCORCH_OK) return st;
        a.B = Bp;
        a.ldb = kSliceCols;
        a.b_tile_stride = (int64_t)plan->k * kSliceCols;
    }
    if (grid > 0) {
        kernel_fn fn = pick_fused(mp.V, mp.G, mp.T, plan->params.U, plan->params.NT, mp.UA);
        if (plan->n_hot > 0 && mp.V == 4 && !mp.UA && mp.xcd_slices == 0 && mp.G >= 8 && plan->params.U >= 8 &&
            (plan->params.NT & 1)) {
            // hot/cold variant: rows of B outside the plan's hot set are read with the streaming policy
            a.hotmask = reinterpret_cast<const uint32_t *>(ws + plan->layout.off_hotmask);
            a.b_bytes = (int64_t)plan->k * ldb * 4;
            fn = pick_fused_hot(mp.G, mp.T, a.b_bytes < (1ll << 32) ? plan->tuning.cold : 0);
        }
        hipLaunchKernelGGL(fn, dim3((uint32_t)grid), dim3(kBlock), 0, stream, a);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return hip_fail(e, "launch spmm_fused_kernel");
    }
    if (plan->n_split > 0 && !fold) {
        FixupArgs f{};
        f.split = reinterpret_cast<const int4 *>(ws + plan->layout.off_split);
        f.partials = a.partials;
        f.C = C;
        f.ldc = ldc;
        f.n = plan->n;
        f.n_split = plan->n_split;
        f.partial_stride = plan->layout.partial_stride;
        f.bias = bias;
        f.act = act;
        hipLaunchKernelGGL(spmm_fixup_kernel, dim3((uint32_t)plan->n_split), dim3(kBlock), 0, stream, f);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return hip_fail(e, "launch spmm_fixup_kernel");
    }
    return SCORCH_OK;
}

scorch_status_t launch_natural(int32_t m, int32_t k, int32_t n, const int32_t *rowptr, const int32_t *colidx,
                               const float *vals, const float *B, int64_t ldb, float *C, int64_t ldc,
                               hipStream_t stream) {
    // Column slices dealt over the XCDs (tile_of_workgroup) need no plan, only the shape: with B of 8 MB or more every
    // XCD walks all rows for one slice of columns at a time, so that the part of B it gathers from is 1/s of B.  Measured
    // on the plan-free call: uniform 1 % pattern, n = 128: 90 -> 69 us with 64-column slices; pruned 4096 x 16384 weight,
    // n = 2048: 5.03 -> 2.26 ms with 128-column slices (64 columns: 3.0 ms, 32: 4.3 ms, 256: 4.2 ms); mid-size graph,
    // n = 128: 168 -> 166 us.  A ragged last slice costs more than it gains, hence the multiples.
    int slice_cols = 0;
    if ((int64_t)k * n * 4 >= (8ll << 20)) {
        if (n >= 256 && n % 128 == 0) slice_cols = 128;
        else if (n >= 128 && n % 64 == 0) slice_cols = 64;
    }
    const Mapping mp = pick_mapping(n, B, ldb, C, ldc, slice_cols);
    ExecArgs a{};
    a.rowptr = rowptr;
    a.colidx = colidx;
    a.vals = vals;
    a.B = B;
    a.C = C;
    a.ldb = ldb;
    a.ldc = ldc;
    a.m = m;
    a.n = n;
    a.xcd_slices = mp.xcd_slices;
    // rows per wavefront: 4 once that leaves a workgroup for every compute unit (measured: 1, 2, 4, 8, 16 rows on the
    // five benchmark workloads; 4 is within 1 % of the best of each that has 16 384 rows or more)
    // (narrow lane groups, i.e. many groups per wavefront: up to one row per group)
    const int64_t rows_cap = std::max(4, std::min(kNaturalRowsMax, kWave / mp.G));
    a.rows_per_wave = (int32_t)std::min<int64_t>(rows_cap, std::max<int64_t>(1, m / 4096));
    a.nb_wave = (int32_t)ceil_div64(m, (int64_t)kWavesPerBlock * a.rows_per_wave);
    a.ncoltiles = mp.ncoltiles;
    const int64_t grid = grid_size(mp, a.nb_wave);
    if (grid > 0x7fffffffLL) {
        set_error("launch grid of %lld workgroups exceeds the HIP limit", (long long)grid);
        return SCORCH_ERR_UNSUPPORTED;
    }
    kernel_fn fn = pick_natural(mp.V, mp.G, mp.T, mp.UA);
    hipLaunchKernelGGL(fn, dim3((uint32_t)grid), dim3(kBlock), 0, stream, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return hip_fail(e, "launch spmm_natural_kernel");
    return SCORCH_OK;
}

}  // namespace scorch
