// Device-side helpers shared by the SpMM and SDDMM kernels (gfx950, 64-wide wavefronts).
#pragma once

#include "spmm_internal.h"

namespace scorch {

template <int V> struct Vec;
template <> struct Vec<1> { using type = float; };
template <> struct Vec<2> { typedef float type __attribute__((ext_vector_type(2))); };
template <> struct Vec<4> { typedef float type __attribute__((ext_vector_type(4))); };
// The same vectors at float alignment: gfx950 takes a global_load/store_dwordx4 at any 4-byte aligned address, so a
// row of B or C that is not 16-byte aligned (odd n or leading dimension) can still move four floats per lane.
template <int V> struct VecU { using type = typename Vec<V>::type; };
template <> struct VecU<4> { typedef float type __attribute__((ext_vector_type(4), aligned(4))); };

template <int V> __device__ __forceinline__ typename Vec<V>::type vzero() {
    typename Vec<V>::type z;
    if constexpr (V == 1) z = 0.f;
    else for (int i = 0; i < V; ++i) z[i] = 0.f;
    return z;
}
template <int V> __device__ __forceinline__ void vfma(typename Vec<V>::type &acc, float a, const typename Vec<V>::type &x) {
    if constexpr (V == 1) acc = __builtin_fmaf(a, x, acc);
    else {
#pragma unroll
        for (int i = 0; i < V; ++i) acc[i] = __builtin_fmaf(a, x[i], acc[i]);
    }
}
template <int V> __device__ __forceinline__ void vadd(typename Vec<V>::type &acc, const typename Vec<V>::type &x) {
    if constexpr (V == 1) acc += x;
    else {
#pragma unroll
        for (int i = 0; i < V; ++i) acc[i] += x[i];
    }
}
// Value held by lane (lane ^ OFF), OFF a power of two below 64.  Distances 1 and 2 are DPP quad
// permutes, 4..16 a ds_swizzle in bit-mask mode (stays inside a 32-lane half, no LDS memory touched),
// 32 a ds_bpermute.
template <int OFF> __device__ __forceinline__ float lane_xor(float x) {
    static_assert(OFF >= 1 && OFF < 64 && (OFF & (OFF - 1)) == 0, "lane distance must be a power of two below 64");
    const int xi = __float_as_int(x);
    int r;
    if constexpr (OFF == 1) r = __builtin_amdgcn_mov_dpp(xi, 0xB1, 0xF, 0xF, true);       // quad_perm [1,0,3,2]
    else if constexpr (OFF == 2) r = __builtin_amdgcn_mov_dpp(xi, 0x4E, 0xF, 0xF, true);  // quad_perm [2,3,0,1]
    else if constexpr (OFF < 32) r = __builtin_amdgcn_ds_swizzle(xi, (OFF << 10) | 0x1F);  // and 0x1f, or 0, xor OFF
    else r = __builtin_amdgcn_ds_bpermute(((int)(threadIdx.x & 63) ^ OFF) << 2, xi);
    return __int_as_float(r);
}
template <int V, int OFF> __device__ __forceinline__ typename Vec<V>::type vlane_xor(const typename Vec<V>::type &x) {
    typename Vec<V>::type r;
    if constexpr (V == 1) r = lane_xor<OFF>(x);
    else {
#pragma unroll
        for (int i = 0; i < V; ++i) r[i] = lane_xor<OFF>(x[i]);
    }
    return r;
}
template <int V, bool UA = false> __device__ __forceinline__ typename Vec<V>::type vload(const float *p) {
    if constexpr (UA) return *reinterpret_cast<const typename VecU<V>::type *>(p);
    else return *reinterpret_cast<const typename Vec<V>::type *>(p);
}
template <int V, bool NT, bool UA = false> __device__ __forceinline__ void vstore(float *p, const typename Vec<V>::type &x) {
    if constexpr (UA) {
        auto *q = reinterpret_cast<typename VecU<V>::type *>(p);
        if constexpr (NT) __builtin_nontemporal_store(x, q);
        else *q = x;
    } else {
        auto *q = reinterpret_cast<typename Vec<V>::type *>(p);
        if constexpr (NT) __builtin_nontemporal_store(x, q);
        else *q = x;
    }
}
// Fused epilogue of a GCN-style layer: v + bias[c..c+V), then the activation (0 identity, 1 ReLU).
// `bias_c` already points at the lane's first column, or is nullptr.
template <int V> __device__ __forceinline__ typename Vec<V>::type apply_epilogue(typename Vec<V>::type v, const float *bias_c,
                                                                              int act) {
    if (bias_c) {
        if constexpr (V == 1) v += bias_c[0];
        else {
#pragma unroll
            for (int i = 0; i < V; ++i) v[i] += bias_c[i];
        }
    }
    if (act == 1) {
        if constexpr (V == 1) v = fmaxf(v, 0.f);
        else {
#pragma unroll
            for (int i = 0; i < V; ++i) v[i] = fmaxf(v[i], 0.f);
        }
    }
    return v;
}

// The same with the lane's V bias values already in registers (loops that store many rows per wavefront read them once).
template <int V> __device__ __forceinline__ typename Vec<V>::type apply_epilogue_reg(typename Vec<V>::type v, bool has_bias,
                                                                                  typename Vec<V>::type bias, int act) {
    if (has_bias) v += bias;
    if (act == 1) {
        if constexpr (V == 1) v = fmaxf(v, 0.f);
        else {
#pragma unroll
            for (int i = 0; i < V; ++i) v[i] = fmaxf(v[i], 0.f);
        }
    }
    return v;
}

template <bool NT> __device__ __forceinline__ int ld_idx(const int32_t *p) {
    if constexpr (NT) return __builtin_nontemporal_load(p);
    else return *p;
}
template <bool NT> __device__ __forceinline__ float ld_val(const float *p) {
    if constexpr (NT) return __builtin_nontemporal_load(p);
    else return *p;
}

// Orders LDS writes before later LDS reads of other lanes of the same wavefront.  LDS operations
// of one wavefront execute in program order, so only the compiler has to be held back.
__device__ __forceinline__ void wave_lds_sync() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

}  // namespace scorch
