// Bandwidth probes for the benchmark's "practical peak" figures (gfx950).  BENCHMARK INFRASTRUCTURE ONLY: built into
// its own shared library (libscorch_probes.so), never linked into libscorch_spmm.so, never called by the product path.
//
// The minimum-traffic model prices an SpMM against the 8 TB/s the memory is specified for.  What the chip delivers
// to the access patterns an SpMM is made of is measured here, in the same process and on the same stream as the
// benchmark's timed steps:
//   stream read   every lane reads consecutive 16-byte vectors of a large buffer
//   copy          the same with a streaming store of what was read
//   LDS read      every lane of a 1024-thread workgroup reads 16-byte vectors out of LDS (what bounds the panel kernel)
//   row gather    a group of lanes reads one whole row (256, 400 or 512 bytes) of a table at a pseudo-random row index,
//                 U rows in flight per group -- the access pattern of C_i += A_ij * B_j with random j (the SpMM of the
//                 paper, Section 4.2, on a graph without locality) -- from tables that fit one die's L2, that fit the
//                 memory-side cache, and that exceed both
// All pointers are device pointers owned by the caller; every call enqueues on `stream` and returns; return value 0 or
// a negative number for a bad argument or a failed launch.
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef float f4 __attribute__((ext_vector_type(4)));
typedef float f4u __attribute__((ext_vector_type(4), aligned(4)));

namespace {

constexpr int kBlock = 256;

// the sum is only stored when it equals a value it cannot take by accident: keeps the loads alive, writes nothing
__device__ __forceinline__ void sink_store(float *sink, const f4 &acc) {
    if (acc.x + acc.y + acc.z + acc.w == 12345.678f) sink[0] = acc.x;
}

__global__ __launch_bounds__(kBlock) void probe_read_kernel(const f4 *__restrict__ src, size_t n4, int reps, float *sink) {
    f4 acc = {0.f, 0.f, 0.f, 0.f};
    const size_t stride = (size_t)gridDim.x * kBlock;
    for (int r = 0; r < reps; ++r)
        for (size_t i = (size_t)blockIdx.x * kBlock + threadIdx.x; i < n4; i += stride) acc += src[i];
    sink_store(sink, acc);
}

__global__ __launch_bounds__(kBlock) void probe_copy_kernel(const f4 *__restrict__ src, f4 *__restrict__ dst, size_t n4) {
    const size_t stride = (size_t)gridDim.x * kBlock;
    for (size_t i = (size_t)blockIdx.x * kBlock + threadIdx.x; i < n4; i += stride) __builtin_nontemporal_store(src[i], dst + i);
}

__device__ __forceinline__ uint32_t hash32(uint32_t x) {
    x ^= x >> 16;
    x *= 0x7feb352dU;
    x ^= x >> 15;
    x *= 0x846ca68bU;
    x ^= x >> 16;
    return x;
}

// 32 lanes per row (8 lanes x 16 bytes per 128 bytes of row), `active` of them inside the row, 8 rows in flight per group
__global__ __launch_bounds__(kBlock) void probe_gather_kernel(const float *__restrict__ table, uint32_t rows, uint32_t ld,
                                                              int active, int iters, float *sink) {
    constexpr int G = 32, U = 8;
    const int lane = threadIdx.x & 63, grp = lane / G, lig = lane % G;
    const uint32_t gid = (blockIdx.x * 4u + (threadIdx.x >> 6)) * (64 / G) + grp;
    f4 acc = {0.f, 0.f, 0.f, 0.f};
    if (lig >= active) return;
    for (int it = 0; it < iters; it += U) {
        f4 x[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const uint32_t r = hash32(gid * 7919u + (uint32_t)(it + u) * 104729u) % rows;
            x[u] = *reinterpret_cast<const f4u *>(table + (size_t)r * ld + lig * 4);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) acc += x[u];
    }
    sink_store(sink, acc);
}

// every wavefront of a 1024-thread workgroup reads 16-byte vectors from a 64 KB LDS array, consecutive lanes consecutive
// vectors (the pattern of the panel kernel's reads), 8 reads in flight per lane
__global__ __launch_bounds__(1024) void probe_lds_kernel(int iters, float *sink) {
    __shared__ f4 s_buf[4096];
    for (int i = threadIdx.x; i < 4096; i += 1024) s_buf[i] = f4{(float)i, 1.f, 2.f, 3.f};
    __syncthreads();
    f4 acc = {0.f, 0.f, 0.f, 0.f};
    const int lane = threadIdx.x & 63;
    int row = (threadIdx.x >> 6) * 7;
    for (int it = 0; it < iters; it += 8) {
        f4 x[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            x[u] = s_buf[((row + u * 5) & 63) * 64 + lane];
        }
        row += 41;
#pragma unroll
        for (int u = 0; u < 8; ++u) acc += x[u];
    }
    sink_store(sink, acc);
}

}  // namespace

extern "C" {

// Reads `bytes` (multiple of 16) at `src` `reps` times.  Useful bytes = bytes * reps.
int scorch_probe_stream_read(const void *src, size_t bytes, int reps, float *sink, void *stream) {
    if (!src || !sink || bytes % 16 || reps < 1) return -1;
    hipLaunchKernelGGL(probe_read_kernel, dim3(256 * 16), dim3(kBlock), 0, static_cast<hipStream_t>(stream),
                       static_cast<const f4 *>(src), bytes / 16, reps, sink);
    return hipGetLastError() == hipSuccess ? 0 : -4;
}

// Copies `bytes` (multiple of 16) from src to dst.  Useful bytes = 2 * bytes (read + written).
int scorch_probe_copy(const void *src, void *dst, size_t bytes, void *stream) {
    if (!src || !dst || bytes % 16) return -1;
    hipLaunchKernelGGL(probe_copy_kernel, dim3(256 * 32), dim3(kBlock), 0, static_cast<hipStream_t>(stream),
                       static_cast<const f4 *>(src), static_cast<f4 *>(dst), bytes / 16);
    return hipGetLastError() == hipSuccess ? 0 : -4;
}

// `groups` lane groups (multiple of 8) each gather `iters` (multiple of 8) rows of `row_floats` floats (multiple of 4,
// at most 128) from a table of `rows` rows with row stride `ld` floats (>= row_floats).  Useful bytes = groups * iters *
// row_floats * 4.  Row indices are a hash of (group, iteration): uniform over the table, the same at every call.
int scorch_probe_row_gather(const float *table, uint32_t rows, uint32_t ld, int row_floats, int64_t groups, int iters,
                            float *sink, void *stream) {
    if (!table || !sink || rows == 0 || row_floats < 4 || row_floats > 128 || row_floats % 4 || ld < (uint32_t)row_floats ||
        groups <= 0 || groups % 8 || iters <= 0 || iters % 8 || groups / 8 > 0x7fffffff)
        return -1;
    hipLaunchKernelGGL(probe_gather_kernel, dim3((uint32_t)(groups / 8)), dim3(kBlock), 0, static_cast<hipStream_t>(stream),
                       table, rows, ld, row_floats / 4, iters, sink);
    return hipGetLastError() == hipSuccess ? 0 : -4;
}

// `blocks` workgroups of 1024 threads each read `iters` (multiple of 8) 16-byte vectors per thread from LDS.  Useful
// bytes = blocks * 1024 * iters * 16.
int scorch_probe_lds_read(int blocks, int iters, float *sink, void *stream) {
    if (!sink || blocks <= 0 || iters <= 0 || iters % 8) return -1;
    hipLaunchKernelGGL(probe_lds_kernel, dim3((uint32_t)blocks), dim3(1024), 0, static_cast<hipStream_t>(stream), iters, sink);
    return hipGetLastError() == hipSuccess ? 0 : -4;
}

}  // extern "C"
