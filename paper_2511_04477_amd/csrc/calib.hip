// Measurement helpers for the benchmark: streaming read, plain copy, empty launch.
// Nothing here is on the GEMV path.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "spqt_calib.h"

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

template <int UNROLL>
__global__ __launch_bounds__(256) void read_kernel(const u32x4 *__restrict__ src, size_t n16,
                                                   uint32_t *sink) {
    const size_t stride = (size_t)gridDim.x * 256;
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    u32x4 acc = {0u, 0u, 0u, 0u};
    for (; i + (UNROLL - 1) * stride < n16; i += UNROLL * stride) {
        u32x4 v[UNROLL];
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) v[u] = __builtin_nontemporal_load(src + i + u * stride);
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) acc ^= v[u];
    }
    for (; i < n16; i += stride) acc ^= __builtin_nontemporal_load(src + i);
    const uint32_t x = acc.x ^ acc.y ^ acc.z ^ acc.w;
    if (x == 0x9E3779B9u) *sink = x;
}

// Same bytes, but every wavefront owns one contiguous slice and walks it 1 KB at a time (the
// access order of a GEMV wavefront that owns a contiguous range of columns).
template <int UNROLL>
__global__ __launch_bounds__(256) void read_blocked_kernel(const u32x4 *__restrict__ src, size_t n16,
                                                           uint32_t *sink) {
    const size_t waves = (size_t)gridDim.x * 4;
    const size_t wave = (size_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    const size_t per = (n16 / 64 + waves - 1) / waves * 64;      // 16-byte units per wave, multiple of 64
    size_t i = wave * per + (threadIdx.x & 63);
    const size_t stop = (wave + 1) * per < n16 ? (wave + 1) * per : n16;
    u32x4 acc = {0u, 0u, 0u, 0u};
    for (; i + (UNROLL - 1) * 64 < stop; i += UNROLL * 64) {
        u32x4 v[UNROLL];
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) v[u] = __builtin_nontemporal_load(src + i + u * 64);
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) acc ^= v[u];
    }
    for (; i < stop; i += 64) acc ^= __builtin_nontemporal_load(src + i);
    const uint32_t x = acc.x ^ acc.y ^ acc.z ^ acc.w;
    if (x == 0x9E3779B9u) *sink = x;
}

// Reads only the listed 128-byte lines (ascending list), 8 lines per wavefront load, each wavefront
// owning a contiguous slice of the list: the memory access pattern of the sparse GEMV with no
// arithmetic at all.
template <int UNROLL>
__global__ __launch_bounds__(256) void read_lines_kernel(const uint8_t *__restrict__ src,
                                                         const int32_t *__restrict__ lines, int n_lines,
                                                         uint32_t *sink) {
    const int waves = gridDim.x * 4;
    const int wave = blockIdx.x * 4 + (threadIdx.x >> 6);
    const int lane = threadIdx.x & 63, cg = lane >> 3, seg = lane & 7;
    const int per = ((n_lines + waves - 1) / waves + 7) / 8 * 8;
    int i = wave * per;
    const int stop = (wave + 1) * per < n_lines ? (wave + 1) * per : n_lines;
    u32x4 acc = {0u, 0u, 0u, 0u};
    for (; i < stop; i += UNROLL * 8) {
        int line[UNROLL];
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            const int e = i + u * 8 + cg;
            line[u] = lines[e < stop ? e : stop - 1];
        }
        u32x4 v[UNROLL];
#pragma unroll
        for (int u = 0; u < UNROLL; ++u)
            v[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(src + (size_t)line[u] * 128 + seg * 16));
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) acc ^= v[u];
    }
    const uint32_t x = acc.x ^ acc.y ^ acc.z ^ acc.w;
    if (x == 0x9E3779B9u) *sink = x;
}

__global__ __launch_bounds__(256) void copy_kernel(u32x4 *__restrict__ dst, const u32x4 *__restrict__ src,
                                                   size_t n16) {
    const size_t stride = (size_t)gridDim.x * 256;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}

__global__ void empty_kernel() {}

}  // namespace

extern "C" int spqt_calib_read(const void *src_dev, size_t bytes, uint32_t *sink_dev, int blocks,
                               int unroll, void *stream) {
    if (!src_dev || !sink_dev || bytes == 0 || bytes % 16 || (uintptr_t)src_dev % 16) return -1;
    const size_t n16 = bytes / 16;
    if (blocks <= 0) blocks = 256 * 8;
    hipStream_t st = (hipStream_t)stream;
    const u32x4 *src = (const u32x4 *)src_dev;
    switch (unroll) {
        case 1: hipLaunchKernelGGL(read_kernel<1>, dim3(blocks), dim3(256), 0, st, src, n16, sink_dev); break;
        case 2: hipLaunchKernelGGL(read_kernel<2>, dim3(blocks), dim3(256), 0, st, src, n16, sink_dev); break;
        case 4: hipLaunchKernelGGL(read_kernel<4>, dim3(blocks), dim3(256), 0, st, src, n16, sink_dev); break;
        case 8: hipLaunchKernelGGL(read_kernel<8>, dim3(blocks), dim3(256), 0, st, src, n16, sink_dev); break;
        case 16: hipLaunchKernelGGL(read_kernel<16>, dim3(blocks), dim3(256), 0, st, src, n16, sink_dev); break;
        default: return -1;
    }
    return hipGetLastError() == hipSuccess ? 0 : -5;
}

extern "C" int spqt_calib_read_blocked(const void *src_dev, size_t bytes, uint32_t *sink_dev, int blocks,
                                       int unroll, void *stream) {
    if (!src_dev || !sink_dev || bytes == 0 || bytes % 16 || (uintptr_t)src_dev % 16) return -1;
    const size_t n16 = bytes / 16;
    if (blocks <= 0) blocks = 512;
    hipStream_t st = (hipStream_t)stream;
    const u32x4 *src = (const u32x4 *)src_dev;
    switch (unroll) {
        case 2: hipLaunchKernelGGL(read_blocked_kernel<2>, dim3(blocks), dim3(256), 0, st, src, n16, sink_dev); break;
        case 4: hipLaunchKernelGGL(read_blocked_kernel<4>, dim3(blocks), dim3(256), 0, st, src, n16, sink_dev); break;
        case 8: hipLaunchKernelGGL(read_blocked_kernel<8>, dim3(blocks), dim3(256), 0, st, src, n16, sink_dev); break;
        case 16: hipLaunchKernelGGL(read_blocked_kernel<16>, dim3(blocks), dim3(256), 0, st, src, n16, sink_dev); break;
        default: return -1;
    }
    return hipGetLastError() == hipSuccess ? 0 : -5;
}

extern "C" int spqt_calib_read_lines(const void *src_dev, const int32_t *lines_dev, int n_lines,
                                     uint32_t *sink_dev, int blocks, int unroll, void *stream) {
    if (!src_dev || !lines_dev || !sink_dev || n_lines <= 0 || (uintptr_t)src_dev % 128) return -1;
    if (blocks <= 0) blocks = 512;
    hipStream_t st = (hipStream_t)stream;
    const uint8_t *src = (const uint8_t *)src_dev;
    switch (unroll) {
        case 2: hipLaunchKernelGGL(read_lines_kernel<2>, dim3(blocks), dim3(256), 0, st, src, lines_dev, n_lines, sink_dev); break;
        case 4: hipLaunchKernelGGL(read_lines_kernel<4>, dim3(blocks), dim3(256), 0, st, src, lines_dev, n_lines, sink_dev); break;
        case 8: hipLaunchKernelGGL(read_lines_kernel<8>, dim3(blocks), dim3(256), 0, st, src, lines_dev, n_lines, sink_dev); break;
        case 16: hipLaunchKernelGGL(read_lines_kernel<16>, dim3(blocks), dim3(256), 0, st, src, lines_dev, n_lines, sink_dev); break;
        default: return -1;
    }
    return hipGetLastError() == hipSuccess ? 0 : -5;
}

extern "C" int spqt_calib_copy(void *dst_dev, const void *src_dev, size_t bytes, int blocks, void *stream) {
    if (!dst_dev || !src_dev || bytes == 0 || bytes % 16 || (uintptr_t)src_dev % 16 || (uintptr_t)dst_dev % 16)
        return -1;
    if (blocks <= 0) blocks = 256 * 8;
    hipLaunchKernelGGL(copy_kernel, dim3(blocks), dim3(256), 0, (hipStream_t)stream, (u32x4 *)dst_dev,
                       (const u32x4 *)src_dev, bytes / 16);
    return hipGetLastError() == hipSuccess ? 0 : -5;
}

extern "C" int spqt_calib_empty(void *stream) {
    hipLaunchKernelGGL(empty_kernel, dim3(1), dim3(64), 0, (hipStream_t)stream);
    return hipGetLastError() == hipSuccess ? 0 : -5;
}
