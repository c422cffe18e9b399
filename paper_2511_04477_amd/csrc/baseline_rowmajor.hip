// Comparison kernel for the benchmark only: int4 GEMV straight from the ROW-MAJOR source format
// (the layout before repacking), dense or with a naive per-weight sparsity test.
//
// Paper Section 6.1 / 6.3: the row-wise kernel is the baseline the zigzag kernel's dense speed is
// compared with, and "naive skipping" on the row-wise layout is the first ablation - every
// weight's activation is tested where it is used, but a row-major line mixes the weights of 256
// different columns, so no memory traffic can be skipped and the test is pure overhead.
//
// One wavefront owns 2 or 4 consecutive rows (4 when that still gives every CU a workgroup).  A row is K/2 contiguous bytes: the 64 lanes
// read 1 KB of it per step (16 bytes = 32 consecutive k per lane, fully coalesced), so a
// quantization group of 128 columns is 4 lanes wide and every lane applies its own group's
// scale.  x is staged once per workgroup in LDS as fp16 pairs {x[k], x[k+4]}, the pairing in
// which a 32-bit word's nibbles {i, i+4} come out of one mask; codes become fp16 through the
// 0x6400 exponent trick (1024 + nibble, minus 1032) and are multiplied two at a time with
// fp32 accumulation (v_dot2_f32_f16).
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "spqt_calib.h"

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));

constexpr int kWaves = 8;
constexpr int kGroup = 128;
constexpr int kStepCols = 64 * 32;     // columns one wavefront step covers

__device__ __forceinline__ f16x2 as_h2(uint32_t v) { return __builtin_bit_cast(f16x2, v); }
__device__ __forceinline__ uint32_t as_u32(f16x2 v) { return __builtin_bit_cast(uint32_t, v); }

// SKIP: test every weight's activation against the threshold where the weight is used.
template <bool SKIP, int kRowsPerWave>
__global__ __launch_bounds__(kWaves * 64) void rowmajor_gemv_kernel(
    const uint8_t *__restrict__ q, const uint16_t *__restrict__ scales, const uint16_t *__restrict__ x,
    float *__restrict__ y, int M, int K, float thr) {
    extern __shared__ uint32_t xs[];      // K/2 words: word 4*(k/8) + i = {x[8*(k/8) + i], x[8*(k/8) + i + 4]}
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    for (int p = tid; p < K / 8; p += kWaves * 64) {       // 8 consecutive x per lane and trip
        const u32x4 v = *reinterpret_cast<const u32x4 *>(x + 8 * p);   // {x0,x1} {x2,x3} {x4,x5} {x6,x7}
        u32x4 o;
        o.x = (v.x & 0xFFFFu) | (v.z << 16);      // {x0, x4}
        o.y = (v.x >> 16) | (v.z & 0xFFFF0000u);  // {x1, x5}
        o.z = (v.y & 0xFFFFu) | (v.w << 16);      // {x2, x6}
        o.w = (v.y >> 16) | (v.w & 0xFFFF0000u);  // {x3, x7}
        *reinterpret_cast<u32x4 *>(&xs[4 * p]) = o;
    }
    __syncthreads();

    const int NG = K / kGroup;
    const size_t row_bytes = (size_t)K / 2;
    // codes as fp16 without a shift per nibble: after one XOR (two's complement -> offset binary),
    // nibbles {0,4} masked in place under exponent 0x6400 read 1024 + n, nibbles {1,5} masked in
    // place (bits 4..7) read 1024 + 16 n; the latter's sums are scaled by 1/16 once per row step.
    const f16x2 off1 = {(_Float16)1032.0f, (_Float16)1032.0f};
    const f16x2 off16 = {(_Float16)1152.0f, (_Float16)1152.0f};
    {
        const int row0 = (blockIdx.x * kWaves + wave) * kRowsPerWave;
        if (row0 >= M) return;
        float acc[kRowsPerWave];
#pragma unroll
        for (int r = 0; r < kRowsPerWave; ++r) acc[r] = 0.0f;
        for (int k0 = 0; k0 < K; k0 += kStepCols) {
            const int k = k0 + lane * 32;              // this lane's 32 columns
            const bool live = k < K;                   // K % 128 == 0, so a lane is all in or all out
            const int kc = live ? k : 0;
            u32x4 w[kRowsPerWave];
            uint32_t sc[kRowsPerWave];
#pragma unroll
            for (int r = 0; r < kRowsPerWave; ++r) {
                const int row = row0 + r < M ? row0 + r : M - 1;
                w[r] = *reinterpret_cast<const u32x4 *>(q + (size_t)row * row_bytes + kc / 2);
                sc[r] = scales[(size_t)row * NG + kc / kGroup];
            }
            uint32_t xp[16];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const u32x4 v = *reinterpret_cast<const u32x4 *>(&xs[kc / 2 + 4 * j]);
                xp[4 * j + 0] = v.x; xp[4 * j + 1] = v.y; xp[4 * j + 2] = v.z; xp[4 * j + 3] = v.w;
            }
#pragma unroll
            for (int r = 0; r < kRowsPerWave; ++r) {
                float part = 0.0f, part16 = 0.0f;
#pragma unroll
                for (int d = 0; d < 4; ++d) {
                    const uint32_t word = w[r][d] ^ 0x88888888u;
                    const uint32_t word8 = word >> 8;
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        // nibbles i and i+4 of the word
                        const uint32_t src = i < 2 ? word : word8;
                        const bool high = (i & 1) != 0;
                        const uint32_t n = (src & (high ? 0x00F000F0u : 0x000F000Fu)) | 0x64006400u;
                        const f16x2 c = as_h2(n) - (high ? off16 : off1);   // code, or 16 * code
                        uint32_t xw = xp[4 * d + i];
                        if (SKIP) {
                            // naive skipping: the test sits where the weight is used, once per weight
                            const f16x2 xv = as_h2(xw);
                            const uint32_t lo = __builtin_fabsf((float)xv.x) < thr ? 0u : 0x0000FFFFu;
                            const uint32_t hi = __builtin_fabsf((float)xv.y) < thr ? 0u : 0xFFFF0000u;
                            xw &= lo | hi;
                        }
                        if (high) part16 = __builtin_amdgcn_fdot2(c, as_h2(xw), part16, false);
                        else part = __builtin_amdgcn_fdot2(c, as_h2(xw), part, false);
                    }
                }
                part += part16 * 0.0625f;
                const float s = (float)__builtin_bit_cast(_Float16, (uint16_t)sc[r]);
                acc[r] += live ? part * s : 0.0f;
            }
        }
#pragma unroll
        for (int r = 0; r < kRowsPerWave; ++r) {
            float v = acc[r];
#pragma unroll
            for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m);
            if (lane == 0 && row0 + r < M) y[row0 + r] = v;
        }
    }
}

}  // namespace

extern "C" int spqt_calib_rowmajor_gemv(const void *q_rowmajor_dev, const void *scales_dev, int64_t M, int64_t K,
                                        const void *x_dev, float threshold, int skip, float *y_dev,
                                        void *stream) {
    if (!q_rowmajor_dev || !scales_dev || !x_dev || !y_dev) return -1;
    if (M <= 0 || K <= 0 || K % kGroup != 0 || K > 32768 || M > (1 << 24)) return -1;   // x must fit 64 KB of LDS
    if ((uintptr_t)q_rowmajor_dev % 16 != 0 || (uintptr_t)scales_dev % 2 != 0 || (uintptr_t)x_dev % 2 != 0) return -1;
    if (threshold != threshold) return -1;
    const int rows = M >= 256 * kWaves * 4 ? 4 : 2;      // rows per wavefront
    const int grid = (int)((M + kWaves * rows - 1) / (kWaves * rows));
    const size_t lds = (size_t)K * 2;
    hipStream_t st = (hipStream_t)stream;
    const uint8_t *qp = (const uint8_t *)q_rowmajor_dev;
    const uint16_t *sp = (const uint16_t *)scales_dev, *xp = (const uint16_t *)x_dev;
    const dim3 g(grid), b(kWaves * 64);
    if (skip && rows == 4) hipLaunchKernelGGL((rowmajor_gemv_kernel<true, 4>), g, b, lds, st, qp, sp, xp, y_dev, (int)M, (int)K, threshold);
    else if (skip) hipLaunchKernelGGL((rowmajor_gemv_kernel<true, 2>), g, b, lds, st, qp, sp, xp, y_dev, (int)M, (int)K, threshold);
    else if (rows == 4) hipLaunchKernelGGL((rowmajor_gemv_kernel<false, 4>), g, b, lds, st, qp, sp, xp, y_dev, (int)M, (int)K, threshold);
    else hipLaunchKernelGGL((rowmajor_gemv_kernel<false, 2>), g, b, lds, st, qp, sp, xp, y_dev, (int)M, (int)K, threshold);
    return hipGetLastError() == hipSuccess ? 0 : -5;
}
