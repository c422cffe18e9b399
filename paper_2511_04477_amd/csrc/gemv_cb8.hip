// spqt_cb8_gemv, spqt_cb8_gemv_rows, spqt_cb8_gemv_fused: the column-block GEMV for 8-bit codes ("ZZ-CB32-W8", spqt_colblock.h).
//
// Paper Section 4.1.3 states that the column-wise layout carries over to other bit-widths.  The kernel
// body is the one all widths other than 4 share (colblock_width.hpp); this file holds what 8 bits
// decide.  One column's 128-byte run is 128 rows, so a block-row is 128 rows high, a lane owns 16 rows
// (half a 32-row block) and keeps 16 accumulators.
//
// Codes become floats without a conversion instruction: v_perm_b32 puts byte b under the fp16
// exponent 0x64 (value 1024 + b, exact), two codes per permute, and v_fma_mix_f32 multiplies a
// half of that pair by the staged x * s in fp32.  The stored byte is q + 128, so every product
// carries (q + 1152) * xs; the lane sums the xs it used and 1152 times that sum comes off at the end.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "colblock_width.hpp"
#include "spqt_colblock.h"

namespace {

using namespace spqt;

// One (a, b) pair of the first fold level (lanes l and l ^ 8, see fold8_x8): returns the register
// that holds a's pair sum in lanes with bit 3 clear and b's in lanes with bit 3 set.
__device__ __forceinline__ float fold8(float a, float b) {
    asm volatile("s_nop 1\n\t" SPQT_FOLD8("%0", "%1") : "+v"(b) : "v"(a));
    return b;
}

struct W8 {
    static constexpr int kRows = SPQT_CB8_TILE_ROWS;           // 128 rows per block-row
    static constexpr int kBlocks = kRows / SPQT_CB_BLOCK_ROWS; // 4 fp16 scales per column
    static constexpr int kScaleBytes = kGroup * 2 * kBlocks;   // 1024
    static constexpr int kChunkBytes = SPQT_CB8_CHUNK_BYTES;
    static constexpr int kAcc = 16;
    static constexpr float kCodeBias = 1024.0f + 128.0f;
    typedef u32x2 Scales;
    typedef float Mine;      // a lane's 16 rows lie in one block
    typedef float Sums;

    static __device__ __forceinline__ Sums zero_sums() { return 0.0f; }
    static __device__ __forceinline__ Scales load_scales(const uint8_t *p) { return *reinterpret_cast<const u32x2 *>(p); }
    static __device__ __forceinline__ void stage(float xf, Scales sv, float *dst) {
        *reinterpret_cast<f32x4 *>(dst) =
            f32x4{xf * half_bits_to_float(sv.x & 0xFFFFu), xf * half_bits_to_float(sv.x >> 16),
                  xf * half_bits_to_float(sv.y & 0xFFFFu), xf * half_bits_to_float(sv.y >> 16)};
    }
    static __device__ __forceinline__ Mine read_mine(const float *col, int seg) { return col[seg >> 1]; }

    // Four codes of one dword (rows 4d .. 4d+3 of the lane's 16): acc[i] += (1024 + byte_i) * xs.
    static __device__ __forceinline__ void fma_bytes(uint32_t w, float xs, float *acc) {
        const f16x2 p01 = as_f16x2(__builtin_amdgcn_perm(0x64646464u, w, 0x04010400u));   // {b0, 0x64, b1, 0x64}
        const f16x2 p23 = as_f16x2(__builtin_amdgcn_perm(0x64646464u, w, 0x04030402u));   // {b2, 0x64, b3, 0x64}
        acc[0] = __builtin_fmaf((float)p01.x, xs, acc[0]);
        acc[1] = __builtin_fmaf((float)p01.y, xs, acc[1]);
        acc[2] = __builtin_fmaf((float)p23.x, xs, acc[2]);
        acc[3] = __builtin_fmaf((float)p23.y, xs, acc[3]);
    }
    static __device__ __forceinline__ void step(u32x4 w, Mine xs, float *acc, Sums &bs) {
        fma_bytes(w.x, xs, acc + 0);
        fma_bytes(w.y, xs, acc + 4);
        fma_bytes(w.z, xs, acc + 8);
        fma_bytes(w.w, xs, acc + 12);
        bs += xs;
    }
    // Fold the 16 accumulators of the 8 lanes that read the same rows, halving the live values at each
    // level: lane (cg, seg) ends with the complete sums of rows 16 seg + 2 rev(cg) + j, j = 0, 1 (rev
    // reverses the three bits of cg).  Once per kernel, so no batched asm blocks here.
    static __device__ __forceinline__ void finish(const float *acc, Sums bs, int seg, int cgr, float *red) {
        float v[8], u[4], r2[2];
#pragma unroll
        for (int i = 0; i < 8; ++i) v[i] = fold8(acc[i], acc[i + 8]);
#pragma unroll
        for (int i = 0; i < 4; ++i) u[i] = fold16(v[i], v[i + 4]);
#pragma unroll
        for (int i = 0; i < 2; ++i) r2[i] = fold32(u[i], u[i + 2]);
        const float bias = sum_over_columns(bs) * kCodeBias;
        red[16 * seg + 2 * cgr + 0] = r2[0] - bias;
        red[16 * seg + 2 * cgr + 1] = r2[1] - bias;
    }
};
static_assert(W8::kChunkBytes == W8::kScaleBytes + kGroup * 128, "chunk size");

template <int WAVES, bool DENSE, bool FUSED, int BATCH>
__global__ __launch_bounds__(WAVES * 64) void spqt_cb8_gemv_kernel(
    const uint8_t *__restrict__ packed, const uint16_t *__restrict__ x, const int32_t *__restrict__ idx,
    const int32_t *__restrict__ count, float *__restrict__ y, void *partials, int32_t *ws_flags, int K, int NC, int S,
    int T, int M, float thr) {
    colblock_width_gemv<W8, WAVES, DENSE, FUSED, BATCH>(packed, x, idx, count, y, partials, ws_flags, K, NC, S, T, M, thr);
}

#define SPQT_CB8_LAUNCH(W, D, F, B)                                                                                \
    hipLaunchKernelGGL((spqt_cb8_gemv_kernel<W, D, F, B>), dim3(grid), dim3(W * 64), 0, st, pk, xp, idx_dev, count_dev, \
                       (float *)y_dev, partials, ws_flags, (int)K, NC, S, T, m_and_flags, thr)
// mode 0 = index list, 1 = dense, 2 = one launch (one activation row)
#define SPQT_CB8_MODES(W, B)                                   \
    do {                                                         \
        if (md == 0) SPQT_CB8_LAUNCH(W, false, false, B);          \
        else if (md == 1) SPQT_CB8_LAUNCH(W, true, false, B);      \
        else SPQT_CB8_LAUNCH(W, false, true, 1);                   \
    } while (0)
#define SPQT_CB8_ROWS(W)                          \
    do {                                            \
        switch (batch) {                            \
            case 1: SPQT_CB8_MODES(W, 1); break;      \
            case 2: SPQT_CB8_MODES(W, 2); break;      \
            case 3: SPQT_CB8_MODES(W, 3); break;      \
            default: SPQT_CB8_MODES(W, 4); break;     \
        }                                           \
    } while (0)

int run8(int mode, int batch, const void *packed_dev, int64_t M, int64_t K, const void *x_dev, const int32_t *idx_dev,
         const int32_t *count_dev, float thr, void *y_dev, void *workspace_dev, size_t workspace_bytes, void *stream,
         const spqt_launch_cfg *cfg) {
    // same targets as the 4-bit column-block kernel: about 512 (list) / 1024 (dense) workgroups of
    // 4 wavefronts, 256 on matrices large enough to be bandwidth-bound; S a power of two <= 16
    const int64_t T64 = (M + W8::kRows - 1) / W8::kRows;
    const bool big = M > 0 && K > 0 && (size_t)M * (size_t)K >= ((size_t)64 << 20);
    const int64_t target = big && batch == 1 ? 256 : (mode == 1 && batch == 1 ? 1024 : 512);
    int S0 = 1;
    while (S0 * 2 <= 16 && (int64_t)S0 * 2 * T64 <= target) S0 *= 2;
    while (mode == 2 && S0 > 1 && (int64_t)S0 * 4 * kPassCols > K) S0 /= 2;   // one launch: at least one unit per wavefront
    hipStream_t st = (hipStream_t)stream;
    const uint8_t *pk = (const uint8_t *)packed_dev;
    const uint16_t *xp = (const uint16_t *)x_dev;
    return colblock_width_run<W8>(
        mode, batch, SPQT_MAX_SPLITS, S0, packed_dev, M, K, x_dev, idx_dev, count_dev, y_dev, workspace_dev, workspace_bytes, cfg,
        [&](int waves, int md, int grid, void *partials, int32_t *ws_flags, int NC, int S, int T, int m_and_flags) {
            switch (waves) {
                case 1: SPQT_CB8_ROWS(1); break;
                case 2: SPQT_CB8_ROWS(2); break;
                default: SPQT_CB8_ROWS(4); break;
            }
            return hipGetLastError();
        });
}

}  // namespace

extern "C" int spqt_cb8_gemv(const void *packed_dev, int64_t M, int64_t K, const void *x_dev,
                             const int32_t *idx_dev, const int32_t *count_dev, void *y_dev,
                             void *workspace_dev, size_t workspace_bytes, void *stream,
                             const spqt_launch_cfg *cfg) {
    return run8(idx_dev ? 0 : 1, 1, packed_dev, M, K, x_dev, idx_dev, count_dev, 0.0f, y_dev, workspace_dev, workspace_bytes,
                stream, cfg);
}

extern "C" int spqt_cb8_gemv_fused(const void *packed_dev, int64_t M, int64_t K, const void *x_dev, float threshold,
                                   void *y_dev, void *workspace_dev, size_t workspace_bytes, void *stream,
                                   const spqt_launch_cfg *cfg) {
    if (threshold != threshold) return SPQT_EINVAL;
    return run8(2, 1, packed_dev, M, K, x_dev, nullptr, nullptr, threshold, y_dev, workspace_dev, workspace_bytes, stream, cfg);
}

extern "C" int spqt_cb8_gemv_rows(const void *packed_dev, int64_t M, int64_t K, const void *x_dev, int batch,
                                  const int32_t *idx_dev, const int32_t *count_dev, void *y_dev,
                                  void *workspace_dev, size_t workspace_bytes, void *stream,
                                  const spqt_launch_cfg *cfg) {
    return run8(idx_dev ? 0 : 1, batch, packed_dev, M, K, x_dev, idx_dev, count_dev, 0.0f, y_dev, workspace_dev,
                workspace_bytes, stream, cfg);
}
