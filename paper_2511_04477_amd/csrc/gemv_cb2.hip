// spqt_cb2_gemv, spqt_cb2_gemv_rows, spqt_cb2_gemv_fused: the column-block GEMV for 2-bit codes ("ZZ-CB32-W2", spqt_colblock.h).
//
// Paper Section 4.1.3 states that the column-wise layout carries over to other bit-widths, 2 to 8 bits.
// The kernel body is the one all widths other than 4 share (colblock_width.hpp); this file holds what
// 2 bits decide.  One column's 128-byte run is 512 rows, so a block-row is 512 rows high, a lane owns 64
// rows (two 32-row blocks) and keeps 64 accumulators.
//
// Codes become floats without a conversion instruction.  A 2-bit field that lies inside the 10
// mantissa bits of an fp16 half, all other bits masked away, IS the fp16 subnormal code * 4^j * 2^-24
// (j = 0..4 for bits 2j, 2j + 1): one v_and_b32 isolates the same field of both halves of a dword and
// v_fma_mix_f32 multiplies either half by the staged x * s in fp32; the factor 4^j * 2^-24 is the same for
// every column and comes off the accumulator once at the end.  The three fields that reach into the
// exponent bits are brought down by one shift of the dword by 10 first.  The level of code c is
// (c - 1.5) * s: the lane sums the x * s it used per block and 1.5 times that sum comes off at the end.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "colblock_width.hpp"
#include "spqt_colblock.h"

namespace {

using namespace spqt;

typedef float f32x2 __attribute__((ext_vector_type(2)));

constexpr int kMaxSplits2 = 16;                            // keeps the exchange words inside spqt_workspace_bytes
constexpr int kMaxRows2 = SPQT_CB2_MAX_BATCH;              // activation rows spqt_cb2_gemv_rows takes

struct W2 {
    static constexpr int kRows = SPQT_CB2_TILE_ROWS;           // 512 rows per block-row
    static constexpr int kBlocks = kRows / SPQT_CB_BLOCK_ROWS; // 16 fp16 scales per column
    static constexpr int kScaleBytes = kGroup * 2 * kBlocks;   // 4096
    static constexpr int kChunkBytes = SPQT_CB2_CHUNK_BYTES;
    static constexpr int kAcc = 64;
    struct Scales { u32x4 lo, hi; };
    typedef f32x2 Mine;      // a lane's 64 rows are blocks 2 seg and 2 seg + 1
    typedef f32x2 Sums;

    static __device__ __forceinline__ Sums zero_sums() { return f32x2{0.0f, 0.0f}; }
    static __device__ __forceinline__ Scales load_scales(const uint8_t *p) {
        const u32x4 *sp = reinterpret_cast<const u32x4 *>(p);
        return Scales{sp[0], sp[1]};
    }
    static __device__ __forceinline__ void stage8(float xf, u32x4 v, float *dst) {
        f32x4 *d = reinterpret_cast<f32x4 *>(dst);
        d[0] = f32x4{xf * half_bits_to_float(v.x & 0xFFFFu), xf * half_bits_to_float(v.x >> 16),
                     xf * half_bits_to_float(v.y & 0xFFFFu), xf * half_bits_to_float(v.y >> 16)};
        d[1] = f32x4{xf * half_bits_to_float(v.z & 0xFFFFu), xf * half_bits_to_float(v.z >> 16),
                     xf * half_bits_to_float(v.w & 0xFFFFu), xf * half_bits_to_float(v.w >> 16)};
    }
    static __device__ __forceinline__ void stage(float xf, Scales sv, float *dst) {
        stage8(xf, sv.lo, dst);
        stage8(xf, sv.hi, dst + 8);
    }
    static __device__ __forceinline__ Mine read_mine(const float *col, int seg) {
        return *reinterpret_cast<const f32x2 *>(col + 2 * seg);
    }

    // Sixteen codes of one dword (rows 16 d .. 16 d + 15 of the lane's 64): acc[i] += field_i * xs, where
    // field_i is code_i * 4^p(i) * 2^-24 with p(i) = i % 8 for the five fields inside the mantissa and
    // i % 8 - 5 for the three brought down by the shift.  The factor 4^p * 2^-24 is the same for every
    // column, so it stays in the accumulator until the end of the kernel (field_weight).
    static __device__ __forceinline__ void fma_codes(uint32_t w, float xs, float *acc) {
        const uint32_t w10 = w >> 10;
#pragma unroll
        for (int j = 0; j < 5; ++j) {
            const f16x2 p = as_f16x2(w & (0x00030003u << (2 * j)));           // codes j and 8 + j
            acc[j] = __builtin_fmaf((float)p.x, xs, acc[j]);
            acc[8 + j] = __builtin_fmaf((float)p.y, xs, acc[8 + j]);
        }
#pragma unroll
        for (int j = 5; j < 8; ++j) {
            const f16x2 p = as_f16x2(w10 & (0x00030003u << (2 * (j - 5))));   // codes j and 8 + j, ten bits lower
            acc[j] = __builtin_fmaf((float)p.x, xs, acc[j]);
            acc[8 + j] = __builtin_fmaf((float)p.y, xs, acc[8 + j]);
        }
    }
    // What accumulator i has to be multiplied by to read code * xs: 2^24 / 4^p(i).
    static __device__ __forceinline__ constexpr float field_weight(int i) {
        const int p = (i & 7) < 5 ? (i & 7) : (i & 7) - 5;
        return kTwo24 / (float)(1 << (2 * p));
    }
    // One column: the lane's 16 bytes are 64 rows, the first 32 of block 2 seg, the rest of block 2 seg + 1.
    static __device__ __forceinline__ void step(u32x4 w, Mine xs, float *acc, Sums &bs) {
        fma_codes(w.x, xs.x, acc + 0);
        fma_codes(w.y, xs.x, acc + 16);
        fma_codes(w.z, xs.y, acc + 32);
        fma_codes(w.w, xs.y, acc + 48);
        bs += xs;
    }
    // accumulator i is row 64 seg + i; each half of them is one block and folds like the 4-bit kernel's 32
    static __device__ __forceinline__ void finish(float *acc, Sums bs, int seg, int cgr, float *red) {
        float r0[4], r1[4];
#pragma unroll
        for (int i = 0; i < 64; ++i) acc[i] *= field_weight(i);
        fold_columns(acc + 0, r0);
        fold_columns(acc + 32, r1);
        const float bias0 = sum_over_columns(bs.x) * 1.5f;
        const float bias1 = sum_over_columns(bs.y) * 1.5f;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            red[64 * seg + 4 * cgr + j] = r0[j] - bias0;
            red[64 * seg + 32 + 4 * cgr + j] = r1[j] - bias1;
        }
    }
};
static_assert(W2::kChunkBytes == W2::kScaleBytes + kGroup * 128, "chunk size");

template <int WAVES, bool DENSE, bool FUSED, int BATCH>
__global__ __launch_bounds__(WAVES * 64) void spqt_cb2_gemv_kernel(
    const uint8_t *__restrict__ packed, const uint16_t *__restrict__ x, const int32_t *__restrict__ idx,
    const int32_t *__restrict__ count, float *__restrict__ y, void *partials, int32_t *ws_flags, int K, int NC, int S,
    int T, int M, float thr) {
    colblock_width_gemv<W2, WAVES, DENSE, FUSED, BATCH>(packed, x, idx, count, y, partials, ws_flags, K, NC, S, T, M, thr);
}

#define SPQT_CB2_LAUNCH(W, D, F, B)                                                                                \
    hipLaunchKernelGGL((spqt_cb2_gemv_kernel<W, D, F, B>), dim3(grid), dim3(W * 64), 0, st, pk, xp, idx_dev, count_dev, \
                       (float *)y_dev, partials, ws_flags, (int)K, NC, S, T, m_and_flags, thr)
// mode 0 = index list, 1 = dense, 2 = one launch (one activation row)
#define SPQT_CB2_MODES(W, B)                                   \
    do {                                                         \
        if (md == 0) SPQT_CB2_LAUNCH(W, false, false, B);          \
        else if (md == 1) SPQT_CB2_LAUNCH(W, true, false, B);      \
        else SPQT_CB2_LAUNCH(W, false, true, 1);                   \
    } while (0)
#define SPQT_CB2_ROWS(W)                          \
    do {                                            \
        switch (batch) {                            \
            case 1: SPQT_CB2_MODES(W, 1); break;      \
            case 2: SPQT_CB2_MODES(W, 2); break;      \
            default: SPQT_CB2_MODES(W, 3); break;     \
        }                                           \
    } while (0)

int run2(int mode, int batch, const void *packed_dev, int64_t M, int64_t K, const void *x_dev, const int32_t *idx_dev,
         const int32_t *count_dev, float thr, void *y_dev, void *workspace_dev, size_t workspace_bytes, void *stream,
         const spqt_launch_cfg *cfg) {
    // a fourth activation row's 64 accumulators no longer fit the register file next to two stages of weights
    if (batch > kMaxRows2) return SPQT_ESHAPE;
    // about one workgroup of 4 wavefronts per CU: the 64 accumulators per activation row and two stages
    // of weights leave room for one wavefront per SIMD; S a power of two <= 16
    const int64_t T64 = (M + W2::kRows - 1) / W2::kRows;
    int S0 = 1;
    while (S0 * 2 <= kMaxSplits2 && (int64_t)S0 * 2 * T64 <= 256) S0 *= 2;
    while (S0 > 1 && (int64_t)S0 * 4 * kPassCols > K) S0 /= 2;      // at least one full pass (or unit) per wavefront when dense
    hipStream_t st = (hipStream_t)stream;
    const uint8_t *pk = (const uint8_t *)packed_dev;
    const uint16_t *xp = (const uint16_t *)x_dev;
    return colblock_width_run<W2>(
        mode, batch, kMaxSplits2, S0, packed_dev, M, K, x_dev, idx_dev, count_dev, y_dev, workspace_dev, workspace_bytes, cfg,
        [&](int waves, int md, int grid, void *partials, int32_t *ws_flags, int NC, int S, int T, int m_and_flags) {
            switch (waves) {
                case 1: SPQT_CB2_ROWS(1); break;
                case 2: SPQT_CB2_ROWS(2); break;
                default: SPQT_CB2_ROWS(4); break;
            }
            return hipGetLastError();
        });
}

}  // namespace

extern "C" int spqt_cb2_gemv(const void *packed_dev, int64_t M, int64_t K, const void *x_dev,
                             const int32_t *idx_dev, const int32_t *count_dev, void *y_dev,
                             void *workspace_dev, size_t workspace_bytes, void *stream,
                             const spqt_launch_cfg *cfg) {
    return run2(idx_dev ? 0 : 1, 1, packed_dev, M, K, x_dev, idx_dev, count_dev, 0.0f, y_dev, workspace_dev, workspace_bytes,
                stream, cfg);
}

extern "C" int spqt_cb2_gemv_fused(const void *packed_dev, int64_t M, int64_t K, const void *x_dev, float threshold,
                                   void *y_dev, void *workspace_dev, size_t workspace_bytes, void *stream,
                                   const spqt_launch_cfg *cfg) {
    if (threshold != threshold) return SPQT_EINVAL;
    return run2(2, 1, packed_dev, M, K, x_dev, nullptr, nullptr, threshold, y_dev, workspace_dev, workspace_bytes, stream, cfg);
}

extern "C" int spqt_cb2_gemv_rows(const void *packed_dev, int64_t M, int64_t K, const void *x_dev, int batch,
                                  const int32_t *idx_dev, const int32_t *count_dev, void *y_dev,
                                  void *workspace_dev, size_t workspace_bytes, void *stream,
                                  const spqt_launch_cfg *cfg) {
    return run2(idx_dev ? 0 : 1, batch, packed_dev, M, K, x_dev, idx_dev, count_dev, 0.0f, y_dev, workspace_dev,
                workspace_bytes, stream, cfg);
}
