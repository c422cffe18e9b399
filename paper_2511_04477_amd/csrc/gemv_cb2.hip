// spqt_cb2_gemv: the column-block GEMV for 2-bit codes ("ZZ-CB32-W2", spqt_colblock.h).
//
// Paper Section 4.1.3 states that the column-wise layout carries over to other bit-widths, 2 to 8 bits.
// What the 4-bit kernels are built around is kept: one activation column's weights of a block-row are
// ONE 128-byte run, read by 8 lanes with one 16-byte load each, 8 columns per wavefront load, 64
// list entries per pass.  With 2-bit codes that run is 512 rows, so a block-row is 512 rows high,
// a lane owns 64 rows (two 32-row blocks) and keeps 64 accumulators.  Everything else follows
// spqt_cb_gemv_kernel: even split of the index list over the S x WAVES wavefronts of a block-row
// (Section 4.2.3), the scales folded into x by the lane that owns the list entry, two-stage
// software pipeline with unpredicated clamped loads, one fold of the 8 column-lanes at the end,
// reduction through LDS and the tagged-word exchange.  Batch 1; list-driven or dense.
//
// Codes become floats without a conversion instruction.  A 2-bit field that lies inside the 10
// mantissa bits of an fp16 half, all other bits masked away, IS the fp16 subnormal code * 4^j * 2^-24
// (j = 0..4 for bits 2j, 2j + 1): one v_and_b32 isolates the same field of both halves of a dword and
// v_fma_mix_f32 multiplies either half by the staged x * s in fp32; the factor 4^j * 2^-24 is the same for
// every column and comes off the accumulator once at the end.  The three fields that
// reach into the exponent bits are brought down by one shift of the dword by 10 first.  The level of code
// c is (c - 1.5) * s: the lane sums the x * s it used per block and 1.5 times that sum comes off at the end.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "gemv_common.hpp"
#include "spqt_colblock.h"

namespace {

using namespace spqt;

typedef float f32x2 __attribute__((ext_vector_type(2)));

constexpr int kRows2 = SPQT_CB2_TILE_ROWS;                 // 512 rows per block-row
constexpr int kBlocks2 = kRows2 / SPQT_CB_BLOCK_ROWS;      // 16 blocks, one fp16 scale each
constexpr int kScaleBytes2 = kGroup * 2 * kBlocks2;        // 128 columns x 16 fp16 scales
constexpr int kChunkBytes2 = SPQT_CB2_CHUNK_BYTES;
static_assert(kChunkBytes2 == kScaleBytes2 + kGroup * 128, "chunk size");
constexpr int kMaxSplits2 = 16;                            // keeps the exchange words inside spqt_workspace_bytes

// Sixteen codes of one dword (rows 16 d .. 16 d + 15 of the lane's 64): acc[i] += field_i * xs, where field_i
// is code_i * 4^p(i) * 2^-24 with p(i) = i % 8 for the five fields inside the mantissa and i % 8 - 5 for the
// three brought down by the shift.  The factor 4^p * 2^-24 is the same for every column, so it stays in
// the accumulator until the end of the kernel (field_weight).
__device__ __forceinline__ void fma_codes2(uint32_t w, float xs, float *acc) {
    const uint32_t w10 = w >> 10;
#pragma unroll
    for (int j = 0; j < 5; ++j) {
        const f16x2 p = as_f16x2(w & (0x00030003u << (2 * j)));        // codes j and 8 + j
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
__device__ __forceinline__ constexpr float field_weight(int i) {
    const int p = (i & 7) < 5 ? (i & 7) : (i & 7) - 5;
    return kTwo24 / (float)(1 << (2 * p));
}

// One column step: the lane's 16 bytes are 64 rows, the first 32 of block 2 seg (xs0), the rest of
// block 2 seg + 1 (xs1).
__device__ __forceinline__ void fma_step2(u32x4 w, float xs0, float xs1, float *acc) {
    fma_codes2(w.x, xs0, acc + 0);
    fma_codes2(w.y, xs0, acc + 16);
    fma_codes2(w.z, xs1, acc + 32);
    fma_codes2(w.w, xs1, acc + 48);
}

template <int WAVES, bool DENSE>
__global__ __launch_bounds__(WAVES * 64) void spqt_cb2_gemv_kernel(
    const uint8_t *__restrict__ packed, const uint16_t *__restrict__ x,
    const int32_t *__restrict__ idx, const int32_t *__restrict__ count, float *__restrict__ y,
    void *partials, int32_t *ws_flags, int K, int NC, int S, int T, int M) {
    __shared__ uint32_t stage_off[WAVES][kPassCols];                                     // byte offset of each column
    __shared__ __attribute__((aligned(16))) float stage_xs[WAVES][kPassCols][kBlocks2];  // x * scale per block
    __shared__ __attribute__((aligned(16))) float red[WAVES][1][kRows2];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int cg = lane >> 3;      // column of the step this lane reads
    const int seg = lane & 7;      // 64-row segment of the block-row this lane reads
    const int cgr = ((cg & 1) << 2) | (cg & 2) | (cg >> 2);
    const uint32_t seg16 = (uint32_t)seg * 16u;
    // all S workgroups of a block-row on one XCD (workgroups go to the 8 XCDs round-robin)
    const int xcd = blockIdx.x & 7;
    const int slot_id = blockIdx.x >> 3;
    const int t = xcd + 8 * (slot_id / S);
    const int s = slot_id % S;
    if (t >= T) return;

    const int n_raw = DENSE ? K : __builtin_amdgcn_readfirstlane(*count);
    const int n_ns = n_raw < 0 ? 0 : (n_raw > K ? K : n_raw);
    const int parts = S * WAVES;
    const int part = s * WAVES + wave;
    int pos = (int)(((int64_t)n_ns * part) / parts);
    const int end = (int)(((int64_t)n_ns * (part + 1)) / parts);

    const uint8_t *row_base = packed + (size_t)t * NC * kChunkBytes2;

    float acc[64];
    float bsum0 = 0.0f, bsum1 = 0.0f;
#pragma unroll
    for (int i = 0; i < 64; ++i) acc[i] = 0.0f;

    if (pos < end) {
        auto fetch_k = [&](int p) -> int {
            const int e = p + lane;
            if (DENSE) return e < end ? e : 0;
            return idx[e < end ? e : end - 1];
        };
        // FETCH stage of the pass at list position p: the next pass's entries, this pass's x, scales
        // and weights.  Lanes past the pass point at its first column and later carry x = 0.
        auto fetch = [&](int kk, int p, u32x4(&w)[8], int &n_out, uint32_t &xraw_out, u32x4(&sv_out)[2], int &k_after) {
            const int left = end - p;
            const int n = left < 0 ? 0 : (left < kPassCols ? left : kPassCols);
            k_after = fetch_k(p + kPassCols);
            const int k_first = n ? __builtin_amdgcn_readfirstlane(kk) : 0;
            const int kc = lane < n ? kk : k_first;
            const uint32_t chunk_off = (uint32_t)(kc >> 7) * (uint32_t)kChunkBytes2;
            const uint32_t col = (uint32_t)(kc & (kGroup - 1));
            xraw_out = x[kc];
            const u32x4 *sp = reinterpret_cast<const u32x4 *>(row_base + (size_t)(chunk_off + col * 32u));
            sv_out[0] = sp[0];
            sv_out[1] = sp[1];
            stage_off[wave][lane] = chunk_off + (uint32_t)kScaleBytes2 + col * 128u;
            __builtin_amdgcn_wave_barrier();
            uint32_t off[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) off[u] = stage_off[wave][u * 8 + cg] + seg16;
#pragma unroll
            for (int u = 0; u < 8; ++u)
                w[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(row_base + (size_t)off[u]));
            n_out = n;
        };
        // MULTIPLY stage: the lane that owns list entry `lane` stages the 16 products x * s_b of
        // its column (0 for a filler entry); every lane then reads the products of its own two blocks.
        auto multiply = [&](int n, uint32_t xraw, const u32x4(&sv)[2], const u32x4(&w)[8]) {
            const float xf = lane < n ? half_bits_to_float(xraw) : 0.0f;
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const u32x4 v = sv[h];
                f32x4 *dst = reinterpret_cast<f32x4 *>(&stage_xs[wave][lane][8 * h]);
                dst[0] = f32x4{xf * half_bits_to_float(v.x & 0xFFFFu), xf * half_bits_to_float(v.x >> 16),
                               xf * half_bits_to_float(v.y & 0xFFFFu), xf * half_bits_to_float(v.y >> 16)};
                dst[1] = f32x4{xf * half_bits_to_float(v.z & 0xFFFFu), xf * half_bits_to_float(v.z >> 16),
                               xf * half_bits_to_float(v.w & 0xFFFFu), xf * half_bits_to_float(v.w >> 16)};
            }
            __builtin_amdgcn_wave_barrier();
            f32x2 xl[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) xl[u] = *reinterpret_cast<const f32x2 *>(&stage_xs[wave][u * 8 + cg][2 * seg]);
            fma_step2(w[0], xl[0].x, xl[0].y, acc);
            bsum0 += xl[0].x;
            bsum1 += xl[0].y;
#pragma unroll
            for (int u = 1; u < 8; ++u)
                if (u * 8 < n) {
                    fma_step2(w[u], xl[u].x, xl[u].y, acc);
                    bsum0 += xl[u].x;
                    bsum1 += xl[u].y;
                }
            __builtin_amdgcn_wave_barrier();
        };

        u32x4 wA[8], wB[8];
        u32x4 svA[2], svB[2];
        uint32_t xrA, xrB;
        int nA, nB, kA, kB;
        kA = fetch_k(pos);
        fetch(kA, pos, wA, nA, xrA, svA, kB);
        if (pos + nA >= end) {
            multiply(nA, xrA, svA, wA);      // the whole slice is one pass
        } else {
            for (;;) {
                const int posB = pos + nA;
                fetch(kB, posB, wB, nB, xrB, svB, kA);
                multiply(nA, xrA, svA, wA);
                if (posB >= end) break;
                const int posA = posB + nB;
                fetch(kA, posA, wA, nA, xrA, svA, kB);
                multiply(nB, xrB, svB, wB);
                if (posA >= end) break;
                pos = posA;
            }
        }
    }

    // accumulator i is row 64 seg + i; each half of them is one block and folds like the 4-bit kernel's 32
    float r0[4], r1[4];
#pragma unroll
    for (int i = 0; i < 64; ++i) acc[i] *= field_weight(i);
    fold_columns(acc + 0, r0);
    fold_columns(acc + 32, r1);
    const float bias0 = sum_over_columns(bsum0) * 1.5f;
    const float bias1 = sum_over_columns(bsum1) * 1.5f;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        red[wave][0][64 * seg + 4 * cgr + j] = r0[j] - bias0;
        red[wave][0][64 * seg + 32 + 4 * cgr + j] = r1[j] - bias1;
    }
    __syncthreads();
    combine_block_row<WAVES, 1, kRows2>(&red[0][0][0], tid, t, s, S, partials, ws_flags, y, M);
}

template <int WAVES>
hipError_t launch2(bool dense, int grid, hipStream_t stream, const uint8_t *packed, const uint16_t *x,
                   const int32_t *idx, const int32_t *count, float *y, void *partials, int32_t *ws_flags, int K,
                   int NC, int S, int T, int m_and_flags) {
    if (dense)
        hipLaunchKernelGGL((spqt_cb2_gemv_kernel<WAVES, true>), dim3(grid), dim3(WAVES * 64), 0, stream, packed, x, idx,
                           count, y, partials, ws_flags, K, NC, S, T, m_and_flags);
    else
        hipLaunchKernelGGL((spqt_cb2_gemv_kernel<WAVES, false>), dim3(grid), dim3(WAVES * 64), 0, stream, packed, x, idx,
                           count, y, partials, ws_flags, K, NC, S, T, m_and_flags);
    return hipGetLastError();
}

}  // namespace

extern "C" int spqt_cb2_gemv(const void *packed_dev, int64_t M, int64_t K, const void *x_dev,
                             const int32_t *idx_dev, const int32_t *count_dev, void *y_dev,
                             void *workspace_dev, size_t workspace_bytes, void *stream,
                             const spqt_launch_cfg *cfg) {
    if (!packed_dev || !x_dev || !y_dev) return SPQT_EINVAL;
    if (idx_dev && !count_dev) return SPQT_EINVAL;
    if (int rc = check_shape(M, K, kGroup)) return rc;
    if (cfg && (cfg->flags & ~SPQT_CFG_Y_FP16)) return SPQT_EINVAL;
    const int y_half = cfg && (cfg->flags & SPQT_CFG_Y_FP16) ? 1 : 0;
    if ((uintptr_t)packed_dev % 128 != 0 || (uintptr_t)x_dev % 2 != 0 || (uintptr_t)y_dev % (y_half ? 2 : 4) != 0)
        return SPQT_EALIGN;
    const int64_t T64 = (M + kRows2 - 1) / kRows2;
    // about one workgroup of 4 wavefronts per CU: the 64 accumulators and two stages of weights leave
    // room for one wavefront per SIMD; S a power of two <= 16
    int S = 1;
    while (S * 2 <= kMaxSplits2 && (int64_t)S * 2 * T64 <= 256) S *= 2;
    while (S > 1 && (int64_t)S * 4 * kPassCols > K) S /= 2;      // at least one full pass per wavefront when dense
    int waves = 4;
    if (cfg) {
        if (cfg->splits) S = cfg->splits;
        if (cfg->waves) waves = cfg->waves;
    }
    if (S < 1 || S > kMaxSplits2) return SPQT_EINVAL;
    if (waves != 1 && waves != 2 && waves != 4 && waves != 8) return SPQT_EINVAL;
    size_t need = 0;
    spqt_workspace_bytes(M, K, 1, &need);
    void *partials = nullptr;
    int32_t *ws_flags = nullptr;
    if (S > 1) {
        if (!workspace_dev) return SPQT_EINVAL;
        if (workspace_bytes < need) return SPQT_ESIZE;
        if ((uintptr_t)workspace_dev % 256 != 0) return SPQT_EALIGN;
        ws_flags = (int32_t *)workspace_dev;
        partials = (void *)((uint8_t *)workspace_dev + counter_bytes(M));
    }
    const int T = (int)T64, NC = (int)(K / kGroup);
    const int grid = 8 * ((T + 7) / 8) * S;
    hipStream_t st = (hipStream_t)stream;
    const uint8_t *pk = (const uint8_t *)packed_dev;
    const uint16_t *xp = (const uint16_t *)x_dev;
    const int m_and_flags = (int)M | (y_half ? kHalfOutputBit : 0);
    hipError_t err;
    switch (waves) {
        case 1: err = launch2<1>(idx_dev == nullptr, grid, st, pk, xp, idx_dev, count_dev, (float *)y_dev, partials, ws_flags, (int)K, NC, S, T, m_and_flags); break;
        case 2: err = launch2<2>(idx_dev == nullptr, grid, st, pk, xp, idx_dev, count_dev, (float *)y_dev, partials, ws_flags, (int)K, NC, S, T, m_and_flags); break;
        case 8: err = launch2<8>(idx_dev == nullptr, grid, st, pk, xp, idx_dev, count_dev, (float *)y_dev, partials, ws_flags, (int)K, NC, S, T, m_and_flags); break;
        default: err = launch2<4>(idx_dev == nullptr, grid, st, pk, xp, idx_dev, count_dev, (float *)y_dev, partials, ws_flags, (int)K, NC, S, T, m_and_flags); break;
    }
    return err == hipSuccess ? SPQT_OK : SPQT_EHIP;
}
