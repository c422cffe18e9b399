// spqt_cb8_gemv: the column-block GEMV for 8-bit codes ("ZZ-CB32-W8", spqt_colblock.h).
//
// Paper Section 4.1.3 states that the column-wise layout carries over to other bit-widths.  What
// the 4-bit kernels are built around is kept: one activation column's weights of a block-row are
// ONE 128-byte run, read by 8 lanes with one 16-byte load each, 8 columns per wavefront load, 64
// list entries per pass.  With 8-bit codes that run is 128 rows, so a block-row is 128 rows high,
// a lane owns 16 rows (half a 32-row block) and keeps 16 accumulators.  Everything else follows
// spqt_cb_gemv_kernel: even split of the index list over the S x WAVES wavefronts of a block-row
// (Section 4.2.3), the scale folded into x by the lane that owns the list entry, two-stage
// software pipeline with unpredicated clamped loads, one fold of the 8 column-lanes at the end,
// reduction through LDS and the tagged-word exchange.  Batch 1; list-driven or dense.
//
// Codes become floats without a conversion instruction: v_perm_b32 puts byte b under the fp16
// exponent 0x64 (value 1024 + b, exact), two codes per permute, and v_fma_mix_f32 multiplies a
// half of that pair by the staged x * s in fp32.  The stored byte is q + 128, so every product
// carries (q + 1152) * xs; the lane sums the xs it used and 1152 times that sum comes off at the end.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "gemv_common.hpp"
#include "spqt_colblock.h"

namespace {

using namespace spqt;

constexpr int kRows8 = SPQT_CB8_TILE_ROWS;                 // 128 rows per block-row
constexpr int kScaleBytes8 = kGroup * 8;                   // 128 columns x 4 fp16 scales
constexpr int kChunkBytes8 = SPQT_CB8_CHUNK_BYTES;
static_assert(kChunkBytes8 == kScaleBytes8 + kGroup * 128, "chunk size");
constexpr float kCodeBias = 1024.0f + 128.0f;

// Four codes of one dword (rows 4d .. 4d+3 of the lane's 16): acc[i] += (1024 + byte_i) * xs.
__device__ __forceinline__ void fma_bytes(uint32_t w, float xs, float *acc) {
    const f16x2 p01 = as_f16x2(__builtin_amdgcn_perm(0x64646464u, w, 0x04010400u));   // {b0, 0x64, b1, 0x64}
    const f16x2 p23 = as_f16x2(__builtin_amdgcn_perm(0x64646464u, w, 0x04030402u));   // {b2, 0x64, b3, 0x64}
    acc[0] = __builtin_fmaf((float)p01.x, xs, acc[0]);
    acc[1] = __builtin_fmaf((float)p01.y, xs, acc[1]);
    acc[2] = __builtin_fmaf((float)p23.x, xs, acc[2]);
    acc[3] = __builtin_fmaf((float)p23.y, xs, acc[3]);
}

__device__ __forceinline__ void fma_step8(u32x4 w, float xs, float *acc) {
    fma_bytes(w.x, xs, acc + 0);
    fma_bytes(w.y, xs, acc + 4);
    fma_bytes(w.z, xs, acc + 8);
    fma_bytes(w.w, xs, acc + 12);
}

// One (a, b) pair of the first fold level (lanes l and l ^ 8, see fold8_x8): returns the register
// that holds a's pair sum in lanes with bit 3 clear and b's in lanes with bit 3 set.
__device__ __forceinline__ float fold8(float a, float b) {
    asm volatile("s_nop 1\n\t" SPQT_FOLD8("%0", "%1") : "+v"(b) : "v"(a));
    return b;
}

// Fold the 16 accumulators of the 8 lanes that read the same rows, halving the live values at
// each level: lane (cg, seg) ends with the complete sums of rows 16 seg + 2 rev(cg) + j, j = 0, 1
// (rev reverses the three bits of cg).  Once per kernel, so no batched asm blocks here.
__device__ __forceinline__ void fold_columns16(const float *acc, float *out2) {
    float v[8], u[4];
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] = fold8(acc[i], acc[i + 8]);
#pragma unroll
    for (int i = 0; i < 4; ++i) u[i] = fold16(v[i], v[i + 4]);
#pragma unroll
    for (int i = 0; i < 2; ++i) out2[i] = fold32(u[i], u[i + 2]);
}

template <int WAVES, bool DENSE>
__global__ __launch_bounds__(WAVES * 64) void spqt_cb8_gemv_kernel(
    const uint8_t *__restrict__ packed, const uint16_t *__restrict__ x,
    const int32_t *__restrict__ idx, const int32_t *__restrict__ count, float *__restrict__ y,
    void *partials, int32_t *ws_flags, int K, int NC, int S, int T, int M) {
    __shared__ uint32_t stage_off[WAVES][kPassCols];                          // byte offset of each column
    __shared__ __attribute__((aligned(16))) float stage_xs[WAVES][kPassCols][4];   // x * scale per block
    __shared__ __attribute__((aligned(16))) float red[WAVES][1][kRows8];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int cg = lane >> 3;      // column of the step this lane reads
    const int seg = lane & 7;      // 16-row segment of the block-row this lane reads
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

    const uint8_t *row_base = packed + (size_t)t * NC * kChunkBytes8;

    float acc[16];
    float bsum = 0.0f;
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[i] = 0.0f;

    if (pos < end) {
        auto fetch_k = [&](int p) -> int {
            const int e = p + lane;
            if (DENSE) return e < end ? e : 0;
            return idx[e < end ? e : end - 1];
        };
        // FETCH stage of the pass at list position p: the next pass's entries, this pass's x, scales
        // and weights.  Lanes past the pass point at its first column and later carry x = 0.
        auto fetch = [&](int kk, int p, u32x4(&w)[8], int &n_out, uint32_t &xraw_out, u32x2 &sv_out, int &k_after) {
            const int left = end - p;
            const int n = left < 0 ? 0 : (left < kPassCols ? left : kPassCols);
            k_after = fetch_k(p + kPassCols);
            const int k_first = n ? __builtin_amdgcn_readfirstlane(kk) : 0;
            const int kc = lane < n ? kk : k_first;
            const uint32_t chunk_off = (uint32_t)(kc >> 7) * (uint32_t)kChunkBytes8;
            const uint32_t col = (uint32_t)(kc & (kGroup - 1));
            xraw_out = x[kc];
            sv_out = *reinterpret_cast<const u32x2 *>(row_base + (size_t)(chunk_off + col * 8u));
            stage_off[wave][lane] = chunk_off + (uint32_t)kScaleBytes8 + col * 128u;
            __builtin_amdgcn_wave_barrier();
            uint32_t off[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) off[u] = stage_off[wave][u * 8 + cg] + seg16;
#pragma unroll
            for (int u = 0; u < 8; ++u)
                w[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(row_base + (size_t)off[u]));
            n_out = n;
        };
        // MULTIPLY stage: the lane that owns list entry `lane` stages the 4 products x * s_b of its
        // column (0 for a filler entry); every lane then reads the product of its own block.
        auto multiply = [&](int n, uint32_t xraw, u32x2 sv, const u32x4(&w)[8]) {
            const float xf = lane < n ? half_bits_to_float(xraw) : 0.0f;
            *reinterpret_cast<f32x4 *>(stage_xs[wave][lane]) =
                f32x4{xf * half_bits_to_float(sv.x & 0xFFFFu), xf * half_bits_to_float(sv.x >> 16),
                      xf * half_bits_to_float(sv.y & 0xFFFFu), xf * half_bits_to_float(sv.y >> 16)};
            __builtin_amdgcn_wave_barrier();
            float xl[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) xl[u] = stage_xs[wave][u * 8 + cg][seg >> 1];
            fma_step8(w[0], xl[0], acc);
            bsum += xl[0];
#pragma unroll
            for (int u = 1; u < 8; ++u)
                if (u * 8 < n) {
                    fma_step8(w[u], xl[u], acc);
                    bsum += xl[u];
                }
            __builtin_amdgcn_wave_barrier();
        };

        u32x4 wA[8], wB[8];
        u32x2 svA, svB;
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

    float r2[2];
    fold_columns16(acc, r2);
    const float bias = sum_over_columns(bsum) * kCodeBias;
    red[wave][0][16 * seg + 2 * cgr + 0] = r2[0] - bias;
    red[wave][0][16 * seg + 2 * cgr + 1] = r2[1] - bias;
    __syncthreads();
    combine_block_row<WAVES, 1, kRows8>(&red[0][0][0], tid, t, s, S, partials, ws_flags, y, M);
}

template <int WAVES>
hipError_t launch8(bool dense, int grid, hipStream_t stream, const uint8_t *packed, const uint16_t *x,
                   const int32_t *idx, const int32_t *count, float *y, void *partials, int32_t *ws_flags, int K,
                   int NC, int S, int T, int m_and_flags) {
    if (dense)
        hipLaunchKernelGGL((spqt_cb8_gemv_kernel<WAVES, true>), dim3(grid), dim3(WAVES * 64), 0, stream, packed, x, idx,
                           count, y, partials, ws_flags, K, NC, S, T, m_and_flags);
    else
        hipLaunchKernelGGL((spqt_cb8_gemv_kernel<WAVES, false>), dim3(grid), dim3(WAVES * 64), 0, stream, packed, x, idx,
                           count, y, partials, ws_flags, K, NC, S, T, m_and_flags);
    return hipGetLastError();
}

}  // namespace

extern "C" int spqt_cb8_gemv(const void *packed_dev, int64_t M, int64_t K, const void *x_dev,
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
    const int64_t T64 = (M + kRows8 - 1) / kRows8;
    // same targets as the 4-bit column-block kernel: about 512 (list) / 1024 (dense) workgroups of
    // 4 wavefronts, 256 on matrices large enough to be bandwidth-bound; S a power of two <= 16
    const bool big = (size_t)M * (size_t)K >= ((size_t)64 << 20);
    const int64_t target = big ? 256 : (idx_dev ? 512 : 1024);
    int S = 1;
    while (S * 2 <= 16 && (int64_t)S * 2 * T64 <= target) S *= 2;
    int waves = 4;
    if (cfg) {
        if (cfg->splits) S = cfg->splits;
        if (cfg->waves) waves = cfg->waves;
    }
    if (S < 1 || S > SPQT_MAX_SPLITS) return SPQT_EINVAL;
    if (waves != 1 && waves != 2 && waves != 4) return SPQT_EINVAL;
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
        case 1: err = launch8<1>(idx_dev == nullptr, grid, st, pk, xp, idx_dev, count_dev, (float *)y_dev, partials, ws_flags, (int)K, NC, S, T, m_and_flags); break;
        case 2: err = launch8<2>(idx_dev == nullptr, grid, st, pk, xp, idx_dev, count_dev, (float *)y_dev, partials, ws_flags, (int)K, NC, S, T, m_and_flags); break;
        default: err = launch8<4>(idx_dev == nullptr, grid, st, pk, xp, idx_dev, count_dev, (float *)y_dev, partials, ws_flags, (int)K, NC, S, T, m_and_flags); break;
    }
    return err == hipSuccess ? SPQT_OK : SPQT_EHIP;
}
