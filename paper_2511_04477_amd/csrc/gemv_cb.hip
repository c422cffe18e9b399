// spqt_cb_gemv: batch-1 GEMV over the column-block variant of the zigzag layout, reading only
// the kept columns.
//
// Paper Section 4.1.2: the quantization groups run along a column (a superblock is 256
// consecutive rows of one column, in blocks of 32), so a skipped activation entry skips whole
// superblocks together with their scales; Section 4.2.2: one superblock row = 256 outputs is
// shared by n1 threadgroups x n2 simdgroups that keep partial sums locally and combine them
// once; Section 4.2.3: the compacted index list is split evenly over them.
//
// Mapping onto gfx950 (wave64), same skeleton as gemv.hip:
//   - lane (cg, seg) = (lane/8, lane%8) of a step reads bytes [16 seg, 16 seg + 16) of column cg
//     of the step: the 32 rows of ONE quantization block.  The block's scale is therefore a
//     per-lane scalar, and it is folded into the activation before the multiply:
//     acc[row] += n * (x * s * 2^24) with the stored code n taken as an fp16 subnormal.
//   - a pass is simply the next (up to) 64 entries of the wavefront's slice of the index list:
//     there is no group structure to respect, no per-group fold, no flush.  The lane that owns
//     entry l loads x and the 8 scales of its column (one 16-byte load) and stages the 8
//     products in LDS; a lane picks up the product of its own (column, block) per step.
//   - the 32 accumulators run through the whole slice; the 8 column-lanes are folded once at
//     the end, and the offset-binary bias (stored = q + 8) is removed there as -8 * (sum of
//     x * s of the lane's block over the slice).
//   - two-stage software pipeline, unpredicated clamped loads, reduction through LDS and the
//     tagged-word workspace exactly as in gemv.hip.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "gemv_common.hpp"
#include "spqt_colblock.h"

namespace {

using namespace spqt;

constexpr int kCbScaleBytes = kGroup * 16;                 // 128 columns x 8 fp16 scales
constexpr int kCbChunkBytes = SPQT_CB_CHUNK_BYTES;
static_assert(kCbChunkBytes == kCbScaleBytes + kGroup * kColBytes, "chunk size");

// FUSED: the kernel applies the sparsity test itself instead of reading an index list (as
// spqt_gemv_fused does for the group layout): a wavefront's slice is a static range of
// 64-column units; lane l tests column 64u + l, a ballot gives the kept set, mbcnt the rank,
// and the kept columns are staged in rank order.
// BATCH activation rows share the (union) index list and ONE pass over the weights; every row has
// its own staged products, accumulators and bias sum.
//
// KQ: the K-quant flavour of the format (Section 4.1.1): the 16 header bytes of a column hold two
// fp16 superblock scales d, dmin and eight 6-bit block scales and minima; a weight is
// (d * sc_b) * q - dmin * m_b with a plain code q in 0..15.  The owner of a list entry decodes the
// header into the 8 effective scales and the 8 effective minima of its column, both times x; the
// multiply is unchanged, and the minima take the place of the offset-binary bias.
template <int WAVES, bool DENSE, bool FUSED, int BATCH, bool KQ = false>
__global__ __launch_bounds__(WAVES * 64) void spqt_cb_gemv_kernel(
    const uint8_t *__restrict__ packed, const uint16_t *__restrict__ x,
    const int32_t *__restrict__ idx, const int32_t *__restrict__ count, float *__restrict__ y,
    void *partials, int32_t *ws_flags, int K, int NC, int S, int T, int M, float thr) {
    // One staging area per wavefront is enough: offsets are written and read back inside a FETCH
    // stage, products inside a MULTIPLY stage, and a wavefront runs its stages one after the other.
    __shared__ uint32_t stage_off[WAVES][kPassCols];                               // byte offset of each column
    __shared__ __attribute__((aligned(16))) float stage_xs[WAVES][BATCH][kPassCols][8];  // x * scale * 2^24 per block
    __shared__ __attribute__((aligned(16))) float stage_xm[KQ ? WAVES : 1][BATCH][KQ ? kPassCols : 1][8];  // x * minimum * 2^24
    __shared__ __attribute__((aligned(16))) float red[WAVES][BATCH][kTileRows];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int cg = lane >> 3;
    const int seg = lane & 7;
    const int cgr = ((cg & 1) << 2) | (cg & 2) | (cg >> 2);
    const uint32_t seg16 = (uint32_t)seg * 16u;
    // all S workgroups of a block-row on one XCD (workgroups go to the 8 XCDs round-robin)
    const int xcd = blockIdx.x & 7;
    const int slot_id = blockIdx.x >> 3;
    const int t = xcd + 8 * (slot_id / S);
    const int s = slot_id % S;
    if (t >= T) return;

    // (a count outside 0..K cannot come from spqt_gather; clamping keeps a corrupt one inside idx)
    const int n_raw = FUSED ? K / kPassCols : (DENSE ? K : __builtin_amdgcn_readfirstlane(*count));
    const int n_ns = n_raw < 0 ? 0 : (n_raw > K ? K : n_raw);
    const int parts = S * WAVES;
    const int part = s * WAVES + wave;
    int pos = (int)(((int64_t)n_ns * part) / parts);
    const int end = (int)(((int64_t)n_ns * (part + 1)) / parts);

    const uint8_t *row_base = packed + (size_t)t * NC * kCbChunkBytes;

    float acc[BATCH][32];   // this lane's 32 rows, summed over its columns of the whole slice
    float bsum[BATCH];      // sum of the staged products this lane multiplied with (its block)
#pragma unroll
    for (int b = 0; b < BATCH; ++b) {
        bsum[b] = 0.0f;
#pragma unroll
        for (int i = 0; i < 32; ++i) acc[b][i] = 0.0f;
    }

    if (pos < end) {
        auto fetch_k = [&](int p) -> int {
            const int e = p + lane;
            if (DENSE) return e < end ? e : 0;
            return idx[e < end ? e : end - 1];
        };

        // FETCH stage of the pass at list position p (kk = its entries): request the next pass's
        // entries, this pass's x, scales and weights.  Lanes past the pass point at its first
        // column and later carry x = 0; past the end of the slice the stage degenerates to n = 0
        // with harmless re-reads.
        auto fetch = [&](int kk, int p, int slot, u32x4(&w)[8], int &n_out, uint32_t(&xraw_out)[BATCH],
                         u32x4 &sv_out, int &k_after) {
            const int left = end - p;
            const int n = left < 0 ? 0 : (left < kPassCols ? left : kPassCols);
            k_after = fetch_k(p + kPassCols);
            const int k_first = n ? __builtin_amdgcn_readfirstlane(kk) : 0;
            const int kc = lane < n ? kk : k_first;
            const uint32_t chunk_off = (uint32_t)(kc >> 7) * (uint32_t)kCbChunkBytes;
            const uint32_t col = (uint32_t)(kc & (kGroup - 1));
#pragma unroll
            for (int b = 0; b < BATCH; ++b) xraw_out[b] = x[(size_t)b * K + kc];
            sv_out = *reinterpret_cast<const u32x4 *>(row_base + (size_t)(chunk_off + col * 16u));
            stage_off[wave][lane] = chunk_off + (uint32_t)kCbScaleBytes + col * (uint32_t)kColBytes;
            __builtin_amdgcn_wave_barrier();
            uint32_t off[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) off[u] = stage_off[wave][u * 8 + cg] + seg16;
#pragma unroll
            for (int u = 0; u < 8; ++u)
                w[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(row_base + (size_t)off[u]));
            n_out = n;
        };

        // MULTIPLY stage of a fetched pass: the lane that owns list entry `ent` stages the 8
        // products x * s_b * 2^24 of its column (xf = x * 2^24, or 0 for a filler entry), per row.
        auto multiply = [&](int n, const float(&xf)[BATCH], int ent, u32x4 sv, int slot, const u32x4(&w)[8]) {
            float sc[8], mn[8];
            if (KQ) {
                const float d = half_bits_to_float(sv.x & 0xFFFFu), dm = half_bits_to_float(sv.x >> 16);
                const uint64_t lo = (uint64_t)sv.y | ((uint64_t)sv.z << 32);
                const uint32_t hi = sv.w;
#pragma unroll
                for (int b = 0; b < 8; ++b) {
                    const int ps = 6 * b, pm = 48 + 6 * b;      // compile-time bit positions
                    const uint32_t fs = (uint32_t)(lo >> ps) & 63u;
                    uint32_t fm;
                    if (pm + 6 <= 64) fm = (uint32_t)(lo >> pm) & 63u;
                    else if (pm >= 64) fm = (hi >> (pm - 64)) & 63u;
                    else fm = ((uint32_t)(lo >> pm) | (hi << (64 - pm))) & 63u;
                    sc[b] = d * (float)fs;
                    mn[b] = dm * (float)fm;
                }
            } else {
                sc[0] = half_bits_to_float(sv.x & 0xFFFFu);
                sc[1] = half_bits_to_float(sv.x >> 16);
                sc[2] = half_bits_to_float(sv.y & 0xFFFFu);
                sc[3] = half_bits_to_float(sv.y >> 16);
                sc[4] = half_bits_to_float(sv.z & 0xFFFFu);
                sc[5] = half_bits_to_float(sv.z >> 16);
                sc[6] = half_bits_to_float(sv.w & 0xFFFFu);
                sc[7] = half_bits_to_float(sv.w >> 16);
            }
#pragma unroll
            for (int b = 0; b < BATCH; ++b) {
                f32x4 *dst = reinterpret_cast<f32x4 *>(stage_xs[wave][b][ent]);
                dst[0] = f32x4{xf[b] * sc[0], xf[b] * sc[1], xf[b] * sc[2], xf[b] * sc[3]};
                dst[1] = f32x4{xf[b] * sc[4], xf[b] * sc[5], xf[b] * sc[6], xf[b] * sc[7]};
                if (KQ) {
                    f32x4 *dm4 = reinterpret_cast<f32x4 *>(stage_xm[wave][b][ent]);
                    dm4[0] = f32x4{xf[b] * mn[0], xf[b] * mn[1], xf[b] * mn[2], xf[b] * mn[3]};
                    dm4[1] = f32x4{xf[b] * mn[4], xf[b] * mn[5], xf[b] * mn[6], xf[b] * mn[7]};
                }
            }
            __builtin_amdgcn_wave_barrier();
            if (BATCH == 1) {
                float xl[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) xl[u] = stage_xs[wave][0][u * 8 + cg][seg];
                float xb[8];     // what step u adds to the bias sum: the product itself, or x * minimum
#pragma unroll
                for (int u = 0; u < 8; ++u) xb[u] = KQ ? stage_xm[wave][0][u * 8 + cg][seg] : xl[u];
                fma_step<false>(w[0], xl[0], acc[0]);
                bsum[0] += xb[0];
#pragma unroll
                for (int u = 1; u < 8; ++u)
                    if (u * 8 < n) {
                        fma_step<false>(w[u], xl[u], acc[0]);
                        bsum[0] += xb[u];
                    }
            } else {
#pragma unroll
                for (int u = 0; u < 8; ++u)
                    if (u == 0 || u * 8 < n) {
#pragma unroll
                        for (int b = 0; b < BATCH; ++b) {
                            const float xl = stage_xs[wave][b][u * 8 + cg][seg];
                            fma_step<false>(w[u], xl, acc[b]);
                            bsum[b] += KQ ? stage_xm[wave][b][u * 8 + cg][seg] : xl;
                        }
                    }
            }
            __builtin_amdgcn_wave_barrier();
        };
        auto multiply_list = [&](int n, const uint32_t(&xraw)[BATCH], u32x4 sv, int slot, const u32x4(&w)[8]) {
            float xf[BATCH];
#pragma unroll
            for (int b = 0; b < BATCH; ++b) xf[b] = lane < n ? half_bits_to_float(xraw[b]) * kTwo24 : 0.0f;
            multiply(n, xf, lane, sv, slot, w);
        };

        u32x4 wA[8], wB[8], svA, svB;
        int nA, nB;
        if (FUSED) {
            // FETCH stage of unit u (xr = this lane's x[64u + lane], requested one stage earlier):
            // threshold, rank, stage the offsets, request the next unit's x, this unit's scales
            // (every lane its own column's) and weights.
            auto fetch_unit = [&](uint32_t xr, int u, int slot, u32x4(&w)[8], int &n_out, float(&xf_out)[BATCH],
                                  int &ent_out, u32x4 &sv_out, uint32_t &xr_next) {
                const bool any = u < end;
                const float xv = half_bits_to_float(xr);
                const bool keep = any && !(__builtin_fabsf(xv) < thr);
                const uint64_t mask = __ballot(keep);
                const int n = __builtin_amdgcn_readfirstlane((int)__popcll(mask));
                const int rank = (int)__builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32),
                                                                __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
                {
                    const int c = (u + 1) * kPassCols + lane;
                    xr_next = x[c < K ? c : K - 1];
                }
                const int uu = any ? u : 0;
                const uint32_t chunk_off = (uint32_t)(uu >> 1) * (uint32_t)kCbChunkBytes;
                const uint32_t col_own = (uint32_t)((uu & 1) * kPassCols + lane);
                const uint32_t col_first = (uint32_t)((uu & 1) * kPassCols + (n ? (int)__builtin_ctzll(mask) : 0));
                sv_out = *reinterpret_cast<const u32x4 *>(row_base + (size_t)(chunk_off + col_own * 16u));
                // kept columns go to entries 0..n-1 in ascending order; the other lanes fill entries
                // n..63 with the unit's first kept column and x = 0
                const int entry = keep ? rank : n + lane - rank;
                stage_off[wave][entry] =
                    chunk_off + (uint32_t)kCbScaleBytes + (keep ? col_own : col_first) * (uint32_t)kColBytes;
                __builtin_amdgcn_wave_barrier();
                uint32_t off[8];
#pragma unroll
                for (int v = 0; v < 8; ++v) off[v] = stage_off[wave][v * 8 + cg] + seg16;
#pragma unroll
                for (int v = 0; v < 8; ++v)
                    w[v] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(row_base + (size_t)off[v]));
                n_out = n;
                xf_out[0] = keep ? xv * kTwo24 : 0.0f;
                ent_out = entry;
            };
            float xfA[BATCH], xfB[BATCH];
            int entA, entB;
            uint32_t xa = x[pos * kPassCols + lane], xb;
            fetch_unit(xa, pos, 0, wA, nA, xfA, entA, svA, xb);
            for (;;) {
                const int uB = pos + 1;
                fetch_unit(xb, uB, 1, wB, nB, xfB, entB, svB, xa);
                if (nA > 0) multiply(nA, xfA, entA, svA, 0, wA);
                if (uB >= end) break;
                const int uA = uB + 1;
                fetch_unit(xa, uA, 0, wA, nA, xfA, entA, svA, xb);
                if (nB > 0) multiply(nB, xfB, entB, svB, 1, wB);
                if (uA >= end) break;
                pos = uA;
            }
        } else {
            uint32_t xrA[BATCH], xrB[BATCH];
            int kA, kB;
            kA = fetch_k(pos);
            fetch(kA, pos, 0, wA, nA, xrA, svA, kB);
            if (pos + nA >= end) {
                multiply_list(nA, xrA, svA, 0, wA);      // the whole slice is one pass
            } else {
                for (;;) {
                    const int posB = pos + nA;
                    fetch(kB, posB, 1, wB, nB, xrB, svB, kA);
                    multiply_list(nA, xrA, svA, 0, wA);
                    if (posB >= end) break;
                    const int posA = posB + nB;
                    fetch(kA, posA, 0, wA, nA, xrA, svA, kB);
                    multiply_list(nB, xrB, svB, 1, wB);
                    if (posA >= end) break;
                    pos = posA;
                }
            }
        }
    }

    // fold the 8 column-lanes once and remove the bias.  The products are already in true units
    // (code * 2^-24 times x * s * 2^24); the staged values the bias sums are still scaled by 2^24.
#pragma unroll
    for (int b = 0; b < BATCH; ++b) {
        float r4[4];
        fold_columns(acc[b], r4);
        const float bias = sum_over_columns(bsum[b]) * ((KQ ? 1.0f : 8.0f) / kTwo24);
        reinterpret_cast<f32x4 *>(red[wave][b])[8 * seg + cgr] =
            f32x4{r4[0] - bias, r4[1] - bias, r4[2] - bias, r4[3] - bias};
    }
    __syncthreads();
    combine_block_row<WAVES, BATCH>(&red[0][0][0], tid, t, s, S, partials, ws_flags, y, M);
}

template <int WAVES, int BATCH>
hipError_t launch_cb_batch(int mode, int grid, hipStream_t stream, const uint8_t *packed, const uint16_t *x,
                           const int32_t *idx, const int32_t *count, float *y, void *partials, int32_t *ws_flags,
                           int K, int NC, int S, int T, int M, int y_half) {
    const dim3 g(grid), b(WAVES * 64);
    if (mode == 3)        // K-quant flavour, index list
        hipLaunchKernelGGL((spqt_cb_gemv_kernel<WAVES, false, false, BATCH, true>), g, b, 0, stream, packed, x, idx, count, y,
                           partials, ws_flags, K, NC, S, T, M | (y_half ? kHalfOutputBit : 0), 0.0f);
    else if (mode == 4)   // K-quant flavour, dense
        hipLaunchKernelGGL((spqt_cb_gemv_kernel<WAVES, true, false, BATCH, true>), g, b, 0, stream, packed, x, idx, count, y,
                           partials, ws_flags, K, NC, S, T, M | (y_half ? kHalfOutputBit : 0), 0.0f);
    else if (mode == 0)   // index list
        hipLaunchKernelGGL((spqt_cb_gemv_kernel<WAVES, false, false, BATCH>), g, b, 0, stream, packed, x, idx, count, y,
                           partials, ws_flags, K, NC, S, T, M | (y_half ? kHalfOutputBit : 0), 0.0f);
    else                  // dense
        hipLaunchKernelGGL((spqt_cb_gemv_kernel<WAVES, true, false, BATCH>), g, b, 0, stream, packed, x, idx, count, y,
                           partials, ws_flags, K, NC, S, T, M | (y_half ? kHalfOutputBit : 0), 0.0f);
    return hipGetLastError();
}

template <int WAVES>
hipError_t launch_cb(int mode, int batch, int grid, hipStream_t stream, const uint8_t *packed, const uint16_t *x,
                     const int32_t *idx, const int32_t *count, float *y, void *partials, int32_t *ws_flags,
                     int K, int NC, int S, int T, int M, float thr, int y_half) {
    if (mode == 5) {      // K-quant flavour, threshold inside the kernel (batch 1)
        hipLaunchKernelGGL((spqt_cb_gemv_kernel<WAVES, false, true, 1, true>), dim3(grid), dim3(WAVES * 64), 0, stream, packed,
                           x, idx, count, y, partials, ws_flags, K, NC, S, T, M | (y_half ? kHalfOutputBit : 0), thr);
        return hipGetLastError();
    }
    if (mode == 2) {      // threshold inside the kernel (batch 1)
        hipLaunchKernelGGL((spqt_cb_gemv_kernel<WAVES, false, true, 1>), dim3(grid), dim3(WAVES * 64), 0, stream, packed,
                           x, idx, count, y, partials, ws_flags, K, NC, S, T, M | (y_half ? kHalfOutputBit : 0), thr);
        return hipGetLastError();
    }
    switch (batch) {
        case 1: return launch_cb_batch<WAVES, 1>(mode, grid, stream, packed, x, idx, count, y, partials, ws_flags, K, NC, S, T, M, y_half);
        case 2: return launch_cb_batch<WAVES, 2>(mode, grid, stream, packed, x, idx, count, y, partials, ws_flags, K, NC, S, T, M, y_half);
        case 3: return launch_cb_batch<WAVES, 3>(mode, grid, stream, packed, x, idx, count, y, partials, ws_flags, K, NC, S, T, M, y_half);
        default: return launch_cb_batch<WAVES, 4>(mode, grid, stream, packed, x, idx, count, y, partials, ws_flags, K, NC, S, T, M, y_half);
    }
}

int run_cb(int mode, int batch, const void *packed_dev, int64_t M, int64_t K, const void *x_dev, const int32_t *idx_dev,
           const int32_t *count_dev, float threshold, void *y_dev, void *workspace_dev, size_t workspace_bytes,
           void *stream, const spqt_launch_cfg *cfg) {
    if (!packed_dev || !x_dev || !y_dev) return SPQT_EINVAL;
    if (int rc = check_shape(M, K, kGroup)) return rc;
    if (batch < 1 || batch > SPQT_MAX_BATCH) return SPQT_ESHAPE;
    if (cfg && (cfg->flags & ~SPQT_CFG_Y_FP16)) return SPQT_EINVAL;
    const int y_half = cfg && (cfg->flags & SPQT_CFG_Y_FP16) ? 1 : 0;
    if ((uintptr_t)packed_dev % 128 != 0 || (uintptr_t)x_dev % 2 != 0 || (uintptr_t)y_dev % (y_half ? 2 : 4) != 0)
        return SPQT_EALIGN;
    spqt_launch_cfg c;
    choose_cfg(M, K, batch, (mode != 1 && mode != 4) ? Kernel::list_groups : Kernel::dense, &c);
    {
        // Measured on MI355X (sweep of S per shape, 50 % and dense): this kernel has no per-group
        // work, so on matrices large enough to be bandwidth-bound (>= 64 MB packed) fewer, longer
        // slices win for the batch-1 list-driven and dense kernels: about 256 workgroups instead of 512 / 1024.
        const int64_t T64 = tiles(M);
        if (mode != 2 && mode != 5 && batch == 1 && (size_t)M * (size_t)K / 2 >= ((size_t)64 << 20))
            while (c.splits > 1 && (int64_t)c.splits * T64 > 256) c.splits /= 2;
    }
    if (cfg) {
        if (cfg->splits) c.splits = cfg->splits;
        if (cfg->waves) c.waves = cfg->waves;
    }
    if (c.splits < 1 || c.splits > SPQT_MAX_SPLITS) return SPQT_EINVAL;
    if (c.waves != 1 && c.waves != 2 && c.waves != 4) return SPQT_EINVAL;
    size_t need = 0;
    spqt_workspace_bytes(M, K, batch, &need);
    void *partials = nullptr;
    int32_t *ws_flags = nullptr;
    if (c.splits > 1) {
        if (!workspace_dev) return SPQT_EINVAL;
        if (workspace_bytes < need) return SPQT_ESIZE;
        if ((uintptr_t)workspace_dev % 256 != 0) return SPQT_EALIGN;
        ws_flags = (int32_t *)workspace_dev;
        partials = (void *)((uint8_t *)workspace_dev + counter_bytes(M));
    }
    const int T = (int)tiles(M), NC = (int)(K / kGroup);
    const int grid = 8 * ((T + 7) / 8) * c.splits;
    hipStream_t st = (hipStream_t)stream;
    const uint8_t *pk = (const uint8_t *)packed_dev;
    const uint16_t *xp = (const uint16_t *)x_dev;
    hipError_t err;
    switch (c.waves) {
        case 1: err = launch_cb<1>(mode, batch, grid, st, pk, xp, idx_dev, count_dev, (float *)y_dev, partials, ws_flags, (int)K, NC, c.splits, T, (int)M, threshold, y_half); break;
        case 2: err = launch_cb<2>(mode, batch, grid, st, pk, xp, idx_dev, count_dev, (float *)y_dev, partials, ws_flags, (int)K, NC, c.splits, T, (int)M, threshold, y_half); break;
        default: err = launch_cb<4>(mode, batch, grid, st, pk, xp, idx_dev, count_dev, (float *)y_dev, partials, ws_flags, (int)K, NC, c.splits, T, (int)M, threshold, y_half); break;
    }
    return err == hipSuccess ? SPQT_OK : SPQT_EHIP;
}

}  // namespace

extern "C" int spqt_cb_gemv(const void *packed_dev, int64_t M, int64_t K, const void *x_dev, int batch,
                            const int32_t *idx_dev, const int32_t *count_dev, void *y_dev,
                            void *workspace_dev, size_t workspace_bytes, void *stream,
                            const spqt_launch_cfg *cfg) {
    if (idx_dev && !count_dev) return SPQT_EINVAL;
    return run_cb(idx_dev ? 0 : 1, batch, packed_dev, M, K, x_dev, idx_dev, count_dev, 0.0f, y_dev, workspace_dev,
                  workspace_bytes, stream, cfg);
}

extern "C" int spqt_cb_gemv_fused(const void *packed_dev, int64_t M, int64_t K, const void *x_dev,
                                  float threshold, void *y_dev, void *workspace_dev, size_t workspace_bytes,
                                  void *stream, const spqt_launch_cfg *cfg) {
    if (threshold != threshold) return SPQT_EINVAL;
    return run_cb(2, 1, packed_dev, M, K, x_dev, nullptr, nullptr, threshold, y_dev, workspace_dev,
                  workspace_bytes, stream, cfg);
}

extern "C" int spqt_cbk_gemv_fused(const void *packed_dev, int64_t M, int64_t K, const void *x_dev,
                                   float threshold, void *y_dev, void *workspace_dev, size_t workspace_bytes,
                                   void *stream, const spqt_launch_cfg *cfg) {
    if (threshold != threshold) return SPQT_EINVAL;
    return run_cb(5, 1, packed_dev, M, K, x_dev, nullptr, nullptr, threshold, y_dev, workspace_dev,
                  workspace_bytes, stream, cfg);
}

extern "C" int spqt_cbk_gemv(const void *packed_dev, int64_t M, int64_t K, const void *x_dev, int batch,
                             const int32_t *idx_dev, const int32_t *count_dev, void *y_dev,
                             void *workspace_dev, size_t workspace_bytes, void *stream,
                             const spqt_launch_cfg *cfg) {
    if (idx_dev && !count_dev) return SPQT_EINVAL;
    return run_cb(idx_dev ? 3 : 4, batch, packed_dev, M, K, x_dev, idx_dev, count_dev, 0.0f, y_dev, workspace_dev,
                  workspace_bytes, stream, cfg);
}
