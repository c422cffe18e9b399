// spqt_gemv: batch-1 GEMV over zigzag-packed group-wise int4 weights that reads only the
// kept columns.
//
// Paper Section 4.2.2 (zigzag kernel): row parallelism is M/256 (one block-row = 256
// outputs), and inside a block-row n1 threadgroups x n2 simdgroups each walk a segment of
// the column blocks, keep partial sums locally, and combine them once at the end instead of
// contending on the output with atomics.  Section 4.2.3 (load balancing): with sparsity the
// segment is not a static column range but an even slice of the compacted index list
// idx[0:n_ns], so every simdgroup gets about n_ns / (n1*n2) kept columns.
//
// This file holds the dense kernel, the kernel for several activation rows and the one-launch mode.
// With an index list and ONE activation row the library launches gemv_list.hip instead, which forms its
// passes differently (only a row of 8 slots must be of one group); this file's list mode for one row
// stays reachable with SPQT_CFG_GROUP_PASSES.
//
// Mapping onto gfx950 (wave64):
//   - grid = T*S workgroups of WAVES wavefronts; workgroup (t, s) works on block-row t, and
//     wavefront j = s*WAVES + w of the S*WAVES that share the block-row takes
//     idx[n_ns*j/(S*WAVES) : n_ns*(j+1)/(S*WAVES)).
//   - a wavefront step is one 16-byte load per lane = 8 kept columns x 128 bytes: lane
//     (cg, seg) = (lane/8, lane%8) reads bytes [16 seg, 16 seg+16) of column cg of the step,
//     i.e. 32 consecutive rows of one column, and keeps 32 fp32 accumulators.
//   - the slice is consumed in passes of up to 64 columns that belong to ONE quantization
//     group (idx is ascending, so a group is a contiguous run of the list).  Lane l of a pass
//     owns list entry pos+l: it computes the column's byte offset and fetches its x, and both
//     are staged in LDS so that every lane can pick up the pair of the column it reads in a
//     step.  The index entries of the next pass are requested before the weights of this one.
//   - int4 -> float costs no conversion instruction: a stored code n in 0..15 masked in
//     place at bit 0..3 (or 4..7) of a 16-bit half IS the fp16 subnormal n*2^-24 (or
//     16n*2^-24).
//   - the multiply-accumulate runs on the matrix cores, used as 4-wide dot-product units rather
//     than for a tiled GEMM: v_mfma_f32_4x4x4_16B_f16 computes, per group of 4 adjacent lanes
//     (which read the same columns), D[m][n] += sum over 4 k of A[m][k] * B[k][n] with n = the
//     lane (its own rows), k = four of the pass's columns, m = the activation row.  B is one
//     row's codes at 4 columns (the subnormals above, two columns per register after one
//     v_perm_b32), A the raw fp16 x of those columns - exact products, fp32 accumulation.  The
//     kernel was bound by VALU issue (8 multiply-adds + 5 unpack instructions per 8 codes and
//     activation row); on the matrix cores 8 codes cost 6 VALU instructions and 2 matrix
//     instructions for ALL activation rows.  With one activation row, x sits in row v of A for
//     the v-th of 4 consecutive rows of W, so the 4 results share one accumulator tuple.
//     (Building with -DSPQT_SINGLE_ROW_ON_MATRIX_CORES=0 gives the plain v_fma_mix_f32 multiply
//     for one activation row: x pre-scaled by 2^24 or 2^20, one instruction per code.)
//   - per pass: the 8 column-lanes are folded with a transposing butterfly (bank-masked DPP
//     adds, then permlane16/32 swaps), leaving each lane 4 rows that are added to the group's
//     running sums.  Folding every pass instead of once per group keeps the 32 accumulators
//     local to the multiply stage (nothing wide is carried around the loop), which is worth
//     more in registers and copies than the ~56 instructions an extra fold costs.
//   - per group: the offset-binary bias (stored = q + 8) is removed as -8 * (sum of the
//     group's kept x), and the fp16 group scale is applied once per (row, group):
//     y_acc += scale * (sum - bias).
//   - WAVES wavefronts are combined through LDS, the S workgroups of a block-row through a
//     workspace of tagged words: the workgroup with the highest index adds the others' partial
//     sums in fixed order and writes y.  No floating-point atomics, so results are reproducible.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <mutex>

#include "rowpass.hpp"

namespace {

using namespace spqt;

#ifndef SPQT_SINGLE_ROW_ON_MATRIX_CORES
#define SPQT_SINGLE_ROW_ON_MATRIX_CORES 1
#endif
constexpr bool kMatrixCoreSingleRow = SPQT_SINGLE_ROW_ON_MATRIX_CORES != 0;

// BATCH activation rows share one pass over the weights: the index list is the union of the
// rows' kept columns, every dequantized code is multiplied by each row's own x, and each row
// has its own accumulators, bias sum and output.
//
// FUSED: the kernel thresholds x itself instead of reading an index list.  The slice of a
// wavefront is then a static range of 64-column units (K/64 units split evenly over the S*WAVES
// wavefronts of the block-row); each unit is one pass: lane l tests column 64u + l, a ballot
// gives the kept set, mbcnt the rank of every kept column, and the (offset, x) pairs are written
// to the staging slot in rank order - the same compacted form the index-list path stages.
// FUSED == 2 is an ablation: same test, same static ranges, but NO compaction - a dropped column
// keeps its slot in the pass with x = 0 (and re-reads a kept column's line), so skipping saves
// memory traffic but not one multiply step.
template <int WAVES, bool DENSE, int BATCH, int FUSED>
__global__ __launch_bounds__(WAVES * 64) void spqt_gemv_kernel(
    const uint8_t *__restrict__ packed, const uint16_t *__restrict__ x,
    const int32_t *__restrict__ idx, const int32_t *__restrict__ count, float *__restrict__ y,
    void *partials, int32_t *ws_flags, int K, int NG, int S, int T, int M, float thr) {
    // Two staging slots per wave (the pass being multiplied and the pass being fetched).
    __shared__ uint32_t stage_off[WAVES][2][kPassCols];      // byte offset of each column of the pass
    __shared__ float stage_x[WAVES][2][BATCH][kPassCols];    // its x per batch row, pre-scaled by 2^24
    __shared__ __attribute__((aligned(16))) float red[WAVES][BATCH][kTileRows];
    // Several activation rows: x as fp16, laid out [column group cg][row b, padded to 4][step u] so that a
    // lane fetches the 8 values of its column group and its matrix-core row with one 16-byte read.
    __shared__ __attribute__((aligned(16))) uint16_t stage_xh[BATCH > 1 ? WAVES : 1][2][8][4][8];
    // One activation row on the matrix cores: x as fp16, [column group cg][step u].
    __shared__ __attribute__((aligned(16))) uint16_t stage_x1[kMatrixCoreSingleRow && BATCH == 1 ? WAVES : 1][2][8][8];

    SPQT_TL_BEGIN();
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int cg = lane >> 3;      // column of the step this lane reads
    const int seg = lane & 7;      // 32-row segment of the tile this lane reads
    const int cgr = ((cg & 1) << 2) | (cg & 2) | (cg >> 2);   // cg with its three bits reversed
    const uint32_t seg16 = (uint32_t)seg * 16u;              // this lane's bytes inside a column run
    const uint32_t sc_off = (uint32_t)(seg * 64 + cgr * 8);  // this lane's 4 scales inside a chunk
    // Workgroups are handed to the 8 XCDs round-robin by index.  Keep all S workgroups of a
    // block-row on ONE XCD (same index mod 8): their partial sums then stay in that XCD's
    // L2 instead of bouncing between dies.  Only a matter of speed, never of correctness.
    const int xcd = blockIdx.x & 7;
    const int slot = blockIdx.x >> 3;          // position among this XCD's workgroups
    const int t = xcd + 8 * (slot / S);        // block-row
    const int s = slot % S;
    if (t >= T) return;

    // Even split of the index list over the S*WAVES wavefronts of this block-row.
    // (a count outside 0..K cannot come from spqt_gather; clamping keeps a corrupt one inside idx)
    const int n_raw = FUSED ? K / kPassCols : (DENSE ? K : __builtin_amdgcn_readfirstlane(*count));
    const int n_ns = n_raw < 0 ? 0 : (n_raw > K ? K : n_raw);
    SPQT_TL(1);
    const int parts = S * WAVES;
    const int part = s * WAVES + wave;
    int pos = (int)(((int64_t)n_ns * part) / parts);
    const int end = (int)(((int64_t)n_ns * (part + 1)) / parts);

    // quantization groups of 128 or 64 columns: NG tells which (K % 128 == 0 either way)
    const int log2g = (NG << 7) == K ? 7 : 6;
    const int chunk_b = kScaleBytes + (kColBytes << log2g);
    const uint8_t *row_base = packed + (size_t)t * NG * chunk_b;
    if (BATCH > 1) {   // rows BATCH..3 of the fp16 staging area are never written: they must read as zero
        reinterpret_cast<u32x4 *>(&stage_xh[wave][0][0][0][0])[lane] = u32x4{0u, 0u, 0u, 0u};
        __builtin_amdgcn_wave_barrier();
    }

    float yacc[BATCH][4];   // rows 32 seg + 4 rev(cg) + j, scaled and summed over groups
#pragma unroll
    for (int b = 0; b < BATCH; ++b)
#pragma unroll
        for (int j = 0; j < 4; ++j) yacc[b][j] = 0.0f;

    if (pos < end) {
        // List entry p + lane, or -1 past the slice.  The load itself is never predicated
        // (the index is clamped): every pass issues the same number of memory operations, so
        // the multiply stage can wait for exactly its own loads while the next pass's fly.
        auto fetch_k = [&](int p) -> int {
            const int e = p + lane;
            if (DENSE) return e < end ? e : -1;
            const int v = idx[e < n_ns ? e : n_ns - 1];
            return e < end ? v : -1;
        };

        float gacc[BATCH][4];           // current group, rows 32 seg + 4 rev(cg) + j, unscaled
        float xsum[BATCH];              // current group: pre-scaled x of the columns this lane staged
#pragma unroll
        for (int b = 0; b < BATCH; ++b) {
            xsum[b] = 0.0f;
#pragma unroll
            for (int j = 0; j < 4; ++j) gacc[b][j] = 0.0f;
        }
        bool fresh = true;              // nothing accumulated for the current group yet

        // FETCH stage of the pass that starts at list position p (kk = fetch_k(p)): delimit the
        // pass (the run of entries that share the group of idx[p], at most 64), request the
        // NEXT pass's entries, this pass's x, its weights (8 steps, always) and its scales.
        // Past the end of the slice (p >= end) it degenerates to n = 0 with harmless re-reads.
        // Everything of the FETCH stage but the weight loads: hands back where they go.
        auto fetch_head = [&](int kk, int p, int slot, const uint8_t *&chunk_out, uint32_t(&off)[8], int &n_out,
                              int &g_out, uint32_t(&xraw_out)[BATCH], u32x2 &sc_out, int &k_after) {
            const bool any = p < end;
            const int g = any ? (__builtin_amdgcn_readfirstlane(kk) >> log2g) : 0;
            const bool in = any && ((kk >> log2g) == g);
            const int n = __builtin_amdgcn_readfirstlane((int)__popcll(__ballot(in)));
            k_after = fetch_k(p + n);
            // Lanes outside the pass point at the pass's first column and later carry x = 0:
            // they re-read a line that is being fetched anyway.
            const uint32_t koff_in = (uint32_t)(kk & ((1 << log2g) - 1)) * kColBytes;
            const uint32_t koff_first = any ? (uint32_t)__builtin_amdgcn_readfirstlane((int)koff_in) : 0u;
#pragma unroll
            for (int b = 0; b < BATCH; ++b) xraw_out[b] = x[(size_t)b * K + (in ? kk : 0)];
            stage_off[wave][slot][lane] = in ? koff_in : koff_first;
            const uint8_t *chunk = row_base + (size_t)g * chunk_b;   // wave-uniform base
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int u = 0; u < 8; ++u) off[u] = stage_off[wave][slot][u * 8 + cg] + seg16;
            sc_out = *reinterpret_cast<const u32x2 *>(chunk + (size_t)sc_off);
            chunk_out = chunk;
            n_out = n;
            g_out = g;
        };
        auto fetch = [&](int kk, int p, int slot, u32x4(&w)[8], int &n_out, int &g_out,
                         uint32_t(&xraw_out)[BATCH], u32x2 &sc_out, int &k_after) {
            const uint8_t *chunk;
            uint32_t off[8];
            fetch_head(kk, p, slot, chunk, off, n_out, g_out, xraw_out, sc_out, k_after);
#pragma unroll
            for (int u = 0; u < 8; ++u)
                w[u] = __builtin_nontemporal_load(
                    reinterpret_cast<const u32x4 *>(chunk + kScaleBytes + (size_t)off[u]));
        };

        // MULTIPLY stage for several activation rows, on the matrix cores.  v_mfma_f32_4x4x4_16B_f16 runs
        // 16 independent 4x4x4 products, one per group of 4 adjacent lanes; those 4 lanes share their
        // column group cg, so for them "k" can be 4 of the pass's steps (4 columns), "n" the lane itself
        // (its own 32 rows, one row per instruction) and "m" the activation row: A = x of row (lane & 3)
        // at the 4 columns (raw fp16 bits, exact), B = this lane's code of one row at the 4 columns as
        // fp16 subnormals (code * 2^-24, or 16 * code * 2^-24 from the upper bits of a byte), D = the
        // 4 activation rows' partial sums for that row of W.  Two such quads of steps make a pass.
        // With chunk_next != nullptr the registers of a quad are refilled with the next pass's
        // weights as soon as the quad has been consumed.
        auto multiply_rows = [&](int n, const uint32_t(&xraw)[BATCH], int slot, u32x4(&w)[8],
                                 const uint8_t *chunk_next, const uint32_t *off_next) {
#pragma unroll
            for (int b = 0; b < BATCH; ++b) {
                if (FUSED) {    // the fused fetch head has already staged x; xraw carries this lane's share of the bias sum
                    xsum[b] += as_float(xraw[b]);
                } else {
                    const uint32_t hb = lane < n ? xraw[b] : 0u;
                    xsum[b] += half_bits_to_float(hb) * kTwo24;
                    stage_xh[wave][slot][lane & 7][b][lane >> 3] = (uint16_t)hb;
                }
            }
            __builtin_amdgcn_wave_barrier();
            const u32x4 xa = *reinterpret_cast<const u32x4 *>(&stage_xh[wave][slot][cg][lane & 3][0]);
            f32x4 accq[32];     // accq[8 d + p][b]: row 8 d + p of the lane's 32, activation row b
#pragma unroll
            for (int quad = 0; quad < 2; ++quad) {
                if (quad == 0 || n > 32) {
                    const f16x4 a = as_f16x4(quad == 0 ? u32x2{xa.x, xa.y} : u32x2{xa.z, xa.w});
#pragma unroll
                    for (int d = 0; d < 4; ++d) {
                        const uint32_t w0 = w[4 * quad + 0][d], w1 = w[4 * quad + 1][d];
                        const uint32_t w2 = w[4 * quad + 2][d], w3 = w[4 * quad + 3][d];
#pragma unroll
                        for (int half = 0; half < 2; ++half) {
                            u32x2 b[4];
                            if (half) code_rows<1>(w0, w1, w2, w3, b);
                            else code_rows<0>(w0, w1, w2, w3, b);
                            const int q = 8 * d + 4 * half;
                            const f32x4 zero = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
                            for (int p = 0; p < 4; ++p)
                                accq[q + p] = __builtin_amdgcn_mfma_f32_4x4x4f16(a, as_f16x4(b[p]), quad ? accq[q + p] : zero, 0, 0, 0);
                        }
                    }
                }
                if (chunk_next) {
#pragma unroll
                    for (int u = 4 * quad; u < 4 * quad + 4; ++u)
                        w[u] = __builtin_nontemporal_load(
                            reinterpret_cast<const u32x4 *>(chunk_next + kScaleBytes + (size_t)off_next[u]));
                }
            }
            // the products are code * 2^-24 * x (16 times that in the odd rows of a byte)
#pragma unroll
            for (int b = 0; b < BATCH; ++b) {
                float col[32], r4[4];
#pragma unroll
                for (int q = 0; q < 32; ++q) col[q] = accq[q][b];
                fold_columns(col, r4);
#pragma unroll
                for (int j = 0; j < 4; ++j) gacc[b][j] = __builtin_fmaf(r4[j], (j & 1) ? kTwo24 * 0.0625f : kTwo24, gacc[b][j]);
            }
            fresh = false;
            __builtin_amdgcn_wave_barrier();
        };

        // MULTIPLY stage for ONE activation row on the matrix cores (row_products in rowpass.hpp: x sits in
        // row v of A for the v-th of four consecutive rows of W, so a lane's 32 rows need 32 registers).
        auto multiply_one = [&](int n, uint32_t xraw, int slot, u32x4(&w)[8]) {
            if (FUSED) {    // the fused fetch stage has already staged x; xraw carries this lane's share
                xsum[0] += as_float(xraw);
            } else {
                const uint32_t hb = lane < n ? xraw : 0u;
                xsum[0] += half_bits_to_float(hb) * kTwo24;
                stage_x1[wave][slot][lane & 7][lane >> 3] = (uint16_t)hb;
            }
            __builtin_amdgcn_wave_barrier();
            const u32x4 xa = *reinterpret_cast<const u32x4 *>(&stage_x1[wave][slot][cg][0]);
            f32x4 accq[8];      // accq[2 d + half][p]: row 8 d + 4 half + p of the lane's 32
            row_products(w, xa, n > 32, f32x4{0.0f, 0.0f, 0.0f, 0.0f}, lane, accq);
            float col[32], r4[4];
#pragma unroll
            for (int q = 0; q < 32; ++q) col[q] = accq[q >> 2][q & 3];
            fold_columns(col, r4);
#pragma unroll
            for (int j = 0; j < 4; ++j) gacc[0][j] = __builtin_fmaf(r4[j], (j & 1) ? kTwo24 * 0.0625f : kTwo24, gacc[0][j]);
            fresh = false;
            __builtin_amdgcn_wave_barrier();
        };

        // MULTIPLY stage of a fetched pass.
        // With chunk_next != nullptr the stage is "rolling": as soon as step u has been consumed, the
        // registers of w[u] receive step u of the NEXT pass (whose FETCH head has already run), so
        // the next pass's weights fly during this pass's arithmetic without a second buffer.
        auto multiply = [&](int n, const uint32_t(&xraw)[BATCH], int slot, u32x4(&w)[8],
                            const uint8_t *chunk_next = nullptr, const uint32_t *off_next = nullptr) {
            if (BATCH > 1) {
                multiply_rows(n, xraw, slot, w, chunk_next, off_next);
                return;
            }
            if (kMatrixCoreSingleRow) {
                multiply_one(n, xraw[0], slot, w);
                return;
            }
            if (FUSED) {    // the fused fetch stage has already staged x; xraw carries this lane's share
                xsum[0] += as_float(xraw[0]);
            } else {
#pragma unroll
                for (int b = 0; b < BATCH; ++b) {
                    const float xs = lane < n ? half_bits_to_float(xraw[b]) * kTwo24 : 0.0f;
                    xsum[b] += xs;
                    stage_x[wave][slot][b][lane] = xs;
                }
            }
            __builtin_amdgcn_wave_barrier();
            // The pass's products live only inside this stage: the first step overwrites the 32
            // accumulators, the others add to them, and the fold at the end leaves 4 sums per lane.
            float acc[BATCH][32];
            {
                float xl[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) xl[u] = stage_x[wave][slot][0][u * 8 + cg];
                fma_step<true>(w[0], xl[0], acc[0]);
#pragma unroll
                for (int u = 1; u < 8; ++u)
                    if (u * 8 < n) fma_step<false>(w[u], xl[u], acc[0]);
            }
#pragma unroll
            for (int b = 0; b < BATCH; ++b) {
                float r4[4];
                fold_columns(acc[b], r4);
#pragma unroll
                for (int j = 0; j < 4; ++j) gacc[b][j] += r4[j];
            }
            fresh = false;
            __builtin_amdgcn_wave_barrier();
        };

        // Fold the finished group (whose scales are `sc`) into yacc.
        auto flush = [&](u32x2 sc) {
            if (FUSED && fresh) return;   // no kept column in this group's share: nothing accumulated
            const uint32_t s01 = sc.x, s23 = sc.y;
            const f16x2 h01 = as_f16x2(s01), h23 = as_f16x2(s23);
#pragma unroll
            for (int b = 0; b < BATCH; ++b) {
                const float bias = wave_sum(xsum[b]) * (-8.0f / kTwo24);
                yacc[b][0] = __builtin_fmaf((float)h01.x, gacc[b][0] + bias, yacc[b][0]);
                yacc[b][1] = __builtin_fmaf((float)h01.y, gacc[b][1] + bias, yacc[b][1]);
                yacc[b][2] = __builtin_fmaf((float)h23.x, gacc[b][2] + bias, yacc[b][2]);
                yacc[b][3] = __builtin_fmaf((float)h23.y, gacc[b][3] + bias, yacc[b][3]);
                xsum[b] = 0.0f;
#pragma unroll
                for (int j = 0; j < 4; ++j) gacc[b][j] = 0.0f;
            }
            fresh = true;
        };

        // Two-stage software pipeline over the passes, buffers A and B alternating.
        u32x4 wA[8], wB[8];
        u32x2 scA, scB;
        uint32_t xrA[BATCH], xrB[BATCH];
        int nA, nB, gA, gB, kA, kB;
        if (FUSED && BATCH > 1) {
            // One launch for several activation rows: a column of the unit is kept if ANY row keeps it;
            // with the own-sets flag every row then contributes only where it keeps the column itself
            // (its x is staged as 0 elsewhere), which is that row's batch-1 result.
            const bool own = (M & kOwnSetsBit) != 0;
            const int upg = log2g - 6;                      // log2 of the 64-column units per group
            // FETCH head of unit u (xr[b] = this lane's x[b][64u + lane], requested one stage earlier):
            // everything of the fetch stage but the weight loads.
            auto fetch_head_unit = [&](const uint32_t(&xr)[BATCH], int u, int slot, const uint8_t *&chunk_out,
                                       uint32_t(&off)[8], int &n_out, int &g_out, uint32_t(&xs_out)[BATCH],
                                       u32x2 &sc_out, uint32_t(&xr_next)[BATCH]) {
                const bool any = u < end;
                const int g = any ? (u >> upg) : 0;
                bool kb[BATCH];
                bool keep = false;
#pragma unroll
                for (int b = 0; b < BATCH; ++b) {
                    kb[b] = any && !(__builtin_fabsf(half_bits_to_float(xr[b])) < thr);
                    keep = keep || kb[b];
                }
                const uint64_t mask = __ballot(keep);
                const int n = __builtin_amdgcn_readfirstlane((int)__popcll(mask));
                const int rank = (int)__builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32),
                                                                __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
                {   // next unit's x (index clamped: the value is unused past the slice)
                    const int c = (u + 1) * kPassCols + lane;
#pragma unroll
                    for (int b = 0; b < BATCH; ++b) xr_next[b] = x[(size_t)b * K + (c < K ? c : K - 1)];
                }
                const int first_lane = n ? (int)__builtin_ctzll(mask) : 0;
                const int uin = u & ((1 << upg) - 1);             // unit inside its group
                const uint32_t koff_first = (uint32_t)((uin * kPassCols + first_lane) * kColBytes);
                const uint32_t koff_own = (uint32_t)((uin * kPassCols + lane) * kColBytes);
                const int entry = keep ? rank : n + lane - rank;
                stage_off[wave][slot][entry] = keep ? koff_own : koff_first;
#pragma unroll
                for (int b = 0; b < BATCH; ++b) {
                    const bool use = keep && (!own || kb[b]);
                    xs_out[b] = as_u32(use ? half_bits_to_float(xr[b]) * kTwo24 : 0.0f);
                    stage_xh[wave][slot][entry & 7][b][entry >> 3] = use ? (uint16_t)xr[b] : (uint16_t)0;
                }
                const uint8_t *chunk = row_base + (size_t)g * chunk_b;   // wave-uniform base
                __builtin_amdgcn_wave_barrier();
#pragma unroll
                for (int v = 0; v < 8; ++v) off[v] = stage_off[wave][slot][v * 8 + cg] + seg16;
                sc_out = *reinterpret_cast<const u32x2 *>(chunk + (size_t)sc_off);
                chunk_out = chunk;
                n_out = n;
                g_out = g;
            };
            uint32_t xc[BATCH], xn[BATCH];
#pragma unroll
            for (int b = 0; b < BATCH; ++b) xc[b] = x[(size_t)b * K + pos * kPassCols + lane];
            {
                const uint8_t *chunk0;
                uint32_t off0[8];
                fetch_head_unit(xc, pos, 0, chunk0, off0, nA, gA, xrA, scA, xn);
#pragma unroll
                for (int v = 0; v < 8; ++v)
                    wA[v] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(chunk0 + kScaleBytes + (size_t)off0[v]));
            }
            int slot = 0, u = pos;
            for (;;) {
                const int uN = u + 1;
                const uint8_t *chunkN;
                uint32_t offN[8], xsN[BATCH], xnn[BATCH];
                u32x2 scN;
                int nN, gN;
                fetch_head_unit(xn, uN, slot ^ 1, chunkN, offN, nN, gN, xsN, scN, xnn);
                multiply(nA, xrA, slot, wA, chunkN, offN);
                if (uN >= end) {
                    flush(scA);
                    break;
                }
                if (gN != gA) flush(scA);
                u = uN;
                nA = nN;
                gA = gN;
                scA = scN;
                slot ^= 1;
#pragma unroll
                for (int b = 0; b < BATCH; ++b) {
                    xrA[b] = xsN[b];
                    xn[b] = xnn[b];
                }
            }
        } else if (FUSED) {
            // FETCH stage of unit u (xr = this lane's x[64u + lane], requested one stage earlier):
            // threshold, rank, stage, request the next unit's x, the weights and the scales.
            auto fetch_unit = [&](uint32_t xr, int u, int slot, u32x4(&w)[8], int &n_out, int &g_out,
                                  u32x2 &sc_out, uint32_t &xr_next, uint32_t &xs_bits) {
                const bool any = u < end;
                const int upg = log2g - 6;                      // log2 of the 64-column units per group
                const int g = any ? (u >> upg) : 0;
                const float xf = half_bits_to_float(xr);
                const bool keep = any && !(__builtin_fabsf(xf) < thr);
                const uint64_t mask = __ballot(keep);
                const int n = __builtin_amdgcn_readfirstlane((int)__popcll(mask));
                const int rank = (int)__builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32),
                                                                __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
                {   // next unit's x (index clamped: the value is unused past the slice)
                    const int c = (u + 1) * kPassCols + lane;
                    xr_next = x[c < K ? c : K - 1];
                }
                // kept columns go to entries 0..n-1 in ascending order; the other lanes fill entries
                // n..63 with the pass's first kept column and x = 0
                const int first_lane = n ? (int)__builtin_ctzll(mask) : 0;
                const int uin = u & ((1 << upg) - 1);             // unit inside its group
                const uint32_t koff_first = (uint32_t)((uin * kPassCols + first_lane) * kColBytes);
                const uint32_t koff_own = (uint32_t)((uin * kPassCols + lane) * kColBytes);
                const int entry = FUSED == 2 ? lane : (keep ? rank : n + lane - rank);
                const float xs = keep ? xf * kTwo24 : 0.0f;
                xs_bits = as_u32(xs);   // added to the group's bias sum when the unit is multiplied
                stage_off[wave][slot][entry] = keep ? koff_own : koff_first;
                if (kMatrixCoreSingleRow) stage_x1[wave][slot][entry & 7][entry >> 3] = keep ? (uint16_t)xr : (uint16_t)0;
                else stage_x[wave][slot][0][entry] = xs;
                const uint8_t *chunk = row_base + (size_t)g * chunk_b;   // wave-uniform base
                __builtin_amdgcn_wave_barrier();
                uint32_t off[8];
#pragma unroll
                for (int v = 0; v < 8; ++v) off[v] = stage_off[wave][slot][v * 8 + cg] + seg16;
#pragma unroll
                for (int v = 0; v < 8; ++v)
                    w[v] = __builtin_nontemporal_load(
                        reinterpret_cast<const u32x4 *>(chunk + kScaleBytes + (size_t)off[v]));
                sc_out = *reinterpret_cast<const u32x2 *>(chunk + (size_t)sc_off);
                n_out = FUSED == 2 ? (n ? kPassCols : 0) : n;
                g_out = g;
            };
            uint32_t xa = x[pos * kPassCols + lane], xb;
            fetch_unit(xa, pos, 0, wA, nA, gA, scA, xb, xrA[0]);
            for (;;) {
                const int uB = pos + 1;
                fetch_unit(xb, uB, 1, wB, nB, gB, scB, xa, xrB[0]);
                if (nA > 0) multiply(nA, xrA, 0, wA);
                if (uB >= end) {
                    flush(scA);
                    break;
                }
                if (gB != gA) flush(scA);
                const int uA = uB + 1;
                fetch_unit(xa, uA, 0, wA, nA, gA, scA, xb, xrA[0]);
                if (nB > 0) multiply(nB, xrB, 1, wB);
                if (uA >= end) {
                    flush(scB);
                    break;
                }
                if (gA != gB) flush(scB);
                pos = uA;
            }
        } else {
        kA = fetch_k(pos);
        SPQT_TL_WAIT(2);
        fetch(kA, pos, 0, wA, nA, gA, xrA, scA, kB);
        SPQT_TL_WAIT(3);
        if (BATCH > 1) {
            // Several activation rows: the accumulators take most of the register file, so there is
            // one weight buffer, refilled step by step while the pass is being multiplied.
            int slot = 0;
            for (;;) {
                const int posN = pos + nA;
                const uint8_t *chunkN;
                uint32_t offN[8], xrN[BATCH];
                u32x2 scN;
                int nN, gN, kC;
                fetch_head(kB, posN, slot ^ 1, chunkN, offN, nN, gN, xrN, scN, kC);
                multiply(nA, xrA, slot, wA, chunkN, offN);
                if (posN >= end) {
                    flush(scA);
                    break;
                }
                if (gN != gA) flush(scA);
                pos = posN;
                nA = nN;
                gA = gN;
                scA = scN;
                kB = kC;
                slot ^= 1;
#pragma unroll
                for (int b = 0; b < BATCH; ++b) xrA[b] = xrN[b];
            }
        } else if (pos + nA >= end) {
            // the whole slice is one pass (small matrices): nothing to overlap with
            multiply(nA, xrA, 0, wA);
            flush(scA);
        } else
        for (;;) {
            const int posB = pos + nA;
            fetch(kB, posB, 1, wB, nB, gB, xrB, scB, kA);
            multiply(nA, xrA, 0, wA);
            if (posB >= end) {
                flush(scA);
                break;
            }
            if (gB != gA) flush(scA);
            const int posA = posB + nB;
            fetch(kA, posA, 0, wA, nA, gA, xrA, scA, kB);
            multiply(nB, xrB, 1, wB);
            if (posA >= end) {
                flush(scB);
                break;
            }
            if (gA != gB) flush(scB);
            pos = posA;
        }
        }
    }

    SPQT_TL(4);
    // ---- combine the WAVES wavefronts through LDS ------------------------------------------
#pragma unroll
    for (int b = 0; b < BATCH; ++b)
        reinterpret_cast<f32x4 *>(red[wave][b])[8 * seg + cgr] = f32x4{yacc[b][0], yacc[b][1], yacc[b][2], yacc[b][3]};
    __syncthreads();
    SPQT_TL(5);
    combine_block_row<WAVES, BATCH>(&red[0][0][0], tid, t, s, S, partials, ws_flags, y, M);
    SPQT_TL_END(WAVES, wave, lane, S > 1 && s == S - 1);
}

SPQT_TL_SETTER(spqt_timeline_set_gemv)


__global__ void spqt_fill_zero_kernel(uint32_t *p, size_t n_words) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n_words) p[i] = 0u;
}

template <int WAVES, int BATCH>
hipError_t launch(bool dense, int grid, hipStream_t stream, const uint8_t *packed, const uint16_t *x,
                  const int32_t *idx, const int32_t *count, float *y, void *partials,
                  int32_t *ws_flags, int K, int NG, int S, int T, int M, int y_half) {
    if (dense)
        hipLaunchKernelGGL((spqt_gemv_kernel<WAVES, true, BATCH, 0>), dim3(grid), dim3(WAVES * 64), 0, stream,
                           packed, x, idx, count, y, partials, ws_flags, K, NG, S, T, M | (y_half ? kHalfOutputBit : 0), 0.0f);
    else
        hipLaunchKernelGGL((spqt_gemv_kernel<WAVES, false, BATCH, 0>), dim3(grid), dim3(WAVES * 64), 0, stream,
                           packed, x, idx, count, y, partials, ws_flags, K, NG, S, T, M | (y_half ? kHalfOutputBit : 0), 0.0f);
    return hipGetLastError();
}

template <int WAVES>
hipError_t launch_fused(bool compact, int grid, hipStream_t stream, const uint8_t *packed, const uint16_t *x,
                        float thr, float *y, void *partials, int32_t *ws_flags, int K, int NG, int S, int T, int M,
                        int y_half) {
    if (compact)
        hipLaunchKernelGGL((spqt_gemv_kernel<WAVES, false, 1, 1>), dim3(grid), dim3(WAVES * 64), 0, stream,
                           packed, x, (const int32_t *)nullptr, (const int32_t *)nullptr, y, partials, ws_flags, K,
                           NG, S, T, M | (y_half ? kHalfOutputBit : 0), thr);
    else
        hipLaunchKernelGGL((spqt_gemv_kernel<WAVES, false, 1, 2>), dim3(grid), dim3(WAVES * 64), 0, stream,
                           packed, x, (const int32_t *)nullptr, (const int32_t *)nullptr, y, partials, ws_flags, K,
                           NG, S, T, M | (y_half ? kHalfOutputBit : 0), thr);
    return hipGetLastError();
}

// One launch for 2..4 activation rows (4 wavefronts per workgroup).
hipError_t launch_fused_rows(int batch, int grid, hipStream_t stream, const uint8_t *packed, const uint16_t *x, float thr,
                             float *y, void *partials, int32_t *ws_flags, int K, int NG, int S, int T, int m_and_flags) {
    const int32_t *none = nullptr;
    switch (batch) {
        case 2: hipLaunchKernelGGL((spqt_gemv_kernel<4, false, 2, 1>), dim3(grid), dim3(256), 0, stream, packed, x, none, none, y, partials, ws_flags, K, NG, S, T, m_and_flags, thr); break;
        case 3: hipLaunchKernelGGL((spqt_gemv_kernel<4, false, 3, 1>), dim3(grid), dim3(256), 0, stream, packed, x, none, none, y, partials, ws_flags, K, NG, S, T, m_and_flags, thr); break;
        default: hipLaunchKernelGGL((spqt_gemv_kernel<4, false, 4, 1>), dim3(grid), dim3(256), 0, stream, packed, x, none, none, y, partials, ws_flags, K, NG, S, T, m_and_flags, thr); break;
    }
    return hipGetLastError();
}

template <int WAVES>
hipError_t launch_batch(int batch, bool dense, int grid, hipStream_t stream, const uint8_t *packed,
                        const uint16_t *x, const int32_t *idx, const int32_t *count, float *y,
                        void *partials, int32_t *ws_flags, int K, int NG, int S, int T, int M, int y_half) {
    switch (batch) {
        case 1: return launch<WAVES, 1>(dense, grid, stream, packed, x, idx, count, y, partials, ws_flags, K, NG, S, T, M, y_half);
        case 2: return launch<WAVES, 2>(dense, grid, stream, packed, x, idx, count, y, partials, ws_flags, K, NG, S, T, M, y_half);
        case 3: return launch<WAVES, 3>(dense, grid, stream, packed, x, idx, count, y, partials, ws_flags, K, NG, S, T, M, y_half);
        default: return launch<WAVES, 4>(dense, grid, stream, packed, x, idx, count, y, partials, ws_flags, K, NG, S, T, M, y_half);
    }
}

}  // namespace

extern "C" int spqt_workspace_bytes(int64_t M, int64_t K, int batch, size_t *out_bytes) {
    if (!out_bytes) return SPQT_EINVAL;
    if (int rc = check_shape(M, K, kGroup)) return rc;
    if (batch < 1 || batch > SPQT_MAX_BATCH) return SPQT_ESHAPE;
    *out_bytes = counter_bytes(M) + (size_t)tiles(M) * kTileRows * SPQT_MAX_SPLITS * 2 * sizeof(float) * (size_t)batch;
    return SPQT_OK;
}

extern "C" int spqt_workspace_init(void *workspace_dev, size_t workspace_bytes, void *stream) {
    if (!workspace_dev || workspace_bytes < 256) return SPQT_EINVAL;
    if ((uintptr_t)workspace_dev % 256 != 0) return SPQT_EALIGN;
    // The poison flag and every exchange word start at zero: clear all of it.
    size_t words = workspace_bytes / 4;
    hipLaunchKernelGGL(spqt_fill_zero_kernel, dim3((unsigned)((words + 255) / 256)), dim3(256), 0,
                       (hipStream_t)stream, (uint32_t *)workspace_dev, words);
    return hipGetLastError() == hipSuccess ? SPQT_OK : SPQT_EHIP;
}

extern "C" int spqt_default_cfg(int64_t M, int64_t K, int batch, int sparse, spqt_launch_cfg *out) {
    if (!out) return SPQT_EINVAL;
    if (int rc = check_shape(M, K, kGroup)) return rc;
    if (batch < 1 || batch > SPQT_MAX_BATCH) return SPQT_ESHAPE;
    choose_cfg(M, K, batch, !sparse ? Kernel::dense : (batch == 1 ? Kernel::list_rows : Kernel::list_groups), out);
    return SPQT_OK;
}

namespace {

// spqt_gemv_ex, and the allocation-free variant: `tight` accepts a workspace that holds just the
// exchange words this launch shape touches instead of the size spqt_workspace_bytes reports.
int gemv_run(const void *packed_dev, int64_t M, int64_t K, int group, const void *x_dev, int batch,
             const int32_t *idx_dev, const int32_t *count_dev, void *y_dev, void *workspace_dev,
             size_t workspace_bytes, void *stream, const spqt_launch_cfg *cfg, bool tight) {
    if (!packed_dev || !x_dev || !y_dev) return SPQT_EINVAL;
    if (idx_dev && !count_dev) return SPQT_EINVAL;
    if (int rc = check_shape(M, K, group)) return rc;
    if (batch < 1 || batch > SPQT_MAX_BATCH) return SPQT_ESHAPE;
    const int y_half = cfg && (cfg->flags & SPQT_CFG_Y_FP16) ? 1 : 0;
    if ((uintptr_t)packed_dev % 128 != 0 || (uintptr_t)x_dev % 2 != 0 || (uintptr_t)y_dev % (y_half ? 2 : 4) != 0)
        return SPQT_EALIGN;

    const bool dense = idx_dev == nullptr;
    // one activation row and an index list: row-aligned passes unless the caller asks for the other kernel
    const bool row_passes = !dense && batch == 1 && !(cfg && (cfg->flags & SPQT_CFG_GROUP_PASSES));
    spqt_launch_cfg c;
    choose_cfg(M, K, batch, dense ? Kernel::dense : (row_passes ? Kernel::list_rows : Kernel::list_groups), &c);
    if (cfg) {
        if (cfg->splits) c.splits = cfg->splits;
        if (cfg->waves) c.waves = cfg->waves;
    }
    if (c.splits < 1 || c.splits > SPQT_MAX_SPLITS) return SPQT_EINVAL;
    // 8 wavefronts per workgroup (two per SIMD) exist for the index-list kernel with one activation row only
    if (c.waves != 1 && c.waves != 2 && c.waves != 4 && !(c.waves == 8 && row_passes)) return SPQT_EINVAL;

    size_t need = 0;
    spqt_workspace_bytes(M, K, batch, &need);
    if (tight) need = exchange_bytes(tiles(M), kTileRows, c.splits, batch);
    void *partials = nullptr;
    int32_t *ws_flags = nullptr;
    if (c.splits > 1) {
        if (!workspace_dev) return SPQT_EINVAL;
        if (workspace_bytes < need) return SPQT_ESIZE;
        if ((uintptr_t)workspace_dev % 256 != 0) return SPQT_EALIGN;
        ws_flags = (int32_t *)workspace_dev;
        partials = (void *)((uint8_t *)workspace_dev + counter_bytes(M));
    }

    const int T = (int)tiles(M), NG = (int)(K / group);
    const int grid = 8 * ((T + 7) / 8) * c.splits;
    hipStream_t st = (hipStream_t)stream;
    hipError_t err;
    const uint8_t *pk = (const uint8_t *)packed_dev;
    const uint16_t *xp = (const uint16_t *)x_dev;
    if (row_passes) {
        err = launch_gemv_list(c.waves, grid, st, pk, xp, idx_dev, count_dev, (float *)y_dev, partials, ws_flags, (int)K, NG,
                               c.splits, T, (int)M | (y_half ? kHalfOutputBit : 0));
        return err == hipSuccess ? SPQT_OK : SPQT_EHIP;
    }
    switch (c.waves) {
        case 1: err = launch_batch<1>(batch, dense, grid, st, pk, xp, idx_dev, count_dev, (float *)y_dev, partials, ws_flags, (int)K, NG, c.splits, T, (int)M, y_half); break;
        case 2: err = launch_batch<2>(batch, dense, grid, st, pk, xp, idx_dev, count_dev, (float *)y_dev, partials, ws_flags, (int)K, NG, c.splits, T, (int)M, y_half); break;
        default: err = launch_batch<4>(batch, dense, grid, st, pk, xp, idx_dev, count_dev, (float *)y_dev, partials, ws_flags, (int)K, NG, c.splits, T, (int)M, y_half); break;
    }
    if (err != hipSuccess) return SPQT_EHIP;
    return SPQT_OK;
}

// Exchange words for callers that cannot bring a workspace: one array per GPU, in the library's own
// image, zero when the image is loaded and put back to zero by every call that used it.
constexpr size_t kStaticScratchBytes = SPQT_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
constexpr int kMaxDevices = 64;
std::mutex scratch_mutex;
void *scratch_of_device[kMaxDevices];   // this process's address of `scratch` on each GPU, once known

// The array's name is only a host-side handle: its device address comes from the runtime, per GPU.
int static_scratch(void **out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return SPQT_EHIP;
    std::lock_guard<std::mutex> lock(scratch_mutex);
    if (!scratch_of_device[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return SPQT_EHIP;
        scratch_of_device[dev] = p;
    }
    *out = scratch_of_device[dev];
    return SPQT_OK;
}

}  // namespace

extern "C" int spqt_gemv_ex(const void *packed_dev, int64_t M, int64_t K, int group, const void *x_dev,
                            int batch, const int32_t *idx_dev, const int32_t *count_dev, void *y_dev,
                            void *workspace_dev, size_t workspace_bytes, void *stream,
                            const spqt_launch_cfg *cfg) {
    return gemv_run(packed_dev, M, K, group, x_dev, batch, idx_dev, count_dev, y_dev, workspace_dev,
                    workspace_bytes, stream, cfg, false);
}

extern "C" int spqt_gemv_static(const void *packed_dev, int64_t M, int64_t K, int group, const void *x_dev,
                                int batch, const int32_t *idx_dev, const int32_t *count_dev, float *y_dev,
                                void *stream) {
    // Shape errors first, so that a bad call never touches the runtime.
    if (int rc = check_shape(M, K, group)) return rc;
    if (batch < 1 || batch > SPQT_MAX_BATCH) return SPQT_ESHAPE;
    spqt_launch_cfg c;
    const bool dense = idx_dev == nullptr;
    choose_cfg(M, K, batch, dense ? Kernel::dense : (batch == 1 ? Kernel::list_rows : Kernel::list_groups), &c);
    if (c.splits > 1 && exchange_bytes(tiles(M), kTileRows, c.splits, batch) > kStaticScratchBytes) return SPQT_ESIZE;
    void *ws = nullptr;
    if (int rc = static_scratch(&ws)) return rc;
    return gemv_run(packed_dev, M, K, group, x_dev, batch, idx_dev, count_dev, y_dev, ws, kStaticScratchBytes,
                    stream, nullptr, true);
}

extern "C" int spqt_gemv_fused(const void *packed_dev, int64_t M, int64_t K, int group, const void *x_dev,
                               float threshold, void *y_dev, void *workspace_dev, size_t workspace_bytes,
                               void *stream, const spqt_launch_cfg *cfg) {
    if (!packed_dev || !x_dev || !y_dev) return SPQT_EINVAL;
    if (threshold != threshold) return SPQT_EINVAL;
    if (int rc = check_shape(M, K, group)) return rc;
    const int y_half = cfg && (cfg->flags & SPQT_CFG_Y_FP16) ? 1 : 0;
    if ((uintptr_t)packed_dev % 128 != 0 || (uintptr_t)x_dev % 2 != 0 || (uintptr_t)y_dev % (y_half ? 2 : 4) != 0)
        return SPQT_EALIGN;
    // Static column ranges by default; even shares of the kept columns (gemv_bal.hip) when the caller asks
    // for them - that kernel reads x 16 bytes at a time and holds all of it in LDS (64 KB).
    const bool even_shares = cfg && (cfg->flags & SPQT_CFG_EVEN_SHARES);
    if (even_shares && ((cfg->flags & SPQT_CFG_NO_COMPACTION) || K > 32768 || (uintptr_t)x_dev % 16 != 0)) return SPQT_EINVAL;
    const bool static_ranges = !even_shares;
    spqt_launch_cfg c;
    choose_cfg(M, K, 1, static_ranges ? Kernel::fused : Kernel::list_rows, &c);
    if (cfg) {
        if (cfg->splits) c.splits = cfg->splits;
        if (cfg->waves) c.waves = cfg->waves;
    }
    if (c.splits < 1 || c.splits > SPQT_MAX_SPLITS) return SPQT_EINVAL;
    if (c.waves != 1 && c.waves != 2 && c.waves != 4) return SPQT_EINVAL;
    size_t need = 0;
    spqt_workspace_bytes(M, K, 1, &need);
    void *partials = nullptr;
    int32_t *ws_flags = nullptr;
    if (c.splits > 1) {
        if (!workspace_dev) return SPQT_EINVAL;
        if (workspace_bytes < need) return SPQT_ESIZE;
        if ((uintptr_t)workspace_dev % 256 != 0) return SPQT_EALIGN;
        ws_flags = (int32_t *)workspace_dev;
        partials = (void *)((uint8_t *)workspace_dev + counter_bytes(M));
    }
    const int T = (int)tiles(M), NG = (int)(K / group);
    const int grid = 8 * ((T + 7) / 8) * c.splits;
    const bool compact = !(cfg && (cfg->flags & SPQT_CFG_NO_COMPACTION));
    hipStream_t st = (hipStream_t)stream;
    const uint8_t *pk = (const uint8_t *)packed_dev;
    const uint16_t *xp = (const uint16_t *)x_dev;
    hipError_t err;
    if (!static_ranges) {
        err = launch_gemv_bal(c.waves, grid, st, pk, xp, threshold, (float *)y_dev, partials, ws_flags, (int)K, NG,
                              c.splits, T, (int)M | (y_half ? kHalfOutputBit : 0));
        return err == hipSuccess ? SPQT_OK : SPQT_EHIP;
    }
    switch (c.waves) {
        case 1: err = launch_fused<1>(compact, grid, st, pk, xp, threshold, (float *)y_dev, partials, ws_flags, (int)K, NG, c.splits, T, (int)M, y_half); break;
        case 2: err = launch_fused<2>(compact, grid, st, pk, xp, threshold, (float *)y_dev, partials, ws_flags, (int)K, NG, c.splits, T, (int)M, y_half); break;
        default: err = launch_fused<4>(compact, grid, st, pk, xp, threshold, (float *)y_dev, partials, ws_flags, (int)K, NG, c.splits, T, (int)M, y_half); break;
    }
    return err == hipSuccess ? SPQT_OK : SPQT_EHIP;
}

extern "C" int spqt_gemv_fused_rows(const void *packed_dev, int64_t M, int64_t K, int group, const void *x_dev, int batch,
                                    float threshold, int own_sets, void *y_dev, void *workspace_dev,
                                    size_t workspace_bytes, void *stream, const spqt_launch_cfg *cfg) {
    if (batch == 1) return spqt_gemv_fused(packed_dev, M, K, group, x_dev, threshold, y_dev, workspace_dev, workspace_bytes, stream, cfg);
    if (!packed_dev || !x_dev || !y_dev) return SPQT_EINVAL;
    if (threshold != threshold) return SPQT_EINVAL;
    if (int rc = check_shape(M, K, group)) return rc;
    if (batch < 1 || batch > SPQT_MAX_BATCH) return SPQT_ESHAPE;
    if (cfg && (cfg->flags & ~SPQT_CFG_Y_FP16)) return SPQT_EINVAL;
    const int y_half = cfg && (cfg->flags & SPQT_CFG_Y_FP16) ? 1 : 0;
    if ((uintptr_t)packed_dev % 128 != 0 || (uintptr_t)x_dev % 2 != 0 || (uintptr_t)y_dev % (y_half ? 2 : 4) != 0)
        return SPQT_EALIGN;
    spqt_launch_cfg c;
    choose_cfg(M, K, batch, Kernel::fused, &c);
    if (cfg) {
        if (cfg->splits) c.splits = cfg->splits;
        if (cfg->waves && cfg->waves != 4) return SPQT_EINVAL;   // this kernel is built for 4 wavefronts per workgroup
    }
    if (c.splits < 1 || c.splits > SPQT_MAX_SPLITS) return SPQT_EINVAL;
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
    const int T = (int)tiles(M), NG = (int)(K / group);
    const int grid = 8 * ((T + 7) / 8) * c.splits;
    const int mf = (int)M | (y_half ? kHalfOutputBit : 0) | (own_sets ? kOwnSetsBit : 0);
    hipError_t err = launch_fused_rows(batch, grid, (hipStream_t)stream, (const uint8_t *)packed_dev, (const uint16_t *)x_dev,
                                       threshold, (float *)y_dev, partials, ws_flags, (int)K, NG, c.splits, T, mf);
    return err == hipSuccess ? SPQT_OK : SPQT_EHIP;
}

extern "C" int spqt_gemv(const void *packed_dev, int64_t M, int64_t K, int group, const void *x_dev,
                         int batch, const int32_t *idx_dev, const int32_t *count_dev, float *y_dev,
                         void *workspace_dev, size_t workspace_bytes, void *stream) {
    return spqt_gemv_ex(packed_dev, M, K, group, x_dev, batch, idx_dev, count_dev, y_dev, workspace_dev,
                        workspace_bytes, stream, nullptr);
}
