// The column-block GEMV for bit-widths other than 4 (gemv_cb8.hip, gemv_cb2.hip): one kernel body, the
// width-specific parts supplied by a format type F.
//
// Paper Section 4.1.3 states that the column-wise layout carries over to other bit-widths.  What the
// 4-bit kernels are built around is kept at every width: one activation column's weights of a block-row
// are ONE 128-byte run, read by 8 lanes with one 16-byte load each, 8 columns per wavefront load, 64
// list entries per pass; the height of a block-row follows from the width (128 bytes of codes).
// Everything else follows spqt_cb_gemv_kernel: even split of the index list over the S x WAVES
// wavefronts of a block-row (Section 4.2.3), the scales folded into x by the lane that owns the list
// entry, two-stage software pipeline with unpredicated clamped loads, one fold of the 8 column-lanes at
// the end, reduction through LDS and the tagged-word exchange.  Three modes: list-driven, dense (every
// column, no list), and ONE-LAUNCH (FUSED, one activation row): the kernel applies the sparsity test of
// Section 2 itself on static 64-column units - lane l tests column 64 u + l, a ballot gives the kept set,
// mbcnt the rank, and the kept columns are staged in rank order - so no index list exists.
// BATCH activation rows (Section 3.3: small beams) share the union index list and ONE pass over the
// weights; every row has its own staged products, accumulators and offset sums.
//
// A format type F provides
//   kRows, kBlocks            rows of a block-row, 32-row blocks in it (one fp16 scale each per column)
//   kScaleBytes, kChunkBytes  scale bytes per 128-column chunk (2 * kBlocks per column), chunk size
//   kAcc                      accumulators per lane (rows per lane = kRows / 8)
//   Scales                    the raw scale bytes of one column, as loaded (load_scales)
//   stage(xf, sv, dst)        dst[b] = xf * scale_b for the kBlocks blocks, by the lane that owns the entry
//   Mine                      the staged products of the block(s) a lane's rows lie in (read_mine)
//   step(w, mine, acc, bs)    one column: acc += code-fields * mine, bs += mine
//   finish(acc, bs, seg, cgr, red)   fold the 8 column-lanes, undo field weights and code offset, rows to red
#ifndef SPQT_COLBLOCK_WIDTH_HPP
#define SPQT_COLBLOCK_WIDTH_HPP

#include "gemv_common.hpp"

namespace spqt {

template <class F, int WAVES, bool DENSE, bool FUSED, int BATCH = 1>
__device__ __forceinline__ void colblock_width_gemv(const uint8_t *__restrict__ packed, const uint16_t *__restrict__ x,
                                                    const int32_t *__restrict__ idx, const int32_t *__restrict__ count,
                                                    float *__restrict__ y, void *partials, int32_t *ws_flags, int K, int NC,
                                                    int S, int T, int M, float thr) {
    __shared__ uint32_t stage_off[WAVES][kPassCols];                                          // byte offset of each column
    static_assert(!FUSED || BATCH == 1, "the one-launch mode takes one activation row");
    __shared__ __attribute__((aligned(16))) float stage_xs[WAVES][BATCH][kPassCols][F::kBlocks];   // x * scale per block
    __shared__ __attribute__((aligned(16))) float red[WAVES][BATCH][F::kRows];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int cg = lane >> 3;      // column of the step this lane reads
    const int seg = lane & 7;      // eighth of the block-row this lane reads
    const int cgr = ((cg & 1) << 2) | (cg & 2) | (cg >> 2);
    const uint32_t seg16 = (uint32_t)seg * 16u;
    // all S workgroups of a block-row on one XCD (workgroups go to the 8 XCDs round-robin)
    const int xcd = blockIdx.x & 7;
    const int slot_id = blockIdx.x >> 3;
    const int t = xcd + 8 * (slot_id / S);
    const int s = slot_id % S;
    if (t >= T) return;

    // what is split evenly: the kept-column list, all columns, or (one launch) the 64-column units
    const int n_raw = FUSED ? K / kPassCols : (DENSE ? K : __builtin_amdgcn_readfirstlane(*count));
    const int n_ns = n_raw < 0 ? 0 : (n_raw > K ? K : n_raw);
    const int parts = S * WAVES;
    const int part = s * WAVES + wave;
    int pos = (int)(((int64_t)n_ns * part) / parts);
    const int end = (int)(((int64_t)n_ns * (part + 1)) / parts);

    const uint8_t *row_base = packed + (size_t)t * NC * F::kChunkBytes;

    float acc[BATCH][F::kAcc];
    typename F::Sums bs[BATCH];
#pragma unroll
    for (int b = 0; b < BATCH; ++b) {
        bs[b] = F::zero_sums();
#pragma unroll
        for (int i = 0; i < F::kAcc; ++i) acc[b][i] = 0.0f;
    }

    if (pos < end) {
        // The weights of the 64 staged columns: 8 loads of 8 columns each.
        auto load_weights = [&](u32x4(&w)[8]) {
            uint32_t off[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) off[u] = stage_off[wave][u * 8 + cg] + seg16;
#pragma unroll
            for (int u = 0; u < 8; ++u)
                w[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(row_base + (size_t)off[u]));
        };
        // MULTIPLY stage: the lane that owns entry `ent` stages the products x * s_b of its column
        // (xf = 0 for a filler entry); every lane then reads the products of its own block(s).
        auto multiply = [&](int n, const float(&xf)[BATCH], int ent, typename F::Scales sv, const u32x4(&w)[8]) {
#pragma unroll
            for (int b = 0; b < BATCH; ++b) F::stage(xf[b], sv, stage_xs[wave][b][ent]);
            __builtin_amdgcn_wave_barrier();
            if (BATCH == 1) {
                typename F::Mine xl[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) xl[u] = F::read_mine(stage_xs[wave][0][u * 8 + cg], seg);
                F::step(w[0], xl[0], acc[0], bs[0]);
#pragma unroll
                for (int u = 1; u < 8; ++u)
                    if (u * 8 < n) F::step(w[u], xl[u], acc[0], bs[0]);
            } else {
#pragma unroll
                for (int u = 0; u < 8; ++u)
                    if (u == 0 || u * 8 < n) {
#pragma unroll
                        for (int b = 0; b < BATCH; ++b)
                            F::step(w[u], F::read_mine(stage_xs[wave][b][u * 8 + cg], seg), acc[b], bs[b]);
                    }
            }
            __builtin_amdgcn_wave_barrier();
        };

        u32x4 wA[8], wB[8];
        typename F::Scales svA, svB;
        int nA, nB;
        if (FUSED) {
            // FETCH stage of unit u (xr = this lane's x[64 u + lane], requested one stage earlier):
            // threshold, rank, stage the offsets, request the next unit's x, this unit's scales (every
            // lane its own column's) and weights.  Kept columns go to entries 0..n-1 in ascending order;
            // the other lanes fill entries n..63 with the unit's first kept column and x = 0.
            auto fetch_unit = [&](uint32_t xr, int u, u32x4(&w)[8], int &n_out, float(&xf_out)[BATCH], int &ent_out,
                                  typename F::Scales &sv_out, uint32_t &xr_next) {
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
                const uint32_t chunk_off = (uint32_t)(uu >> 1) * (uint32_t)F::kChunkBytes;
                const uint32_t col_own = (uint32_t)((uu & 1) * kPassCols + lane);
                const uint32_t col_first = (uint32_t)((uu & 1) * kPassCols + (n ? (int)__builtin_ctzll(mask) : 0));
                sv_out = F::load_scales(row_base + (size_t)(chunk_off + col_own * (uint32_t)(2 * F::kBlocks)));
                const int entry = keep ? rank : n + lane - rank;
                stage_off[wave][entry] = chunk_off + (uint32_t)F::kScaleBytes + (keep ? col_own : col_first) * 128u;
                __builtin_amdgcn_wave_barrier();
                load_weights(w);
                n_out = n;
                xf_out[0] = keep ? xv : 0.0f;
                ent_out = entry;
            };
            float xfA[BATCH], xfB[BATCH];
            int entA, entB;
            uint32_t xa = x[pos * kPassCols + lane], xb;
            fetch_unit(xa, pos, wA, nA, xfA, entA, svA, xb);
            for (;;) {
                const int uB = pos + 1;
                fetch_unit(xb, uB, wB, nB, xfB, entB, svB, xa);
                if (nA > 0) multiply(nA, xfA, entA, svA, wA);
                if (uB >= end) break;
                const int uA = uB + 1;
                fetch_unit(xa, uA, wA, nA, xfA, entA, svA, xb);
                if (nB > 0) multiply(nB, xfB, entB, svB, wB);
                if (uA >= end) break;
                pos = uA;
            }
        } else {
            auto fetch_k = [&](int p) -> int {
                const int e = p + lane;
                if (DENSE) return e < end ? e : 0;
                return idx[e < end ? e : end - 1];
            };
            // FETCH stage of the pass at list position p: the next pass's entries, this pass's x, scales
            // and weights.  Lanes past the pass point at its first column and later carry x = 0.
            auto fetch = [&](int kk, int p, u32x4(&w)[8], int &n_out, uint32_t(&xraw_out)[BATCH], typename F::Scales &sv_out,
                             int &k_after) {
                const int left = end - p;
                const int n = left < 0 ? 0 : (left < kPassCols ? left : kPassCols);
                k_after = fetch_k(p + kPassCols);
                const int k_first = n ? __builtin_amdgcn_readfirstlane(kk) : 0;
                const int kc = lane < n ? kk : k_first;
                const uint32_t chunk_off = (uint32_t)(kc >> 7) * (uint32_t)F::kChunkBytes;
                const uint32_t col = (uint32_t)(kc & (kGroup - 1));
#pragma unroll
                for (int b = 0; b < BATCH; ++b) xraw_out[b] = x[(size_t)b * K + kc];
                sv_out = F::load_scales(row_base + (size_t)(chunk_off + col * (uint32_t)(2 * F::kBlocks)));
                stage_off[wave][lane] = chunk_off + (uint32_t)F::kScaleBytes + col * 128u;
                __builtin_amdgcn_wave_barrier();
                load_weights(w);
                n_out = n;
            };
            auto multiply_list = [&](int n, const uint32_t(&xraw)[BATCH], typename F::Scales sv, const u32x4(&w)[8]) {
                float xf[BATCH];
#pragma unroll
                for (int b = 0; b < BATCH; ++b) xf[b] = lane < n ? half_bits_to_float(xraw[b]) : 0.0f;
                multiply(n, xf, lane, sv, w);
            };
            uint32_t xrA[BATCH], xrB[BATCH];
            int kA, kB;
            kA = fetch_k(pos);
            fetch(kA, pos, wA, nA, xrA, svA, kB);
            if (pos + nA >= end) {
                multiply_list(nA, xrA, svA, wA);      // the whole slice is one pass
            } else {
                for (;;) {
                    const int posB = pos + nA;
                    fetch(kB, posB, wB, nB, xrB, svB, kA);
                    multiply_list(nA, xrA, svA, wA);
                    if (posB >= end) break;
                    const int posA = posB + nB;
                    fetch(kA, posA, wA, nA, xrA, svA, kB);
                    multiply_list(nB, xrB, svB, wB);
                    if (posA >= end) break;
                    pos = posA;
                }
            }
        }
    }

#pragma unroll
    for (int b = 0; b < BATCH; ++b) F::finish(acc[b], bs[b], seg, cgr, red[wave][b]);
    __syncthreads();
    combine_block_row<WAVES, BATCH, F::kRows>(&red[0][0][0], tid, t, s, S, partials, ws_flags, y, M);
}

// Host side shared by the entry points: argument checks, launch shape, workspace, grid.  `launch` starts the
// kernel for (waves, mode) with mode 0 = index list, 1 = dense, 2 = one launch (batch 1 only).
template <class F, class Launch>
int colblock_width_run(int mode, int batch, int max_splits, int default_splits, const void *packed_dev, int64_t M, int64_t K,
                       const void *x_dev, const int32_t *idx_dev, const int32_t *count_dev, void *y_dev,
                       void *workspace_dev, size_t workspace_bytes, const spqt_launch_cfg *cfg, Launch launch) {
    if (!packed_dev || !x_dev || !y_dev) return SPQT_EINVAL;
    if (mode == 0 && !count_dev) return SPQT_EINVAL;
    if (int rc = check_shape(M, K, kGroup)) return rc;
    if (batch < 1 || batch > SPQT_MAX_BATCH || (mode == 2 && batch != 1)) return SPQT_ESHAPE;
    if (cfg && (cfg->flags & ~SPQT_CFG_Y_FP16)) return SPQT_EINVAL;
    const int y_half = cfg && (cfg->flags & SPQT_CFG_Y_FP16) ? 1 : 0;
    if ((uintptr_t)packed_dev % 128 != 0 || (uintptr_t)x_dev % 2 != 0 || (uintptr_t)y_dev % (y_half ? 2 : 4) != 0)
        return SPQT_EALIGN;
    const int64_t T64 = (M + F::kRows - 1) / F::kRows;
    int S = default_splits, waves = 4;
    if (cfg) {
        if (cfg->splits) S = cfg->splits;
        if (cfg->waves) waves = cfg->waves;
    }
    if (S < 1 || S > max_splits) return SPQT_EINVAL;
    if (waves != 1 && waves != 2 && waves != 4) return SPQT_EINVAL;
    size_t need = 0;
    spqt_workspace_bytes(M, K, batch, &need);
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
    const int m_and_flags = (int)M | (y_half ? kHalfOutputBit : 0);
    const hipError_t err = launch(waves, mode, grid, partials, ws_flags, NC, S, T, m_and_flags);
    return err == hipSuccess ? SPQT_OK : SPQT_EHIP;
}

}  // namespace spqt
#endif
