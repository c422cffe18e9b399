// The load-balanced sparse GEMV for ONE activation row with row-aligned passes (paper Section 4.2.3:
// every wavefront of a block-row takes an even slice of the kept-column list; Section 4.2.2: partial
// sums stay local and are combined once).
//
// The kernel in gemv.hip consumes its slice in passes whose columns all belong to ONE quantization
// group, so that the 8 column-lanes can be folded before the group's scale is applied.  With
// sparsity a group rarely fills the 64 slots of a pass (at 50 % a group of 128 keeps about 64
// columns: one full pass and a nearly empty one), and the empty slots still cost their load and
// multiply issue.  Here a pass is 8 ROWS of 8 slots, and only a row must be of one group:
//   - lane (cg, seg) = (lane / 8, lane % 8) reads, in its 8 steps, bytes [16 seg, 16 seg + 16) of the 8
//     columns of ROW cg - 32 consecutive rows of W at 8 consecutive list entries;
//   - the list entries are dealt to the rows in order: a row takes up to 8 consecutive entries of
//     one group, a new group starts a new row.  A group boundary therefore costs the rest of one
//     row (3.5 slots on average) instead of the rest of a pass; a pass that would need a ninth row
//     ends early and the next pass starts there;
//   - the 4 columns of a matrix-core product (v_mfma_f32_4x4x4_16B_f16, used as in gemv.hip) are 4
//     adjacent slots of one row, so every product is inside one group.  The lane's 32 row sums of a
//     pass are scaled by the 32 fp16 scales of (its rows, its row's group) - 64 contiguous bytes of
//     the chunk header - and added to 32 running sums; the 8 column-lanes are folded ONCE, at the end
//     of the slice, instead of once per pass;
//   - the offset-binary bias (stored = q + 8) enters as the initial value of the accumulators:
//     -8 * (sum of the row's 8 x), in the accumulator's units.
// Same pipeline as gemv.hip (a pass is fetched while the previous one is multiplied), same exchange
// between the workgroups of a block-row, same results up to rounding order.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "rowpass.hpp"

namespace {

using namespace spqt;

template <int WAVES>
__global__ __launch_bounds__(WAVES * 64) void spqt_gemv_list_kernel(
    const uint8_t *__restrict__ packed, const uint16_t *__restrict__ x, const int32_t *__restrict__ idx,
    const int32_t *__restrict__ count, float *__restrict__ y, void *partials, int32_t *ws_flags, int K, int NG,
    int S, int T, int M) {
    // Two staging slots per wave (the pass being multiplied and the pass being fetched).
    __shared__ __attribute__((aligned(16))) uint32_t stage_off[WAVES][2][kPassCols];   // byte offset of each slot's column in the block-row
    __shared__ __attribute__((aligned(16))) uint16_t stage_x[WAVES][2][8][8];          // x of each slot, [row][slot in row]
    __shared__ int32_t stage_grp[WAVES][2][8];                                         // group of each row
    __shared__ __attribute__((aligned(16))) float red[WAVES][1][kTileRows];

    SPQT_TL_BEGIN();
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int cg = lane >> 3;      // row of the pass this lane reads
    const int seg = lane & 7;      // 32-row segment of the tile this lane reads
    const int cgr = ((cg & 1) << 2) | (cg & 2) | (cg >> 2);   // cg with its three bits reversed
    const uint32_t seg16 = (uint32_t)seg * 16u;
    const uint64_t upto = (2ull << lane) - 1ull;              // bits 0..lane
    // all S workgroups of a block-row on one XCD (same index mod 8), as in gemv.hip
    const int xcd = blockIdx.x & 7;
    const int slot_x = blockIdx.x >> 3;
    const int t = xcd + 8 * (slot_x / S);
    const int s = slot_x % S;
    if (t >= T) return;

    const int n_raw = __builtin_amdgcn_readfirstlane(*count);
    const int n_ns = n_raw < 0 ? 0 : (n_raw > K ? K : n_raw);
    SPQT_TL(1);
    const int parts = S * WAVES;
    const int part = s * WAVES + wave;
    // even shares [n_ns * part / parts, n_ns * (part + 1) / parts); 32-bit arithmetic when the products fit
    int pos, end;
    if (n_ns < (1 << 23)) {
        pos = (int)(((uint32_t)n_ns * (uint32_t)part) / (uint32_t)parts);
        end = (int)(((uint32_t)n_ns * (uint32_t)(part + 1)) / (uint32_t)parts);
    } else {
        pos = (int)(((int64_t)n_ns * part) / parts);
        end = (int)(((int64_t)n_ns * (part + 1)) / parts);
    }
    // A list of all K columns is the identity (the entries are distinct columns in ascending order): the
    // FIRST pass then does not wait for its entries, which takes a dependent memory access off the start
    // (later passes request theirs a pass ahead anyway, with the unconditional load the pipeline counts on).
    const bool all_kept = n_ns == K;

    const int log2g = (NG << 7) == K ? 7 : 6;
    const int chunk_b = kScaleBytes + (kColBytes << log2g);
    const uint8_t *row_base = packed + (size_t)t * NG * chunk_b;

    float acc[32];   // rows 32 seg + i of the block-row, this lane's rows of the passes, scaled, in units of 2^-24 (even i) or 2^-20 (odd i)
#pragma unroll
    for (int i = 0; i < 32; ++i) acc[i] = 0.0f;

    if (pos < end) {
        // List entry p + lane, or -1 past the slice (the load itself is never predicated).
        auto fetch_k = [&](int p) -> int {
            const int e = p + lane;
            const int v = idx[e < n_ns ? e : n_ns - 1];
            return e < end ? v : -1;
        };

        // FETCH stage of the pass that starts at list position p < end (kk = fetch_k(p)): deal the entries
        // to rows, request the next pass's entries, this pass's x, its weights and its rows' scales.
        auto fetch = [&](int kk, int p, int slot, u32x4(&w)[8], u32x4(&sc)[4], int &n_out, bool &hi_out,
                         int &k_after, uint32_t &xraw, int &where) {
            const RowDeal d = deal_rows(kk, log2g, lane, upto);
            const bool take = d.take;
            const int g = d.g, row = d.row, col = d.col, n = d.n;
            k_after = fetch_k(p + n);
            where = take ? row * 8 + col : -1;
            hi_out = d.hi;
            xraw = x[take ? kk : 0];
            const uint32_t off_own = (uint32_t)g * (uint32_t)chunk_b + (uint32_t)(kk & ((1 << log2g) - 1)) * kColBytes;
            // Slots no entry lands in point at the pass's first column (a line that is fetched anyway)
            // and carry x = 0; rows no entry lands in take the first row's group.
            const uint32_t off_first = (uint32_t)__builtin_amdgcn_readfirstlane((int)off_own);
            const int g_first = __builtin_amdgcn_readfirstlane(g);
            stage_off[wave][slot][lane] = off_first;
            if (lane < 8) stage_grp[wave][slot][lane] = g_first;
            __builtin_amdgcn_wave_barrier();
            if (take) {
                stage_off[wave][slot][where] = off_own;
                if (col == 0) stage_grp[wave][slot][row] = g;
            }
            __builtin_amdgcn_wave_barrier();
            const u32x4 o0 = *reinterpret_cast<const u32x4 *>(&stage_off[wave][slot][cg * 8]);
            const u32x4 o1 = *reinterpret_cast<const u32x4 *>(&stage_off[wave][slot][cg * 8 + 4]);
            const int grow = stage_grp[wave][slot][cg];
            const uint8_t *wp = row_base + kScaleBytes + seg16;
            w[0] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(wp + (size_t)o0.x));
            w[1] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(wp + (size_t)o0.y));
            w[2] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(wp + (size_t)o0.z));
            w[3] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(wp + (size_t)o0.w));
            w[4] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(wp + (size_t)o1.x));
            w[5] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(wp + (size_t)o1.y));
            w[6] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(wp + (size_t)o1.z));
            w[7] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(wp + (size_t)o1.w));
            // the 32 scales of rows 32 seg .. 32 seg + 31 for this lane's row of the pass
            const u32x4 *scp = reinterpret_cast<const u32x4 *>(row_base + (size_t)grow * chunk_b + (size_t)seg * 64);
#pragma unroll
            for (int i = 0; i < 4; ++i) sc[i] = scp[i];
            n_out = n;
        };

        // MULTIPLY stage of a fetched pass: x goes to its slots, then the shared row-pass multiply.
        auto multiply = [&](int slot, u32x4(&w)[8], u32x4(&sc)[4], bool hi, uint32_t xraw, int where) {
            if (lane < 32) reinterpret_cast<uint32_t *>(&stage_x[wave][slot][0][0])[lane] = 0u;
            __builtin_amdgcn_wave_barrier();
            if (where >= 0) (&stage_x[wave][slot][0][0])[where] = (uint16_t)xraw;
            __builtin_amdgcn_wave_barrier();
            const u32x4 xa = *reinterpret_cast<const u32x4 *>(&stage_x[wave][slot][cg][0]);
            multiply_row_pass(w, sc, xa, hi, lane, acc);
            __builtin_amdgcn_wave_barrier();
        };

        // Two-stage software pipeline over the passes, buffers A and B alternating.
        u32x4 wA[8], wB[8], scA[4], scB[4];
        uint32_t xrA, xrB;
        int nA, nB, kA, kB, whA, whB;
        bool hiA, hiB;
        if (all_kept) kA = pos + lane < end ? pos + lane : -1;
        else kA = fetch_k(pos);
        SPQT_TL_WAIT(2);
        fetch(kA, pos, 0, wA, scA, nA, hiA, kB, xrA, whA);
        SPQT_TL_WAIT(3);
        for (;;) {
            const int posB = pos + nA;
            if (posB >= end) {
                multiply(0, wA, scA, hiA, xrA, whA);
                break;
            }
            fetch(kB, posB, 1, wB, scB, nB, hiB, kA, xrB, whB);
            multiply(0, wA, scA, hiA, xrA, whA);
            const int posA = posB + nB;
            if (posA >= end) {
                multiply(1, wB, scB, hiB, xrB, whB);
                break;
            }
            fetch(kA, posA, 0, wA, scA, nA, hiA, kB, xrA, whA);
            multiply(1, wB, scB, hiB, xrB, whB);
            pos = posA;
        }
    }

    SPQT_TL(4);
    // the 8 column-lanes are folded: lane (cg, seg) ends with rows 32 seg + 4 rev(cg) + j (the fold only adds
    // rows whose index is equal mod 4, so odd and even rows stay apart), then back to true units
    float r4[4];
    fold_columns(acc, r4);
    reinterpret_cast<f32x4 *>(red[wave][0])[8 * seg + cgr] =
        f32x4{r4[0] * kTwo24, r4[1] * (kTwo24 * 0.0625f), r4[2] * kTwo24, r4[3] * (kTwo24 * 0.0625f)};
    __syncthreads();
    SPQT_TL(5);
    combine_block_row<WAVES, 1>(&red[0][0][0], tid, t, s, S, partials, ws_flags, y, M);
    SPQT_TL_END(WAVES, wave, lane, S > 1 && s == S - 1);
}

}  // namespace

namespace spqt {

SPQT_TL_SETTER(spqt_timeline_set_list)

hipError_t launch_gemv_list(int waves, int grid, hipStream_t stream, const uint8_t *packed, const uint16_t *x,
                            const int32_t *idx, const int32_t *count, float *y, void *partials, int32_t *ws_flags,
                            int K, int NG, int S, int T, int m_and_flags) {
    switch (waves) {
        case 1: hipLaunchKernelGGL((spqt_gemv_list_kernel<1>), dim3(grid), dim3(64), 0, stream, packed, x, idx, count, y, partials, ws_flags, K, NG, S, T, m_and_flags); break;
        case 2: hipLaunchKernelGGL((spqt_gemv_list_kernel<2>), dim3(grid), dim3(128), 0, stream, packed, x, idx, count, y, partials, ws_flags, K, NG, S, T, m_and_flags); break;
        case 8: hipLaunchKernelGGL((spqt_gemv_list_kernel<8>), dim3(grid), dim3(512), 0, stream, packed, x, idx, count, y, partials, ws_flags, K, NG, S, T, m_and_flags); break;
        default: hipLaunchKernelGGL((spqt_gemv_list_kernel<4>), dim3(grid), dim3(256), 0, stream, packed, x, idx, count, y, partials, ws_flags, K, NG, S, T, m_and_flags); break;
    }
    return hipGetLastError();
}

}  // namespace spqt
