// Row-aligned passes: the two stages every kernel for ONE activation row and a kept-column list shares
// (gemv_list.hip takes the list from spqt_gather, gemv_bal.hip builds it inside the kernel).
//
// A pass is 8 rows of 8 slots; lane (cg, seg) = (lane / 8, lane % 8) reads, in its 8 steps, bytes
// [16 seg, 16 seg + 16) of the 8 columns of ROW cg - 32 consecutive rows of W at 8 consecutive list
// entries.  Only a row must be of one quantization group: the lane's 32 row sums of a pass are scaled by
// the 32 fp16 scales of (its rows, its row's group) before anything is folded across lanes.
// (Paper Section 4.2.3: every wavefront consumes an even slice of the kept-column list; Section 4.2.2:
// partial sums stay local and are combined once.)
#ifndef SPQT_ROWPASS_HPP
#define SPQT_ROWPASS_HPP

#include "gemv_common.hpp"

namespace spqt {

typedef _Float16 h2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ h2 as_h2(uint32_t bits) { return __builtin_bit_cast(h2, bits); }

// How the (up to) 64 candidate list entries of a pass are dealt to its rows.
struct RowDeal {
    bool take;      // this lane's candidate belongs to the pass
    int row, col;   // its row (0..7) and slot inside the row (0..7)
    int g;          // its quantization group
    int n;          // entries the pass takes (wave-uniform): the next pass starts n entries further
    bool hi;        // some row uses its slots 4..7 (wave-uniform): the second quad of products is needed
};

// Lane l holds candidate column kk (or -1 past the slice); candidates are consecutive list entries.
// A row takes up to 8 consecutive entries of one group, a new group starts a new row, and entries that
// would need a ninth row wait for the next pass.  All with wave-wide bit tricks, no loop: `start` =
// group differs from the previous lane's, ballot -> each lane finds the start of its run by clz on the
// masked ballot, rank = distance to it, a second ballot of rank % 8 == 0 counts rows.
__device__ __forceinline__ RowDeal deal_rows(int kk, int log2g, int lane, uint64_t upto) {
    RowDeal d;
    const bool cand = kk >= 0;
    d.g = kk >> log2g;
    const int gprev = __builtin_amdgcn_ds_bpermute((lane - 1) << 2, d.g);
    const bool start = cand && (lane == 0 || d.g != gprev);               // first entry of a run of one group
    const uint64_t starts = __ballot(start);
    const int first = 63 - (int)__builtin_clzll((starts & upto) | 1ull);  // where this entry's run starts
    const int rank = lane - first;                                        // position inside the run
    const bool newrow = cand && (rank & 7) == 0;
    const uint64_t rows = __ballot(newrow);
    d.row = (int)__builtin_popcountll(rows & upto) - 1;
    d.take = cand && d.row < 8;
    d.n = __builtin_amdgcn_readfirstlane((int)__popcll(__ballot(d.take)));
    d.col = rank & 7;
    d.hi = __ballot(d.take && d.col >= 4) != 0ull;
    return d;
}

// The products of one pass for ONE activation row on the matrix cores: w[u] = the lane's 16 bytes (32 rows)
// of column slot u, xa = the raw fp16 x of the 8 slots, accq[2 d + half][p] = init[p] + sum over the slots
// of code(row 8 d + 4 half + p, slot) * x(slot), codes as fp16 subnormals (code * 2^-24 in even rows,
// 16 * code * 2^-24 in odd rows).  second_quad == false skips slots 4..7 (wave-uniform).
//
// v_mfma_f32_4x4x4_16B_f16 computes 16 independent 4x4x4 products, one per group of 4 adjacent lanes
// (which read the same columns): D[m][n] += sum over 4 k of A[m][k] * B[k][n] with n = the lane (its own
// rows), k = four slots, m = the activation row.  B is one row's codes at 4 columns (code_rows), A the raw
// fp16 x of those columns - exact products, fp32 accumulation.  A 4x4x4 product has room for 4 rows of A
// and only one is needed: x is placed in row v of A (zeros elsewhere) for the v-th of four consecutive
// rows of W, so the four results land in the four registers of ONE accumulator tuple and a lane's 32
// rows need 8 tuples.
__device__ __forceinline__ void row_products(const u32x4 (&w)[8], u32x4 xa, bool second_quad, f32x4 init, int lane,
                                             f32x4 (&accq)[8]) {
#pragma unroll
    for (int quad = 0; quad < 2; ++quad) {
        if (quad == 0 || second_quad) {
            f16x4 a[4];
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const bool mine = (lane & 3) == v;
                a[v] = as_f16x4(u32x2{mine ? (quad ? xa.z : xa.x) : 0u, mine ? (quad ? xa.w : xa.y) : 0u});
            }
#pragma unroll
            for (int d = 0; d < 4; ++d) {
                const uint32_t w0 = w[4 * quad + 0][d], w1 = w[4 * quad + 1][d];
                const uint32_t w2 = w[4 * quad + 2][d], w3 = w[4 * quad + 3][d];
#pragma unroll
                for (int half = 0; half < 2; ++half) {
                    u32x2 b[4];
                    if (half) code_rows<1>(w0, w1, w2, w3, b);
                    else code_rows<0>(w0, w1, w2, w3, b);
                    f32x4 c = quad ? accq[2 * d + half] : init;
#pragma unroll
                    for (int p = 0; p < 4; ++p) c = __builtin_amdgcn_mfma_f32_4x4x4f16(a[p], as_f16x4(b[p]), c, 0, 0, 0);
                    accq[2 * d + half] = c;
                }
            }
        }
    }
}

// MULTIPLY stage of a row-aligned pass: w[u] = the lane's 16 bytes of slot u of its row, sc = the 32 fp16
// scales of (its 32 rows, its row's group), xa = the raw fp16 x of its row's 8 slots (0 in unused slots).
// acc[i] += scale_i * sum over the row's slots of code(row i, slot) * x(slot), in units of 2^-24 (even i)
// or 2^-20 (odd i); the bias of the offset-binary codes enters as the products' initial value.
__device__ __forceinline__ void multiply_row_pass(const u32x4 (&w)[8], const u32x4 (&sc)[4], u32x4 xa, bool hi,
                                                  int lane, float (&acc)[32]) {
    // bias: -8 * (sum of the row's x), as the accumulators' initial value
    const h2 ones = {(_Float16)1.0f, (_Float16)1.0f};
    float xs = __builtin_amdgcn_fdot2(as_h2(xa.x), ones, 0.0f, false);
    xs = __builtin_amdgcn_fdot2(as_h2(xa.y), ones, xs, false);
    xs = __builtin_amdgcn_fdot2(as_h2(xa.z), ones, xs, false);
    xs = __builtin_amdgcn_fdot2(as_h2(xa.w), ones, xs, false);
    const float be = xs * (-8.0f / kTwo24), bo = xs * (-128.0f / kTwo24);
    f32x4 accq[8];
    row_products(w, xa, hi, f32x4{be, bo, be, bo}, lane, accq);
    // scale and add: row i = 4 tq + p of the lane's 32; its scale is half i of the 64 bytes
#pragma unroll
    for (int i = 0; i < 32; i += 2) {
        const h2 sh = as_h2(sc[i >> 3][(i >> 1) & 3]);
        acc[i] = __builtin_fmaf((float)sh.x, accq[i >> 2][i & 3], acc[i]);
        acc[i + 1] = __builtin_fmaf((float)sh.y, accq[i >> 2][(i & 3) + 1], acc[i + 1]);
    }
}

}  // namespace spqt
#endif
