// spqt_gemv_fused, one activation row: sparsity test, compaction and load-balanced GEMV in ONE launch.
//
// Paper Section 4.2.3: every simdgroup that works on a block-row gets an EVEN share of the kept-column
// list (about n_ns / (n1 * n2) columns), so the work is balanced however the kept columns are spread;
// Section 2: a column is sparse iff |x_i| < threshold.  The paper builds the list with a kernel of its
// own; here every workgroup derives what it needs of the list from x itself, which removes that
// launch and the dependent global reads count -> index entries -> weights from the GEMV's start:
//   1. COUNT.  The workgroup's wavefronts bring the whole x into LDS (loads that write LDS directly, 512
//      columns = 8 fp16 per lane at a time), threshold it and leave the kept count of every 512-column
//      step in LDS (x is at most 64 KB here and sits in L2; this is popcounts only, three steps packed in
//      one word so that one lane reduction serves three steps).
//   2. SPLIT.  Every wavefront scans the step counts (at most 128), which gives n_ns and, for its own even
//      share [n_ns * j / (S * WAVES), n_ns * (j + 1) / (S * WAVES)) of the kept columns in ascending order,
//      the step in which the share begins - the very partition the index-list kernel takes from idx.
//   3. LIST.  The wavefront compacts the steps of its share, one at a time and only as the passes need
//      them, into a ring of (column, x) pairs in LDS: an exclusive scan of the lanes' kept counts ranks the
//      kept columns, and an entry whose rank falls inside the share is written at rank - share start.
//      The next step's x is requested one refill ahead, so no pass ever waits on a dependent global read.
//   4. GEMV.  Row-aligned passes over the ring exactly as gemv_list.hip forms them over idx (rowpass.hpp),
//      same two-stage pipeline, same exchange between the workgroups of a block-row; for the same launch
//      shape the two kernels perform the same arithmetic in the same order.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "rowpass.hpp"

namespace {

using namespace spqt;

constexpr int kStepCols = 512;            // columns one wavefront step thresholds: 8 per lane
constexpr int kXsSteps = 64;              // steps of x kept in LDS: K <= 32768 (larger K: static column ranges)
constexpr int kPackSteps = 3;             // step counts packed in one 32-bit word (10 bits each, a count is <= 512)
constexpr int kRing = 1024;               // ring entries per wavefront; a refill adds at most 512 to at most 63 live ones

typedef short s16x2 __attribute__((ext_vector_type(2)));

// The sparsity test |x| < thr on fp16 bit patterns.  For an fp16 x and an fp32 thr, |x| < thr holds iff
// |x| < c, c being the smallest fp16 value >= thr (c = 0 for thr <= 0: nothing is below it; c = +inf for
// thr above the largest finite fp16), and for non-negative fp16 values the order of the values is the
// order of their bit patterns, NaN patterns lying above +inf: so the test is (bits & 0x7FFF) < bits(c)
// as 15-bit integers, two halves of a dword at a time - exactly the result of the fp32 comparison
// (NaN and, at any finite threshold, Inf are kept; an entry equal to the threshold is kept).
__device__ __forceinline__ uint32_t threshold_bits(float thr) {
    if (!(thr > 0.0f)) return 0u;
    const _Float16 h = (_Float16)thr;                       // round to nearest even
    uint32_t b = __builtin_bit_cast(uint16_t, h);
    if ((float)h < thr) b += 1u;                            // next fp16 up (from the largest finite one: +inf)
    return b | (b << 16);
}
// Sign bits (bit 15 / bit 31) set where the half is DROPPED.
__device__ __forceinline__ uint32_t dropped_signs(uint32_t two_halves, uint32_t c2) {
    const s16x2 d = __builtin_bit_cast(s16x2, two_halves & 0x7FFF7FFFu) - __builtin_bit_cast(s16x2, c2);
    return __builtin_bit_cast(uint32_t, d) & 0x80008000u;
}
// Number of dropped entries among the eight fp16 values of v.
__device__ __forceinline__ int dropped_count8(u32x4 v, uint32_t c2) {
    return (int)__popc(dropped_signs(v.x, c2) | (dropped_signs(v.y, c2) >> 1) | (dropped_signs(v.z, c2) >> 2) |
                       (dropped_signs(v.w, c2) >> 3));
}
// Bit i set iff entry i of the eight fp16 values of v is KEPT.
__device__ __forceinline__ uint32_t keep_bits8(u32x4 v, uint32_t c2) {
    const uint32_t u = (dropped_signs(v.x, c2) >> 15) | (dropped_signs(v.y, c2) >> 13) | (dropped_signs(v.z, c2) >> 11) |
                       (dropped_signs(v.w, c2) >> 9);
    return ~(u | (u >> 15)) & 0xFFu;
}

// Inclusive prefix sum over the 64 lanes (Hillis-Steele with DPP row shifts, then the row totals);
// total = the sum over all lanes (wave-uniform).
__device__ __forceinline__ int wave_inclusive_scan(int v, int lane, int &total) {
    v += __builtin_amdgcn_update_dpp(0, v, 0x111, 0xf, 0xf, true);   // row_shr:1
    v += __builtin_amdgcn_update_dpp(0, v, 0x112, 0xf, 0xf, true);   // row_shr:2
    v += __builtin_amdgcn_update_dpp(0, v, 0x114, 0xf, 0xf, true);   // row_shr:4
    v += __builtin_amdgcn_update_dpp(0, v, 0x118, 0xf, 0xf, true);   // row_shr:8
    // totals of the rows of 16 lanes
    const int t0 = __builtin_amdgcn_readlane(v, 15), t1 = __builtin_amdgcn_readlane(v, 31);
    const int t2 = __builtin_amdgcn_readlane(v, 47), t3 = __builtin_amdgcn_readlane(v, 63);
    const int row = lane >> 4;
    total = t0 + t1 + t2 + t3;
    return v + (row > 0 ? t0 : 0) + (row > 1 ? t1 : 0) + (row > 2 ? t2 : 0);
}
// Sum over the 64 lanes (wave-uniform).
__device__ __forceinline__ int wave_total(int v) {
    v += __builtin_amdgcn_update_dpp(0, v, 0x111, 0xf, 0xf, true);
    v += __builtin_amdgcn_update_dpp(0, v, 0x112, 0xf, 0xf, true);
    v += __builtin_amdgcn_update_dpp(0, v, 0x114, 0xf, 0xf, true);
    v += __builtin_amdgcn_update_dpp(0, v, 0x118, 0xf, 0xf, true);
    return __builtin_amdgcn_readlane(v, 15) + __builtin_amdgcn_readlane(v, 31) + __builtin_amdgcn_readlane(v, 47) +
           __builtin_amdgcn_readlane(v, 63);
}

template <int WAVES>
__global__ __launch_bounds__(WAVES * 64) void spqt_gemv_bal_kernel(
    const uint8_t *__restrict__ packed, const uint16_t *__restrict__ x, float thr, float *__restrict__ y,
    void *partials, int32_t *ws_flags, int K, int NG, int S, int T, int M) {
    __shared__ __attribute__((aligned(16))) uint32_t stage_off[WAVES][2][kPassCols];   // byte offset of each slot's column in the block-row
    __shared__ __attribute__((aligned(16))) uint16_t stage_x[WAVES][2][8][8];          // x of each slot, [row][slot in row]
    __shared__ int32_t stage_grp[WAVES][2][8];                                         // group of each row
    __shared__ __attribute__((aligned(16))) float red[WAVES][1][kTileRows];
    // kept columns per step: word [w][q][row of 16 lanes] holds, 10 bits each, that row's counts of the steps
    // w + WAVES * (3 q + r), r = 0..2 (the steps wavefront w thresholds, three at a time)
    __shared__ __attribute__((aligned(16))) uint32_t count_part[WAVES][(kXsSteps / WAVES + kPackSteps - 1) / kPackSteps + 1][4];
    __shared__ uint32_t ring[WAVES][kRing + 64];                                       // the wavefront's share of the list: column | x bits << 16 (+ 64 dummy entries)
    __shared__ __attribute__((aligned(16))) u32x4 xs[kXsSteps * 64];                   // x, [step][lane]

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

    // 1. COUNT: x into LDS, then the kept columns of every 512-column step (every workgroup does all of x).
    const int nsteps = (K + kStepCols - 1) / kStepCols;      // <= kXsSteps (checked on the host)
    const uint32_t c2 = threshold_bits(thr);
    const int my_steps = (nsteps - wave + WAVES - 1) / WAVES;             // steps wave, wave + WAVES, ...
#pragma unroll 1
    for (int i = 0; i < my_steps; ++i) {
        const int j = wave + i * WAVES;
        const int c = j * kStepCols + lane * 8;
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(x + (c < K ? c : 0)),
                                         (__attribute__((address_space(3))) void *)&xs[j * 64], 16, 0, 0);
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#pragma unroll 1
    for (int q = 0; q * kPackSteps < my_steps; ++q) {
        uint32_t packed = 0;
#pragma unroll
        for (int r = 0; r < kPackSteps; ++r) {
            const int i = q * kPackSteps + r;
            const int j = wave + (i < my_steps ? i : my_steps - 1) * WAVES;
            const u32x4 v = xs[j * 64 + lane];
            const bool valid = i < my_steps && j * kStepCols + lane * 8 < K;
            packed |= (uint32_t)(valid ? 8 - dropped_count8(v, c2) : 0) << (10 * r);
        }
        // sums over the rows of 16 lanes end up in lanes 15, 31, 47, 63
        packed += __builtin_amdgcn_update_dpp(0u, packed, 0x111, 0xf, 0xf, true);   // row_shr:1
        packed += __builtin_amdgcn_update_dpp(0u, packed, 0x112, 0xf, 0xf, true);   // row_shr:2
        packed += __builtin_amdgcn_update_dpp(0u, packed, 0x114, 0xf, 0xf, true);   // row_shr:4
        packed += __builtin_amdgcn_update_dpp(0u, packed, 0x118, 0xf, 0xf, true);   // row_shr:8
        if ((lane & 15) == 15) count_part[wave][q][lane >> 4] = packed;
    }
    __syncthreads();
    SPQT_TL(1);

    // 2. SPLIT: prefix sums of the step counts; this wavefront's even share of the n_ns kept columns.
    int c0 = 0;                                                 // kept columns of step `lane`
    {
        const int j = lane < nsteps ? lane : 0;
        const int i = j / WAVES;
        const u32x4 p = *reinterpret_cast<const u32x4 *>(count_part[j % WAVES][i / kPackSteps]);
        c0 = lane < nsteps ? (int)(((p.x + p.y + p.z + p.w) >> (10 * (i % kPackSteps))) & 0x3FFu) : 0;
    }
    int n_ns;
    const int p0 = wave_inclusive_scan(c0, lane, n_ns);
    const int parts = S * WAVES;
    const int part = s * WAVES + wave;
    // n_ns <= 32768 and part < parts <= 256: the products fit 32 bits
    const int begin = (int)(((uint32_t)n_ns * (uint32_t)part) / (uint32_t)parts);     // ranks [begin, begin + total) of the kept columns
    const int total = (int)(((uint32_t)n_ns * (uint32_t)(part + 1)) / (uint32_t)parts) - begin;

    const int log2g = (NG << 7) == K ? 7 : 6;
    const int chunk_b = kScaleBytes + (kColBytes << log2g);
    const uint8_t *row_base = packed + (size_t)t * NG * chunk_b;

    float acc[32];   // rows 32 seg + i of the block-row, this lane's rows of the passes, scaled, in units of 2^-24 (even i) or 2^-20 (odd i)
#pragma unroll
    for (int i = 0; i < 32; ++i) acc[i] = 0.0f;

    if (total > 0) {
        // the step in which rank `begin` lies, and the kept columns before that step
        int step = (int)__builtin_ctzll(__ballot(p0 > begin));
        int rank_base = __builtin_amdgcn_readlane(p0 - c0, step);
        int filled = 0;                       // entries of the share written to the ring so far

        // 3. LIST: compact one more step into the ring (entries rank - begin, for ranks inside the share).
        // Every lane writes all eight of its entries; those that are dropped or outside the share go to a
        // dummy entry behind the ring, which keeps the code free of branches.
        auto refill = [&]() {
            const u32x4 v = xs[step * 64 + lane];
            const int col0 = step * kStepCols + lane * 8;
            const uint32_t m = col0 < K ? keep_bits8(v, c2) : 0u;
            int kept_here;
            const int incl = wave_inclusive_scan((int)__popc(m), lane, kept_here);
            const int e0 = rank_base + incl - (int)__popc(m) - begin;      // entry of this lane's first kept column
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int e = e0 + (int)__popc(m & ((1u << i) - 1u));
                const bool ok = ((m >> i) & 1u) && (uint32_t)e < (uint32_t)total;
                const uint32_t xb = (i & 1) ? (v[i >> 1] & 0xFFFF0000u) : (v[i >> 1] << 16);
                ring[wave][ok ? (e & (kRing - 1)) : kRing + lane] = (uint32_t)(col0 + i) | xb;
            }
            rank_base += kept_here;
            const int upto_rank = rank_base - begin;
            filled = upto_rank < 0 ? 0 : (upto_rank > total ? total : upto_rank);
            ++step;
            __builtin_amdgcn_wave_barrier();
        };

        // Entry p + lane of the share: its column, or -1 past the share.  The ring must hold it: refill first.
        auto fetch_k = [&](int p, uint32_t &xk) -> int {
            const int need = p + 64 < total ? p + 64 : total;
            while (filled < need && step < nsteps) refill();
            const int e = p + lane;
            const uint32_t v = ring[wave][e & (kRing - 1)];
            xk = v >> 16;
            return e < total ? (int)(v & 0xFFFFu) : -1;
        };

        // FETCH stage of the pass that starts at entry p < total: deal the entries to rows, request the
        // pass's weights and its rows' scales.
        auto fetch = [&](int p, int slot, u32x4(&w)[8], u32x4(&sc)[4], int &n_out, bool &hi_out, uint32_t &xraw,
                         int &where) {
            const int kk = fetch_k(p, xraw);
            const RowDeal d = deal_rows(kk, log2g, lane, upto);
            where = d.take ? d.row * 8 + d.col : -1;
            hi_out = d.hi;
            const uint32_t off_own = (uint32_t)d.g * (uint32_t)chunk_b + (uint32_t)(kk & ((1 << log2g) - 1)) * kColBytes;
            // Slots no entry lands in point at the pass's first column (a line that is fetched anyway)
            // and carry x = 0; rows no entry lands in take the first row's group.
            const uint32_t off_first = (uint32_t)__builtin_amdgcn_readfirstlane((int)off_own);
            const int g_first = __builtin_amdgcn_readfirstlane(d.g);
            stage_off[wave][slot][lane] = off_first;
            if (lane < 8) stage_grp[wave][slot][lane] = g_first;
            __builtin_amdgcn_wave_barrier();
            if (d.take) {
                stage_off[wave][slot][where] = off_own;
                if (d.col == 0) stage_grp[wave][slot][d.row] = d.g;
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
            n_out = d.n;
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

        // 4. GEMV: two-stage software pipeline over the passes, buffers A and B alternating.
        u32x4 wA[8], wB[8], scA[4], scB[4];
        uint32_t xrA, xrB;
        int nA, nB, whA, whB;
        bool hiA, hiB;
        int pos = 0;
        fetch(pos, 0, wA, scA, nA, hiA, xrA, whA);
        SPQT_TL(2);
        SPQT_TL_WAIT(3);
        for (;;) {
            const int posB = pos + nA;
            if (posB >= total) {
                multiply(0, wA, scA, hiA, xrA, whA);
                break;
            }
            fetch(posB, 1, wB, scB, nB, hiB, xrB, whB);
            multiply(0, wA, scA, hiA, xrA, whA);
            const int posA = posB + nB;
            if (posA >= total) {
                multiply(1, wB, scB, hiB, xrB, whB);
                break;
            }
            fetch(posA, 0, wA, scA, nA, hiA, xrA, whA);
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

SPQT_TL_SETTER(spqt_timeline_set_bal)

hipError_t launch_gemv_bal(int waves, int grid, hipStream_t stream, const uint8_t *packed, const uint16_t *x, float thr,
                           float *y, void *partials, int32_t *ws_flags, int K, int NG, int S, int T, int m_and_flags) {
    switch (waves) {
        case 1: hipLaunchKernelGGL((spqt_gemv_bal_kernel<1>), dim3(grid), dim3(64), 0, stream, packed, x, thr, y, partials, ws_flags, K, NG, S, T, m_and_flags); break;
        case 2: hipLaunchKernelGGL((spqt_gemv_bal_kernel<2>), dim3(grid), dim3(128), 0, stream, packed, x, thr, y, partials, ws_flags, K, NG, S, T, m_and_flags); break;
        default: hipLaunchKernelGGL((spqt_gemv_bal_kernel<4>), dim3(grid), dim3(256), 0, stream, packed, x, thr, y, partials, ws_flags, K, NG, S, T, m_and_flags); break;
    }
    return hipGetLastError();
}

}  // namespace spqt
