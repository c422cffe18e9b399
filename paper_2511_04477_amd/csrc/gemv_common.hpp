// Device helpers shared by the GEMV kernels (gemv.hip, gemv_cb.hip): the int4 multiply step,
// the transposing lane folds, wave sums, and the exchange of partial sums between the
// workgroups of a block-row.  Not part of the C ABI.
#ifndef SPQT_GEMV_COMMON_HPP
#define SPQT_GEMV_COMMON_HPP

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "spqt_internal.h"

namespace spqt {

typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kPassCols = 64;                  // most columns one pass covers (8 steps)
constexpr float kTwo24 = 16777216.0f;          // 2^24: undoes the fp16 subnormal exponent
constexpr int kHalfOutputBit = 1 << 30;        // in the kernels' M argument: y is fp16, not fp32
constexpr int kOwnSetsBit = 1 << 29;           // in the kernels' M argument: every activation row keeps its own set
constexpr int kRowsMask = (1 << 25) - 1;       // the bits of that argument that hold M (M <= 2^24)
#ifdef SPQT_TEST_GIVE_UP
// Test build (libspqt_giveup.so): the producers publish nothing and the reducer's wait is a handful of polls, so
// the give-up path of combine_block_row runs on every launch with several workgroups per block-row - and every
// kernel still ends normally.
constexpr int kMaxPolls = 4;
constexpr bool kMuteProducers = true;
#else
constexpr int kMaxPolls = 1 << 18;             // bound on the reducer's wait for one batch of partials
constexpr bool kMuteProducers = false;
#endif

// Per-wavefront wall-clock stamps for the timeline build (-DSPQT_TIMELINE=1, libspqt_timeline.so): every
// wavefront records when it started (0), knew its share of the list (1), had issued its first pass (2),
// had that pass's weights (3, with a forced wait that the product build does not have), left its loop (4),
// passed the workgroup's LDS reduction (5) and finished (6); word 7 tells whether it belongs to the
// reducing workgroup and where it ran.  The product build compiles all of it away.
#ifdef SPQT_TIMELINE
static __device__ unsigned long long *spqt_tl_buf = nullptr;   // one per translation unit, set by its setter
#define SPQT_TL_BEGIN() unsigned long long tl_[8] = {0, 0, 0, 0, 0, 0, 0, 0}; tl_[0] = wall_clock64()
#define SPQT_TL(i) tl_[i] = wall_clock64()
#define SPQT_TL_WAIT(i) do { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); tl_[i] = wall_clock64(); } while (0)
#define SPQT_TL_END(WAVES_, wave_, lane_, reducer_)                                                              \
    do {                                                                                                         \
        tl_[6] = wall_clock64();                                                                                 \
        if (spqt_tl_buf && (lane_) == 0) {                                                                       \
            unsigned long long *d_ = spqt_tl_buf + ((size_t)blockIdx.x * (WAVES_) + (wave_)) * 8;                \
            for (int i_ = 0; i_ < 7; ++i_) d_[i_] = tl_[i_];                                                     \
            d_[7] = (unsigned long long)((reducer_) ? 1 : 0) |                                                   \
                    ((unsigned long long)__builtin_amdgcn_s_getreg(63492) << 8) |        /* HW_ID */             \
                    ((unsigned long long)(__builtin_amdgcn_s_getreg(63508) & 15) << 40); /* XCC_ID */            \
        }                                                                                                        \
    } while (0)
#define SPQT_TL_SETTER(name)                                                                          \
    extern "C" int name(void *p) { return (int)hipMemcpyToSymbol(HIP_SYMBOL(spqt_tl_buf), &p, sizeof(p)); }
#else
#define SPQT_TL_BEGIN()
#define SPQT_TL(i)
#define SPQT_TL_WAIT(i)
#define SPQT_TL_END(WAVES_, wave_, lane_, reducer_)
#define SPQT_TL_SETTER(name)
#endif

__device__ __forceinline__ float half_bits_to_float(uint32_t h16) {
    return (float)__builtin_bit_cast(_Float16, (uint16_t)h16);
}

// Bit casts go through by-value parameters on purpose: __builtin_bit_cast applied directly
// to a vector-element expression (v.y, v[i]) reads the vector's first element instead.
__device__ __forceinline__ float as_float(uint32_t bits) { return __builtin_bit_cast(float, bits); }
__device__ __forceinline__ uint32_t as_u32(float f) { return __builtin_bit_cast(uint32_t, f); }
__device__ __forceinline__ f16x2 as_f16x2(uint32_t bits) { return __builtin_bit_cast(f16x2, bits); }
__device__ __forceinline__ f16x4 as_f16x4(u32x2 bits) { return __builtin_bit_cast(f16x4, bits); }

// Eight codes of one dword: acc[i] (+)= n_i * x for nibble i (row 8d+i of the lane's 32 rows).
// xlo = x * 2^24 pairs with nibbles sitting at bits 0..3 of a half, xhi = x * 2^20 with
// nibbles at bits 4..7 (value 16 n * 2^-24).  INIT overwrites the accumulators (first step of
// a pass) instead of adding to them.
template <bool INIT>
__device__ __forceinline__ void fma_codes(uint32_t w, float xlo, float xhi, float *acc) {
    const uint32_t w8 = w >> 8;
    const f16x2 a = as_f16x2(w & 0x000F000Fu);    // nibbles 0, 4
    const f16x2 b = as_f16x2(w & 0x00F000F0u);    // nibbles 1, 5
    const f16x2 c = as_f16x2(w8 & 0x000F000Fu);   // nibbles 2, 6
    const f16x2 d = as_f16x2(w8 & 0x00F000F0u);   // nibbles 3, 7
    acc[0] = __builtin_fmaf((float)a.x, xlo, INIT ? 0.0f : acc[0]);
    acc[4] = __builtin_fmaf((float)a.y, xlo, INIT ? 0.0f : acc[4]);
    acc[1] = __builtin_fmaf((float)b.x, xhi, INIT ? 0.0f : acc[1]);
    acc[5] = __builtin_fmaf((float)b.y, xhi, INIT ? 0.0f : acc[5]);
    acc[2] = __builtin_fmaf((float)c.x, xlo, INIT ? 0.0f : acc[2]);
    acc[6] = __builtin_fmaf((float)c.y, xlo, INIT ? 0.0f : acc[6]);
    acc[3] = __builtin_fmaf((float)d.x, xhi, INIT ? 0.0f : acc[3]);
    acc[7] = __builtin_fmaf((float)d.y, xhi, INIT ? 0.0f : acc[7]);
}

template <bool INIT>
__device__ __forceinline__ void fma_step(u32x4 w, float xl, float *acc) {
    const float xh = xl * 0.0625f;
    fma_codes<INIT>(w.x, xl, xh, acc + 0);
    fma_codes<INIT>(w.y, xl, xh, acc + 8);
    fma_codes<INIT>(w.z, xl, xh, acc + 16);
    fma_codes<INIT>(w.w, xl, xh, acc + 24);
}

// The three levels of the column fold are written as asm blocks: the lane swaps work in place
// on both of their registers (no copies), and the wait states a swap or DPP read needs after a
// VALU write of its operand are paid once per block instead of once per instruction.

// Level 1, lane pairs (l, l^8) inside every row of 16 lanes: afterwards lanes with bit 3 clear
// hold a summed over the pair, lanes with bit 3 set hold b summed over the pair - in b's
// register.  Two bank-masked DPP adds per (a, b).
#define SPQT_FOLD8(B, A)                                                              \
    "v_add_f32_dpp " B ", " B ", " B " row_ror:8 row_mask:0xf bank_mask:0xc\n\t"      \
    "v_add_f32_dpp " B ", " A ", " A " row_ror:8 row_mask:0xf bank_mask:0x3\n\t"
__device__ __forceinline__ void fold8_x8(const float *a, float *b) {
    asm volatile("s_nop 1\n\t" SPQT_FOLD8("%0", "%8") SPQT_FOLD8("%1", "%9") SPQT_FOLD8("%2", "%10")
                     SPQT_FOLD8("%3", "%11") SPQT_FOLD8("%4", "%12") SPQT_FOLD8("%5", "%13")
                         SPQT_FOLD8("%6", "%14") SPQT_FOLD8("%7", "%15")
                 : "+v"(b[0]), "+v"(b[1]), "+v"(b[2]), "+v"(b[3]), "+v"(b[4]), "+v"(b[5]), "+v"(b[6]), "+v"(b[7])
                 : "v"(a[0]), "v"(a[1]), "v"(a[2]), "v"(a[3]), "v"(a[4]), "v"(a[5]), "v"(a[6]), "v"(a[7]));
}

// Level 2, lane pairs (l, l^16): v_permlane16_swap exchanges the odd rows of its first operand
// with the even rows of its second, so a + b afterwards is, in lanes with bit 4 clear, the old a
// summed over the pair and, in the others, the old b summed over the pair.
__device__ __forceinline__ void swap16_x8(float *a, float *b) {
    asm volatile("s_nop 1\n\t"
                 "v_permlane16_swap_b32 %0, %8\n\tv_permlane16_swap_b32 %1, %9\n\t"
                 "v_permlane16_swap_b32 %2, %10\n\tv_permlane16_swap_b32 %3, %11\n\t"
                 "v_permlane16_swap_b32 %4, %12\n\tv_permlane16_swap_b32 %5, %13\n\t"
                 "v_permlane16_swap_b32 %6, %14\n\tv_permlane16_swap_b32 %7, %15"
                 : "+v"(a[0]), "+v"(a[1]), "+v"(a[2]), "+v"(a[3]), "+v"(a[4]), "+v"(a[5]), "+v"(a[6]), "+v"(a[7]),
                   "+v"(b[0]), "+v"(b[1]), "+v"(b[2]), "+v"(b[3]), "+v"(b[4]), "+v"(b[5]), "+v"(b[6]), "+v"(b[7]));
}
// Level 3, lane pairs (l, l^32), same idea with the two halves of the wave.
__device__ __forceinline__ void swap32_x4(float *a, float *b) {
    asm volatile("s_nop 1\n\t"
                 "v_permlane32_swap_b32 %0, %4\n\tv_permlane32_swap_b32 %1, %5\n\t"
                 "v_permlane32_swap_b32 %2, %6\n\tv_permlane32_swap_b32 %3, %7"
                 : "+v"(a[0]), "+v"(a[1]), "+v"(a[2]), "+v"(a[3]), "+v"(b[0]), "+v"(b[1]), "+v"(b[2]), "+v"(b[3]));
}
__device__ __forceinline__ float fold16(float a, float b) {
    asm volatile("s_nop 1\n\tv_permlane16_swap_b32 %0, %1" : "+v"(a), "+v"(b));
    return a + b;
}
__device__ __forceinline__ float fold32(float a, float b) {
    asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1" : "+v"(a), "+v"(b));
    return a + b;
}

// Fold the 32 accumulators of the 8 lanes that read the same rows (lanes seg, seg+8, ...,
// seg+56), halving the number of live values at each of the three levels.  Lane (cg, seg)
// ends with the complete sums of rows 32 seg + 4 rev(cg) + j, j = 0..3, where rev reverses
// the three bits of cg (level 1 splits on lane bit 3, level 2 on bit 4, level 3 on bit 5).
// acc is clobbered.
__device__ __forceinline__ void fold_columns(float *acc, float *out4) {
    fold8_x8(acc + 0, acc + 16);      // pairs (i, i+16), i = 0..7   -> acc[16..23]
    fold8_x8(acc + 8, acc + 24);      // pairs (i, i+16), i = 8..15  -> acc[24..31]
    swap16_x8(acc + 16, acc + 24);    // pairs (16+i, 24+i)
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[i] = acc[16 + i] + acc[24 + i];
    swap32_x4(acc + 0, acc + 4);      // pairs (i, 4+i)
#pragma unroll
    for (int i = 0; i < 4; ++i) out4[i] = acc[i] + acc[4 + i];
}

template <int CTRL>
__device__ __forceinline__ float dpp_move(float v) {
    return as_float(__builtin_amdgcn_update_dpp(0u, as_u32(v), CTRL, 0xf, 0xf, false));
}

// Sum over the 64 lanes, returned in every lane: xor-butterfly inside rows of 16 with DPP
// (quad permutes, half-row and row mirrors), then across rows with the permlane swaps.
__device__ __forceinline__ float wave_sum(float v) {
    v += dpp_move<0xB1>(v);    // quad_perm [1,0,3,2]: lane ^ 1
    v += dpp_move<0x4E>(v);    // quad_perm [2,3,0,1]: lane ^ 2
    v += dpp_move<0x141>(v);   // row_half_mirror: the other quad of the 8
    v += dpp_move<0x140>(v);   // row_mirror: the other half of the row
    v = fold16(v, v);
    v = fold32(v, v);
    return v;
}

// Sum over the 8 lanes that read the same rows of a column run (lanes seg, seg + 8, ..., seg + 56).
__device__ __forceinline__ float sum_over_columns(float v) {
    v += dpp_move<0x128>(v);   // row_ror:8 - the lane 8 further inside the row of 16
    v = fold16(v, v);
    v = fold32(v, v);
    return v;
}

// Matrix-core B operands for 4 consecutive rows of W at 4 columns.  w0..w3 are the same dword of 4
// steps (4 columns, 8 rows each); HALF picks rows 0..3 or 4..7 of the dword.  One v_perm_b32 puts the
// same 16 bits of two columns side by side; masked in place, b[p] holds row p's code at the 4
// columns as fp16 subnormals: code * 2^-24 for p = 0, 2 and 16 * code * 2^-24 for p = 1, 3.
template <int HALF>
__device__ __forceinline__ void code_rows(uint32_t w0, uint32_t w1, uint32_t w2, uint32_t w3, u32x2 (&b)[4]) {
    constexpr uint32_t sel = HALF ? 0x07060302u : 0x05040100u;
    const uint32_t t01 = __builtin_amdgcn_perm(w1, w0, sel);
    const uint32_t t23 = __builtin_amdgcn_perm(w3, w2, sel);
    const uint32_t s01 = t01 >> 8, s23 = t23 >> 8;
    b[0] = u32x2{t01 & 0x000F000Fu, t23 & 0x000F000Fu};
    b[1] = u32x2{t01 & 0x00F000F0u, t23 & 0x00F000F0u};
    b[2] = u32x2{s01 & 0x000F000Fu, s23 & 0x000F000Fu};
    b[3] = u32x2{s01 & 0x00F000F0u, s23 & 0x00F000F0u};
}

// The one-launch kernel for one activation row: list built in the kernel, even shares (gemv_bal.hip).
hipError_t launch_gemv_bal(int waves, int grid, hipStream_t stream, const uint8_t *packed, const uint16_t *x, float thr,
                           float *y, void *partials, int32_t *ws_flags, int K, int NG, int S, int T, int m_and_flags);

// The index-list kernel for one activation row with row-aligned passes (gemv_list.hip).
hipError_t launch_gemv_list(int waves, int grid, hipStream_t stream, const uint8_t *packed, const uint16_t *x,
                            const int32_t *idx, const int32_t *count, float *y, void *partials, int32_t *ws_flags,
                            int K, int NG, int S, int T, int m_and_flags);

// Combine the S workgroups of block-row t (paper Section 4.2.2: the partial sums of the
// threadgroups that share a superblock row are reduced once at the end, without atomics on y).
// `red` holds this workgroup's [WAVES][BATCH][ROWS] partial sums in LDS (already synchronised);
// ROWS is the height of a block-row (256 for the 4-bit layouts).
// Every workgroup but the last (s == S-1) publishes its ROWS partial sums as 64-bit words
// {value, kWordTag} with device-scope stores and is done: no wait, no counter.  The last one adds
// the others' words in index order, polling a word until it carries the tag, then its own sums,
// writes y, and stores zero back into every word it consumed - so between calls the exchange area
// is all zeros whatever M, launch shape or kernel the calls had, and a word with the tag is always
// one of THIS call.  A 64-bit store is a single access: value and tag arrive together.  The
// reducer has the highest index of its block-row and workgroups are dispatched in index order, so
// everything it waits for is running or finished; the wait is bounded anyway, and a give-up
// poisons y with NaN instead of hanging and raises the workspace's poison flag (word 0 of its
// head): a late word of the abandoned call could otherwise be taken for a later call's, so from
// then on every call on that workspace yields NaN until spqt_workspace_init clears it.
constexpr uint32_t kWordTag = 0x5B07C0DEu;
template <int WAVES, int BATCH, int ROWS = kTileRows>
__device__ __forceinline__ void combine_block_row(const float *red, int tid, int t, int s, int S, void *partials,
                                                  int32_t *ws_flags, float *__restrict__ y, int m_and_flags) {
    // One kernel argument carries both (M <= 2^24): every extra scalar argument costs the
    // four-row kernels, which sit at the register limit, a spill.
    const int M = m_and_flags & kRowsMask;
    const bool y_half = (m_and_flags & kHalfOutputBit) != 0;
    constexpr int kOut = BATCH * ROWS;           // values one workgroup contributes: [BATCH][ROWS]
    constexpr int kThreads = WAVES * 64;
    constexpr int kPerThread = (kOut + kThreads - 1) / kThreads;
    // A thread that owns several values handles 2 of them together, so that the reducer's loads for
    // all of them are in flight at once (one round trip instead of one per value).
    constexpr int kTogether = kPerThread < 2 ? kPerThread : 2;
    unsigned long long *slots = reinterpret_cast<unsigned long long *>(partials) + (size_t)t * S * kOut;
    const bool reducer = S > 1 && s == S - 1;
    uint32_t poisoned = 0u;
    if (reducer) poisoned = __hip_atomic_load(reinterpret_cast<uint32_t *>(ws_flags), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    for (int r0 = tid; r0 < kOut; r0 += kTogether * kThreads) {
        int r[kTogether];
        bool real[kTogether];
        float sum[kTogether];
#pragma unroll
        for (int i = 0; i < kTogether; ++i) {
            const bool have = r0 + i * kThreads < kOut;
            r[i] = have ? r0 + i * kThreads : r0;
            real[i] = have && t * ROWS + (r[i] % ROWS) < M;   // rows past M are the last block-row's zero padding
            sum[i] = 0.0f;
#pragma unroll
            for (int w2 = 0; w2 < WAVES; ++w2) sum[i] += red[w2 * kOut + r[i]];
        }
        // fp32 output, or the same value rounded to fp16 (nearest even) when the caller asked for it
        auto store_y = [&](int i, float v) {
            const size_t y_at = (size_t)(r[i] / ROWS) * M + t * ROWS + (r[i] % ROWS);
            if (y_half) reinterpret_cast<_Float16 *>(y)[y_at] = (_Float16)v;
            else y[y_at] = v;
        };
        if (S == 1) {
#pragma unroll
            for (int i = 0; i < kTogether; ++i)
                if (real[i]) store_y(i, sum[i]);
        } else if (!reducer) {
#pragma unroll
            for (int i = 0; i < kTogether; ++i) {
                if (i > 0 && r[i] == r[0]) continue;   // a clamped duplicate: already published
                if (kMuteProducers) continue;
                const unsigned long long word = ((unsigned long long)kWordTag << 32) | as_u32(sum[i]);
                __hip_atomic_store(slots + (size_t)s * kOut + r[i], word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        } else {
            float total[kTogether];
#pragma unroll
            for (int i = 0; i < kTogether; ++i) total[i] = 0.0f;
            bool gave_up = false;
            for (int p0 = 0; p0 < S - 1; p0 += 16) {
                unsigned long long v[kTogether][16];
                int polls = 0;
                bool all_here;
                do {
                    // unconditional loads back to back (clamped index), then one check
#pragma unroll
                    for (int i = 0; i < kTogether; ++i)
#pragma unroll
                        for (int j = 0; j < 16; ++j) {
                            const int p = p0 + j < S - 1 ? p0 + j : S - 2;
                            v[i][j] = __hip_atomic_load(slots + (size_t)p * kOut + r[i], __ATOMIC_RELAXED,
                                                        __HIP_MEMORY_SCOPE_AGENT);
                        }
                    uint32_t missing = 0u;
#pragma unroll
                    for (int i = 0; i < kTogether; ++i)
#pragma unroll
                        for (int j = 0; j < 16; ++j) missing |= (uint32_t)(v[i][j] >> 32) ^ kWordTag;
                    all_here = missing == 0u;
                } while (!all_here && ++polls < kMaxPolls);
                gave_up = gave_up || !all_here;
#pragma unroll
                for (int i = 0; i < kTogether; ++i)
#pragma unroll
                    for (int j = 0; j < 16; ++j)
                        if (p0 + j < S - 1) {
                            total[i] += as_float((uint32_t)v[i][j]);
                            // consumed: the word goes back to zero for whatever call comes next
                            __hip_atomic_store(slots + (size_t)(p0 + j) * kOut + r[i], 0ull, __ATOMIC_RELAXED,
                                               __HIP_MEMORY_SCOPE_AGENT);
                        }
            }
            if (gave_up) __hip_atomic_store(reinterpret_cast<uint32_t *>(ws_flags), 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#pragma unroll
            for (int i = 0; i < kTogether; ++i)
                if (real[i]) store_y(i, (gave_up || poisoned) ? __builtin_nanf("") : total[i] + sum[i]);
        }
    }
}

}  // namespace spqt
#endif
