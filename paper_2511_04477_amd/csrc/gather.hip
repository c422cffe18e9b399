// spqt_gather: threshold the hidden state and compact the surviving column indices.
//
// Paper Section 4.2.3 ("Sparse index collecting kernel design"): a binary mask of the
// entries that pass the threshold is prefix-summed and every active entry writes its index
// to the position the scan gives it, so the list is contiguous.  The paper scans 1024-entry
// segments with a Blelloch scan and orders the segments through a global atomic counter,
// which makes the order depend on arrival.  Here the list must be ascending and
// reproducible, so there are no atomics: workgroup b owns the 4096-entry segment b of x,
// ranks its kept entries with wave64 primitives (ballot + mbcnt inside a 512-entry wave
// step, eight wave totals through LDS), and obtains its base offset by simply counting
// the kept entries of all earlier segments itself (x is at most 128 KB and sits in L2 after
// the first touch; counting needs no ballots, only popcounts).
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "spqt_internal.h"

namespace {

constexpr int kWaves = 8;
constexpr int kThreads = kWaves * 64;
constexpr int kPerLane = 8;                        // one 16-byte load of fp16 per lane
constexpr int kStep = 64 * kPerLane;               // entries one wave covers
constexpr int kSegment = kWaves * kStep;           // entries one workgroup ranks: 4096

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float half_bits_to_float(uint32_t h16) {
    return (float)__builtin_bit_cast(_Float16, (uint16_t)h16);
}

// Bit i of the result is set iff entry i of the eight fp16 values in v is kept:
// kept == !(|x| < thr), evaluated in fp32 (Section 2: sparse iff |x_i| < threshold).
__device__ __forceinline__ uint32_t keep_bits(u32x4 v, float thr) {
    uint32_t m = 0;
#pragma unroll
    for (int d = 0; d < 4; ++d) {
        const uint32_t word = v[d];
        const float lo = half_bits_to_float(word & 0xFFFFu);
        const float hi = half_bits_to_float(word >> 16);
        m |= (uint32_t)(!(__builtin_fabsf(lo) < thr)) << (2 * d);
        m |= (uint32_t)(!(__builtin_fabsf(hi) < thr)) << (2 * d + 1);
    }
    return m;
}

// Keep mask of the eight entries starting at `first` (all rows of the batch OR-ed), or 0 past K.
template <int BATCH>
__device__ __forceinline__ uint32_t mask_at(const uint16_t *__restrict__ x, int K, int first, float thr) {
    u32x4 v[BATCH];
#pragma unroll
    for (int b = 0; b < BATCH; ++b) v[b] = *reinterpret_cast<const u32x4 *>(x + (size_t)b * K + first);
    uint32_t m = 0;
#pragma unroll
    for (int b = 0; b < BATCH; ++b) m |= keep_bits(v[b], thr);
    return m;
}

// The eight fp16 values of v with the entries whose bit in `keep` is clear replaced by +0.
__device__ __forceinline__ u32x4 zero_dropped(u32x4 v, uint32_t keep) {
    u32x4 out;
#pragma unroll
    for (int d = 0; d < 4; ++d) {
        const uint32_t lo = (keep >> (2 * d)) & 1u ? 0x0000FFFFu : 0u;
        const uint32_t hi = (keep >> (2 * d + 1)) & 1u ? 0xFFFF0000u : 0u;
        out[d] = v[d] & (lo | hi);
    }
    return out;
}

// MASKED: besides the union list, write a copy of x in which every row has ITS OWN dropped
// entries set to zero.  A GEMV over the union list fed this copy gives each row the sum over
// that row's kept columns only (a dropped entry of a listed column contributes 0 * w).
template <int BATCH, bool MASKED = false>
__global__ __launch_bounds__(kThreads) void spqt_gather_kernel(const uint16_t *__restrict__ x, int K,
                                                               float thr, int32_t *__restrict__ idx,
                                                               int32_t *__restrict__ count,
                                                               uint16_t *__restrict__ x_masked = nullptr) {
    __shared__ int wave_total[kWaves];
    __shared__ int wave_before[kWaves];
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int seg = blockIdx.x;
    const int lane_first = wave * kStep + lane * kPerLane;   // inside a segment

    // This workgroup's own segment: lane l of wave w owns entries 8l..8l+7 of wave step w, so
    // ranks follow (wave, lane, bit) order = ascending index.
    const int first = seg * kSegment + lane_first;
    // K % 8 == 0, so a lane's eight entries are all inside x or all past its end
    uint32_t m = 0u;
    if (MASKED) {
        if (first < K) {
#pragma unroll
            for (int b = 0; b < BATCH; ++b) {
                const u32x4 v = *reinterpret_cast<const u32x4 *>(x + (size_t)b * K + first);
                const uint32_t kb = keep_bits(v, thr);
                *reinterpret_cast<u32x4 *>(x_masked + (size_t)b * K + first) = zero_dropped(v, kb);
                m |= kb;
            }
        }
    } else {
        m = first < K ? mask_at<BATCH>(x, K, first, thr) : 0u;
    }

    // Kept entries of all earlier segments, counted by this workgroup itself.
    // (Earlier segments are complete - only the last one can be ragged - so these loads need no
    // bounds test and can all be in flight together.)
    int before = 0;
#pragma unroll 4
    for (int p = 0; p < seg; ++p) before += __popc(mask_at<BATCH>(x, K, p * kSegment + lane_first, thr));
#pragma unroll
    for (int s = 1; s < 64; s <<= 1) before += __shfl_xor(before, s);

    int rank = 0, total = 0;
#pragma unroll
    for (int j = 0; j < kPerLane; ++j) {
        const uint64_t ballot = __ballot((m >> j) & 1u);
        rank += __builtin_amdgcn_mbcnt_hi((uint32_t)(ballot >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)ballot, 0u));
        total += __popcll(ballot);
    }
    if (lane == 0) {
        wave_total[wave] = total;
        wave_before[wave] = before;
    }
    __syncthreads();
    int base = 0, all = 0;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
        const int t = wave_total[w];
        base += wave_before[w] + ((w < wave) ? t : 0);
        all += wave_before[w] + t;
    }
    if (seg == (int)gridDim.x - 1 && threadIdx.x == 0) *count = all;

    int pos = base + rank;
#pragma unroll
    for (int j = 0; j < kPerLane; ++j)
        if ((m >> j) & 1u) idx[pos++] = first + j;
}

int run_gather(const void *x_dev, int64_t K, int batch, float threshold, int32_t *idx_out_dev,
               int32_t *count_out_dev, void *x_masked_dev, void *stream) {
    if (!x_dev || !idx_out_dev || !count_out_dev) return SPQT_EINVAL;
    if (K <= 0 || K % spqt::kGroup != 0 || K > SPQT_GATHER_MAX_K) return SPQT_ESHAPE;
    if (batch < 1 || batch > SPQT_MAX_BATCH) return SPQT_ESHAPE;
    if (threshold != threshold) return SPQT_EINVAL;   // NaN threshold has no meaning
    if ((uintptr_t)x_dev % 16 != 0 || (uintptr_t)idx_out_dev % 4 != 0) return SPQT_EALIGN;
    if ((uintptr_t)x_masked_dev % 16 != 0) return SPQT_EALIGN;
    const int segments = (int)((K + kSegment - 1) / kSegment);
    const dim3 grid(segments), block(kThreads);
    hipStream_t st = (hipStream_t)stream;
    const uint16_t *x = (const uint16_t *)x_dev;
    if (x_masked_dev) {
        uint16_t *xm = (uint16_t *)x_masked_dev;
        switch (batch) {
            case 1: hipLaunchKernelGGL((spqt_gather_kernel<1, true>), grid, block, 0, st, x, (int)K, threshold, idx_out_dev, count_out_dev, xm); break;
            case 2: hipLaunchKernelGGL((spqt_gather_kernel<2, true>), grid, block, 0, st, x, (int)K, threshold, idx_out_dev, count_out_dev, xm); break;
            case 3: hipLaunchKernelGGL((spqt_gather_kernel<3, true>), grid, block, 0, st, x, (int)K, threshold, idx_out_dev, count_out_dev, xm); break;
            default: hipLaunchKernelGGL((spqt_gather_kernel<4, true>), grid, block, 0, st, x, (int)K, threshold, idx_out_dev, count_out_dev, xm); break;
        }
        return hipGetLastError() == hipSuccess ? SPQT_OK : SPQT_EHIP;
    }
    switch (batch) {
        case 1: hipLaunchKernelGGL((spqt_gather_kernel<1, false>), grid, block, 0, st, x, (int)K, threshold, idx_out_dev, count_out_dev, (uint16_t *)nullptr); break;
        case 2: hipLaunchKernelGGL((spqt_gather_kernel<2, false>), grid, block, 0, st, x, (int)K, threshold, idx_out_dev, count_out_dev, (uint16_t *)nullptr); break;
        case 3: hipLaunchKernelGGL((spqt_gather_kernel<3, false>), grid, block, 0, st, x, (int)K, threshold, idx_out_dev, count_out_dev, (uint16_t *)nullptr); break;
        default: hipLaunchKernelGGL((spqt_gather_kernel<4, false>), grid, block, 0, st, x, (int)K, threshold, idx_out_dev, count_out_dev, (uint16_t *)nullptr); break;
    }
    return hipGetLastError() == hipSuccess ? SPQT_OK : SPQT_EHIP;
}

}  // namespace

extern "C" int spqt_gather(const void *x_dev, int64_t K, int batch, float threshold,
                           int32_t *idx_out_dev, int32_t *count_out_dev, void *stream) {
    return run_gather(x_dev, K, batch, threshold, idx_out_dev, count_out_dev, nullptr, stream);
}

extern "C" int spqt_gather_rows(const void *x_dev, int64_t K, int batch, float threshold,
                                int32_t *idx_out_dev, int32_t *count_out_dev, void *x_masked_out_dev,
                                void *stream) {
    if (!x_masked_out_dev || !x_dev) return SPQT_EINVAL;
    if (K > 0 && batch > 0) {   // the copy may not overlap x: other workgroups are still reading it
        const uintptr_t a = (uintptr_t)x_dev, b = (uintptr_t)x_masked_out_dev;
        const uintptr_t bytes = (uintptr_t)K * (uintptr_t)batch * 2u;
        if (a < b + bytes && b < a + bytes) return SPQT_EINVAL;
    }
    return run_gather(x_dev, K, batch, threshold, idx_out_dev, count_out_dev, x_masked_out_dev, stream);
}
