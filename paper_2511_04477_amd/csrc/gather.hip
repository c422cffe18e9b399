// spqt_gather: threshold the hidden state and compact the surviving column indices.
//
// Paper Section 4.2.3 ("Sparse index collecting kernel design"): a binary mask of the
// entries that pass the threshold is prefix-summed and every active entry writes its index
// to the position the scan gives it, so the list is contiguous.  The paper scans 1024-entry
// segments with a Blelloch scan and orders the segments through a global atomic counter,
// which makes the order depend on arrival.  Here the list must be ascending and
// reproducible, and x is at most a few tens of KB, so ONE 1024-lane workgroup does the
// whole vector with wave64 primitives: ballot + mbcnt give each lane its rank inside a
// 512-entry wave step, and sixteen wave totals are combined through LDS.  No atomics.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "spqt_internal.h"

namespace {

constexpr int kWaves = 16;
constexpr int kThreads = kWaves * 64;
constexpr int kPerLane = 8;                        // one 16-byte load of fp16 per lane
constexpr int kStep = 64 * kPerLane;               // entries one wave covers per step
constexpr int kMaxSteps = SPQT_GATHER_MAX_K / (kWaves * kStep);   // 8

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
        float lo = half_bits_to_float(v[d] & 0xFFFFu);
        float hi = half_bits_to_float(v[d] >> 16);
        m |= (uint32_t)(!(__builtin_fabsf(lo) < thr)) << (2 * d);
        m |= (uint32_t)(!(__builtin_fabsf(hi) < thr)) << (2 * d + 1);
    }
    return m;
}

__global__ __launch_bounds__(kThreads) void spqt_gather_kernel(const uint16_t *__restrict__ x, int K,
                                                               int batch, float thr,
                                                               int32_t *__restrict__ idx,
                                                               int32_t *__restrict__ count) {
    __shared__ int wave_total[kWaves];
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;

    // Wave w owns the contiguous span [w*span, (w+1)*span), walked in steps of 512 entries;
    // lane l of a step owns entries 8l..8l+7 of it, so ranks follow (step, lane, bit) order.
    const int steps = (K + kWaves * kStep - 1) / (kWaves * kStep);
    const int span = steps * kStep;

    uint32_t bits[kMaxSteps];      // keep mask of this lane's 8 entries, per step
    int lane_rank[kMaxSteps];      // kept entries of this wave before this lane's, per step
    int total = 0;                 // kept entries of this wave so far

#pragma unroll
    for (int s = 0; s < kMaxSteps; ++s) {
        bits[s] = 0;
        lane_rank[s] = 0;
        if (s < steps) {
            const int first = wave * span + s * kStep + lane * kPerLane;
            uint32_t m = 0;
            if (first < K) {       // K % 8 == 0, so a lane's eight entries are all in or all out
                for (int b = 0; b < batch; ++b) {
                    u32x4 v = *reinterpret_cast<const u32x4 *>(x + (size_t)b * K + first);
                    m |= keep_bits(v, thr);
                }
            }
            bits[s] = m;
            int before = total;
#pragma unroll
            for (int j = 0; j < kPerLane; ++j) {
                uint64_t ballot = __ballot((m >> j) & 1u);
                before += __builtin_amdgcn_mbcnt_hi((uint32_t)(ballot >> 32),
                                                    __builtin_amdgcn_mbcnt_lo((uint32_t)ballot, 0u));
                total += __popcll(ballot);
            }
            lane_rank[s] = before;
        }
    }

    if (lane == 0) wave_total[wave] = total;
    __syncthreads();
    int base = 0, all = 0;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
        int t = wave_total[w];
        base += (w < wave) ? t : 0;
        all += t;
    }
    if (threadIdx.x == 0) *count = all;

#pragma unroll
    for (int s = 0; s < kMaxSteps; ++s) {
        if (s < steps) {
            uint32_t m = bits[s];
            const int first = wave * span + s * kStep + lane * kPerLane;
            int pos = base + lane_rank[s];
#pragma unroll
            for (int j = 0; j < kPerLane; ++j) {
                if ((m >> j) & 1u) idx[pos++] = first + j;
            }
        }
    }
}

}  // namespace

extern "C" int spqt_gather(const void *x_dev, int64_t K, int batch, float threshold,
                           int32_t *idx_out_dev, int32_t *count_out_dev, void *stream) {
    if (!x_dev || !idx_out_dev || !count_out_dev) return SPQT_EINVAL;
    if (K <= 0 || K % spqt::kGroup != 0 || K > SPQT_GATHER_MAX_K) return SPQT_ESHAPE;
    if (batch < 1 || batch > SPQT_MAX_BATCH) return SPQT_ESHAPE;
    if (threshold != threshold) return SPQT_EINVAL;   // NaN threshold has no meaning
    if ((uintptr_t)x_dev % 16 != 0 || (uintptr_t)idx_out_dev % 4 != 0) return SPQT_EALIGN;
    hipLaunchKernelGGL(spqt_gather_kernel, dim3(1), dim3(kThreads), 0, (hipStream_t)stream,
                       (const uint16_t *)x_dev, (int)K, batch, threshold, idx_out_dev, count_out_dev);
    return hipGetLastError() == hipSuccess ? SPQT_OK : SPQT_EHIP;
}
