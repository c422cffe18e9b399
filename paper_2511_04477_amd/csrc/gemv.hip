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
//     16n*2^-24), which v_fma_mix_f32 multiplies by a pre-scaled x*2^24 (x*2^20) into the fp32
//     accumulator - exact products, fp32 accumulation.
//   - per group: the 8 column-lanes are folded with a transposing butterfly (permlane32/16
//     swaps + one DPP rotate), leaving each lane 4 rows; the offset-binary bias (stored =
//     q + 8) is removed there as -8 * (sum of the group's kept x), and the fp16 group scale is
//     applied once per (row, group): y_acc += scale * (sum - bias).
//   - WAVES wavefronts are combined through LDS, the S workgroups of a block-row through a
//     workspace: the last one to arrive adds the partials in fixed order and writes y.  No
//     floating-point atomics, so results are reproducible.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "spqt_internal.h"

namespace {

using namespace spqt;

typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kPassCols = 64;                  // most columns one pass covers (8 steps)
constexpr float kTwo24 = 16777216.0f;          // 2^24: undoes the fp16 subnormal exponent

__device__ __forceinline__ float half_bits_to_float(uint32_t h16) {
    return (float)__builtin_bit_cast(_Float16, (uint16_t)h16);
}

// Bit casts go through by-value parameters on purpose: __builtin_bit_cast applied directly
// to a vector-element expression (v.y, v[i]) reads the vector's first element instead.
__device__ __forceinline__ float as_float(uint32_t bits) { return __builtin_bit_cast(float, bits); }
__device__ __forceinline__ uint32_t as_u32(float f) { return __builtin_bit_cast(uint32_t, f); }
__device__ __forceinline__ f16x2 as_f16x2(uint32_t bits) { return __builtin_bit_cast(f16x2, bits); }

// Eight codes of one dword: acc[i] += n_i * x for nibble i (row 8d+i of the lane's 32 rows).
// xlo = x * 2^24 pairs with nibbles sitting at bits 0..3 of a half, xhi = x * 2^20 with
// nibbles at bits 4..7 (value 16 n * 2^-24).
__device__ __forceinline__ void fma_codes(uint32_t w, float xlo, float xhi, float *acc) {
    const uint32_t w8 = w >> 8;
    const f16x2 a = as_f16x2(w & 0x000F000Fu);    // nibbles 0, 4
    const f16x2 b = as_f16x2(w & 0x00F000F0u);    // nibbles 1, 5
    const f16x2 c = as_f16x2(w8 & 0x000F000Fu);   // nibbles 2, 6
    const f16x2 d = as_f16x2(w8 & 0x00F000F0u);   // nibbles 3, 7
    acc[0] = __builtin_fmaf((float)a.x, xlo, acc[0]);
    acc[4] = __builtin_fmaf((float)a.y, xlo, acc[4]);
    acc[1] = __builtin_fmaf((float)b.x, xhi, acc[1]);
    acc[5] = __builtin_fmaf((float)b.y, xhi, acc[5]);
    acc[2] = __builtin_fmaf((float)c.x, xlo, acc[2]);
    acc[6] = __builtin_fmaf((float)c.y, xlo, acc[6]);
    acc[3] = __builtin_fmaf((float)d.x, xhi, acc[3]);
    acc[7] = __builtin_fmaf((float)d.y, xhi, acc[7]);
}

// a and b are two accumulators of every lane.  Returns, in lanes 0..31, a summed over the
// lane pair (l, l+32) and, in lanes 32..63, b summed over the same pair.
__device__ __forceinline__ float fold32(float a, float b) {
    const u32x2 r = __builtin_amdgcn_permlane32_swap(as_u32(a), as_u32(b), false, false);
    const uint32_t r0 = r.x, r1 = r.y;
    return as_float(r0) + as_float(r1);
}
// Same for the lane pair (l, l^16): lanes with bit 4 clear get a's sum, the others b's.
__device__ __forceinline__ float fold16(float a, float b) {
    const u32x2 r = __builtin_amdgcn_permlane16_swap(as_u32(a), as_u32(b), false, false);
    const uint32_t r0 = r.x, r1 = r.y;
    return as_float(r0) + as_float(r1);
}
// Value of lane l^8 (rotate by 8 inside each row of 16 lanes).
__device__ __forceinline__ float from_xor8(float v) {
    return as_float(__builtin_amdgcn_update_dpp(0u, as_u32(v), 0x128 /* row_ror:8 */, 0xf, 0xf, false));
}

// Fold the 32 accumulators of the 8 lanes that read the same rows (lanes seg, seg+8, ...,
// seg+56).  Lane (cg, seg) ends with the complete sums of rows 32 seg + 4 cg + j, j = 0..3.
__device__ __forceinline__ void fold_columns(const float *acc, bool bit3, float *out4) {
    float v16[16], v8[8];
#pragma unroll
    for (int i = 0; i < 16; ++i) v16[i] = fold32(acc[i], acc[i + 16]);
#pragma unroll
    for (int i = 0; i < 8; ++i) v8[i] = fold16(v16[i], v16[i + 8]);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const float keep = bit3 ? v8[i + 4] : v8[i];
        const float send = bit3 ? v8[i] : v8[i + 4];
        out4[i] = keep + from_xor8(send);
    }
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int m = 1; m < 64; m <<= 1) v += __shfl_xor(v, m);
    return v;
}

template <int WAVES, bool DENSE>
__global__ __launch_bounds__(WAVES * 64) void spqt_gemv_kernel(
    const uint8_t *__restrict__ packed, const uint16_t *__restrict__ x,
    const int32_t *__restrict__ idx, const int32_t *__restrict__ count, float *__restrict__ y,
    float *partials, int32_t *counters, int K, int NG, int S, int T) {
    __shared__ uint32_t stage_off[WAVES][kPassCols];   // byte offset of each column of the pass
    __shared__ float stage_x[WAVES][kPassCols];        // its x, pre-scaled by 2^24
    __shared__ __attribute__((aligned(16))) float red[WAVES][kTileRows];
    __shared__ int is_last;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int cg = lane >> 3;      // column of the step this lane reads
    const int seg = lane & 7;      // 32-row segment of the tile this lane reads
    const bool bit3 = (lane & 8) != 0;
    // Workgroups are handed to the 8 XCDs round-robin by index.  Keep all S workgroups of a
    // block-row on ONE XCD (same index mod 8): their arrival counter then stays in that XCD's
    // L2 instead of bouncing between dies.  Only a matter of speed, never of correctness.
    const int xcd = blockIdx.x & 7;
    const int slot = blockIdx.x >> 3;          // position among this XCD's workgroups
    const int t = xcd + 8 * (slot / S);        // block-row
    const int s = slot % S;
    if (t >= T) return;

    // Even split of the index list over the S*WAVES wavefronts of this block-row.
    const int n_ns = DENSE ? K : __builtin_amdgcn_readfirstlane(*count);
    const int parts = S * WAVES;
    const int part = s * WAVES + wave;
    int pos = (int)(((int64_t)n_ns * part) / parts);
    const int end = (int)(((int64_t)n_ns * (part + 1)) / parts);

    uint32_t *my_off = stage_off[wave];
    float *my_x = stage_x[wave];
    const uint8_t *row_base = packed + (size_t)t * NG * kChunkBytes;

    // list entry pos + lane (-1 past the slice): the column this lane stages in the pass
    auto fetch_k = [&](int p) -> int {
        const int e = p + lane;
        if (e >= end) return -1;
        return DENSE ? e : idx[e];
    };

    float yacc[4] = {0.0f, 0.0f, 0.0f, 0.0f};   // rows 32 seg + 4 cg + j, scaled and summed over groups
    float acc[32];                               // current group, this lane's columns, unscaled
#pragma unroll
    for (int i = 0; i < 32; ++i) acc[i] = 0.0f;
    float xsum = 0.0f;                           // current group: x (pre-scaled) of the columns this lane staged
    u32x2 sc = {0u, 0u};                         // current group: fp16 scales of this lane's 4 rows
    int g_cur = -1;

    // fold the finished group into yacc
    auto flush = [&]() {
        float r4[4];
        fold_columns(acc, bit3, r4);
        const float bias = wave_sum(xsum) * (-8.0f / kTwo24);
        const uint32_t s01 = sc.x, s23 = sc.y;
        const f16x2 h01 = as_f16x2(s01), h23 = as_f16x2(s23);
        yacc[0] = __builtin_fmaf((float)h01.x, r4[0] + bias, yacc[0]);
        yacc[1] = __builtin_fmaf((float)h01.y, r4[1] + bias, yacc[1]);
        yacc[2] = __builtin_fmaf((float)h23.x, r4[2] + bias, yacc[2]);
        yacc[3] = __builtin_fmaf((float)h23.y, r4[3] + bias, yacc[3]);
#pragma unroll
        for (int i = 0; i < 32; ++i) acc[i] = 0.0f;
        xsum = 0.0f;
    };

    int k = fetch_k(pos);
    while (pos < end) {
        // ---- the pass: the run of list entries from pos that share the group of idx[pos] ----
        const int g = __builtin_amdgcn_readfirstlane(k) >> 7;
        const bool in = (k >> 7) == g;
        const int n = __builtin_amdgcn_readfirstlane((int)__popcll(__ballot(in)));
        const int k_next = fetch_k(pos + n);                 // next pass's entries: request early

        const uint32_t koff = in ? (uint32_t)(k & (kGroup - 1)) * kColBytes : 0u;
        uint32_t xraw = 0u;
        if (in) xraw = x[k];
        my_off[lane] = koff;

        const uint8_t *chunk = row_base + (size_t)g * kChunkBytes;
        const uint8_t *cols = chunk + kScaleBytes + seg * 16;
        __builtin_amdgcn_wave_barrier();

        // ---- request this pass's weights: one 16-byte load per lane and step ---------------
        u32x4 w[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            w[u] = u32x4{0u, 0u, 0u, 0u};
            if (u * 8 < n) {                                   // wave-uniform: skip empty steps
                const int e = u * 8 + cg;
                const uint32_t o = my_off[e];
                if (e < n) w[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(cols + o));
            }
        }

        // ---- group change: fold the finished group while the loads are in flight -----------
        if (g != g_cur) {
            if (g_cur >= 0) flush();
            g_cur = g;
            sc = *reinterpret_cast<const u32x2 *>(chunk + seg * 64 + cg * 8);
        }

        const float xs = half_bits_to_float(xraw) * kTwo24;   // 0 for lanes outside the pass
        xsum += xs;
        my_x[lane] = xs;
        __builtin_amdgcn_wave_barrier();

        // ---- multiply-accumulate ------------------------------------------------------------
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            if (u * 8 < n) {
                const float xl = my_x[u * 8 + cg];
                const float xh = xl * 0.0625f;
                fma_codes(w[u].x, xl, xh, acc + 0);
                fma_codes(w[u].y, xl, xh, acc + 8);
                fma_codes(w[u].z, xl, xh, acc + 16);
                fma_codes(w[u].w, xl, xh, acc + 24);
            }
        }
        __builtin_amdgcn_wave_barrier();
        pos += n;
        k = k_next;
    }
    if (g_cur >= 0) flush();

    // ---- combine the WAVES wavefronts through LDS ------------------------------------------
    reinterpret_cast<f32x4 *>(red[wave])[8 * seg + cg] = f32x4{yacc[0], yacc[1], yacc[2], yacc[3]};
    __syncthreads();

    float *my_partial = partials + ((size_t)t * S + s) * kTileRows;
    for (int r = tid; r < kTileRows; r += WAVES * 64) {
        float sum = 0.0f;
#pragma unroll
        for (int w2 = 0; w2 < WAVES; ++w2) sum += red[w2][r];
        if (S == 1)
            y[(size_t)t * kTileRows + r] = sum;
        else
            __hip_atomic_store(my_partial + r, sum, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    if (S == 1) return;

    // ---- combine the S workgroups of this block-row: last arrival adds in fixed order ------
    // The partials are written and read with device-scope atomic accesses (they go through to
    // the device-coherent level instead of staying in one XCD's L2), so the only ordering
    // needed is "my stores have completed before my arrival is counted" and "the count is read
    // before the partials are": a wait on the memory counters plus the workgroup barrier, not a
    // cache-wide write-back and invalidate.
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __syncthreads();
    if (tid == 0) {
        const int prev = __hip_atomic_fetch_add(counters + t, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        is_last = (prev == S - 1);
    }
    __syncthreads();
    if (!is_last) return;
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
    const float *tile_partials = partials + (size_t)t * S * kTileRows;
    for (int r = tid; r < kTileRows; r += WAVES * 64) {
        // request the partials in batches so their latencies overlap; add in index order
        float sum = 0.0f;
        for (int p0 = 0; p0 < S; p0 += 16) {
            float v[16];
#pragma unroll
            for (int j = 0; j < 16; ++j) {
                v[j] = 0.0f;
                if (p0 + j < S)
                    v[j] = __hip_atomic_load(tile_partials + (size_t)(p0 + j) * kTileRows + r,
                                             __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
#pragma unroll
            for (int j = 0; j < 16; ++j) sum += v[j];
        }
        y[(size_t)t * kTileRows + r] = sum;
    }
    if (tid == 0) __hip_atomic_store(counters + t, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__global__ void spqt_fill_zero_kernel(uint32_t *p, size_t n_words) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n_words) p[i] = 0u;
}

template <int WAVES>
hipError_t launch(bool dense, int grid, hipStream_t stream, const uint8_t *packed, const uint16_t *x,
                  const int32_t *idx, const int32_t *count, float *y, float *partials,
                  int32_t *counters, int K, int NG, int S, int T) {
    if (dense)
        hipLaunchKernelGGL((spqt_gemv_kernel<WAVES, true>), dim3(grid), dim3(WAVES * 64), 0, stream,
                           packed, x, idx, count, y, partials, counters, K, NG, S, T);
    else
        hipLaunchKernelGGL((spqt_gemv_kernel<WAVES, false>), dim3(grid), dim3(WAVES * 64), 0, stream,
                           packed, x, idx, count, y, partials, counters, K, NG, S, T);
    return hipGetLastError();
}

}  // namespace

extern "C" int spqt_workspace_bytes(int64_t M, int64_t K, int batch, size_t *out_bytes) {
    if (!out_bytes) return SPQT_EINVAL;
    if (int rc = check_shape(M, K, kGroup)) return rc;
    if (batch < 1 || batch > SPQT_MAX_BATCH) return SPQT_ESHAPE;
    *out_bytes = counter_bytes(M) + (size_t)M * SPQT_MAX_SPLITS * sizeof(float);
    return SPQT_OK;
}

extern "C" int spqt_workspace_init(void *workspace_dev, size_t workspace_bytes, void *stream) {
    if (!workspace_dev || workspace_bytes < 256) return SPQT_EINVAL;
    if ((uintptr_t)workspace_dev % 256 != 0) return SPQT_EALIGN;
    // Only the counters need a defined start value; zero the counter area of the largest
    // shape this workspace could serve (it is a few KB at most) - simply all leading words
    // up to 64 KB or the buffer's end.
    size_t words = (workspace_bytes < 65536 ? workspace_bytes : 65536) / 4;
    hipLaunchKernelGGL(spqt_fill_zero_kernel, dim3((unsigned)((words + 255) / 256)), dim3(256), 0,
                       (hipStream_t)stream, (uint32_t *)workspace_dev, words);
    return hipGetLastError() == hipSuccess ? SPQT_OK : SPQT_EHIP;
}

extern "C" int spqt_default_cfg(int64_t M, int64_t K, int batch, int sparse, spqt_launch_cfg *out) {
    if (!out) return SPQT_EINVAL;
    if (int rc = check_shape(M, K, kGroup)) return rc;
    if (batch < 1 || batch > SPQT_MAX_BATCH) return SPQT_ESHAPE;
    (void)sparse;
    const int64_t T = M / kTileRows, NG = K / kGroup;
    int waves = 4;
    // Aim for ~2048 wavefronts in flight, but keep at least one quantization group of
    // dense work per wavefront.
    int64_t S = (2048 + T * waves - 1) / (T * waves);
    int64_t cap = NG / waves;
    if (cap < 1) cap = 1;
    if (S > cap) S = cap;
    if (S > SPQT_MAX_SPLITS) S = SPQT_MAX_SPLITS;
    if (S < 1) S = 1;
    out->splits = (int)S;
    out->waves = waves;
    return SPQT_OK;
}

extern "C" int spqt_gemv_ex(const void *packed_dev, int64_t M, int64_t K, int group, const void *x_dev,
                            int batch, const int32_t *idx_dev, const int32_t *count_dev, float *y_dev,
                            void *workspace_dev, size_t workspace_bytes, void *stream,
                            const spqt_launch_cfg *cfg) {
    if (!packed_dev || !x_dev || !y_dev) return SPQT_EINVAL;
    if (idx_dev && !count_dev) return SPQT_EINVAL;
    if (int rc = check_shape(M, K, group)) return rc;
    if (batch < 1 || batch > SPQT_MAX_BATCH) return SPQT_ESHAPE;
    if ((uintptr_t)packed_dev % 128 != 0 || (uintptr_t)x_dev % 2 != 0 || (uintptr_t)y_dev % 4 != 0)
        return SPQT_EALIGN;

    spqt_launch_cfg c;
    if (int rc = spqt_default_cfg(M, K, batch, idx_dev != nullptr, &c)) return rc;
    if (cfg) {
        if (cfg->splits) c.splits = cfg->splits;
        if (cfg->waves) c.waves = cfg->waves;
    }
    if (c.splits < 1 || c.splits > SPQT_MAX_SPLITS) return SPQT_EINVAL;
    if (c.waves != 1 && c.waves != 2 && c.waves != 4) return SPQT_EINVAL;

    size_t need = 0;
    spqt_workspace_bytes(M, K, batch, &need);
    float *partials = nullptr;
    int32_t *counters = nullptr;
    if (c.splits > 1) {
        if (!workspace_dev) return SPQT_EINVAL;
        if (workspace_bytes < need) return SPQT_ESIZE;
        if ((uintptr_t)workspace_dev % 256 != 0) return SPQT_EALIGN;
        counters = (int32_t *)workspace_dev;
        partials = (float *)((uint8_t *)workspace_dev + counter_bytes(M));
    }

    const int T = (int)(M / kTileRows), NG = (int)(K / kGroup);
    const int grid = 8 * ((T + 7) / 8) * c.splits;
    const bool dense = idx_dev == nullptr;
    hipStream_t st = (hipStream_t)stream;
    // batch > 1: one pass per row over the shared (union) index list; each row uses its own
    // x values.  Launches on one stream run in order, so they can share the workspace.
    for (int b = 0; b < batch; ++b) {
        const uint16_t *xb = (const uint16_t *)x_dev + (size_t)b * K;
        float *yb = y_dev + (size_t)b * M;
        hipError_t err;
        switch (c.waves) {
            case 1: err = launch<1>(dense, grid, st, (const uint8_t *)packed_dev, xb, idx_dev, count_dev, yb, partials, counters, (int)K, NG, c.splits, T); break;
            case 2: err = launch<2>(dense, grid, st, (const uint8_t *)packed_dev, xb, idx_dev, count_dev, yb, partials, counters, (int)K, NG, c.splits, T); break;
            default: err = launch<4>(dense, grid, st, (const uint8_t *)packed_dev, xb, idx_dev, count_dev, yb, partials, counters, (int)K, NG, c.splits, T); break;
        }
        if (err != hipSuccess) return SPQT_EHIP;
    }
    return SPQT_OK;
}

extern "C" int spqt_gemv(const void *packed_dev, int64_t M, int64_t K, int group, const void *x_dev,
                         int batch, const int32_t *idx_dev, const int32_t *count_dev, float *y_dev,
                         void *workspace_dev, size_t workspace_bytes, void *stream) {
    return spqt_gemv_ex(packed_dev, M, K, group, x_dev, batch, idx_dev, count_dev, y_dev, workspace_dev,
                        workspace_bytes, stream, nullptr);
}
