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
//   - the slice is consumed in passes of up to 128 columns that belong to ONE quantization
//     group (idx is ascending, so a group is a contiguous run of the list).  Per pass the
//     wave stages (byte offset, x) of its columns in LDS, so every lane fetches the pair for
//     its column with one broadcast LDS read per step.
//   - int4 -> float costs no conversion instruction: a stored code n in 0..15 masked in
//     place at bit 0..3 (or 4..7) of a 16-bit half IS the fp16 subnormal n*2^-24 (or
//     16n*2^-24), which v_fma_mix_f32 multiplies by a pre-scaled x*2^24 (x*2^20) into the fp32
//     accumulator - exact products, fp32 accumulation.  The offset-binary bias (stored =
//     q + 8) is removed by starting each pass's accumulators at -8 * sum of the lane's x.
//   - the group scale is applied once per (row, pass): y_acc += scale * acc.
//   - reduction: 8 column-lanes and WAVES wavefronts through LDS, then the S workgroups of a
//     block-row through a workspace; the last one to arrive adds the partials in fixed order
//     and writes y.  No floating-point atomics, so results are reproducible.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "spqt_internal.h"

namespace {

using namespace spqt;

typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kPassCols = 128;                 // most columns one pass stages (one group)
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

template <int WAVES, bool DENSE>
__global__ __launch_bounds__(WAVES * 64) void spqt_gemv_kernel(
    const uint8_t *__restrict__ packed, const uint16_t *__restrict__ x,
    const int32_t *__restrict__ idx, const int32_t *__restrict__ count, float *__restrict__ y,
    float *partials, int32_t *counters, int K, int NG, int S) {
    // Per wave: 8 KB.  During the main loop its first 1 KB stages (offset, x) pairs; after
    // the loop the whole 8 KB receives the wave's 64 x 32 partial sums.
    __shared__ __attribute__((aligned(16))) float lds[WAVES][8 * kTileRows];
    __shared__ int is_last;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int cg = lane >> 3;      // column of the step this lane reads
    const int seg = lane & 7;      // 32-row segment of the tile this lane reads
    const int t = blockIdx.x / S;  // block-row
    const int s = blockIdx.x - t * S;

    // Even split of the index list over the S*WAVES wavefronts of this block-row.
    const int n_ns = DENSE ? K : __builtin_amdgcn_readfirstlane(*count);
    const int parts = S * WAVES;
    const int part = s * WAVES + wave;
    int pos = (int)(((int64_t)n_ns * part) / parts);
    const int end = (int)(((int64_t)n_ns * (part + 1)) / parts);

    u32x2 *stage = reinterpret_cast<u32x2 *>(lds[wave]);
    const uint8_t *row_base = packed + (size_t)t * NG * kChunkBytes;

    float yacc[32];
#pragma unroll
    for (int i = 0; i < 32; ++i) yacc[i] = 0.0f;

    while (pos < end) {
        // ---- stage up to 128 kept columns that share the group of idx[pos] ---------------
        const int e0 = pos + lane, e1 = pos + 64 + lane;
        int k0 = -1, k1 = -1;
        if (e0 < end) k0 = DENSE ? e0 : idx[e0];
        if (e1 < end) k1 = DENSE ? e1 : idx[e1];
        const int g = __builtin_amdgcn_readfirstlane(k0) >> 7;
        const bool in0 = (k0 >> 7) == g, in1 = (k1 >> 7) == g;
        const int n = __builtin_amdgcn_readfirstlane(__popcll(__ballot(in0)) + __popcll(__ballot(in1)));

        float x0 = 0.0f, x1 = 0.0f;
        if (in0) x0 = half_bits_to_float(x[k0]) * kTwo24;
        if (in1) x1 = half_bits_to_float(x[k1]) * kTwo24;
        u32x2 s0v = {in0 ? (uint32_t)(k0 & (kGroup - 1)) * kColBytes : 0u, as_u32(x0)};
        u32x2 s1v = {in1 ? (uint32_t)(k1 & (kGroup - 1)) * kColBytes : 0u, as_u32(x1)};
        stage[lane] = s0v;
        stage[64 + lane] = s1v;

        // Sum of the (pre-scaled) x of the columns this lane will visit: columns 8u + cg.
        float z = x0 + x1;
        z += __shfl_xor(z, 8);
        z += __shfl_xor(z, 16);
        z += __shfl_xor(z, 32);           // lane l now holds the sum over columns = l mod 8
        z = __shfl(z, cg);
        const float bias = z * (-8.0f / kTwo24);

        const uint8_t *chunk = row_base + (size_t)g * kChunkBytes;
        // this lane's 32 scales (rows 32 seg .. 32 seg + 31), 64 bytes
        u32x4 sc[4];
#pragma unroll
        for (int i = 0; i < 4; ++i)
            sc[i] = *reinterpret_cast<const u32x4 *>(chunk + seg * 64 + i * 16);

        float acc[32];
#pragma unroll
        for (int i = 0; i < 32; ++i) acc[i] = bias;

        const uint8_t *cols = chunk + kScaleBytes + seg * 16;
        __builtin_amdgcn_wave_barrier();   // staging writes above, reads below: same wave, LDS is in order

        for (int c0 = 0; c0 < n; c0 += 64) {
            u32x4 w[8];
            float xl[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                w[u] = u32x4{0u, 0u, 0u, 0u};
                xl[u] = 0.0f;
                if (c0 + u * 8 < n) {                     // wave-uniform: skip empty steps
                    const int e = c0 + u * 8 + cg;
                    const u32x2 ox = stage[e];
                    xl[u] = as_float(ox.y);
                    if (e < n)
                        w[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(cols + ox.x));
                }
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                if (c0 + u * 8 < n) {
                    const float xh = xl[u] * 0.0625f;
                    fma_codes(w[u].x, xl[u], xh, acc + 0);
                    fma_codes(w[u].y, xl[u], xh, acc + 8);
                    fma_codes(w[u].z, xl[u], xh, acc + 16);
                    fma_codes(w[u].w, xl[u], xh, acc + 24);
                }
            }
        }
        __builtin_amdgcn_wave_barrier();

        // ---- apply the group scale once per row ------------------------------------------
#pragma unroll
        for (int i = 0; i < 4; ++i) {
#pragma unroll
            for (int d = 0; d < 4; ++d) {
                const f16x2 h = as_f16x2(sc[i][d]);
                const int r = i * 8 + d * 2;
                yacc[r] = __builtin_fmaf((float)h.x, acc[r], yacc[r]);
                yacc[r + 1] = __builtin_fmaf((float)h.y, acc[r + 1], yacc[r + 1]);
            }
        }
        pos += n;
    }

    // ---- reduce: 8 column-lanes x WAVES wavefronts, through LDS -------------------------
    // float index inside a wave's region: ((cg*8 + q)*8 + seg)*4 + j  <->  row 32 seg + 4 q + j
    __builtin_amdgcn_wave_barrier();
    f32x4 *mine = reinterpret_cast<f32x4 *>(lds[wave]);
#pragma unroll
    for (int q = 0; q < 8; ++q)
        mine[(cg * 8 + q) * 8 + seg] = f32x4{yacc[4 * q], yacc[4 * q + 1], yacc[4 * q + 2], yacc[4 * q + 3]};
    __syncthreads();

    // element e of the 256-entry tile vector in "LDS order"; its output row:
    auto row_of = [](int e) { return ((e >> 2) & 7) * 32 + (e >> 5) * 4 + (e & 3); };

    float *my_partial = partials + ((size_t)blockIdx.x) * kTileRows;
    for (int e = tid; e < kTileRows; e += WAVES * 64) {
        float sum = 0.0f;
#pragma unroll
        for (int w = 0; w < WAVES; ++w)
#pragma unroll
            for (int c = 0; c < 8; ++c) sum += lds[w][c * kTileRows + e];
        if (S == 1)
            y[(size_t)t * kTileRows + row_of(e)] = sum;
        else
            __hip_atomic_store(my_partial + e, sum, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    if (S == 1) return;

    // ---- combine the S workgroups of this block-row: last arrival adds in fixed order ----
    __threadfence();
    __syncthreads();
    if (tid == 0) {
        const int prev = __hip_atomic_fetch_add(counters + t, 1, __ATOMIC_ACQ_REL, __HIP_MEMORY_SCOPE_AGENT);
        is_last = (prev == S - 1);
    }
    __syncthreads();
    if (!is_last) return;
    __threadfence();
    const float *tile_partials = partials + (size_t)t * S * kTileRows;
    for (int e = tid; e < kTileRows; e += WAVES * 64) {
        float sum = 0.0f;
        for (int k = 0; k < S; ++k)
            sum += __hip_atomic_load(tile_partials + (size_t)k * kTileRows + e, __ATOMIC_RELAXED,
                                     __HIP_MEMORY_SCOPE_AGENT);
        y[(size_t)t * kTileRows + row_of(e)] = sum;
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
                  int32_t *counters, int K, int NG, int S) {
    if (dense)
        hipLaunchKernelGGL((spqt_gemv_kernel<WAVES, true>), dim3(grid), dim3(WAVES * 64), 0, stream,
                           packed, x, idx, count, y, partials, counters, K, NG, S);
    else
        hipLaunchKernelGGL((spqt_gemv_kernel<WAVES, false>), dim3(grid), dim3(WAVES * 64), 0, stream,
                           packed, x, idx, count, y, partials, counters, K, NG, S);
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
    const int grid = T * c.splits;
    const bool dense = idx_dev == nullptr;
    hipStream_t st = (hipStream_t)stream;
    // batch > 1: one pass per row over the shared (union) index list; each row uses its own
    // x values.  Launches on one stream run in order, so they can share the workspace.
    for (int b = 0; b < batch; ++b) {
        const uint16_t *xb = (const uint16_t *)x_dev + (size_t)b * K;
        float *yb = y_dev + (size_t)b * M;
        hipError_t err;
        switch (c.waves) {
            case 1: err = launch<1>(dense, grid, st, (const uint8_t *)packed_dev, xb, idx_dev, count_dev, yb, partials, counters, (int)K, NG, c.splits); break;
            case 2: err = launch<2>(dense, grid, st, (const uint8_t *)packed_dev, xb, idx_dev, count_dev, yb, partials, counters, (int)K, NG, c.splits); break;
            default: err = launch<4>(dense, grid, st, (const uint8_t *)packed_dev, xb, idx_dev, count_dev, yb, partials, counters, (int)K, NG, c.splits); break;
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
