// Internal helpers shared by the library's translation units (not part of the C ABI).
#ifndef SPQT_INTERNAL_H
#define SPQT_INTERNAL_H

#include <stdint.h>

#include "spqt.h"

namespace spqt {

constexpr int kTileRows = SPQT_TILE_ROWS;          // R: rows per zigzag tile
constexpr int kGroup = SPQT_GROUP;                 // G: columns per quantization group
constexpr int kScaleBytes = 2 * kTileRows;         // fp16 scales at the head of a chunk
constexpr int kColBytes = kTileRows / 2;           // one column of one tile: 128 bytes
constexpr int kChunkBytes = SPQT_CHUNK_BYTES;      // kScaleBytes + kGroup * kColBytes
static_assert(kChunkBytes == kScaleBytes + kGroup * kColBytes, "chunk size");

// Block-rows of a matrix with M rows; the last one is zero-padded when M is not a multiple of 256.
inline int64_t tiles(int64_t M) { return (M + kTileRows - 1) / kTileRows; }

// Bytes reserved at the head of the workspace: word 0 is the poison flag the reducers raise when a
// wait for partial sums is abandoned; the rest keeps the exchange words 256-byte aligned.
inline size_t counter_bytes(int64_t) { return 256; }

// Bytes of exchange words a launch with S workgroups per block-row really touches (64-bit words,
// `rows` outputs per block-row and activation row), head included.
inline size_t exchange_bytes(int64_t n_tiles, int rows, int S, int batch) {
    return 256 + (size_t)n_tiles * (size_t)rows * (size_t)S * (size_t)batch * 8;
}

// Bytes of one chunk (block-row t, group g) of the group layout: 256 fp16 scales + `group` column runs.
inline int chunk_bytes(int group) { return kScaleBytes + group * kColBytes; }

inline int check_shape(int64_t M, int64_t K, int group) {
    if (group != kGroup && group != kGroup / 2) return SPQT_ESHAPE;
    if (M <= 0 || K <= 0 || K % kGroup != 0) return SPQT_ESHAPE;
    if (M > (int64_t)1 << 24 || K > (int64_t)1 << 24) return SPQT_ESHAPE;
    return SPQT_OK;
}

enum class Kernel { dense, list_rows, list_groups, fused };

// Launch shape per kernel, measured on MI355X over the benchmark shapes at 50 % sparsity and dense.
inline void choose_cfg(int64_t M, int64_t K, int batch, Kernel kind, spqt_launch_cfg *out) {
    const int64_t T = tiles(M), NG = K / kGroup;
    const int waves = 4;
    int64_t S = 1;
    if (kind == Kernel::list_rows) {
        // Row-aligned passes (one activation row): fastest with about one workgroup of 4 wavefronts per
        // CU - at most 256 in total - and S any integer up to 16.  More workgroups only shorten every
        // wavefront's slice, and the fixed cost per wavefront (dependent prologue loads, pipeline fill,
        // fold, exchange of partial sums) outweighs the extra parallelism.
        S = 256 / T;
        S = S < 1 ? 1 : (S > 16 ? 16 : S);
        while (S > 1 && S * waves > 4 * NG) --S;
    } else {
        // The others: about 512 (sparse) / 1024 (dense) workgroups in total, S a power of two and at
        // most 16.  Several activation rows need enough accumulator registers that two wavefronts fit per
        // SIMD instead of three: 512 workgroups of 4 wavefronts is then the whole chip, once.
        // The dense batch-1 kernel on matrices large enough to be bandwidth-bound (>= 64 MB packed) is
        // fastest with one wavefront per SIMD: about 256 workgroups.
        const bool big = (size_t)M * (size_t)K / 2 >= ((size_t)64 << 20);
        const int64_t target = batch >= 2 ? 512 : (kind != Kernel::dense ? 512 : (big ? 256 : 1024));
        while (S * 2 <= 16 && S * 2 * T <= target) S *= 2;
        // keep at least a quarter of a quantization group per wavefront
        while (S > 1 && S * waves > 4 * NG) S /= 2;
    }
    out->splits = (int)S;
    out->waves = waves;
    out->flags = 0;
}

}  // namespace spqt
#endif
