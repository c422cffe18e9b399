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

// Bytes reserved at the head of the workspace for the per-block-row epoch counters (two per
// 256 rows: the 8-bit layout's block-rows are 128 rows high).
inline size_t counter_bytes(int64_t M) {
    size_t n = (size_t)tiles(M) * 2 * sizeof(int32_t);
    return (n + 255) & ~(size_t)255;
}

// Bytes of one chunk (block-row t, group g) of the group layout: 256 fp16 scales + `group` column runs.
inline int chunk_bytes(int group) { return kScaleBytes + group * kColBytes; }

inline int check_shape(int64_t M, int64_t K, int group) {
    if (group != kGroup && group != kGroup / 2) return SPQT_ESHAPE;
    if (M <= 0 || K <= 0 || K % kGroup != 0) return SPQT_ESHAPE;
    if (M > (int64_t)1 << 24 || K > (int64_t)1 << 24) return SPQT_ESHAPE;
    return SPQT_OK;
}

}  // namespace spqt
#endif
