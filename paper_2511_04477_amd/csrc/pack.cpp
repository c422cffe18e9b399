// Host-side repacker: row-major group-128 int4 (fp16 scales) <-> zigzag column tiles.
//
// Paper Section 4.1.2: weights are grouped along a column (one block = 256 consecutive
// rows of one column) while blocks are stored row-major by block-row.  This is a pure
// byte/nibble permutation of an already-quantized matrix (no requantization), so it
// round-trips bit-exactly.  The destination layout is documented in spqt.h.
#include <algorithm>
#include <cstring>
#include <thread>
#include <vector>

#include "spqt_internal.h"

using namespace spqt;

namespace {

// Run fn(t) for every block-row t on a few host threads (block-rows are independent).
template <class F>
void for_each_block_row(int64_t T, F fn) {
    unsigned hw = std::thread::hardware_concurrency();
    int nthreads = (int)std::max<int64_t>(1, std::min<int64_t>(std::min<unsigned>(hw ? hw : 1, 16u), T));
    if (nthreads == 1) {
        for (int64_t t = 0; t < T; ++t) fn(t);
        return;
    }
    std::vector<std::thread> pool;
    for (int w = 0; w < nthreads; ++w)
        pool.emplace_back([=]() {
            for (int64_t t = w; t < T; t += nthreads) fn(t);
        });
    for (auto &th : pool) th.join();
}

}  // namespace

extern "C" const char *spqt_status_str(int status) {
    switch (status) {
        case SPQT_OK: return "SPQT_OK";
        case SPQT_EINVAL: return "SPQT_EINVAL: null pointer or bad scalar argument";
        case SPQT_ESHAPE: return "SPQT_ESHAPE: need M >= 1, K % 128 == 0, group 64 or 128, batch in 1..4";
        case SPQT_EALIGN: return "SPQT_EALIGN: device pointer not aligned as required";
        case SPQT_ESIZE: return "SPQT_ESIZE: buffer or workspace too small";
        case SPQT_EHIP: return "SPQT_EHIP: HIP runtime error at launch";
        default: return "SPQT_?: unknown status";
    }
}

extern "C" int spqt_packed_bytes(int64_t M, int64_t K, int group, size_t *out_bytes) {
    if (!out_bytes) return SPQT_EINVAL;
    if (int rc = check_shape(M, K, group)) return rc;
    *out_bytes = (size_t)tiles(M) * (size_t)(K / group) * (size_t)chunk_bytes(group);
    return SPQT_OK;
}

extern "C" int spqt_pack(const uint8_t *q_rowmajor, const uint16_t *scales_rowmajor, int64_t M,
                         int64_t K, int group, void *out_packed, size_t out_bytes) {
    if (!q_rowmajor || !scales_rowmajor || !out_packed) return SPQT_EINVAL;
    size_t need = 0;
    if (int rc = spqt_packed_bytes(M, K, group, &need)) return rc;
    if (out_bytes < need) return SPQT_ESIZE;

    const int64_t T = tiles(M), NG = K / group, row_bytes = K / 2;
    const int G = group, CH = chunk_bytes(group);
    uint8_t *out = static_cast<uint8_t *>(out_packed);
    // Rows M .. 256 T - 1 of the last block-row do not exist: they are stored as weight 0
    // (code 8) under scale bits 0, so any kernel may treat them like real rows.
    const std::vector<uint8_t> zero_row((size_t)row_bytes, 0);

    for_each_block_row(T, [=](int64_t t) {
        for (int64_t g = 0; g < NG; ++g) {
            uint8_t *chunk = out + (size_t)(t * NG + g) * CH;
            // head of the chunk: the 256 scales of this (block-row, group), as stored bits
            uint16_t sc[kTileRows];
            for (int r = 0; r < kTileRows; ++r)
                sc[r] = t * kTileRows + r < M ? scales_rowmajor[(t * kTileRows + r) * NG + g] : (uint16_t)0;
            std::memcpy(chunk, sc, kScaleBytes);   // host is little-endian x86-64
            uint8_t *cols = chunk + kScaleBytes;
            // two source rows at a time fill byte j of every column run of the chunk
            for (int j = 0; j < kTileRows / 2; ++j) {
                const int64_t m = t * kTileRows + 2 * j;
                const uint8_t *even = (m < M ? q_rowmajor + (size_t)m * row_bytes : zero_row.data()) + g * (G / 2);
                const uint8_t *odd = (m + 1 < M ? q_rowmajor + (size_t)(m + 1) * row_bytes : zero_row.data()) + g * (G / 2);
                for (int b = 0; b < G / 2; ++b) {
                    // source byte b carries columns 2b (low) and 2b+1 (high) of one row;
                    // two's complement -> offset binary is a flip of the nibble's top bit
                    uint8_t e = even[b] ^ 0x88, o = odd[b] ^ 0x88;
                    cols[(2 * b) * kColBytes + j] = (uint8_t)((e & 0x0F) | (o << 4));
                    cols[(2 * b + 1) * kColBytes + j] = (uint8_t)((e >> 4) | (o & 0xF0));
                }
            }
        }
    });
    return SPQT_OK;
}

extern "C" int spqt_unpack(const void *packed, int64_t M, int64_t K, int group, uint8_t *q_rowmajor,
                           uint16_t *scales_rowmajor) {
    if (!packed || !q_rowmajor || !scales_rowmajor) return SPQT_EINVAL;
    if (int rc = check_shape(M, K, group)) return rc;

    const int64_t T = tiles(M), NG = K / group, row_bytes = K / 2;
    const int G = group, CH = chunk_bytes(group);
    const uint8_t *in = static_cast<const uint8_t *>(packed);

    for_each_block_row(T, [=](int64_t t) {
        for (int64_t g = 0; g < NG; ++g) {
            const uint8_t *chunk = in + (size_t)(t * NG + g) * CH;
            uint16_t sc[kTileRows];
            std::memcpy(sc, chunk, kScaleBytes);
            for (int r = 0; r < kTileRows && t * kTileRows + r < M; ++r)
                scales_rowmajor[(t * kTileRows + r) * NG + g] = sc[r];
            const uint8_t *cols = chunk + kScaleBytes;
            for (int j = 0; j < kTileRows / 2; ++j) {
                const int64_t m = t * kTileRows + 2 * j;
                if (m >= M) break;                               // padding rows are not written back
                uint8_t *even = q_rowmajor + (size_t)m * row_bytes + g * (G / 2);
                uint8_t *odd = even + row_bytes;
                for (int b = 0; b < G / 2; ++b) {
                    uint8_t c0 = cols[(2 * b) * kColBytes + j];      // rows 2j (low), 2j+1 (high) of column 2b
                    uint8_t c1 = cols[(2 * b + 1) * kColBytes + j];  // same rows of column 2b+1
                    even[b] = (uint8_t)(((c0 & 0x0F) | (c1 << 4)) ^ 0x88);
                    if (m + 1 < M) odd[b] = (uint8_t)(((c0 >> 4) | (c1 & 0xF0)) ^ 0x88);
                }
            }
        }
    });
    return SPQT_OK;
}
