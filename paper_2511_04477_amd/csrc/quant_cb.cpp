// Host-side quantizer for the column-block variant of the zigzag layout.
//
// Paper Section 4.1.2: the quantization groups run along a column (a superblock is 256
// consecutive rows of one column, in blocks of 32 as in Section 4.1.1) and superblocks are
// stored row-major by superblock-row; Section 5: the model is converted offline.  The rule
// (symmetric int4, one fp16 scale per 32-row block) and the byte layout are documented in
// spqt_colblock.h.
#include <algorithm>
#include <cmath>
#include <cstring>
#include <thread>
#include <vector>

#include "spqt_colblock.h"
#include "spqt_internal.h"

using namespace spqt;

namespace {

constexpr int kBlockRows = SPQT_CB_BLOCK_ROWS;
constexpr int kBlocksPerTile = kTileRows / kBlockRows;           // 8
constexpr int kCbScaleBytes = kGroup * kBlocksPerTile * 2;       // 2048
constexpr int kCbChunkBytes = SPQT_CB_CHUNK_BYTES;
static_assert(kCbChunkBytes == kCbScaleBytes + kGroup * kColBytes, "chunk size");

// fp32 -> fp16 bits, round to nearest even (finite inputs; overflow gives infinity).
uint16_t float_to_half_bits(float f) {
    uint32_t u;
    std::memcpy(&u, &f, 4);
    const uint32_t sign = (u >> 16) & 0x8000u;
    const uint32_t a = u & 0x7FFFFFFFu;
    if (a >= 0x47800000u) return (uint16_t)(sign | 0x7C00u);      // >= 65536 (or inf/nan): infinity
    if (a < 0x38800000u) {                                        // below the smallest normal half
        if (a < 0x33000000u) return (uint16_t)sign;               // < 2^-25: zero
        const int shift = 126 - (int)(a >> 23);                   // 14..24
        const uint32_t mant = (a & 0x7FFFFFu) | 0x800000u;
        const uint32_t q = mant >> shift, rem = mant & ((1u << shift) - 1u), half = 1u << (shift - 1);
        return (uint16_t)(sign | (q + ((rem > half || (rem == half && (q & 1u))) ? 1u : 0u)));
    }
    const uint32_t q = (a - 0x38000000u) >> 13, rem = a & 0x1FFFu;
    const uint32_t r = q + ((rem > 0x1000u || (rem == 0x1000u && (q & 1u))) ? 1u : 0u);
    return (uint16_t)(sign | r);                                  // a carry into the exponent is correct
}

float half_bits_to_float(uint16_t h) {
    const uint32_t sign = (uint32_t)(h & 0x8000u) << 16;
    const uint32_t e = (h >> 10) & 0x1Fu, m = h & 0x3FFu;
    uint32_t u;
    if (e == 0) {
        if (m == 0) {
            u = sign;
        } else {
            const float v = (float)m * (1.0f / 16777216.0f);      // m * 2^-24, exact
            std::memcpy(&u, &v, 4);
            u |= sign;
        }
    } else if (e == 31) {
        u = sign | 0x7F800000u | (m << 13);
    } else {
        u = sign | ((e + 112u) << 23) | (m << 13);
    }
    float f;
    std::memcpy(&f, &u, 4);
    return f;
}

template <class F>
void for_each_tile_row(int64_t T, F fn) {
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

int check_cb_shape(int64_t M, int64_t K) { return check_shape(M, K, kGroup); }

// When M is not a multiple of 256 the last block-row is quantized as if the missing rows
// held zero weights: a zero-filled copy [256][K] of that block-row (empty otherwise).
std::vector<float> padded_last_tile(const float *w, int64_t M, int64_t K) {
    std::vector<float> p;
    const int64_t have = M % kTileRows;
    if (have == 0) return p;
    p.assign((size_t)kTileRows * K, 0.0f);
    std::memcpy(p.data(), w + (size_t)(M - have) * K, (size_t)have * K * sizeof(float));
    return p;
}

}  // namespace

extern "C" int spqt_cb_packed_bytes(int64_t M, int64_t K, size_t *out_bytes) {
    if (!out_bytes) return SPQT_EINVAL;
    if (int rc = check_cb_shape(M, K)) return rc;
    *out_bytes = (size_t)tiles(M) * (size_t)(K / kGroup) * (size_t)kCbChunkBytes;
    return SPQT_OK;
}

extern "C" int spqt_cb_quantize(const float *w, int64_t M, int64_t K, void *out_packed, size_t out_bytes) {
    if (!w || !out_packed) return SPQT_EINVAL;
    size_t need = 0;
    if (int rc = spqt_cb_packed_bytes(M, K, &need)) return rc;
    if (out_bytes < need) return SPQT_ESIZE;
    const int64_t T = tiles(M), NC = K / kGroup;
    uint8_t *out = (uint8_t *)out_packed;
    const std::vector<float> padded = padded_last_tile(w, M, K);
    const float *last = padded.empty() ? nullptr : padded.data();
    for_each_tile_row(T, [=](int64_t t) {
        float scale[kBlocksPerTile][kGroup];
        for (int64_t c = 0; c < NC; ++c) {
            uint8_t *chunk = out + (size_t)(t * NC + c) * kCbChunkBytes;
            const float *tile = (last && t == T - 1 ? last : w + (size_t)t * kTileRows * K) + (size_t)c * kGroup;   // row stride K
            for (int b = 0; b < kBlocksPerTile; ++b) {
                float amax[kGroup];
                for (int j = 0; j < kGroup; ++j) amax[j] = 0.0f;
                for (int r = 0; r < kBlockRows; ++r) {
                    const float *row = tile + (size_t)(b * kBlockRows + r) * K;
                    for (int j = 0; j < kGroup; ++j) amax[j] = std::max(amax[j], std::fabs(row[j]));
                }
                for (int j = 0; j < kGroup; ++j) {
                    const uint16_t h = float_to_half_bits(amax[j] / 7.0f);
                    chunk[16 * j + 2 * b] = (uint8_t)(h & 0xFF);
                    chunk[16 * j + 2 * b + 1] = (uint8_t)(h >> 8);
                    scale[b][j] = half_bits_to_float(h);
                }
            }
            uint8_t *codes = chunk + kCbScaleBytes;
            for (int r = 0; r < kTileRows; ++r) {
                const float *row = tile + (size_t)r * K;
                const float *sc = scale[r / kBlockRows];
                for (int j = 0; j < kGroup; ++j) {
                    int q = 0;
                    if (sc[j] > 0.0f) {
                        const float v = std::nearbyintf(row[j] / sc[j]);   // round half to even
                        q = (int)std::min(7.0f, std::max(-8.0f, v));
                    }
                    uint8_t &byte = codes[128 * j + r / 2];
                    const uint8_t n = (uint8_t)(q + 8);
                    byte = (r & 1) ? (uint8_t)((byte & 0x0F) | (n << 4)) : n;   // even row first: overwrites
                }
            }
        }
    });
    return SPQT_OK;
}

extern "C" int spqt_cb_dequantize(const void *packed, int64_t M, int64_t K, float *w_out) {
    if (!packed || !w_out) return SPQT_EINVAL;
    if (int rc = check_cb_shape(M, K)) return rc;
    const int64_t T = tiles(M), NC = K / kGroup;
    const uint8_t *in = (const uint8_t *)packed;
    for_each_tile_row(T, [=](int64_t t) {
        for (int64_t c = 0; c < NC; ++c) {
            const uint8_t *chunk = in + (size_t)(t * NC + c) * kCbChunkBytes;
            float *tile = w_out + (size_t)t * kTileRows * K + (size_t)c * kGroup;
            for (int j = 0; j < kGroup; ++j) {
                for (int r = 0; r < kTileRows && t * kTileRows + r < M; ++r) {
                    const int b = r / kBlockRows;
                    const uint16_t h = (uint16_t)(chunk[16 * j + 2 * b] | (chunk[16 * j + 2 * b + 1] << 8));
                    const uint8_t byte = chunk[kCbScaleBytes + 128 * j + r / 2];
                    const int q = (int)((byte >> (4 * (r & 1))) & 15) - 8;
                    tile[(size_t)r * K + j] = (float)q * half_bits_to_float(h);
                }
            }
        }
    });
    return SPQT_OK;
}

// ---------------------------------------------------------------------------------------------
// K-quant flavour (paper Section 4.1.1: Q4_K's superblock of eight 32-weight blocks with 6-bit block
// scales and minima under two 16-bit superblock scales), on the same column-block geometry.  The
// decode rule is the format's; the min/max quantizer is this build's own.  See spqt_colblock.h.

namespace {

// the 96-bit field string of a superblock header: sc_0..sc_7 then m_0..m_7, 6 bits each
void put_fields(uint8_t *dst12, const int *sc, const int *m) {
    uint64_t lo = 0, hi = 0;      // bits 0..63 and 64..95
    auto put = [&](int pos, uint64_t v) {
        if (pos < 64) {
            lo |= v << pos;
            if (pos > 58) hi |= v >> (64 - pos);
        } else {
            hi |= v << (pos - 64);
        }
    };
    for (int b = 0; b < 8; ++b) put(6 * b, (uint64_t)sc[b]);
    for (int b = 0; b < 8; ++b) put(48 + 6 * b, (uint64_t)m[b]);
    for (int i = 0; i < 8; ++i) dst12[i] = (uint8_t)(lo >> (8 * i));
    for (int i = 0; i < 4; ++i) dst12[8 + i] = (uint8_t)(hi >> (8 * i));
}

void get_fields(const uint8_t *src12, int *sc, int *m) {
    uint64_t lo = 0, hi = 0;
    for (int i = 0; i < 8; ++i) lo |= (uint64_t)src12[i] << (8 * i);
    for (int i = 0; i < 4; ++i) hi |= (uint64_t)src12[8 + i] << (8 * i);
    auto get = [&](int pos) -> int {
        uint64_t v = pos < 64 ? (lo >> pos) : (hi >> (pos - 64));
        if (pos < 64 && pos > 58) v |= hi << (64 - pos);
        return (int)(v & 63u);
    };
    for (int b = 0; b < 8; ++b) sc[b] = get(6 * b);
    for (int b = 0; b < 8; ++b) m[b] = get(48 + 6 * b);
}

}  // namespace

extern "C" int spqt_cbk_quantize(const float *w, int64_t M, int64_t K, void *out_packed, size_t out_bytes) {
    if (!w || !out_packed) return SPQT_EINVAL;
    size_t need = 0;
    if (int rc = spqt_cb_packed_bytes(M, K, &need)) return rc;
    if (out_bytes < need) return SPQT_ESIZE;
    const int64_t T = tiles(M), NC = K / kGroup;
    uint8_t *out = (uint8_t *)out_packed;
    const std::vector<float> padded = padded_last_tile(w, M, K);
    const float *last = padded.empty() ? nullptr : padded.data();
    for_each_tile_row(T, [=](int64_t t) {
        std::vector<float> se_v((size_t)kBlocksPerTile * kGroup), me_v((size_t)kBlocksPerTile * kGroup);
        for (int64_t c = 0; c < NC; ++c) {
            uint8_t *chunk = out + (size_t)(t * NC + c) * kCbChunkBytes;
            const float *tile = (last && t == T - 1 ? last : w + (size_t)t * kTileRows * K) + (size_t)c * kGroup;
            for (int j = 0; j < kGroup; ++j) {
                float scale_b[kBlocksPerTile], min_b[kBlocksPerTile];
                float smax = 0.0f, mmax = 0.0f;
                for (int b = 0; b < kBlocksPerTile; ++b) {
                    float lo = 0.0f, hi = 0.0f;
                    for (int r = 0; r < kBlockRows; ++r) {
                        const float v = tile[(size_t)(b * kBlockRows + r) * K + j];
                        lo = std::min(lo, v);
                        hi = std::max(hi, v);
                    }
                    scale_b[b] = (hi - lo) / 15.0f;
                    min_b[b] = 0.0f - lo;      // +0 for an all-zero block
                    smax = std::max(smax, scale_b[b]);
                    mmax = std::max(mmax, min_b[b]);
                }
                const uint16_t dh = float_to_half_bits(smax / 63.0f), mh = float_to_half_bits(mmax / 63.0f);
                const float d = half_bits_to_float(dh), dm = half_bits_to_float(mh);
                int sc[kBlocksPerTile], mq[kBlocksPerTile];
                for (int b = 0; b < kBlocksPerTile; ++b) {
                    sc[b] = d > 0.0f ? (int)std::min(63.0f, std::max(0.0f, std::nearbyintf(scale_b[b] / d))) : 0;
                    mq[b] = dm > 0.0f ? (int)std::min(63.0f, std::max(0.0f, std::nearbyintf(min_b[b] / dm))) : 0;
                    se_v[(size_t)b * kGroup + j] = d * (float)sc[b];
                    me_v[(size_t)b * kGroup + j] = dm * (float)mq[b];
                }
                uint8_t *head = chunk + 16 * j;
                head[0] = (uint8_t)(dh & 0xFF);
                head[1] = (uint8_t)(dh >> 8);
                head[2] = (uint8_t)(mh & 0xFF);
                head[3] = (uint8_t)(mh >> 8);
                put_fields(head + 4, sc, mq);
            }
            uint8_t *codes = chunk + kCbScaleBytes;
            for (int r = 0; r < kTileRows; ++r) {
                const float *row = tile + (size_t)r * K;
                const float *se = &se_v[(size_t)(r / kBlockRows) * kGroup], *me = &me_v[(size_t)(r / kBlockRows) * kGroup];
                for (int j = 0; j < kGroup; ++j) {
                    int q = 0;
                    if (se[j] > 0.0f) {
                        const float v = std::nearbyintf((row[j] + me[j]) / se[j]);
                        q = (int)std::min(15.0f, std::max(0.0f, v));
                    }
                    uint8_t &byte = codes[128 * j + r / 2];
                    byte = (r & 1) ? (uint8_t)((byte & 0x0F) | (q << 4)) : (uint8_t)q;
                }
            }
        }
    });
    return SPQT_OK;
}

extern "C" int spqt_cbk_dequantize(const void *packed, int64_t M, int64_t K, float *w_out) {
    if (!packed || !w_out) return SPQT_EINVAL;
    if (int rc = check_cb_shape(M, K)) return rc;
    const int64_t T = tiles(M), NC = K / kGroup;
    const uint8_t *in = (const uint8_t *)packed;
    for_each_tile_row(T, [=](int64_t t) {
        for (int64_t c = 0; c < NC; ++c) {
            const uint8_t *chunk = in + (size_t)(t * NC + c) * kCbChunkBytes;
            float *tile = w_out + (size_t)t * kTileRows * K + (size_t)c * kGroup;
            for (int j = 0; j < kGroup; ++j) {
                const uint8_t *head = chunk + 16 * j;
                const float d = half_bits_to_float((uint16_t)(head[0] | (head[1] << 8)));
                const float dm = half_bits_to_float((uint16_t)(head[2] | (head[3] << 8)));
                int sc[kBlocksPerTile], mq[kBlocksPerTile];
                get_fields(head + 4, sc, mq);
                for (int r = 0; r < kTileRows && t * kTileRows + r < M; ++r) {
                    const int b = r / kBlockRows;
                    const uint8_t byte = chunk[kCbScaleBytes + 128 * j + r / 2];
                    const int q = (byte >> (4 * (r & 1))) & 15;
                    tile[(size_t)r * K + j] = (d * (float)sc[b]) * (float)q - dm * (float)mq[b];
                }
            }
        }
    });
    return SPQT_OK;
}

// ---- 8-bit flavour: block-rows of 128 rows, codes stored as q + 128 ---------------------------------

namespace {

constexpr int kRows8 = SPQT_CB8_TILE_ROWS;
constexpr int kBlocks8 = kRows8 / kBlockRows;                    // 4
constexpr int kScaleBytes8 = kGroup * 2 * kBlocks8;              // 1024
constexpr int kChunkBytes8 = SPQT_CB8_CHUNK_BYTES;
static_assert(kChunkBytes8 == kScaleBytes8 + kGroup * kRows8, "8-bit chunk size");

inline int64_t tiles8(int64_t M) { return (M + kRows8 - 1) / kRows8; }

}  // namespace

extern "C" int spqt_cb8_packed_bytes(int64_t M, int64_t K, size_t *out_bytes) {
    if (!out_bytes) return SPQT_EINVAL;
    if (int rc = check_cb_shape(M, K)) return rc;
    *out_bytes = (size_t)tiles8(M) * (size_t)(K / kGroup) * (size_t)kChunkBytes8;
    return SPQT_OK;
}

extern "C" int spqt_cb8_quantize(const float *w, int64_t M, int64_t K, void *out_packed, size_t out_bytes) {
    if (!w || !out_packed) return SPQT_EINVAL;
    size_t need = 0;
    if (int rc = spqt_cb8_packed_bytes(M, K, &need)) return rc;
    if (out_bytes < need) return SPQT_ESIZE;
    const int64_t T = tiles8(M), NC = K / kGroup;
    uint8_t *out = (uint8_t *)out_packed;
    for_each_tile_row(T, [=](int64_t t) {
        for (int64_t c = 0; c < NC; ++c) {
            uint8_t *chunk = out + (size_t)(t * NC + c) * kChunkBytes8;
            for (int j = 0; j < kGroup; ++j) {
                const int64_t k = c * kGroup + j;
                for (int b = 0; b < kBlocks8; ++b) {
                    // rows past M count as zero weights
                    float v[kBlockRows];
                    float amax = 0.0f;
                    for (int r = 0; r < kBlockRows; ++r) {
                        const int64_t m = t * kRows8 + b * kBlockRows + r;
                        v[r] = m < M ? w[(size_t)m * K + k] : 0.0f;
                        amax = std::max(amax, std::fabs(v[r]));
                    }
                    const uint16_t h = float_to_half_bits(amax / 127.0f);
                    chunk[8 * j + 2 * b] = (uint8_t)(h & 0xFF);
                    chunk[8 * j + 2 * b + 1] = (uint8_t)(h >> 8);
                    const float sc = half_bits_to_float(h);
                    for (int r = 0; r < kBlockRows; ++r) {
                        int q = 0;
                        if (sc > 0.0f) q = (int)std::min(127.0f, std::max(-128.0f, std::nearbyintf(v[r] / sc)));
                        chunk[kScaleBytes8 + 128 * j + b * kBlockRows + r] = (uint8_t)(q + 128);
                    }
                }
            }
        }
    });
    return SPQT_OK;
}

extern "C" int spqt_cb8_dequantize(const void *packed, int64_t M, int64_t K, float *w_out) {
    if (!packed || !w_out) return SPQT_EINVAL;
    if (int rc = check_cb_shape(M, K)) return rc;
    const int64_t T = tiles8(M), NC = K / kGroup;
    const uint8_t *in = (const uint8_t *)packed;
    for_each_tile_row(T, [=](int64_t t) {
        for (int64_t c = 0; c < NC; ++c) {
            const uint8_t *chunk = in + (size_t)(t * NC + c) * kChunkBytes8;
            for (int j = 0; j < kGroup; ++j)
                for (int r = 0; r < kRows8 && t * kRows8 + r < M; ++r) {
                    const int b = r / kBlockRows;
                    const uint16_t h = (uint16_t)(chunk[8 * j + 2 * b] | (chunk[8 * j + 2 * b + 1] << 8));
                    const int q = (int)chunk[kScaleBytes8 + 128 * j + r] - 128;
                    w_out[(size_t)(t * kRows8 + r) * K + c * kGroup + j] = (float)q * half_bits_to_float(h);
                }
        }
    });
    return SPQT_OK;
}

// ---- 2-bit flavour: block-rows of 512 rows, four mid-rise levels (c - 1.5) * s ------------------------

namespace {

constexpr int kRows2 = SPQT_CB2_TILE_ROWS;
constexpr int kBlocks2 = kRows2 / kBlockRows;                    // 16
constexpr int kScaleBytes2 = kGroup * 2 * kBlocks2;              // 4096
constexpr int kChunkBytes2 = SPQT_CB2_CHUNK_BYTES;
static_assert(kChunkBytes2 == kScaleBytes2 + kGroup * (kRows2 / 4), "2-bit chunk size");

inline int64_t tiles2(int64_t M) { return (M + kRows2 - 1) / kRows2; }

}  // namespace

extern "C" int spqt_cb2_packed_bytes(int64_t M, int64_t K, size_t *out_bytes) {
    if (!out_bytes) return SPQT_EINVAL;
    if (int rc = check_cb_shape(M, K)) return rc;
    *out_bytes = (size_t)tiles2(M) * (size_t)(K / kGroup) * (size_t)kChunkBytes2;
    return SPQT_OK;
}

extern "C" int spqt_cb2_quantize(const float *w, int64_t M, int64_t K, void *out_packed, size_t out_bytes) {
    if (!w || !out_packed) return SPQT_EINVAL;
    size_t need = 0;
    if (int rc = spqt_cb2_packed_bytes(M, K, &need)) return rc;
    if (out_bytes < need) return SPQT_ESIZE;
    const int64_t T = tiles2(M), NC = K / kGroup;
    uint8_t *out = (uint8_t *)out_packed;
    for_each_tile_row(T, [=](int64_t t) {
        for (int64_t c = 0; c < NC; ++c) {
            uint8_t *chunk = out + (size_t)(t * NC + c) * kChunkBytes2;
            for (int j = 0; j < kGroup; ++j) {
                const int64_t k = c * kGroup + j;
                for (int b = 0; b < kBlocks2; ++b) {
                    // rows past M count as zero weights
                    float v[kBlockRows];
                    float amax = 0.0f;
                    for (int r = 0; r < kBlockRows; ++r) {
                        const int64_t m = t * kRows2 + b * kBlockRows + r;
                        v[r] = m < M ? w[(size_t)m * K + k] : 0.0f;
                        amax = std::max(amax, std::fabs(v[r]));
                    }
                    const uint16_t h = float_to_half_bits(amax / 1.5f);
                    chunk[32 * j + 2 * b] = (uint8_t)(h & 0xFF);
                    chunk[32 * j + 2 * b + 1] = (uint8_t)(h >> 8);
                    const float sc = half_bits_to_float(h);
                    // four rows to a byte, row 4 i + e in bits 2 e, 2 e + 1
                    for (int r = 0; r < kBlockRows; r += 4) {
                        unsigned byte = 0;
                        for (int e = 0; e < 4; ++e) {
                            int code = 0;
                            if (sc > 0.0f) code = (int)std::min(3.0f, std::max(0.0f, std::nearbyintf(v[r + e] / sc + 1.5f)));
                            byte |= (unsigned)code << (2 * e);
                        }
                        chunk[kScaleBytes2 + 128 * j + (b * kBlockRows + r) / 4] = (uint8_t)byte;
                    }
                }
            }
        }
    });
    return SPQT_OK;
}

extern "C" int spqt_cb2_dequantize(const void *packed, int64_t M, int64_t K, float *w_out) {
    if (!packed || !w_out) return SPQT_EINVAL;
    if (int rc = check_cb_shape(M, K)) return rc;
    const int64_t T = tiles2(M), NC = K / kGroup;
    const uint8_t *in = (const uint8_t *)packed;
    for_each_tile_row(T, [=](int64_t t) {
        for (int64_t c = 0; c < NC; ++c) {
            const uint8_t *chunk = in + (size_t)(t * NC + c) * kChunkBytes2;
            for (int j = 0; j < kGroup; ++j)
                for (int r = 0; r < kRows2 && t * kRows2 + r < M; ++r) {
                    const int b = r / kBlockRows;
                    const uint16_t h = (uint16_t)(chunk[32 * j + 2 * b] | (chunk[32 * j + 2 * b + 1] << 8));
                    const int code = (chunk[kScaleBytes2 + 128 * j + r / 4] >> (2 * (r & 3))) & 3;
                    w_out[(size_t)(t * kRows2 + r) * K + c * kGroup + j] = ((float)code - 1.5f) * half_bits_to_float(h);
                }
        }
    });
    return SPQT_OK;
}
