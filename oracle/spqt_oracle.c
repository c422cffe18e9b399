/*
 * CPU oracle for the sparse int4 GEMV path.  TEST INFRASTRUCTURE ONLY.
 *
 * This file is the slow, plain definition of what the GPU library must compute.  It is
 * used by the tests, by the smoke check and by the benchmark's cpu_baseline leg, and by
 * nothing else; the product library never calls it and shares no code with it.
 *
 * What it computes (paper Section 2, "activation sparsity": an entry of the hidden
 * state whose magnitude is under the threshold is treated as zero and its weight column
 * is skipped; Section 4.2.3: the non-sparse entries form an index array idx[0:n_ns]):
 *
 *   Wd[m][k] = scale[m][k/G] * q[m][k]                       (group-wise symmetric int4)
 *   keep[k]  = !(|x[k]| < threshold)                          (union over batch rows)
 *   idx      = ascending list of k with keep[k];  n_ns = its length
 *   y[m]     = sum over kept k, in increasing k, of Wd[m][k] * x[k]      (fp64)
 *
 * The sparse result is by definition the dense quantized GEMV applied to x with the
 * dropped entries zeroed, so the oracle is that definition written out: it dequantizes
 * the row-major weights, applies the mask and runs a naive dot product.  The zigzag
 * layout plays no part in the values; it only appears in the reference packer below,
 * which exists to check the library's packed bytes bit for bit.
 *
 * Every function here is pinned by tests that do not use this file's own formulas
 * (closed forms, library routines, brute force, exact-arithmetic cases); nothing is
 * "parity unpinned".
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* ---- number formats -------------------------------------------------------------- */

/* IEEE-754 binary16 bit pattern -> double, by the textbook field decomposition. */
double spqt_oracle_half_to_double(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int expo = (h >> 10) & 0x1F;
    int frac = h & 0x3FF;
    double v;
    if (expo == 0)
        v = ldexp((double)frac, -24);               /* zero and subnormals: frac * 2^-24 */
    else if (expo == 31)
        v = frac ? NAN : INFINITY;
    else
        v = ldexp(1.0 + (double)frac / 1024.0, expo - 15);
    return sign ? -v : v;
}

/* Source format: element (m,k) sits in byte k/2 of row m; even k in the low nibble, odd k
 * in the high nibble; the nibble is a two's-complement 4-bit integer in [-8, 7]. */
static int source_code(const uint8_t *q_rowmajor, int64_t K, int64_t m, int64_t k)
{
    uint8_t byte = q_rowmajor[m * (K / 2) + k / 2];
    int nib = (k % 2 == 0) ? (byte & 0x0F) : (byte >> 4);
    return nib >= 8 ? nib - 16 : nib;
}

/* ---- step 1: dequantize one row (no zigzag involved) ------------------------------ */

void spqt_oracle_dequant_row(const uint8_t *q_rowmajor, const uint16_t *scales, int64_t K,
                             int group, int64_t m, double *out_row)
{
    int64_t NG = K / group;
    for (int64_t k = 0; k < K; ++k) {
        double s = spqt_oracle_half_to_double(scales[m * NG + k / group]);
        out_row[k] = s * (double)source_code(q_rowmajor, K, m, k);
    }
}

/* ---- step 2: threshold mask (Section 2: sparse iff |x_i| < threshold) ------------- */

/* x: fp16 bits [batch][K].  keep[k] = 1 if ANY batch row has !(|x_b[k]| < thr).
 * The comparison is done in fp32 (fp16 -> fp32 is exact; thr is fp32).  NaN is kept. */
void spqt_oracle_mask(const uint16_t *x, int64_t K, int batch, float thr, uint8_t *keep)
{
    for (int64_t k = 0; k < K; ++k) {
        int any = 0;
        for (int b = 0; b < batch; ++b) {
            float xf = (float)spqt_oracle_half_to_double(x[(int64_t)b * K + k]);
            if (!(fabsf(xf) < thr))
                any = 1;
        }
        keep[k] = (uint8_t)any;
    }
}

/* ---- step 3: index list (Section 4.2.3: idx[0:n_ns]) ------------------------------ */

/* Writes the kept indices in ascending order; returns n_ns.  idx must hold K entries. */
int64_t spqt_oracle_gather(const uint16_t *x, int64_t K, int batch, float thr, int32_t *idx)
{
    uint8_t *keep = (uint8_t *)malloc((size_t)K);
    int64_t n = 0;
    spqt_oracle_mask(x, K, batch, thr, keep);
    for (int64_t k = 0; k < K; ++k)
        if (keep[k])
            idx[n++] = (int32_t)k;
    free(keep);
    return n;
}

/* ---- step 4: masked dot products --------------------------------------------------- */

/* y: fp64 [batch][M].  Each batch row uses its own x values on the shared kept set. */
void spqt_oracle_gemv(const uint8_t *q_rowmajor, const uint16_t *scales, int64_t M, int64_t K,
                      int group, const uint16_t *x, int batch, float thr, double *y)
{
    uint8_t *keep = (uint8_t *)malloc((size_t)K);
    double *xd = (double *)malloc(sizeof(double) * (size_t)K * (size_t)batch);
    spqt_oracle_mask(x, K, batch, thr, keep);
    for (int64_t i = 0; i < (int64_t)batch * K; ++i)
        xd[i] = spqt_oracle_half_to_double(x[i]);

#pragma omp parallel
    {
        double *row = (double *)malloc(sizeof(double) * (size_t)K);
#pragma omp for schedule(static)
        for (int64_t m = 0; m < M; ++m) {
            spqt_oracle_dequant_row(q_rowmajor, scales, K, group, m, row);
            for (int b = 0; b < batch; ++b) {
                double acc = 0.0;
                for (int64_t k = 0; k < K; ++k)
                    if (keep[k])
                        acc += row[k] * xd[(int64_t)b * K + k];
                y[(int64_t)b * M + m] = acc;
            }
        }
        free(row);
    }
    free(xd);
    free(keep);
}

/* Same, for a chosen list of output rows only (sampled checks at full size). */
void spqt_oracle_gemv_rows(const uint8_t *q_rowmajor, const uint16_t *scales, int64_t M,
                           int64_t K, int group, const uint16_t *x, int batch, float thr,
                           const int64_t *rows, int64_t n_rows, double *y_rows)
{
    uint8_t *keep = (uint8_t *)malloc((size_t)K);
    double *row = (double *)malloc(sizeof(double) * (size_t)K);
    (void)M;
    spqt_oracle_mask(x, K, batch, thr, keep);
    for (int64_t i = 0; i < n_rows; ++i) {
        spqt_oracle_dequant_row(q_rowmajor, scales, K, group, rows[i], row);
        for (int b = 0; b < batch; ++b) {
            double acc = 0.0;
            for (int64_t k = 0; k < K; ++k)
                if (keep[k])
                    acc += row[k] * spqt_oracle_half_to_double(x[(int64_t)b * K + k]);
            y_rows[(int64_t)b * n_rows + i] = acc;
        }
    }
    free(row);
    free(keep);
}

/* ---- load-balanced partition of the index list (Section 4.2.3, Figure 6) ---------- */

/* Part j of `parts` gets idx[begin:end); the parts are disjoint, cover [0, n_ns) in order
 * and their sizes differ by at most one (about n_ns / parts each). */
void spqt_oracle_partition(int64_t n_ns, int64_t parts, int64_t j, int64_t *begin, int64_t *end)
{
    *begin = (n_ns * j) / parts;
    *end = (n_ns * (j + 1)) / parts;
}

/* ---- reference packer: row-major source -> zigzag tiles ----------------------------
 *
 * The paper fixes the block order (Section 4.1.2: blocks are grouped along a column -
 * one block is 256 consecutive rows of one column - and the blocks are stored row-major:
 * all columns of block-row 0, then block-row 1, ...).  Everything finer is this build's
 * choice, because the quantization groups stay along K (no requantization):
 *
 *   R = 256 rows per tile, G columns per quantization group (128 in the workloads of record; the
 *   paper says other group sizes work the same way, Section 4.1.3, and G = 64 is the second one
 *   built: read 64 for 128 in the column range and the size of a chunk below),
 *   T = ceil(M / R) block-rows, NG = K / G groups.  When M is not a multiple of R the rows
 *   M .. R*T-1 of the last block-row do not exist; they are stored as weight 0 (code 8) under
 *   scale bits 0 (the paper states no rule for a ragged edge; zero padding is this build's).
 *   One chunk per (t, g), at byte offset (t*NG + g) * CH, CH = 2*R + G*R/2 = 16896.
 *     bytes [0, 512):              fp16 bits of scale[256 t + r][g], r = 0..255, little endian
 *     bytes [512 + 128 c + j]:     column k = 128 g + c (c = 0..127), j = 0..127:
 *                                  low nibble  = code of row 256 t + 2 j
 *                                  high nibble = code of row 256 t + 2 j + 1
 *                                  stored code = (q + 8) & 15   (offset binary)
 *
 * So one activation column's 256 weights of a block-row are one aligned 128-byte run and
 * the scales they need sit at the head of the same chunk.
 */
#define ZZ_R 256
#define ZZ_G 128
#define ZZ_CH (2 * ZZ_R + ZZ_G * ZZ_R / 2)

int64_t spqt_oracle_packed_bytes_g(int64_t M, int64_t K, int G)
{
    return ((M + ZZ_R - 1) / ZZ_R) * (K / G) * (int64_t)(2 * ZZ_R + G * ZZ_R / 2);
}

int64_t spqt_oracle_packed_bytes(int64_t M, int64_t K)
{
    return spqt_oracle_packed_bytes_g(M, K, ZZ_G);
}

static void set_nibble(uint8_t *byte, int high, int value)
{
    if (high)
        *byte = (uint8_t)((*byte & 0x0F) | ((value & 0x0F) << 4));
    else
        *byte = (uint8_t)((*byte & 0xF0) | (value & 0x0F));
}

static int get_nibble(uint8_t byte, int high)
{
    return high ? (byte >> 4) : (byte & 0x0F);
}

int spqt_oracle_pack_g(const uint8_t *q_rowmajor, const uint16_t *scales, int64_t M, int64_t K,
                       int G, uint8_t *out)
{
    if (M <= 0 || K <= 0 || (G != 64 && G != 128) || K % G)
        return -1;
    int64_t T = (M + ZZ_R - 1) / ZZ_R, NG = K / G, CH = 2 * ZZ_R + G * ZZ_R / 2;
    memset(out, 0, (size_t)spqt_oracle_packed_bytes_g(M, K, G));
    for (int64_t t = 0; t < T; ++t)
        for (int64_t g = 0; g < NG; ++g) {
            uint8_t *chunk = out + (t * NG + g) * CH;
            for (int r = 0; r < ZZ_R; ++r) {
                uint16_t s = (t * ZZ_R + r < M) ? scales[(t * ZZ_R + r) * NG + g] : 0;
                chunk[2 * r] = (uint8_t)(s & 0xFF);
                chunk[2 * r + 1] = (uint8_t)(s >> 8);
            }
            for (int c = 0; c < G; ++c)
                for (int j = 0; j < ZZ_R / 2; ++j)
                    for (int half = 0; half < 2; ++half) {
                        int64_t m = t * ZZ_R + 2 * j + half;
                        int64_t k = g * G + c;
                        int q = (m < M) ? source_code(q_rowmajor, K, m, k) : 0;
                        set_nibble(&chunk[512 + 128 * c + j], half, q + 8);
                    }
        }
    return 0;
}

int spqt_oracle_pack(const uint8_t *q_rowmajor, const uint16_t *scales, int64_t M, int64_t K,
                     uint8_t *out)
{
    return spqt_oracle_pack_g(q_rowmajor, scales, M, K, ZZ_G, out);
}

int spqt_oracle_unpack_g(const uint8_t *packed, int64_t M, int64_t K, int G, uint8_t *q_rowmajor,
                         uint16_t *scales)
{
    if (M <= 0 || K <= 0 || (G != 64 && G != 128) || K % G)
        return -1;
    int64_t T = (M + ZZ_R - 1) / ZZ_R, NG = K / G, CH = 2 * ZZ_R + G * ZZ_R / 2;
    memset(q_rowmajor, 0, (size_t)(M * (K / 2)));
    for (int64_t t = 0; t < T; ++t)
        for (int64_t g = 0; g < NG; ++g) {
            const uint8_t *chunk = packed + (t * NG + g) * CH;
            for (int r = 0; r < ZZ_R && t * ZZ_R + r < M; ++r)
                scales[(t * ZZ_R + r) * NG + g] =
                    (uint16_t)(chunk[2 * r] | ((uint16_t)chunk[2 * r + 1] << 8));
            for (int c = 0; c < G; ++c)
                for (int j = 0; j < ZZ_R / 2; ++j)
                    for (int half = 0; half < 2; ++half) {
                        int64_t m = t * ZZ_R + 2 * j + half;
                        int64_t k = g * G + c;
                        if (m >= M)
                            continue; /* padding row */
                        int q = get_nibble(chunk[512 + 128 * c + j], half) - 8; /* [-8,7] */
                        set_nibble(&q_rowmajor[m * (K / 2) + k / 2], (int)(k % 2), q);
                    }
        }
    return 0;
}

int spqt_oracle_unpack(const uint8_t *packed, int64_t M, int64_t K, uint8_t *q_rowmajor,
                       uint16_t *scales)
{
    return spqt_oracle_unpack_g(packed, M, K, ZZ_G, q_rowmajor, scales);
}

int spqt_oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* How many threads the row loops may use from now on (timing legs: one thread, then all); no arithmetic
 * depends on it - every output row is computed by one thread in the same order either way. */
void spqt_oracle_set_threads(int n)
{
#ifdef _OPENMP
    if (n >= 1) omp_set_num_threads(n);
#else
    (void)n;
#endif
}
