/*
 * libspqt - column-block variant of the zigzag layout: the quantization groups themselves
 * run along a column, as in the paper (Section 4.1.2: one superblock is 256 consecutive
 * rows of ONE column, split like Q4_K into eight blocks of 32 weights, Section 4.1.1;
 * superblocks are stored row-major by superblock-row), and the model is re-quantized
 * offline into this form (Section 5).  A skipped activation column then skips its scales
 * too, and the GEMV needs no per-group bookkeeping: the scale of a block is folded into the
 * activation value before the multiply.
 *
 * Where the paper leaves the encoding open this build keeps what it uses elsewhere:
 * symmetric int4, fp16 scales (one per 32-row block; 4.5 bits per weight like Q4_K):
 *
 *     scale  s = fp16( max|w| over the block / 7 )          fp32 arithmetic, round to nearest even
 *     code   q = clamp( rint( w / float(s) ), -8, 7 )       fp32, round half to even;
 *            q = 0 for every weight of a block whose scale rounds to zero
 *     value  q * float(s)
 *
 * Packed form ("ZZ-CB32"): T = ceil(M/256) superblock-rows, NC = K/128 chunks of 128 columns;
 * chunk (t, c) at byte offset (t*NC + c) * 18432:
 *     bytes [16 j + 2 b], j = 0..127, b = 0..7   fp16 scale (little endian) of rows
 *                                                256t + 32b .. +31 of column 128c + j
 *     bytes [2048 + 128 j + i], i = 0..127       column 128c + j: low nibble = code of row
 *                                                256t + 2i, high nibble = row 256t + 2i + 1,
 *                                                stored code = q + 8
 * total = T*NC*18432 bytes (= M*K/2 + M*K/16 when M % 256 == 0).  When M is not a multiple of
 * 256 the quantizers treat the missing rows of the last superblock-row as zero weights and the
 * dequantizers and kernels never write them back.  Conventions (status codes, HOST/DEVICE,
 * streams, shapes M >= 1 and K % 128 == 0) are those of spqt.h.
 */
#ifndef SPQT_COLBLOCK_H
#define SPQT_COLBLOCK_H

#include "spqt.h"

#ifdef __cplusplus
extern "C" {
#endif

#define SPQT_CB_BLOCK_ROWS 32
#define SPQT_CB_CHUNK_BYTES 18432

/* Size in bytes of the packed column-block form of an M x K matrix. */
int spqt_cb_packed_bytes(int64_t M, int64_t K, size_t *out_bytes);

/* HOST, offline, once per matrix (Section 5: the offline quantizer that emits the zigzag
 * layout).  Quantizes fp32 weights by the rule above and writes the packed form.
 *   w_rowmajor   float[M][K], finite values.
 *   out_packed   caller-owned, out_bytes >= spqt_cb_packed_bytes (else SPQT_ESIZE); fully
 *                overwritten. */
int spqt_cb_quantize(const float *w_rowmajor, int64_t M, int64_t K, void *out_packed, size_t out_bytes);

/* HOST.  The values the packed form stands for: w_out[m][k] = q * float(s), float[M][K]. */
int spqt_cb_dequantize(const void *packed, int64_t M, int64_t K, float *w_out);

/* DEVICE, async.  y[b][m] = sum over the listed columns k of q[m][k] * s[m/32][k] * x[b][k], fp32
 * accumulation (Section 4.2.2 / 4.2.3: same block-row parallelism and even split of the index
 * list as spqt_gemv).
 *   packed_dev     device copy of spqt_cb_quantize's output, 128-byte aligned.
 *   x_dev          fp16[batch][K], batch in 1..SPQT_MAX_BATCH (rows share the union index list
 *                  and one pass over the weights).
 *   idx_dev        int32 kept-column list from spqt_gather (ascending), or NULL for the
 *                  dense kernel, which visits every column and reads neither idx nor count.
 *   count_dev      int32[1] n_ns on the device (ignored when idx_dev == NULL).
 *   y_dev          fp32[batch][M] (fp16 with SPQT_CFG_Y_FP16), fully overwritten.
 *   workspace_dev  as for spqt_gemv: >= spqt_workspace_bytes(M, K, batch), prepared once by
 *                  spqt_workspace_init.
 *   cfg            launch shape or NULL (flags: 0 or SPQT_CFG_Y_FP16).
 * Deterministic; same bounded wait and NaN-on-give-up behaviour as spqt_gemv. */
int spqt_cb_gemv(const void *packed_dev, int64_t M, int64_t K, const void *x_dev, int batch,
                 const int32_t *idx_dev, const int32_t *count_dev, void *y_dev, void *workspace_dev,
                 size_t workspace_bytes, void *stream, const spqt_launch_cfg *cfg);

/* DEVICE, async.  Gather and GEMV in ONE launch (the column-block counterpart of
 * spqt_gemv_fused): the kernel applies the sparsity test of Section 2 to x itself on static
 * 64-column ranges, compacts the kept columns with a wavefront ballot and multiplies; no index
 * list exists.  Same y as spqt_gather followed by spqt_cb_gemv up to summation order. */
int spqt_cb_gemv_fused(const void *packed_dev, int64_t M, int64_t K, const void *x_dev, float threshold,
                       void *y_dev, void *workspace_dev, size_t workspace_bytes, void *stream,
                       const spqt_launch_cfg *cfg);

/* ---- K-quant flavour of the column-block layout --------------------------------------------
 * Section 4.1.1 names the paper's format: Q4_K - a superblock of 256 weights in eight blocks of 32,
 * 4-bit codes, 6-bit block scales, a 16-bit superblock scale and min - and gives no more.  The per-block
 * 6-bit minimum, the second 16-bit superblock scale for the minima and the decode formula
 * (d * sc_b) * q - dmin * m_b with q in 0..15 are this build's reading, taken from the public K-quant
 * format.  Here the superblock is 256 consecutive rows of one column (Section 4.1.2).  The quantizer is this build's own
 * plain min/max rule, in fp32 with round to nearest even:
 *     lo_b = min(min w, 0), hi_b = max(max w, 0), scale_b = (hi_b - lo_b) / 15, min_b = 0 - lo_b
 *     d = fp16(max_b scale_b / 63), dmin = fp16(max_b min_b / 63)
 *     sc_b = clamp(rint(scale_b / d), 0, 63), m_b = clamp(rint(min_b / dmin), 0, 63)   (0 if d / dmin is 0)
 *     q = clamp(rint((w + dmin*m_b) / (d*sc_b)), 0, 15)                                (0 if d*sc_b is 0)
 * Packed form: the geometry of ZZ-CB32 (chunk (t, c) at (t*NC + c) * 18432); the 16 header bytes
 * of column j at [16 j]: d (fp16), dmin (fp16), then a 96-bit little-endian bit string sc_0..sc_7,
 * m_0..m_7 of 6 bits each; codes at [2048 + 128 j + i] as plain nibbles (low = row 2i). */
int spqt_cbk_quantize(const float *w_rowmajor, int64_t M, int64_t K, void *out_packed, size_t out_bytes);

/* HOST.  w_out[m][k] = (d * sc_b) * q - dmin * m_b, float[M][K]. */
int spqt_cbk_dequantize(const void *packed, int64_t M, int64_t K, float *w_out);

/* DEVICE, async.  As spqt_cb_gemv (batch 1..SPQT_MAX_BATCH), on spqt_cbk_quantize's output. */
int spqt_cbk_gemv(const void *packed_dev, int64_t M, int64_t K, const void *x_dev, int batch,
                  const int32_t *idx_dev, const int32_t *count_dev, void *y_dev, void *workspace_dev,
                  size_t workspace_bytes, void *stream, const spqt_launch_cfg *cfg);

/* DEVICE, async.  As spqt_cb_gemv_fused (gather and GEMV in one launch, batch 1), on
 * spqt_cbk_quantize's output. */
int spqt_cbk_gemv_fused(const void *packed_dev, int64_t M, int64_t K, const void *x_dev, float threshold,
                        void *y_dev, void *workspace_dev, size_t workspace_bytes, void *stream,
                        const spqt_launch_cfg *cfg);

/* ---- 8-bit flavour of the column-block layout ("ZZ-CB32-W8") --------------------------------
 * Section 4.1.3 states that the layout carries over to other bit-widths without giving one.  This
 * reading keeps one activation column's weights of a block-row in ONE 128-byte run, so a
 * block-row is 128 rows high; blocks stay 32 rows with one fp16 scale (fp32, round to nearest even):
 *     s = fp16(max|w| / 127),  q = clamp(rint(w / float(s)), -128, 127)  (0 if s is 0),  value q * float(s)
 * Packed form: T = ceil(M/128), NC = K/128, chunk (t, c) at (t*NC + c) * 17408:
 *     bytes [8 j + 2 b], b = 0..3         fp16 scale of rows 128t + 32b .. +31 of column 128c + j
 *     bytes [1024 + 128 j + i], i < 128   code of row 128t + i of column 128c + j, stored q + 128
 * Rows past M in the last block-row are quantized as zero weights and never written back. */
#define SPQT_CB8_TILE_ROWS 128
#define SPQT_CB8_CHUNK_BYTES 17408
int spqt_cb8_packed_bytes(int64_t M, int64_t K, size_t *out_bytes);
/* HOST, offline.  As spqt_cb_quantize, by the 8-bit rule above. */
int spqt_cb8_quantize(const float *w_rowmajor, int64_t M, int64_t K, void *out_packed, size_t out_bytes);
/* HOST.  w_out[m][k] = q * float(s), float[M][K]. */
int spqt_cb8_dequantize(const void *packed, int64_t M, int64_t K, float *w_out);
/* DEVICE, async.  As spqt_cb_gemv with batch 1, on spqt_cb8_quantize's output.  The workspace
 * has the size spqt_workspace_bytes(M, K, 1) gives and may be the one the other entry points use. */
int spqt_cb8_gemv(const void *packed_dev, int64_t M, int64_t K, const void *x_dev, const int32_t *idx_dev,
                  const int32_t *count_dev, void *y_dev, void *workspace_dev, size_t workspace_bytes,
                  void *stream, const spqt_launch_cfg *cfg);
/* DEVICE, async.  As spqt_cb_gemv for 1..SPQT_MAX_BATCH activation rows (Section 3.3: small beams) that share
 * the union index list and one pass over the weights: x_dev fp16[batch][K], y_dev [batch][M], workspace of
 * spqt_workspace_bytes(M, K, batch). */
int spqt_cb8_gemv_rows(const void *packed_dev, int64_t M, int64_t K, const void *x_dev, int batch,
                       const int32_t *idx_dev, const int32_t *count_dev, void *y_dev, void *workspace_dev,
                       size_t workspace_bytes, void *stream, const spqt_launch_cfg *cfg);
/* DEVICE, async.  As spqt_cb_gemv_fused (gather and GEMV in one launch, batch 1: the sparsity test of
 * Section 2 runs inside the kernel on static 64-column ranges), on spqt_cb8_quantize's output. */
int spqt_cb8_gemv_fused(const void *packed_dev, int64_t M, int64_t K, const void *x_dev, float threshold,
                        void *y_dev, void *workspace_dev, size_t workspace_bytes, void *stream,
                        const spqt_launch_cfg *cfg);

/* ---- 2-bit flavour of the column-block layout ("ZZ-CB32-W2") --------------------------------
 * Section 4.1.3 names 2 to 8 bits as the widths the layout carries over to and gives no format.  This
 * reading again keeps one activation column's weights of a block-row in ONE 128-byte run, so a
 * block-row is 512 rows high; blocks stay 32 rows with one fp16 scale.  Four levels cannot hold a zero
 * level and a symmetric range at once; the rule is the plain mid-rise one, levels -1.5 s, -0.5 s,
 * +0.5 s, +1.5 s (fp32, round to nearest even, ties of rint to even):
 *     s = fp16(max|w| / 1.5),  c = clamp(rint(w / float(s) + 1.5), 0, 3)  (0 if s is 0),  value (c - 1.5) * float(s)
 * Packed form: T = ceil(M/512), NC = K/128, chunk (t, c) at (t*NC + c) * 20480:
 *     bytes [32 j + 2 b], b = 0..15         fp16 scale of rows 512t + 32b .. +31 of column 128c + j
 *     bytes [4096 + 128 j + i], i < 128     codes of rows 512t + 4i + e, e = 0..3, of column 128c + j,
 *                                           row 4i + e in bits 2e, 2e + 1
 * total = T*NC*20480 bytes (2.5 bits per weight when M % 512 == 0).  Rows past M in the last
 * block-row are quantized as zero weights (code 0 under a zero scale) and never written back. */
#define SPQT_CB2_TILE_ROWS 512
#define SPQT_CB2_CHUNK_BYTES 20480
#define SPQT_CB2_MAX_BATCH 3
int spqt_cb2_packed_bytes(int64_t M, int64_t K, size_t *out_bytes);
/* HOST, offline.  As spqt_cb_quantize, by the 2-bit rule above. */
int spqt_cb2_quantize(const float *w_rowmajor, int64_t M, int64_t K, void *out_packed, size_t out_bytes);
/* HOST.  w_out[m][k] = (c - 1.5) * float(s), float[M][K]. */
int spqt_cb2_dequantize(const void *packed, int64_t M, int64_t K, float *w_out);
/* DEVICE, async.  As spqt_cb_gemv with batch 1, on spqt_cb2_quantize's output:
 * y[m] = sum over the listed columns k of (c[m][k] - 1.5) * s[m/32][k] * x[k], fp32 accumulation.
 * cfg->splits at most 16, cfg->waves 1, 2 or 4 (else SPQT_EINVAL).  The workspace has the size
 * spqt_workspace_bytes(M, K, 1) gives and may be the one the other entry points use. */
int spqt_cb2_gemv(const void *packed_dev, int64_t M, int64_t K, const void *x_dev, const int32_t *idx_dev,
                  const int32_t *count_dev, void *y_dev, void *workspace_dev, size_t workspace_bytes,
                  void *stream, const spqt_launch_cfg *cfg);
/* DEVICE, async.  As spqt_cb8_gemv_rows, for 1..SPQT_CB2_MAX_BATCH activation rows (SPQT_ESHAPE beyond: a lane
 * keeps 64 accumulators per row); cfg as for spqt_cb2_gemv. */
int spqt_cb2_gemv_rows(const void *packed_dev, int64_t M, int64_t K, const void *x_dev, int batch,
                       const int32_t *idx_dev, const int32_t *count_dev, void *y_dev, void *workspace_dev,
                       size_t workspace_bytes, void *stream, const spqt_launch_cfg *cfg);
/* DEVICE, async.  As spqt_cb_gemv_fused (gather and GEMV in one launch, batch 1), on spqt_cb2_quantize's
 * output; cfg as for spqt_cb2_gemv. */
int spqt_cb2_gemv_fused(const void *packed_dev, int64_t M, int64_t K, const void *x_dev, float threshold,
                        void *y_dev, void *workspace_dev, size_t workspace_bytes, void *stream,
                        const spqt_launch_cfg *cfg);

#ifdef __cplusplus
}
#endif
#endif /* SPQT_COLBLOCK_H */
