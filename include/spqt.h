/*
 * libspqt - batch-1 decode GEMV over group-wise int4 weights with dynamic activation
 * sparsity, for AMD MI355X (gfx950).  C ABI: plain pointers and sizes only.
 *
 * The three calls follow the paper's problem statement (Section 3.2, "The Operations"):
 * the model is converted once, offline, into the zigzag layout (spqt_pack); at every
 * decode GEMV the hidden state first goes through a sparse-index-collecting kernel with a
 * calibrated threshold (spqt_gather), and the index list together with the hidden state
 * is fed to the GEMV kernel that touches only the listed weight columns (spqt_gemv).
 *
 * Conventions
 *   - Every function returns SPQT_OK (0) or a negative spqt_status.  Nothing throws,
 *     aborts, or synchronizes a stream unless stated.  Argument errors are detected on the
 *     host before anything is launched.
 *   - "HOST" pointers are ordinary host memory; "DEVICE" pointers are device memory of the
 *     current HIP device.  The caller owns every buffer; the library keeps no state.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Device calls
 *     are asynchronous on that stream and never read device results back to the host:
 *     the kept count n_ns stays on the device between spqt_gather and spqt_gemv.
 *   - Shapes: W is M (outputs) x K (inputs).  1 <= M <= 2^24, K % 128 == 0, group 128 or 64,
 *     batch in 1..4; anything else is SPQT_ESHAPE.  M need not be a multiple of the block
 *     height: the last block-row is zero-padded in the packed form (the paper's claim of
 *     generality, Section 4.1.3, fixes no rule for a ragged edge; padding is this build's).
 *
 * Packed layout ("zigzag", paper Section 4.1.2: weights are grouped along a column - one
 * block is 256 consecutive rows of ONE column - and the blocks are stored row-major: all
 * columns of block-row 0, then block-row 1, ...).  The quantization groups stay along K
 * (the source is row-major group-128 int4 and is not requantized), so the unit of storage
 * is one chunk per (block-row t, group g):
 *
 *   (written for group = 128; with group = 64 - the paper's claim that other group sizes work the
 *    same way, Section 4.1.3 - read G = 64 for 128 in NG, in the column range of a chunk and in
 *    its size, 512 + 128 G = 8704)
 *     T = ceil(M/256), NG = K/128, chunk (t, g) at byte offset (t*NG + g) * 16896
 *       bytes [0, 512)          fp16 bits of scale[256t + r][g], r = 0..255, little endian
 *       bytes [512 + 128c + j]  column k = 128g + c, c = 0..127, j = 0..127:
 *                               low nibble  = code of row 256t + 2j
 *                               high nibble = code of row 256t + 2j + 1
 *                               stored code = (q + 8) & 15  (offset binary, q in [-8, 7])
 *     rows M .. 256T-1 (when M % 256 != 0): stored code 8 (weight 0) and scale bits 0
 *     total = T*NG*16896 bytes (= M*K/2 + M*NG*2 when M % 256 == 0).
 *
 * One activation column's 256 weights of a block-row are therefore one aligned 128-byte
 * run (a skipped column is a skipped cache line), and the scales of its group sit at the
 * head of the same chunk.
 */
#ifndef SPQT_H
#define SPQT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    SPQT_OK = 0,
    SPQT_EINVAL = -1, /* null pointer or bad scalar argument */
    SPQT_ESHAPE = -2, /* M, K, group or batch not supported */
    SPQT_EALIGN = -3, /* a device pointer is not aligned as required */
    SPQT_ESIZE = -4,  /* an output buffer or the workspace is too small */
    SPQT_EHIP = -5    /* the HIP runtime reported an error at launch */
} spqt_status;

#define SPQT_TILE_ROWS 256
#define SPQT_GROUP 128            /* default group size; 64 is accepted too */
#define SPQT_CHUNK_BYTES 16896    /* bytes of one chunk at group size 128 */
#define SPQT_MAX_BATCH 4
#define SPQT_MAX_SPLITS 64   /* most workgroups that may share one block-row */
#define SPQT_GATHER_MAX_K 65536

/* Human-readable name of a status code (static storage). */
const char *spqt_status_str(int status);

/* Size in bytes of the packed form of an M x K matrix (layout above). */
int spqt_packed_bytes(int64_t M, int64_t K, int group, size_t *out_bytes);

/* Size in bytes of the device workspace spqt_gemv needs for this shape: a 256-byte head plus, for
 * each of up to SPQT_MAX_SPLITS workgroups that may share a block-row, 256 x batch 64-bit words
 * {partial sum, tag} through which they hand their partial sums to the workgroup that writes y.
 * The workspace must be prepared ONCE with spqt_workspace_init before its first use.  The workgroup
 * that consumes a word puts it back to zero, so every call leaves the workspace all zeros: calls on
 * one stream, or replays of one graph, may share one workspace whatever their M, K, batch, launch
 * shape, kernel (dense / sparse / one launch) or layout (group, column-block, 8-bit), provided it is
 * large enough for each.  Two calls that may overlap in time (different streams) need two workspaces.
 * Word 0 of the head is a poison flag: should a reducer ever abandon its bounded wait (it cannot
 * while the device makes progress), it writes NaN, raises the flag, and every later call on that
 * workspace yields NaN until spqt_workspace_init is run on it again - a late word of the abandoned
 * call could otherwise be mistaken for a later call's. */
int spqt_workspace_bytes(int64_t M, int64_t K, int batch, size_t *out_bytes);

/* DEVICE, async.  Clears the whole workspace (head and exchange words) with a small fill
 * kernel, so it is safe under graph capture. */
int spqt_workspace_init(void *workspace_dev, size_t workspace_bytes, void *stream);

/* HOST, offline, once per matrix (Section 3.2: one-time conversion; Section 4.1.2: the
 * layout).  Pure nibble/byte permutation, no requantization.
 *   q_rowmajor       uint8[M][K/2]; element (m,k) in byte k/2, even k in the low nibble,
 *                    odd k in the high nibble, two's-complement int4.
 *   scales_rowmajor  uint16[M][K/group], IEEE fp16 bit patterns.
 *   out_packed       caller-owned, out_bytes >= spqt_packed_bytes (else SPQT_ESIZE);
 *                    fully overwritten. */
int spqt_pack(const uint8_t *q_rowmajor, const uint16_t *scales_rowmajor, int64_t M, int64_t K,
              int group, void *out_packed, size_t out_bytes);

/* HOST.  Exact inverse of spqt_pack. */
int spqt_unpack(const void *packed, int64_t M, int64_t K, int group, uint8_t *q_rowmajor,
                uint16_t *scales_rowmajor);

/* DEVICE, async.  Sparse index collection (Section 4.2.3, "Sparse index collecting kernel
 * design"; sparsity test of Section 2: an entry is sparse iff |x_i| < threshold).
 *   x_dev          fp16[batch][K], K <= SPQT_GATHER_MAX_K.  For batch > 1 a column is kept
 *                  if ANY row keeps it (union).
 *   threshold      fp32; the comparison is done in fp32.  |x| == threshold is kept, NaN is
 *                  kept, so threshold 0 keeps every column.
 *   idx_out_dev    int32, capacity K entries; receives the kept column indices in ASCENDING
 *                  order, contiguous from entry 0 (entries past n_ns are left untouched).
 *   count_out_dev  int32[1]; receives n_ns.
 * The result is deterministic (no atomics): the same input gives the same bytes. */
int spqt_gather(const void *x_dev, int64_t K, int batch, float threshold, int32_t *idx_out_dev,
                int32_t *count_out_dev, void *stream);

/* DEVICE, async.  spqt_gather for several activation rows that each keep their OWN set (the
 * paper expects a small beam to work, Section 3.3, without saying how the rows' sets combine;
 * spqt_gather's union lets every listed column contribute to every row).  Same idx and count
 * as spqt_gather (the union), and in the same launch a copy of x in which row b has the
 * entries it drops itself, |x[b][k]| < threshold, replaced by +0:
 *   x_masked_out_dev  fp16[batch][K], 16-byte aligned, must not overlap x (else SPQT_EINVAL).
 * Passing the copy instead of x to any GEMV entry point with this idx / count gives
 * y[b] = sum over the columns ROW b keeps - the batch-1 result of every row - at the cost of
 * one pass over the union of columns. */
int spqt_gather_rows(const void *x_dev, int64_t K, int batch, float threshold, int32_t *idx_out_dev,
                     int32_t *count_out_dev, void *x_masked_out_dev, void *stream);

/* Optional launch shape for spqt_gemv_ex (the two hyper-parameters of Section 4.2.2: how
 * many workgroups share a block-row, and how many wavefronts each holds).  0 = choose. */
typedef struct {
    int splits; /* workgroups per block-row, 1..SPQT_MAX_SPLITS (any integer) */
    int waves;  /* wavefronts per workgroup: 1, 2 or 4 */
    int flags;  /* 0, or SPQT_CFG_* bits */
} spqt_launch_cfg;

/* spqt_gemv_fused only - an ablation in the spirit of Section 6.3's "no load balancing"
 * variant: the sparsity test runs inside the kernel on static column ranges and a dropped
 * column is NOT compacted away - it keeps its slot in the wavefront's step with x = 0.
 * Skipping then saves memory traffic but no issue slots.  Same results as the default. */
#define SPQT_CFG_NO_COMPACTION 1

/* spqt_gemv_fused only - every wavefront of a block-row gets an EVEN share of the kept columns (Section
 * 4.2.3: about n_ns / (n1 * n2) each, however the kept columns are spread) instead of an equal column
 * range: every workgroup first counts the kept columns of x per 512-column stretch, which gives n_ns and
 * the column at which each share begins, and each wavefront then compacts the stretches of its share
 * into a small list in LDS as it goes.  For one launch shape the arithmetic is that of spqt_gather
 * followed by spqt_gemv, in the same order: the same y bit for bit.  The counting makes the kernel's
 * start about 1.5 microseconds longer than the index-list kernel's, and building the list costs per column
 * scanned: measured on 28672 x 8192 at 50 % it is faster than spqt_gather + spqt_gemv (by the saved
 * launch) and slower than the static ranges, on evenly spread and on clustered activations alike.  Needs K <= 32768 and x_dev
 * 16-byte aligned (else SPQT_EINVAL); not combinable with SPQT_CFG_NO_COMPACTION. */
#define SPQT_CFG_EVEN_SHARES 16

/* y_dev is IEEE fp16 [batch][M] instead of fp32: the fp32 result rounded to nearest even at the
 * final store (2-byte aligned).  Accumulation and the exchange of partial sums stay fp32. */
#define SPQT_CFG_Y_FP16 4

/* spqt_gemv_ex with an index list and one activation row only - an ablation of how the list is
 * consumed.  By default a pass of 64 column slots is 8 rows of 8 slots and only a ROW must hold
 * columns of one quantization group, so a group boundary wastes the rest of a row.  With this flag
 * the kernel that serves several activation rows is used: a whole pass holds columns of ONE group
 * (its 8 column-lanes are folded before the scale is applied), so a group boundary wastes the rest
 * of a pass - at 50 % sparsity nearly half of the slots.  Same results up to rounding order. */
#define SPQT_CFG_GROUP_PASSES 8

/* DEVICE, async.  y[b][m] = sum over the listed columns k of scale[m][k/group] * q[m][k] *
 * x[b][k], fp32 accumulation (Section 4.2.2 for the dense kernel, Section 4.2.3 for the
 * load-balanced sparse one: the index list is split evenly over all wavefronts that work
 * on a block-row).
 *   packed_dev     device copy of spqt_pack's output, 128-byte aligned (else SPQT_EALIGN).
 *   x_dev          fp16[batch][K].
 *   idx_dev        int32 kept-column list from spqt_gather (distinct columns, ascending), or NULL for
 *                  the dense kernel, which visits every column and reads neither idx nor count.  With one
 *                  activation row a list of n_ns == K entries is taken to be 0..K-1 without being read.
 *   count_dev      int32[1] n_ns on the device (ignored when idx_dev == NULL).
 *   y_dev          fp32[batch][M], fully overwritten (zeros when n_ns == 0).
 *                  Non-finite activations: a kept NaN or +-Inf in x[b] makes EVERY output of row b NaN.
 *                  (The stored codes are q + 8 and the bias is removed as -8 * sum of the kept x, so an
 *                  infinite x meets its opposite infinity; the definition w * x would give +-Inf, and NaN
 *                  only where q == 0.  Finite inputs are what the method is for; this pins the rest.)
 *   workspace_dev  >= spqt_workspace_bytes(M, K, batch) bytes, prepared by
 *                  spqt_workspace_init (else SPQT_ESIZE / SPQT_EINVAL).
 * Deterministic: partial sums are combined in a fixed order, no floating-point atomics.
 * The workgroup that combines a block-row waits for the others' partial sums; the wait is
 * bounded, and if it ever gave up (it cannot while the device makes progress) the affected
 * outputs are NaN rather than silently wrong. */
int spqt_gemv(const void *packed_dev, int64_t M, int64_t K, int group, const void *x_dev,
              int batch, const int32_t *idx_dev, const int32_t *count_dev, float *y_dev,
              void *workspace_dev, size_t workspace_bytes, void *stream);

/* Same, with an explicit launch shape and options (NULL cfg == spqt_gemv).  y_dev is fp32
 * [batch][M] unless cfg->flags has SPQT_CFG_Y_FP16. */
int spqt_gemv_ex(const void *packed_dev, int64_t M, int64_t K, int group, const void *x_dev,
                 int batch, const int32_t *idx_dev, const int32_t *count_dev, void *y_dev,
                 void *workspace_dev, size_t workspace_bytes, void *stream,
                 const spqt_launch_cfg *cfg);

/* DEVICE, async.  spqt_gemv for callers that cannot allocate device memory and therefore cannot bring
 * a workspace: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * Same arguments, kernels, launch shape and results as spqt_gemv; the exchange words live in a fixed
 * array of SPQT_STATIC_SCRATCH_BYTES inside the library's device image (every GPU the library runs on
 * holds its own copy until the process ends).  The call allocates and frees nothing.
 *   - SPQT_ESIZE when the default launch shape for (M, K, batch) needs more exchange words than the
 *     array holds: 256 + ceil(M/256) * 256 * splits * batch * 8 bytes, splits as spqt_default_cfg
 *     reports (a shape that runs with one workgroup per block-row needs none).  The default launch
 *     shapes keep block-rows x splits <= 512, so every shape fits with 1 or 2 activation rows; with
 *     3 or 4 rows the large ones (e.g. 8192 x 28672: 32 block-rows x 16 splits) do not.
 *   - All calls on one GPU share that GPU's array: calls that may overlap in time (different streams,
 *     different host threads) race on it and must use spqt_gemv with workspaces of their own.  Every
 *     call leaves the array all zeros, so successive calls may differ in shape.
 *   - The first call on a GPU looks the array's device address up (no allocation either); make that
 *     call outside graph capture. */
#define SPQT_STATIC_SCRATCH_BYTES ((2u << 20) + 256u)
int spqt_gemv_static(const void *packed_dev, int64_t M, int64_t K, int group, const void *x_dev,
                     int batch, const int32_t *idx_dev, const int32_t *count_dev, float *y_dev,
                     void *stream);

/* DEVICE, async.  Gather and GEMV in ONE launch, batch 1: the kernel applies the sparsity test of
 * Section 2 (sparse iff |x_i| < threshold, compared in fp32) to x itself, compacts the kept
 * columns of each 64-column stretch with a wavefront ballot, and multiplies - no index list
 * is written and n_ns is never materialised.  Same y as spqt_gather followed by spqt_gemv (the
 * summation order differs, so the last bits may).  Because the index list does not exist, the
 * work of a block-row is split into equal COLUMN ranges instead of equal shares of the list
 * (Section 4.2.3): balanced when the kept columns are spread evenly, as with iid activations;
 * SPQT_CFG_EVEN_SHARES selects the kernel that splits the kept columns evenly instead.
 * This is the combination the paper's threshold sharing aims at (Section 5: fewer index collections
 * per layer), taken to one collection per GEMV at no extra launch.
 * Arguments as for spqt_gemv_ex; cfg may be NULL; cfg->flags may hold SPQT_CFG_EVEN_SHARES,
 * SPQT_CFG_NO_COMPACTION, SPQT_CFG_Y_FP16. */
int spqt_gemv_fused(const void *packed_dev, int64_t M, int64_t K, int group, const void *x_dev,
                    float threshold, void *y_dev, void *workspace_dev, size_t workspace_bytes,
                    void *stream, const spqt_launch_cfg *cfg);

/* DEVICE, async.  spqt_gemv_fused for 2..4 activation rows that share one pass over the weights
 * (Section 3.3 expects small beams to work; batch == 1 forwards to spqt_gemv_fused).  A column is
 * visited if ANY row keeps it.
 *   x_dev      fp16[batch][K].
 *   own_sets   0: every row takes every visited column (the union, as spqt_gather + spqt_gemv do);
 *              non-zero: row b takes only the columns it keeps itself, |x[b][k]| >= threshold - the
 *              result spqt_gemv_fused gives for that row alone (as spqt_gather_rows + spqt_gemv do).
 *   y_dev      fp32 (or fp16 with SPQT_CFG_Y_FP16) [batch][M].
 *   cfg        NULL, or splits and SPQT_CFG_Y_FP16; this kernel always runs 4 wavefronts per
 *              workgroup (cfg->waves must be 0 or 4, else SPQT_EINVAL).
 * Workspace as for spqt_gemv with the same batch. */
int spqt_gemv_fused_rows(const void *packed_dev, int64_t M, int64_t K, int group, const void *x_dev,
                         int batch, float threshold, int own_sets, void *y_dev, void *workspace_dev,
                         size_t workspace_bytes, void *stream, const spqt_launch_cfg *cfg);

/* The launch shape spqt_gemv would pick for this shape (host only, no device access): sparse != 0
 * for a call with an index list, 0 for the dense kernel. */
int spqt_default_cfg(int64_t M, int64_t K, int batch, int sparse, spqt_launch_cfg *out);

#ifdef __cplusplus
}
#endif
#endif /* SPQT_H */
