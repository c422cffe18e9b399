/*
 * libspqt_calib - kernels used only by the benchmark to put its numbers in context: what a plain
 * streaming read / copy reaches on this GPU, what an empty launch costs, and a GEMV on the
 * row-major source layout as the comparison the paper measures against.  None is on the GEMV
 * path; the copy kernel of known size is also what hardware byte counters are scaled against.
 * All pointers are DEVICE pointers; calls are asynchronous on `stream` (hipStream_t as void*).
 * Return 0 on success, -1 on bad arguments, -5 if the launch failed.
 */
#ifndef SPQT_CALIB_H
#define SPQT_CALIB_H
#include <stddef.h>
#include <stdint.h>
#ifdef __cplusplus
extern "C" {
#endif
/* Reads `bytes` (multiple of 16, 16-byte aligned) once with `blocks` workgroups of 256 lanes
 * (0 = pick), `unroll` independent 16-byte loads per lane in flight (1, 2, 4, 8 or 16).
 * sink_dev (one uint32) is written only if the XOR of everything read has an unlikely value. */
int spqt_calib_read(const void *src_dev, size_t bytes, uint32_t *sink_dev, int blocks, int unroll,
                    void *stream);
/* Same read, but each wavefront owns one contiguous slice of the buffer and walks it 1 KB at a
 * time, `unroll` (2, 4, 8, 16) loads in flight - the order a GEMV wavefront reads its columns in. */
int spqt_calib_read_blocked(const void *src_dev, size_t bytes, uint32_t *sink_dev, int blocks, int unroll,
                            void *stream);
/* Reads only the 128-byte lines whose numbers are listed in lines_dev (ascending int32, n_lines
 * of them; src_dev 128-byte aligned), 8 lines per wavefront load, each wavefront a contiguous
 * slice of the list - the sparse GEMV's access pattern with no arithmetic. */
int spqt_calib_read_lines(const void *src_dev, const int32_t *lines_dev, int n_lines, uint32_t *sink_dev,
                          int blocks, int unroll, void *stream);
/* Copies `bytes` (multiple of 16) from src to dst: reads bytes, writes bytes. */
int spqt_calib_copy(void *dst_dev, const void *src_dev, size_t bytes, int blocks, void *stream);
/* Comparison kernel (paper Section 6.1 "row-wise" baseline and Section 6.3 "naive skipping"): int4
 * GEMV read straight from the row-major source format of spqt_pack - q uint8[M][K/2] (even k in the
 * low nibble, two's complement), scales fp16[M][K/128] - batch 1, y fp32[M].  skip == 0: dense.
 * skip != 0: every weight's activation is tested against `threshold` where the weight is used
 * (sparse iff |x| < threshold); the result equals the masked GEMV, but no byte of a row-major line
 * can be skipped.  K % 128 == 0, K <= 32768; q 16-byte aligned. */
int spqt_calib_rowmajor_gemv(const void *q_rowmajor_dev, const void *scales_dev, int64_t M, int64_t K,
                             const void *x_dev, float threshold, int skip, float *y_dev, void *stream);
/* Launches one empty workgroup. */
int spqt_calib_empty(void *stream);
#ifdef __cplusplus
}
#endif
#endif
