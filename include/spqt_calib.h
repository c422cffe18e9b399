/*
 * libspqt_calib - three trivial kernels used only by the benchmark to put its numbers in
 * context: what a plain streaming read / copy reaches on this GPU, and what an empty launch
 * costs.  They are not part of the GEMV path and implement nothing from the paper; the copy
 * kernel of known size is also what hardware byte counters are scaled against.
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
/* Launches one empty workgroup. */
int spqt_calib_empty(void *stream);
#ifdef __cplusplus
}
#endif
#endif
