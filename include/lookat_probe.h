/*
 * lookat_probe.h -- measurement aid shipped with the LOOKAT library (not part of the method).
 *
 * The decode path is bound by the HBM read stream (the paper's own argument, Sec. 3.1 /
 * 3.5: bytes loaded per key decide the cost).  To state an achieved bandwidth against
 * what the device can actually deliver, the benchmark times this plain read kernel over
 * the same buffers the decode kernel streams.
 */
#ifndef LOOKAT_PROBE_H
#define LOOKAT_PROBE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Reads `bytes` bytes starting at `src` (device pointer, 16-byte aligned, bytes a
 * multiple of 16) once, with 16-byte loads, 32 bytes per thread, and folds them into a
 * checksum that is written to sink[0] only if it equals a value that seeded data
 * cannot produce in practice (so the reads cannot be optimised away and nothing is
 * written).  `sink` is a device pointer to at least 4 bytes.  Asynchronous on `stream`
 * (a hipStream_t as void*).  Returns 0, or a negative lookat_status from lookat.h.
 */
int lookat_probe_stream_read(const void *src, size_t bytes, uint32_t *sink, void *stream);

/*
 * Writes `bytes` bytes starting at `dst` (device pointer, 16-byte aligned, bytes a multiple of
 * 16) once, with 16-byte stores of the 32-bit pattern `word`, one per thread: the write-stream
 * counterpart, for the kernels whose cost is their output (the materialised tables of
 * lookat_build_lut with many queries, the score block of lookat_score_prefill).  Asynchronous on
 * `stream`.  Returns 0, or a negative lookat_status from lookat.h.
 */
int lookat_probe_stream_write(void *dst, size_t bytes, uint32_t word, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* LOOKAT_PROBE_H */
