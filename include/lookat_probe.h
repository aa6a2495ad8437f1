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

#include "lookat.h"

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

/*
 * The read stream in a chosen launch shape, to look for the shape that streams a buffer fastest (the
 * ceiling a streaming kernel is judged against must not share that kernel's launch head and tail):
 *   threads           workgroup size: 64, 128, 256, 512 or 1024
 *   loads_per_thread  16-byte loads a thread keeps in flight per round: 1, 2, 4, 8 or 16
 *   workgroups        0: as many as cover the buffer in one round (every thread reads once);
 *                     > 0: that many persistent workgroups
 *   contiguous        persistent workgroups only: 0 = rounds strided by the grid (at any time the grid
 *                     reads one contiguous window), 1 = every workgroup owns one contiguous share
 *   nontemporal       1 = loads carry the read-once hint
 * Other arguments and behaviour as lookat_probe_stream_read.  LOOKAT_ERR_UNSUPPORTED for other values.
 */
int lookat_probe_stream_read_shaped(const void *src, size_t bytes, uint32_t *sink, int32_t threads,
                                    int32_t loads_per_thread, int32_t workgroups, int32_t contiguous,
                                    int32_t nontemporal, void *stream);

/* A kernel that does nothing, `workgroups` x `threads`: back-to-back launches of it on one stream give the
 * launch interval of the device and runtime (the floor under any per-launch time measured that way). */
int lookat_probe_empty_launch(int32_t workgroups, int32_t threads, void *stream);

/*
 * lookat_attend_decode (paper Algorithm 1 after the table build; same arguments, same result) on a flat
 * launch geometry with the pieces of a (b,h) merged INSIDE the kernel: the 64-key tiles of all (b,h) form
 * one index space cut into equal shares, one per workgroup (a share may hold the tail of one (b,h), a whole
 * one and the head of the next); every piece of a shared (b,h) publishes (o, max, sum) in the workspace and
 * draws a ticket from that (b,h)'s counter, the last ticket merges and writes `out`.  num_splits = 0: equal
 * shares over the 256 compute units; >= 1: shares of ceil(tiles / num_splits) tiles.
 * A measurement aid: lookat_attend_decode (one range per workgroup, a second launch to merge) measured
 * faster on MI355X at every workload; this entry point keeps that comparison reproducible.
 *   workspace        lookat_probe_attend_decode_ticket_workspace_bytes() bytes, 16-byte aligned; its first
 *                    256-byte-rounded 4*B*H bytes are the ticket counters: ZERO them once after allocation
 *                    and whenever B*H changes (the kernel leaves them at zero)
 *   pieces_per_unit  host pointer or NULL: receives the most pieces a (b,h) is cut into
 * Supported: d_k in {32, 64, 128, 256}, m in {2, 4, 8, 16}.
 */
size_t lookat_probe_attend_decode_ticket_workspace_bytes(const lookat_shape *shape, int64_t L, int32_t num_splits);

int lookat_probe_attend_decode_ticket(const lookat_shape *shape, int64_t L,
                                      const float *lut,
                                      const uint8_t *codes, int64_t code_stride_bh,
                                      const void *values, int64_t value_stride_bh,
                                      float scale, int32_t num_splits,
                                      void *workspace, size_t workspace_bytes,
                                      float *out, float *scores_out,
                                      int32_t *pieces_per_unit,
                                      void *stream);

/*
 * lookat_score_prefill forced onto its lookup-and-sum kernel (per-query tables built and gathered in LDS,
 * paper Sec. 3.5 as written), whatever the shape: lookat_score_prefill itself scores blocks of 24 or more
 * queries as a dense product against the keys' centroids on the matrix cores.  Same arguments, results
 * and error behaviour as lookat_score_prefill; exists so that both kernels can be timed and checked against
 * the oracle on the same inputs.
 */
int lookat_probe_score_prefill_lookup(const lookat_shape *shape, int32_t T, int64_t L,
                                      const void *q, lookat_dtype q_dtype,
                                      const float *codebooks,
                                      const uint8_t *codes, int64_t code_stride_bh,
                                      float *scores,
                                      void *stream);

/*
 * lookat_decode_step with the number of batch entries a workgroup serves chosen by the caller instead of
 * by the library (see lookat_decode_step_entries_per_workgroup): 1 = one (b,h) per 512-thread workgroup;
 * 2 = one 1024-thread workgroup serves (b, h) and (b + 1, h), fetches the head's codebook rows (paper
 * Sec. 3.4 for the new key's codes, Sec. 3.5 for the tables) once and computes both entries' tables and
 * distances from them.  Same arguments, results (bit for bit) and error behaviour as lookat_decode_step;
 * 2 needs an even B and d_k = 64, or d_k = 128 with m > 2 (LOOKAT_ERR_UNSUPPORTED otherwise); any other
 * count: LOOKAT_ERR_SHAPE.
 * Exists so that both instances can be timed and checked on any shape.
 */
int lookat_probe_decode_step_entries(const lookat_shape *shape, int32_t entries_per_workgroup, int64_t L,
                                     const void *q, const void *k_new, lookat_dtype qk_dtype,
                                     const float *codebooks,
                                     uint8_t *codes, int64_t code_stride_bh,
                                     const void *values, int64_t value_stride_bh,
                                     float scale,
                                     float *out,
                                     void *stream);

#ifdef __cplusplus
}
#endif
#endif /* LOOKAT_PROBE_H */
