/*
 * freescale_aux.h - what the library exports BESIDE the method: measurement aids (per-kernel event timing, host
 * phase times, the plain copy that bandwidth counters are calibrated with), the table initialiser of the
 * synthetic workloads, and the hook of the diagnostic workgroup tracer.  Nothing here computes a step of the
 * prioritized update; the operations and their schedules are declared in freescale.h.
 */
#ifndef FREESCALE_AUX_H
#define FREESCALE_AUX_H

#include "freescale.h"

#ifdef __cplusplus
extern "C" {
#endif

/* ---- per-kernel timing of fs_prioritized_step (measurement aid) ---------------------------- */

enum { FS_TIME_REDUCE = 0, FS_TIME_GATHER = 1, FS_TIME_UPDATE_CO = 2, FS_TIME_UPDATE_EX = 3, FS_TIME_KINDS = 4 };

/* slots > 0: one in `every` later steps (fs_prioritized_step, fs_prioritized_step_pipelined)
 * brackets its gather and its two fused reduce+update passes (FS_TIME_UPDATE_CO, FS_TIME_UPDATE_EX;
 * FS_TIME_REDUCE is not produced by the fused path) with HIP events on the stream each is
 * launched on (ring of `slots` sampled steps).  An event record costs the
 * host more than a kernel launch: sample sparsely when the steps themselves are being timed.
 * slots == 0 turns it off (the default) and frees the events. */
int fs_ctx_set_kernel_timing(fs_ctx *ctx, int slots, int every);

/* Waits for all streams, then writes the duration in milliseconds of kernel `which` for each of
 * the steps recorded since timing was enabled (oldest first, at most max_out and at most the
 * ring size) to the HOST array ms_out_host and their number to *n_out_host.  Enabling timing
 * again clears the ring. */
int fs_ctx_get_kernel_timing(fs_ctx *ctx, int which, float *ms_out_host, int max_out, int *n_out_host);

/* Host-side microseconds that fs_prioritized_step_pipelined has spent so far in: [0] waiting for
 * the side-stream thread, [1] recording the fork event and handing over the side work, [2] the
 * wait for the previous side work, [3] enqueueing priority pass and gather, [4] the index-stream
 * thread's enqueueing (fs_unique_ids_ahead), [5] the side-stream thread's enqueueing, [6] number
 * of calls.  Written to the HOST array out7_host; reset != 0 clears the counters. */
int fs_ctx_host_times(fs_ctx *ctx, double *out7_host, int reset);

/* ---- input generation and calibration helpers (not part of the method) ------------------- */

/* Fills a table with the counter-based integer-hash rule of the synthetic workloads:
 * e = row*dim + col; h = mix32(lo32(e) ^ mix32(hi32(e) + 0x9E3779B9));
 * fp32: ((h & 0xFFFF) - 32768) * 2^-22;  bf16: ((h & 0xFF) - 128) * 2^-14. */
int fs_init_table_hash(fs_ctx *ctx, void *table, int64_t num_rows, int32_t dim, fs_dtype dt, fs_stream stream);

/* Reads the rows rows[index[j], :] for j in [0, n) and throws them away (one folded word per wavefront goes to
 * sink [1024] uint32): what the memory system gives whole rows at indexed addresses with nothing else in the way -
 * the ceiling of the step's access pattern, measured beside the step.  rows [num_rows] of row_bytes bytes each
 * (a multiple of 16, at most 1024); an index outside [0, num_rows) reads row 0. */
int fs_stream_row_read(fs_ctx *ctx, const void *rows, int64_t num_rows, int32_t row_bytes, const int64_t *index,
                       int64_t n, uint32_t *sink, fs_stream stream);

/* Plain 16-byte-per-lane copy of n_bytes (multiple of 16) from src to dst: the calibration
 * kernel for bandwidth counters and the achievable-copy ceiling. */
int fs_stream_copy(fs_ctx *ctx, const void *src, void *dst, int64_t n_bytes, fs_stream stream);

#ifdef FS_TRACE
/* Diagnostic builds (-DFS_TRACE) only: every workgroup of the step's kernels appends its kind and its first and
 * last 100 MHz clock reading to buf_dev (zeroed device array of 64-bit words, word 1 = records per lane of the
 * buffer); NULL switches the trace off.  Synchronises the device. */
int fs_debug_trace(fs_ctx *ctx, void *buf_dev);
#endif

#ifdef __cplusplus
}
#endif
#endif /* FREESCALE_AUX_H */
