/*
 * stx_measure.h — measurement aids of libstx: live timing of the library's kernels with HIP events, and two
 * kernels of known memory traffic against which a profiler's hardware byte counters are scaled.  Not part of
 * the method's boundary (stx.h); benchmarks and profiling scripts use them.
 */
#ifndef STX_MEASURE_H
#define STX_MEASURE_H

#include "stx.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Live timing of one kernel, for benchmarks.  stx_profile_kernel: from now on every launch of the kernel
 * called `kernel_name` (e.g. "k_forward_stacked", "k_seg_reduce", "k_sgd_rows", "k_scatter") on this
 * context is bracketed by a pair of HIP events on the context's stream, for at most max_records
 * launches; a null name or max_records == 0 switches timing off.  stx_profile_read: waits for the
 * stream, then *avg_us (host) = mean bracketed time in microseconds and *n (host) = launches recorded;
 * recording restarts from zero.  The name "*" brackets every kernel that has a bracket (all but a few
 * one-workgroup helpers); stx_profile_dump then writes one line "name mean_us launches" per kernel into
 * text (host, text_bytes long, NUL-terminated) and restarts recording.  Bracketing every kernel adds
 * event work to the stream: use it to see where time goes, not to time a whole step.  Not to be used
 * while the stream is being captured into a graph.                                                     */
stx_status stx_profile_kernel(stx_ctx *ctx, const char *kernel_name /* host */, int32_t max_records);
/* Bracket only every `every`-th launch that stx_profile_kernel selects (1 = all, the default after every
 * stx_profile_kernel call).  An event pair costs a few microseconds of stream time: a benchmark that times
 * whole steps and one kernel together samples the kernel sparsely so that the steps are not slowed.    */
stx_status stx_profile_every(stx_ctx *ctx, int32_t every);
/* Both wait for the stream before they read the events. */
stx_status stx_profile_read(stx_ctx *ctx, double *avg_us, int32_t *n);
stx_status stx_profile_dump(stx_ctx *ctx, char *text, size_t text_bytes);

/* Measurement aid: dst[i] = src[i] for n floats (n % 4 == 0, both 16-byte aligned) by a plain
 * grid-stride copy kernel ("k_copy_f32") that reads 4n and writes 4n bytes.  Profilers' hardware byte
 * counters are scaled by what they report for this known traffic.                                     */
stx_status stx_copy_f32(stx_ctx *ctx, float *dst, const float *src, int64_t n);

/* Measurement aid: n_reads scattered reads of 32 bytes each ("k_read_sectors"): read i takes the first 32 bytes
 * of slot (i * 40503) mod n_slots of src, slots slot_bytes apart (a multiple of 16, at least 32; src 16-byte
 * aligned, n_slots * slot_bytes bytes long).  With slot_bytes >= 128 no two lanes of a wavefront share a
 * memory line: the access pattern of the kernels that fetch one packed record or one index per lane.
 * Algorithmic volume: 32 * n_reads bytes read, nothing written (sink: at least 16,384 floats, device; left
 * untouched in practice).                                                                               */
stx_status stx_read_sectors(stx_ctx *ctx, const void *src, int64_t n_slots, int32_t slot_bytes, int64_t n_reads,
                            float *sink);

#ifdef __cplusplus
}
#endif
#endif /* STX_MEASURE_H */
