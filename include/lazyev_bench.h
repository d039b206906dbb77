/*
 * lazyev_bench.h -- measuring aids and tuning knobs around the lazyev library.  None of these
 * is part of the decode path's contract (include/lazyev.h): they exist for bench.py, for the
 * profiles and for tests that force a particular kernel or block split.
 *
 * The knobs and the per-kernel timer act on a context and live in liblazyev.so; the plain
 * streaming probes and the event-cost probe are a library of their own, liblazyev_bench.so.
 */
#ifndef LAZYEV_BENCH_H
#define LAZYEV_BENCH_H

#include "lazyev.h"

#ifdef __cplusplus
extern "C" {
#endif

/* ---- in liblazyev.so ---- */

/* Tuning knobs for how a unit's cache is split over thread blocks.  Results do not depend on
 * them beyond floating-point summation order.
 *   lazyev_set_chunk: entries per block of the vector-ALU attention kernel (a power of two,
 *     64..256; default 128).
 *   lazyev_set_target_blocks: stream blocks per layer call the single-launch attention kernel
 *     aims for, taken literally: each unit gets round(n_blocks / units) blocks, at least one
 *     and at most 64.  Until this is called the library sizes the split from the cache length
 *     (about 16 sub-tiles of 16 entries per wave, at least one block per compute unit, at most
 *     two).
 * Errors: EINVAL. */
int lazyev_set_chunk(lazyev_ctx *ctx, int32_t chunk);
int lazyev_set_target_blocks(lazyev_ctx *ctx, int32_t n_blocks);

/* Tuning knob: attention kernel.
 *   0  vector-ALU split kernel + merge kernel (any supported shape; the only one for fp32 or
 *      head_dim 64);
 *   4  one launch: MFMA stream blocks, the block that finishes a unit last merges the partials
 *      into the output; the tracking rides with the next launch (bf16, head_dim 128).  A block
 *      leaves only the logits of entries that can still reach alpha for the tracking; it leaves
 *      all of them when the caller passes p_out / p_override, with
 *      LAZYEV_SCORE_CURRENT_ATTENTION, or with 8 query heads per KV head;
 *   5  kernel 4 leaving every logit of a call in the workspace for the tracking, 6 kernel 4
 *      leaving only those of the entries that can reach alpha (what 4 does whenever nobody reads
 *      the logits as such; same results bit for bit; for comparison and tests);
 *   1  (default) picks 4 when it applies, else 0.
 * 2 and 3 are not assigned.  Errors: EINVAL. */
int lazyev_set_variant(lazyev_ctx *ctx, int32_t variant);

/* Kernel 4, units of 2..4 blocks: the unit's last block waits for the partial results of the
 * others; the wait is bounded by `ticks` of the GPU's constant 100 MHz counter (default 2000000
 * = 20 ms; the others never wait themselves, so the bound is not reached).  When it is, the block
 * goes on with what it has and the next lazyev_stats returns LAZYEV_EEXCHANGE.  0 makes a block
 * give up when its first look finds a partial missing (a test of that path).  Errors: EINVAL. */
int lazyev_set_spin_ticks(lazyev_ctx *ctx, uint32_t ticks);

/* Test aid.  The single-launch kernel leaves the tracking of a call that nobody asked the weights
 * of as an ACTIVATION LOG: one bit per cache entry and call (bit i of a unit's words: entry i
 * was active, i.e. some head of the group gave it a weight >= alpha; the call's appended entry
 * has no bit), applied to TS / MRI in step order before anything reads them (an eviction,
 * lazyev_stats, lazyev_mri_histogram, a call with p_out / p_override).  lazyev_log_words: 32-bit
 * words per unit, 0 if this configuration keeps no log.  lazyev_log_peek copies the log_words
 * words of unit `unit` (= sequence * n_kv_heads + KV head) of the latest logged call of `layer`
 * (back = 0) or of the one `back` calls before it to `words` (host) and its step to *t (host,
 * nullable); it waits for the stream and applies nothing.  Errors: EINVAL (no such logged
 * call), EHIP. */
int32_t lazyev_log_words(lazyev_ctx *ctx);
int lazyev_log_peek(lazyev_ctx *ctx, int32_t layer, int32_t back, int32_t unit, uint32_t *words, int32_t *t);

/* Profiling aid.  lazyev_profile_arm makes the next n_calls calls that launch kernels
 * (decode_step, or an evict that is due) record HIP events on the stream before, between and
 * after their two kernels.  lazyev_profile_read waits for the stream, adds up the elapsed
 * times of the armed calls since the last read and forgets them:
 *   index 0 attention kernel (the only one of kernel 4), 1 combine + tracking kernel,
 *         2 eviction score/select kernel, 3 eviction row-move kernel.
 * ms_total, launches: (host) arrays of 4.  Errors: EINVAL, EHIP. */
int lazyev_profile_arm(lazyev_ctx *ctx, int32_t n_calls);
int lazyev_profile_read(lazyev_ctx *ctx, double ms_total[4], int64_t launches[4]);

/* ---- in liblazyev_bench.so ---- */

/* Plain streaming kernels of known traffic, for the bandwidth a simple kernel reaches on the
 * same chip and for calibrating hardware byte counters.  lazyev_stream_probe copies `bytes`
 * (a multiple of 16) from src to dst; lazyev_stream_read_probe only reads src (sink: 4 bytes of
 * device memory that is practically never written).  n_blocks blocks of 256 threads, grid-stride.
 * All pointers are device memory.  Asynchronous on `stream`.  Errors: EINVAL, EHIP. */
int lazyev_stream_probe(void *dst, const void *src, size_t bytes, int32_t n_blocks, void *stream);
int lazyev_stream_read_probe(const void *src, size_t bytes, int32_t n_blocks, void *sink,
                             void *stream);

/* Average time, in milliseconds, between two HIP events recorded back to back on `stream`
 * with nothing between them: the fixed cost an event pair adds to the interval measured around
 * a kernel.  Waits for the stream.  ms_avg: (host).  Errors: EINVAL, EHIP. */
int lazyev_event_overhead(int32_t n_pairs, void *stream, double *ms_avg);

#ifdef __cplusplus
}
#endif
#endif /* LAZYEV_BENCH_H */
