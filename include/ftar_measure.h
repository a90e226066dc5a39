/*
 * ftar_measure.h - measurement tooling around the FTAR data path (include/ftar.h).  Nothing here
 * is part of the method: no result ever depends on these calls.  They exist for the benchmark and
 * the tuning tests: launch-shape and cache-policy overrides, kernel durations recorded by the
 * dispatch itself, and bare streaming kernels that show what the GPU's memory system gives for a
 * mix of read and written streams (the ceiling next to which the reduce and ring kernels are
 * judged; paper section 4.2 "Optimizations" only says the kernels must keep many loads in flight).
 *
 * Two libraries export them:
 *   libftar.so          ftar_set_tuning, ftar_time_next_launch  (hooks in the product's launch path)
 *   libftar_measure.so  ftar_probe_stream, ftar_probe_stream_windows, ftar_probe_stream_workgroups
 *                       (bench-only; links against libftar.so and honours both hooks)
 */
#ifndef FTAR_MEASURE_H_
#define FTAR_MEASURE_H_

#include <stddef.h>
#include <stdint.h>

#include "ftar.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Launch shape and cache policy, for measurement only (results never depend on it).
 * blocks_per_cu: workgroups launched per compute unit (0 = each kernel's default);
 * flags: 0 = each kernel's defaults.
 *   0x10 | p      explicit cache policy p: bit 0 non-temporal loads, bit 1 non-temporal stores
 *   0x20          wide tiles in the one-shot reduce
 *   0x40          one launch, however long the call (one-shot reduce, big buckets, ring steps); no soft
 *                 barriers inside the long steps of the persistent ring
 *   0x80          no write windows in the many-source reductions
 *   bits 8..11    vectors per lane and tile in the ring step kernels (2, 4 or 8)
 *   bits 12..15   log2 of the write-window period in 10 ns ticks; bits 16..19: log2(period / window)
 *   0x100000      write windows whenever the kernel has them (also for outputs below 16 MiB and, with four
 *                 or five sources, below 256 MiB)
 *   0x200000      bf16 ReduceScatter lanes take 8 elements (16-byte loads, two partial-sum vectors)
 *   0x400000      the persistent ring keeps its small tile also with few workgroups
 *   bits 24..27   traffic per launch of a long ring step in units of 256 MiB; in the persistent ring, log2 of
 *                 the Mi elements between two soft barriers inside a long step */
void ftar_set_tuning(int blocks_per_cu, int flags);

/* Measurement only: arms two hipEvent_t (passed as void*, either may be NULL) for the NEXT kernel
 * this thread launches through the library.  That dispatch records them itself: `start` when the
 * kernel begins on the GPU, `stop` when it ends, so hipEventElapsedTime(start, stop) is the
 * kernel's own duration.  A one-shot or bucketed reduce that goes out as several launches records
 * `start` with its first and `stop` with its last launch.  The pair is consumed by that call and
 * cleared.  The caller owns the events. */
void ftar_time_next_launch(void* start_event, void* stop_event);

/* Measurement only: a bare streaming kernel over n_read + n_written device buffers of `bytes`
 * bytes each (bufs: HOST array, the read buffers first; 16-byte aligned; bytes a multiple of 32 KiB).
 * The first n_read are read, each of the others receives the xor of the read ones at the same
 * offset (or the 32-bit word `fill` when n_read == 0); with n_written == 0 nothing is stored.
 * It gives this GPU's own ceiling for a mix of streams, next to which the reduce and ring kernels
 * are judged.  Mixes offered: reads only 1/2/4/8/16, writes only 1/2/4/8, r+1 for r = 1,2,3,4,7,8,16,
 * 4+4, 8+8; anything else FTAR_ERR_INVALID_ARG.  Honours ftar_set_tuning and ftar_time_next_launch. */
ftar_status_t ftar_probe_stream(void* const* bufs, int n_read, int n_written, size_t bytes, uint32_t fill,
                                void* stream);

/* Measurement only: n_read buffers read, ONE written (bufs: the read buffers first, then the written
 * one; sizes and alignment as above), the written vectors staged in LDS and written out only inside
 * windows [0, window_ticks) of every period_ticks of the 100 MHz wall clock (10 ns ticks; the period
 * a power of two), or when the stage is full: the bare-stream form of the write windows that the
 * many-source reductions use, next to ftar_probe_stream(n_read, 1) for the plain mix.
 * n_read in 1, 2, 4, 7, 8, 16; anything else FTAR_ERR_INVALID_ARG.  One workgroup per compute unit. */
ftar_status_t ftar_probe_stream_windows(void* const* bufs, int n_read, size_t bytes, unsigned period_ticks,
                                        unsigned window_ticks, void* stream);

/* Measurement only: n_read (1 or 2) buffers read and ONE written (the xor) by exactly n_workgroups
 * workgroups of `threads` lanes, each lane moving vectors_per_lane 16-byte vectors per tile, with
 * ordinary loads and stores: what a few compute units can move, next to the persistent ring at a
 * small compute-unit budget (paper section 4.2 "Optimizations": two thread blocks).  (threads,
 * vectors_per_lane) one of (256, 8), (1024, 8) and, with one read buffer, (256, 32); bytes a multiple of threads *
 * vectors_per_lane * 16; n_workgroups 1..4096; anything else FTAR_ERR_INVALID_ARG.  Ignores
 * ftar_set_tuning; honours ftar_time_next_launch. */
ftar_status_t ftar_probe_stream_workgroups(void* const* bufs, int n_read, size_t bytes, unsigned n_workgroups,
                                           unsigned threads, unsigned vectors_per_lane, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* FTAR_MEASURE_H_ */
