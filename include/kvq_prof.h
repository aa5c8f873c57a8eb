/*
 * kvq_prof.h -- switches of the measurement build of the library (libkvq_prof.so: the same
 * sources compiled with -DKVQ_PROFILE).  They exist for benchmarks and tests only; the library
 * proper (libkvq.so, include/kvq.h) has none of them, and the kernels it launches are the ones
 * the measurement build launches while every switch is off.
 * All switches are process-global and not thread-safe.
 */
#ifndef KVQ_PROF_H
#define KVQ_PROF_H

#include "kvq.h"

#ifdef __cplusplus
extern "C" {
#endif

/* While `before` and `after` (hipEvent_t handles
 * created by the caller) are set, every paged_decode_attn call records `before` on its stream
 * immediately ahead of its split kernel (the kernel that streams the K/V codes) and `after`
 * immediately behind it, so that a benchmark can time that kernel alone.  Pass NULL, NULL to
 * switch the hook off (the initial state).  Process-global and not thread-safe. */
void kvq_profile_split_events(void* before, void* after);

/* While switched on, paged_decode_attn launches a
 * read-only twin of its streaming kernel (same work split, addresses, load instructions and
 * software pipeline, the arithmetic replaced by an XOR of the loaded words) and skips the
 * reduce; `out` is not written and the workspace is scribbled on.  Its duration is the
 * read ceiling of this access pattern on the machine at hand.  Process-global; off initially. */
void kvq_profile_read_ceiling(int on);

/* While switched on, paged_decode_attn launches only
 * its streaming kernel and skips the reduce (`out` is then incomplete), so that a run of calls
 * is a run of back-to-back streaming kernels that two events can bracket.  Off initially. */
void kvq_profile_skip_reduce(int on);

/* 0 makes paged_decode_attn use its streaming kernels also for 128
 * and more query rows per kv head, where it otherwise takes the kernel that shares the
 * dequantization among 128 rows.  On initially.  Process-global. */
void kvq_profile_prefill_kernel(int on);

/* While `buf` (device, 16 x uint64 per launched
 * wavefront, i.e. 16 * 8 * (number of wavefronts) bytes) is registered, every wavefront of the
 * streaming kernel stores in buf[16*w + k]: the shader clock at entry (k = 0), after its first
 * loads are issued (2), after its steady loop (3), after its last group (4) and after its
 * results are stored (5); its hardware placement XCC_ID << 32 | HW_ID (1); the constant
 * 100 MHz clock at entry (6) and exit (7); and the shader clock when the sequence lengths have
 * arrived (8), when the wavefront's range is worked out (9) and when its first block-table
 * entries have arrived (10).  Slots 11-15 are not written.
 * Pass NULL to switch off (the initial state).  Process-global. */
void kvq_profile_wave_clock(void* buf);

#ifdef __cplusplus
}
#endif
#endif /* KVQ_PROF_H */
