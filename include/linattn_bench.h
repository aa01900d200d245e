/*
 * linattn_bench.h -- benchmark instrumentation of liblinattn.so.  Not part of the operator's
 * interface (that is linattn.h): nothing here changes what Eq. 3 / Eq. 5 compute.
 */
#ifndef LINATTN_BENCH_H
#define LINATTN_BENCH_H

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Per-stage timing (the paper reports end-to-end latency only, Sec. 5.2; the roofline accounting
 * of the forward needs the duration of each of its kernels).  `events` points to four hipEvent_t
 * (passed as void*) created by the caller; from then on every linattn_fwd records events[0] before
 * its first stage and events[1..3] after the state pass, the reduction (or, where the reduction is
 * folded into a neighbour, at the same point) and the query pass, on the call's stream.  NULL
 * switches it off (the default).  Process-wide; the setting is taken under the library's lock, but a
 * linattn_fwd running concurrently on another thread may record into either set: use it from the
 * one thread that benchmarks.  The caller keeps the events alive while they are set.
 * Always returns LINATTN_OK.
 */
int linattn_set_stage_events(void* const* events);

#ifdef __cplusplus
}
#endif
#endif /* LINATTN_BENCH_H */
