/*
 * rls - timing aid for benchmarks.  NOT part of the library's interface proper (rls.h) and not part of the
 * paper's method: a benchmark program uses it to time the fused assign + update pass that dominates the
 * k-means calls of Algorithm 1 (Sec. 4.2) on the stream the library launches it on.
 *
 * Unlike everything in rls.h these two calls keep process-wide state (a flag and a pool of HIP events the
 * library creates on first use); a mutex guards that state.  While enabled, every sweep of every host thread
 * records into the one pool, so the figures only mean something when one thread is sweeping.  Leave it
 * disabled (the default) anywhere else: a sweep that is being recorded into a HIP graph must not record events.
 */
#ifndef RLS_BENCH_H
#define RLS_BENCH_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* on != 0: rls_kmeans_sweep[_batched] records a pair of events around every launch of the Lloyd step kernel. */
int32_t rls_profile_enable(int32_t on);
/* Waits for the recorded events; returns the number of launches timed and their summed duration in
 * milliseconds, and forgets them.  RLS_ERR_NULL / RLS_ERR_HIP as in rls.h. */
int32_t rls_profile_read(int32_t *n_launches, double *total_ms);

#ifdef __cplusplus
}
#endif
#endif /* RLS_BENCH_H */
