/*
 * ctm_bench.h -- benchmark diagnostics of libctm.so, kept apart from the operator entry points of ctm.h because they
 * are not for production code: they create HIP events inside operator calls.
 */
#ifndef CTM_BENCH_H
#define CTM_BENCH_H

#include "ctm.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Between ctm_profile_begin() and ctm_profile_end() every operator
 * call made by the calling thread brackets each kernel it launches with HIP events on the
 * call's stream (this creates events, so it is not for production loops).
 * ctm_profile_end() waits for the last event and returns, per kernel class, the summed
 * event-to-event time in milliseconds and the number of launches:
 *   index 0 seed kernel, 1 stacked GEMM + jet rule (one launch per hidden layer), 2 last layer.
 * Either output pointer may be NULL.
 */
int ctm_profile_begin(void);
int ctm_profile_end(double ms[3], long launches[3]);

#ifdef __cplusplus
}
#endif
#endif /* CTM_BENCH_H */
