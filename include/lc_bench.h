/*
 * lc_bench.h -- instrumentation of liblc.so for this repository's benchmark, not part of the library's
 * interface (it may change with the kernels): per-kernel timing with HIP events on the caller's stream.
 */
#ifndef LC_BENCH_H
#define LC_BENCH_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/*
 * lc_profile(1) switches it on and clears the totals, lc_profile(0) switches it off.
 * lc_profile_read copies up to `cap` accumulated kernel times (milliseconds) and
 * launch counts; returns the number of kernel slots.  lc_profile_name(i) names slot i
 * (NULL past the end).
 */
int lc_profile(int enable);
int lc_profile_read(double* ms_total, uint64_t* launches, int cap);
const char* lc_profile_name(int slot);

#ifdef __cplusplus
}
#endif
#endif /* LC_BENCH_H */
