/*
 * pwlq_bench.h - measurement and test aids of libpwlq.  Not part of the
 * quantization interface (pwlq.h): nothing here changes what a call computes.
 * Used by the benchmark driver to time single kernels inside a call and to name
 * them in a kernel trace, and by the tests to choose between two routes to the
 * same result.
 */
#ifndef PWLQ_BENCH_H
#define PWLQ_BENCH_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Counters of the last pwlq_search* call enqueued by the calling thread, for
 * benchmarks: number of tiles, groups and work units.  Any pointer may be NULL. */
void pwlq_last_search_shape(int64_t *n_tiles, int64_t *n_groups, int64_t *n_units);

/* Benchmark aid.  `roles` is a bit mask (0: off, the default).  With bit r set,
 * every call that launches the kernel of role r records HIP events on its own
 * stream right before and after that kernel (role 0: the candidate-evaluation
 * kernel of a search; role 1: the quantize kernel; role 2: the prefix-sum
 * evaluation kernel of a fast search; role 3: the integer inner-product
 * kernel).  pwlq_profile_last_ms waits for the later event of the most recent
 * launch of a role and returns the kernel's duration in milliseconds, or -1 if
 * none was recorded.  Process-wide, not thread-safe. */
void pwlq_profile_enable(int roles);
double pwlq_profile_last_ms(int role);
/* The same for an earlier launch of that role: back = 0 is the most recent one,
 * back = 1 the one before, up to the last 64 recorded launches; -1 beyond. */
double pwlq_profile_ms(int role, int back);

/* Name of the candidate-evaluation kernel that the calling thread's last search launched
 * (role 0 of the event timing): "k_search", or "k_small" for a call small enough to be one
 * fused launch, or "k_fast" for a fast search. */
const char *pwlq_last_search_kernel(void);

/* Test and measurement aid.  A search call of at most this many groups (all of at
 * most 1024 elements, at most 1024 candidates) runs as one fused launch, one
 * workgroup per group; larger calls partition, evaluate and refine in separate
 * launches.  Both routes meet the same definition of the result; this sets the
 * limit (0: never the fused launch; negative: the default, 256) so that one input
 * can be put through both, and returns the limit it replaces.  Process-wide. */
int pwlq_set_small_call_tiles(int tiles);

/* Name of the library's kernels as they appear in a kernel trace, by role:
 * 0 search (dominant), 1 quantize, 2 prefix-sum evaluation, 3 integer inner
 * product.  Returns NULL for other roles. */
const char *pwlq_kernel_name(int role);

#ifdef __cplusplus
}
#endif
#endif /* PWLQ_BENCH_H */
