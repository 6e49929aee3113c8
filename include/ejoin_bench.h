/*
 * ejoin_bench -- measurement hooks of libejoin.so, kept apart from the product interface (ejoin.h):
 * only benchmark programs call these.
 */
#ifndef EJOIN_BENCH_H
#define EJOIN_BENCH_H

#include "ejoin.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Kernel timing.  With profiling on, each join call records HIP events on the call's stream around its
 * preparation kernels (norms and re-layout, FP16 split of the norm terms) and around its Gram/epilogue
 * kernel (the roofline of the join is stated for that kernel: Step 2 of Section 3.1 is where the time
 * goes).  ejoin_last_kernel_ms waits for those events and returns the two durations in milliseconds
 * (host pointers, either may be NULL).  EJOIN_EINVAL if no call has been timed since profiling was set. */
int ejoin_set_profiling(ejoin_ctx* ctx, int on);
int ejoin_last_kernel_ms(ejoin_ctx* ctx, float* prep_ms, float* join_ms);

#ifdef __cplusplus
}
#endif
#endif /* EJOIN_BENCH_H */
