/* libknapattn: hooks for benchmarks and tests.  Not part of the attention
 * interface (include/knapattn.h) and of no use to a training loop: they let a
 * benchmark time one kernel of the backward with events on the launch stream,
 * and read the size of the persistent launches.  Same conventions as
 * knapattn.h (plain C ABI, nothing allocates or synchronises).
 */
#ifndef KNAPATTN_BENCH_H
#define KNAPATTN_BENCH_H

#ifdef __cplusplus
extern "C" {
#endif

/* While both are non-NULL, every backward call made by this thread records
 * `start` right before and `stop` right after its dK/dV kernel (the longest
 * kernel of the path) on the call's stream; the dQ kernel, which runs before
 * it, stays outside the pair.  hipEvent_t passed as void*, owned by the
 * caller.  Pass NULLs to switch it off.  Not for use under graph capture. */
void knap_bwd_profile_events(void* start, void* stop);

/* Number of persistent workgroups the forward / backward kernels are launched
 * with on the current device (<= 0 on error). */
int knap_launch_workgroups(int which /* 0 = forward, 1 = backward dK/dV, 2 = backward dQ */);

#ifdef __cplusplus
}
#endif
#endif /* KNAPATTN_BENCH_H */
