/*
 * aasd_hooks.h - measurement and test hooks of libaasd.  NOT part of the method and not needed by a
 * caller of aasd.h: a benchmark uses them to time one kernel of a call, the tests use them to force
 * every compiled launch shape.  Each hook acts on the calling thread only and is off by default.
 */
#ifndef AASD_HOOKS_H
#define AASD_HOOKS_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/*
 * While two hipEvent_t handles (passed as void*) are set, aasd_align_sample, aasd_verify,
 * aasd_verify_tree and aasd_verify_topk launch their row-sweep kernel (for the one-launch form of
 * aasd_verify: its only kernel) so that `start` takes the time at which the kernel begins and `stop`
 * the time at which it ends (hipExtLaunchKernelGGL's events): their difference is that kernel's own
 * duration, as a profiler's trace gives it.  Where a call launches the kernel several times, `start`
 * belongs to the first and `stop` to the last launch.  NULL, NULL switches it off.
 */
void aasd_hook_sweep_events(void *start, void *stop);
/* The same for the kernel that makes the full-vocabulary draws of AASD_EXTRAS_GUMBEL. */
void aasd_hook_draw_events(void *start, void *stop);

/*
 * Overrides the launch shape that the library would pick for the row sweep: threads per workgroup,
 * 16-byte loads in flight per lane, segments a row is cut into (0 = leave that to the library).
 * Compiled shapes: 256 x {1, 2, 4}, 512 x {2, 4}, 1024 x {1, 2}; segments 1..16.  (0, 0, n) overrides
 * the segments only, (0, 0, 0) switches the override off.  Returns AASD_OK, or an error for a shape
 * that is not compiled (the override is then unchanged).  The workspace queries answer for the shape
 * in force, so set it before asking.  A segment count also caps the workgroups per row of the
 * full-vocabulary draw kernel (which otherwise takes up to 16 while the rows are few).
 */
int aasd_hook_sweep_plan(int32_t threads, int32_t loads, int32_t segments);

/*
 * How many kernels aasd_verify would enqueue for these sizes and flags under the plan in force: 1 (sweep and
 * decisions in one launch: needs AASD_VERIFY_ZEROED_WORKSPACE and a call small enough) or 2; 0 for invalid sizes.
 */
int aasd_hook_verify_launches(int32_t B, int32_t C, int32_t k, int32_t V, int32_t dt, uint32_t flags);

#ifdef __cplusplus
}
#endif
#endif /* AASD_HOOKS_H */
