/*
 * guide_diag.h -- diagnostics of libguide.so that are not part of the method's
 * interface (guide.h): event pairs on the kernels of a call, for programs that
 * report kernel times next to throughput.
 */
#ifndef GUIDE_DIAG_H
#define GUIDE_DIAG_H

#include "guide.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Kernel timing aid.  After
 * guide_profile_enable(ctx, capacity, every), every `every`-th grid evaluation
 * kernel launched by guide_eval_grid (one sample) or guide_eval_select (the
 * first, the every+1-th, ...) carries a pair of HIP events on the call's stream
 * that receive the start and the end of that kernel's dispatch.  When such a
 * guide_eval_select call has one top-k and one Pareto selection over stored
 * columns, the two kernels of its selection passes (filter, finish) carry a
 * pair each as well, so that every dispatch of the call is observed the same
 * way.  `capacity` is the number of pairs (later launches are
 * not timed); capacity 0 switches it off.  A timed launch delays the launches
 * around it by a few microseconds, which is why a caller that also measures
 * throughput times separate calls.  guide_profile_read waits for the recorded
 * events, writes the elapsed milliseconds of each timed kernel, in launch
 * order (three per such guide_eval_select call, one per other call), to
 * ms[0 .. *n) (HOST, room for `capacity` values) and starts over.
 */
int guide_profile_enable(guide_ctx *ctx, uint32_t capacity, uint32_t every);
int guide_profile_read(guide_ctx *ctx, float *ms, uint32_t *n);

#ifdef __cplusplus
}
#endif
#endif /* GUIDE_DIAG_H */
