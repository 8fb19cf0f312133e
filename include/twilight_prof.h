/*
 * twilight_prof.h - opt-in per-kernel timing of the library's launches, for
 * benchmarks.  This is the library's only process-global mutable state: one
 * list of event pairs shared by all threads and streams (calls are serialised
 * by a lock; while timing is on, use one stream at a time).  Off by default;
 * nothing here is needed to use the entry points of twilight.h.
 */
#ifndef TWILIGHT_PROF_H
#define TWILIGHT_PROF_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

struct twilight_kv;   /* twilight.h */

/*
 * A HIP event pair is attached to the
 * kernel's own dispatch (hipExtLaunchKernelGGL: start and stop timestamps of
 * the kernel, no extra packets on the stream).  mode 0 = off (default), 1 =
 * every kernel, 2 = only the kernel id given to twilight_prof_select, at
 * every `every`-th of its launches (the every-th, 2 * every-th, ... since
 * twilight_prof_select), 3 = as 2, and with each of those launches
 * the launch just ahead of it on the stream (the library kernel that preceded
 * the chosen one the last time): a timed kernel's start stamp is taken when
 * its dispatch is reached, which is before an untimed predecessor has
 * drained (1.5 us early on MI355X), not when both carry events.  Timed
 * launches are not meant to be
 * captured into a graph.  While on,
 * each launch adds one record {kernel id, start event, stop event} (at most
 * TW_PROF_MAX_RECORDS between two collects; further launches are not timed).
 * twilight_prof_collect synchronises the events, writes up to `cap` records
 * (kernel id, milliseconds) to the HOST arrays and clears the list; returns
 * the number written.
 */
#define TW_PROF_MAX_RECORDS 65536
#define TW_K_KQUANT_APPEND 0
#define TW_K_PAGE_SCORE 1
#define TW_K_PAGE_SELECT 2
#define TW_K_INT4_SCORE 3
#define TW_K_TOPP 4
#define TW_K_UNION 5
#define TW_K_DECODE 6
#define TW_K_COMBINE 7
#define TW_K_SCORE_TOPP 8         /* scoring + top-p + union in one launch (twilight_select_prune) */
#define TW_K_SELECT_SCORE_TOPP 9  /* page selection as well */
#define TW_K_COUNT 10
int twilight_prof_enable(int mode);
int twilight_prof_select(int kernel_id, int every);
int twilight_prof_collect(int32_t* kernel_ids /*host*/, float* ms /*host*/, int32_t cap);
const char* twilight_kernel_name(int kernel_id);

/*
 * Launch shape of the attention kernel for a cache shape (host only; only
 * kv's shape fields are read): the persistent grid before it is cut to the
 * number of work items, the shortest chunk of list entries per work item
 * (dense != 0: the all-tokens sweep), and the number of items per workgroup
 * beyond which the kernel doubles the chunk (up to 4 x chunk0, at most 512).
 * which = TW_WS_DECODE or TW_WS_DECODE_PER_HEAD.  For reports on how evenly
 * ragged lists spread over the workgroups (Section 4.2, load balancing).
 */
int twilight_decode_plan(const struct twilight_kv* kv, int which, int32_t dense, int32_t* grid /*host, out*/,
                         int32_t* chunk0 /*host, out*/, int32_t* items_per_wg /*host, out*/);

#ifdef __cplusplus
}
#endif
#endif /* TWILIGHT_PROF_H */
