/*
 * loopserve_test_hooks.h -- entry points of libloopserve that exist for its tests only.  They know
 * internals (workspace layout, kernel wait bounds) and are not part of the product interface.
 */
#ifndef LOOPSERVE_TEST_HOOKS_H
#define LOOPSERVE_TEST_HOOKS_H

#include "loopserve.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Copies the retention score [B,Hkv,len] fp32 (column sums of the last n_obs rows, summed over each
 * KV group, Sec. 5.2) that the most recent ls_kv_compress call on this context left in the workspace
 * to `dst_device`.  `shape` must be the shape of that call.
 */
int ls_debug_copy_compress_score(ls_ctx* ctx, const ls_shape* shape, float* dst_device, void* hip_stream);

/*
 * Bound (number of polls) of every wait between the waves of the greedy-loop kernel of ls_select on
 * this context; negative restores the default.  With a bound of 0 a wave that has to wait gives up at
 * once, every wave still leaves the kernel normally, and the heads concerned take the documented
 * LS_STAT_WALK_TIMEOUT path: this is how the tests reach that path from the host.
 */
int ls_debug_set_walk_spin_limit(ls_ctx* ctx, int32_t limit);

/*
 * Copies to the host the work queues that the most recent ls_sparse_prefill call on this context built
 * (one queue per XCD; an item is one block of 128 query rows of one head): host_queue holds 8 arrays of
 * B * Hq * nqb words, (batch * Hq + head) << 16 | row block, of which the first host_qlen[x] are valid;
 * *nqb_out receives the number of row blocks per head.  `shape` must be that call's shape.  Waits for the
 * stream.  The tests use it to check that every item is queued exactly once.
 */
int ls_debug_copy_prefill_queues(ls_ctx* ctx, const ls_shape* shape, uint32_t* host_queue, int32_t* host_qlen,
                                 int32_t* nqb_out, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* LOOPSERVE_TEST_HOOKS_H */
