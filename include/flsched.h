/* flsched.h - C ABI of the asynchronous swap planner: the host-side policy that lets block moves
 * run beside compute (paper section 4.3, "asynchronous swap-in/out": the moves of a query are issued
 * on streams of their own; a query whose blocks are still in flight waits, the queries that are ready
 * run, so transfers hide behind compute).
 *
 * A request is a query together with the block moves it needs before it may run: write-backs that
 * make room (device -> host) and fetches of its adapter pages and prefix KV (host -> device), as the
 * cache manager of flcache.h (or any other host logic) lists them.
 *
 *   fls_submit          the request's write-backs are enqueued on the planner's out stream, its
 *                       fetches on the in stream (the two directions of the host link are
 *                       independent), and an event marks their completion.  Ordering that the
 *                       planner adds by itself: write-backs come after the last compute that the
 *                       caller announced (that compute may still append to the blocks); fetches come
 *                       after the write-backs of all EARLIER requests (the free list may since have
 *                       handed out the blocks they released) and, with FLS_FETCH_INTO_RELEASED,
 *                       after the request's own write-backs too (section 3.2: when the device tier
 *                       is full, swap-out makes the room that swap-in fills); without the flag the
 *                       two directions of one request run side by side.
 *   fls_poll            which of the waiting requests have all their blocks in the device tier now
 *                       (event query, never blocks), in the order of submission: the caller composes
 *                       the next compute batch from these and lets the others wait.
 *   fls_wait_next       blocks until the oldest waiting request is ready (for a caller that has
 *                       nothing else to run).
 *   fls_stream_wait     makes a compute stream wait on the GPU for one request's moves, for a caller
 *                       that decides the batch ahead of time instead of polling.
 *   fls_compute_enqueued  the caller has enqueued a batch's compute on `compute_stream`; later
 *                       write-backs are ordered after it.
 *
 * The in and out streams belong to the device, not to the planner: they are created with the device's
 * first planner and kept for the life of the process, and all planners on a device share them (their
 * moves are then ordered among each other as well, which is harmless).  fls_create wants the pool's
 * device current (FLP_EHIP otherwise).
 *
 * A planner created with `manual = 1` issues nothing and uses no streams: requests complete when the
 * caller says so (fls_complete).  It is the same policy as a discrete-event model, for simulations of
 * arrival patterns on the host and for the tests of the policy itself.
 *
 * Errors: FLP_EINVAL (null pointer, negative count, unknown or duplicate request id, a call that the
 * planner's mode does not have), FLP_ERANGE / FLP_EDUP from the swap lists (nothing was enqueued for
 * that request and it is not recorded), FLP_EHIP.  Text via flp_last_error().  Calls on one planner
 * are serialised by an internal lock; the pool must outlive the planner.
 */
#ifndef FLSCHED_H_
#define FLSCHED_H_

#include "flpool.h"

#ifdef __cplusplus
extern "C" {
#endif

typedef struct fls_sched fls_sched;

typedef struct {
  int64_t submitted, ready_returned, waiting;   /* requests: all, handed to the caller, still waiting  */
  int64_t blocks_in, blocks_out;                /* blocks moved so far                                 */
  int64_t polls, polls_empty;                   /* fls_poll calls, and those that found nothing ready  */
} fls_stats;

flp_status fls_create(flp_pool* pool, int32_t manual, fls_sched** out);
flp_status fls_destroy(fls_sched* s);

#define FLS_FETCH_INTO_RELEASED 1   /* the fetches land in blocks that this request's write-backs release */
#define FLS_UNHURRIED 2             /* the moves have a whole compute step to finish in: they are launched narrow, so that
                                       the kernels running beside them lose less (at about two thirds of the link's rate) */

/* host_ids / dev_ids: n_in pairs for flp_pool_swap_in; out_dev_ids / out_host_ids: n_out pairs for
 * flp_pool_swap_out.  Host arrays, consumed before the call returns.  A request without moves is ready
 * at once.  flags: 0 or a combination of FLS_FETCH_INTO_RELEASED and FLS_UNHURRIED. */
flp_status fls_submit(fls_sched* s, int64_t req_id, int32_t n_in, const int32_t* host_ids, const int32_t* dev_ids,
                      int32_t n_out, const int32_t* out_dev_ids, const int32_t* out_host_ids, int32_t flags);
/* Up to `max` ready requests, oldest first; they leave the planner.  *n_ready may be 0. */
flp_status fls_poll(fls_sched* s, int32_t max, int64_t* ready_ids, int32_t* n_ready);
/* Blocks until the oldest waiting request is ready (returns at once if none waits). Not in manual mode. */
flp_status fls_wait_next(fls_sched* s);
/* GPU-side wait of `compute_stream` for the moves of a waiting request, which leaves the planner as if
 * polled.  Not in manual mode. */
flp_status fls_stream_wait(fls_sched* s, int64_t req_id, void* compute_stream);
flp_status fls_compute_enqueued(fls_sched* s, void* compute_stream);
/* Manual mode only: the moves of `req_id` have completed. */
flp_status fls_complete(fls_sched* s, int64_t req_id);
flp_status fls_get_stats(const fls_sched* s, fls_stats* out);

#ifdef __cplusplus
}
#endif
#endif /* FLSCHED_H_ */
