/*
 * qp_feed.h -- consumer side of the producer/consumer pipeline between frame loading and group-wise prefill
 * (Sec. 3.3 of the QuickVideo paper, "Overlapping ..."): the loader makes the inputs of group after group available
 * in order; the prefill of a group starts as soon as its inputs are there, while the loader works on later groups;
 * the GPU idles only while it waits for the loader. With t_dec / t_prefill the total loading / prefill time and
 * t^g_dec / t^g_prefill the time to load the first group / to prefill the last, the run takes
 *     t_total = max(t_dec + t^g_prefill, t_prefill + t^g_dec) + delta            (the equation of Sec. 3.3)
 * instead of t_dec + t_prefill.
 *
 * A qp_feed is a ring of host slots (pinned memory) with an in-order ready queue:
 *   producer (any host thread)   qp_feed_begin_write -> fill the slot -> qp_feed_publish, ... , qp_feed_close
 *   consumer (one host thread)   qp_feed_consume: for every published group, copy the slot to one of two device
 *                                buffers on the feed's copy stream and call the group function, which enqueues the
 *                                group's prefill on the caller's stream. The copy of group g+1 runs beside the
 *                                compute of group g; a device buffer is overwritten only after the compute that read
 *                                it has finished; a host slot is handed back to the producer when its copy is done.
 * The producer here is whatever fills the slots: the frame loader itself is not part of this library;
 * qp_feed_stub_producer stands in for it with a configurable latency per group.
 *
 * Unlike the rest of the library a feed owns memory and a stream: qp_feed_create allocates the slots (hipHostMalloc;
 * plain malloc with QP_FEED_PAGEABLE) and creates the copy stream and events (default priority) on the current device;
 * qp_feed_destroy releases them. Errors are qp_status values (qp.h); nothing throws.
 */
#ifndef QP_FEED_H_
#define QP_FEED_H_

#include "qp.h"

#ifdef __cplusplus
extern "C" {
#endif

typedef struct qp_feed qp_feed;

enum {
  QP_FEED_PAGEABLE = 1 /* slots in pageable host memory: copies do not overlap compute; also lets the queue
                          (everything except qp_feed_consume) be used on a machine without a GPU */
};

/* The consumer-side calls also return QP_FEED_END (the feed is closed and every published group has been taken) and
 * qp_feed_next QP_FEED_TIMEOUT (nothing was published within the time-out); both are qp_status values of qp.h. */

/* n_slots >= 2 host slots of slot_bytes each. INVALID_ARG on bad sizes, QP_ERR_HIP if an allocation fails. */
qp_status qp_feed_create(int32_t n_slots, size_t slot_bytes, int32_t flags, qp_feed** out);
/* Stops the feed (as qp_feed_stop), joins the stand-in producer's thread if one was started, releases everything.
 * A producer thread of the caller's own must have returned from its last call before this. NULL is ignored. */
void qp_feed_destroy(qp_feed* feed);
/* The consumer gives up: from now on qp_feed_begin_write and qp_feed_publish return QP_FEED_END instead of blocking
 * or publishing, and a producer blocked on a full ring wakes up with that status. qp_feed_consume calls it when it
 * ends with an error (group function failed, group larger than the device buffer, HIP error). Never undone. */
qp_status qp_feed_stop(qp_feed* feed);

/* ---- producer side ------------------------------------------------------------------------------------- */
/* The next slot to fill (host pointer, slot_bytes long). Blocks while all slots are in use (published but not yet
 * copied to the device) and the feed has not been stopped. INVALID_ARG after qp_feed_close or if the previous slot
 * was not published; QP_FEED_END once the feed is stopped (nobody will take the group). */
qp_status qp_feed_begin_write(qp_feed* feed, void** host_slot);
/* The slot obtained last holds `bytes` bytes of the next group (groups are numbered in publication order). */
qp_status qp_feed_publish(qp_feed* feed, size_t bytes);
/* No more groups will be published. */
qp_status qp_feed_close(qp_feed* feed);

/* ---- consumer side ------------------------------------------------------------------------------------- */
/* Host-only primitive: waits up to timeout_ms (negative: for ever) for the next group; returns its slot, size and
 * index. The slot stays in use until qp_feed_release(feed, group). QP_FEED_END / QP_FEED_TIMEOUT as above. */
qp_status qp_feed_next(qp_feed* feed, int32_t timeout_ms, const void** host_slot, size_t* bytes, int32_t* group);
qp_status qp_feed_release(qp_feed* feed, int32_t group); /* hands the group's slot back to the producer */

/* The group function: enqueue the prefill of `group`, whose inputs are `bytes` bytes at device_input (DEVICE
 * pointer, valid until the function enqueued for group + 2 starts), on hip_stream. Must only enqueue. A status other
 * than QP_OK stops the run and is returned by qp_feed_consume. */
typedef qp_status (*qp_group_fn)(void* user, int32_t group, const void* device_input, size_t bytes, void* hip_stream);

typedef struct {
  int32_t groups;             /* groups consumed                                                        */
  double total_ms;            /* host wall clock from the call to the end of the last group's GPU work  */
  double waited_ms;           /* of it, waiting for the producer (summed over groups)                   */
  double first_group_wait_ms; /* of that, before the first group                                        */
} qp_feed_stats;

/* Runs the consumer loop until the feed ends: device_buf0 / device_buf1 (DEVICE, buf_bytes each, 16-byte aligned)
 * alternate as the landing area of the copies. Blocks the calling thread (it waits for the producer and, at the
 * end, for the GPU); the GPU work of the groups is ordered on hip_stream. CAPACITY if a published group is larger
 * than buf_bytes. */
qp_status qp_feed_consume(qp_feed* feed, void* device_buf0, void* device_buf1, size_t buf_bytes, qp_group_fn fn,
                          void* user, void* hip_stream, qp_feed_stats* stats_or_null);

/* ---- stand-in producer ----------------------------------------------------------------------------------- */
/* Starts a host thread that publishes n_groups groups: group g is bytes_per_group[g] bytes copied from
 * host_src + sum of the earlier sizes, made available first_latency_us after the start for group 0 and
 * per_group_latency_us after the previous one for the others (the loader's t^g_dec and its steady rate), then
 * closes the feed. host_src must stay valid until qp_feed_stub_join. One stub per feed. */
qp_status qp_feed_stub_producer(qp_feed* feed, const void* host_src, const size_t* bytes_per_group, int32_t n_groups,
                                int64_t first_latency_us, int64_t per_group_latency_us);
qp_status qp_feed_stub_join(qp_feed* feed, double* producer_ms_or_null); /* waits for the stub thread to finish */

#ifdef __cplusplus
}
#endif
#endif /* QP_FEED_H_ */
