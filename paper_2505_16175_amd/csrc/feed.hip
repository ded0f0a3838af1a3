// qp_feed (qp_feed.h): ring of host slots with an in-order ready queue between a loader thread and the group-wise
// prefill, the consumer loop that overlaps the host->device copy of group g+1 with the compute of group g, and a
// stand-in producer with a configurable latency per group. Host code only.
#include <string.h>

#include <chrono>
#include <condition_variable>
#include <deque>
#include <mutex>
#include <new>
#include <thread>
#include <vector>

#include "qp_feed.h"
#include "qp_internal.h"

using Clock = std::chrono::steady_clock;

struct qp_feed {
  int n_slots = 0;
  size_t slot_bytes = 0;
  int flags = 0;
  std::vector<unsigned char*> slots;
  std::vector<size_t> bytes;  // per slot, of the group it holds
  std::vector<char> busy;     // per slot: published and not yet released
  std::mutex mu;
  std::condition_variable cv;
  long written = 0;  // groups published; group g lives in slot g % n_slots
  long taken = 0;    // groups handed to the consumer
  bool writing = false, closed = false;
  bool stopped = false;  // the consumer has given up (error exit of qp_feed_consume, qp_feed_stop, destroy): producers must not block
  // device side (absent with QP_FEED_PAGEABLE on a machine without a GPU)
  hipStream_t copy = nullptr;
  hipEvent_t copied[2] = {nullptr, nullptr}, computed[2] = {nullptr, nullptr};
  std::vector<hipEvent_t> slot_done;
  // stand-in producer
  std::thread stub;
  bool stub_started = false;
  double stub_ms = 0.0;
};

namespace {

double ms_since(Clock::time_point t0) { return std::chrono::duration<double, std::milli>(Clock::now() - t0).count(); }

qp_status hip_failed(hipError_t e) {
  qp::note_hip_error((int)e);
  (void)hipGetLastError();
  return QP_ERR_HIP;
}

void free_feed(qp_feed* f) {
  for (unsigned char* p : f->slots) {
    if (p == nullptr) continue;
    if (f->flags & QP_FEED_PAGEABLE) free(p);
    else (void)hipHostFree(p);
  }
  for (hipEvent_t e : f->slot_done)
    if (e != nullptr) (void)hipEventDestroy(e);
  for (int i = 0; i < 2; ++i) {
    if (f->copied[i] != nullptr) (void)hipEventDestroy(f->copied[i]);
    if (f->computed[i] != nullptr) (void)hipEventDestroy(f->computed[i]);
  }
  if (f->copy != nullptr) (void)hipStreamDestroy(f->copy);
  delete f;
}

// The copy stream and the events are created on first use by the consumer, so that a pageable feed's queue works
// without a GPU.
qp_status ensure_device_side(qp_feed* f) {
  if (f->copy != nullptr) return QP_OK;
  hipError_t e = hipStreamCreateWithFlags(&f->copy, hipStreamNonBlocking);
  for (int i = 0; i < 2 && e == hipSuccess; ++i) {
    e = hipEventCreateWithFlags(&f->copied[i], hipEventDisableTiming);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&f->computed[i], hipEventDisableTiming);
  }
  f->slot_done.assign(f->n_slots, nullptr);
  for (int i = 0; i < f->n_slots && e == hipSuccess; ++i) e = hipEventCreateWithFlags(&f->slot_done[i], hipEventDisableTiming);
  return e == hipSuccess ? QP_OK : hip_failed(e);
}

}  // namespace

extern "C" {

qp_status qp_feed_create(int32_t n_slots, size_t slot_bytes, int32_t flags, qp_feed** out) {
  if (out == nullptr) return QP_ERR_INVALID_ARG;
  *out = nullptr;
  if (n_slots < 2 || n_slots > 1024 || slot_bytes == 0 || (flags & ~QP_FEED_PAGEABLE)) return QP_ERR_INVALID_ARG;
  qp_feed* f = new (std::nothrow) qp_feed;
  if (f == nullptr) return QP_ERR_CAPACITY;
  f->n_slots = n_slots, f->slot_bytes = slot_bytes, f->flags = flags;
  f->slots.assign(n_slots, nullptr);
  f->bytes.assign(n_slots, 0);
  f->busy.assign(n_slots, 0);
  for (int i = 0; i < n_slots; ++i) {
    if (flags & QP_FEED_PAGEABLE) {
      f->slots[i] = (unsigned char*)malloc(slot_bytes);
      if (f->slots[i] == nullptr) {
        free_feed(f);
        return QP_ERR_CAPACITY;
      }
    } else {
      void* p = nullptr;
      hipError_t e = hipHostMalloc(&p, slot_bytes, hipHostMallocDefault);
      if (e != hipSuccess) {
        free_feed(f);
        return hip_failed(e);
      }
      f->slots[i] = (unsigned char*)p;
    }
    memset(f->slots[i], 0, slot_bytes);  // first touch here, not in the producer's first pass over the ring
  }
  *out = f;
  return QP_OK;
}

qp_status qp_feed_stop(qp_feed* feed) {
  if (feed == nullptr) return QP_ERR_INVALID_ARG;
  std::lock_guard<std::mutex> lk(feed->mu);
  feed->stopped = true;
  feed->cv.notify_all();
  return QP_OK;
}

void qp_feed_destroy(qp_feed* feed) {
  if (feed == nullptr) return;
  // a producer blocked on a full ring (its consumer stopped early) must wake up before its thread is joined
  (void)qp_feed_stop(feed);
  if (feed->stub_started && feed->stub.joinable()) feed->stub.join();
  free_feed(feed);
}

qp_status qp_feed_begin_write(qp_feed* feed, void** host_slot) {
  if (feed == nullptr || host_slot == nullptr) return QP_ERR_INVALID_ARG;
  std::unique_lock<std::mutex> lk(feed->mu);
  if (feed->closed || feed->writing) return QP_ERR_INVALID_ARG;
  const int slot = (int)(feed->written % feed->n_slots);
  feed->cv.wait(lk, [&] { return !feed->busy[slot] || feed->stopped; });
  if (feed->stopped) return QP_FEED_END;  // nobody will take this group
  feed->writing = true;
  *host_slot = feed->slots[slot];
  return QP_OK;
}

qp_status qp_feed_publish(qp_feed* feed, size_t bytes) {
  if (feed == nullptr) return QP_ERR_INVALID_ARG;
  std::lock_guard<std::mutex> lk(feed->mu);
  if (!feed->writing || feed->closed) return QP_ERR_INVALID_ARG;
  if (feed->stopped) {
    feed->writing = false;
    return QP_FEED_END;
  }
  if (bytes > feed->slot_bytes) return QP_ERR_CAPACITY;
  const int slot = (int)(feed->written % feed->n_slots);
  feed->bytes[slot] = bytes;
  feed->busy[slot] = 1;
  feed->written += 1;
  feed->writing = false;
  feed->cv.notify_all();
  return QP_OK;
}

qp_status qp_feed_close(qp_feed* feed) {
  if (feed == nullptr) return QP_ERR_INVALID_ARG;
  std::lock_guard<std::mutex> lk(feed->mu);
  feed->closed = true;
  feed->writing = false;
  feed->cv.notify_all();
  return QP_OK;
}

qp_status qp_feed_next(qp_feed* feed, int32_t timeout_ms, const void** host_slot, size_t* bytes, int32_t* group) {
  if (feed == nullptr || host_slot == nullptr || bytes == nullptr || group == nullptr) return QP_ERR_INVALID_ARG;
  std::unique_lock<std::mutex> lk(feed->mu);
  auto ready = [&] { return feed->taken < feed->written || feed->closed; };
  if (timeout_ms < 0) feed->cv.wait(lk, ready);
  else if (!feed->cv.wait_for(lk, std::chrono::milliseconds(timeout_ms), ready)) return QP_FEED_TIMEOUT;
  if (feed->taken >= feed->written) return QP_FEED_END;  // closed and drained
  const int slot = (int)(feed->taken % feed->n_slots);
  *host_slot = feed->slots[slot];
  *bytes = feed->bytes[slot];
  *group = (int32_t)feed->taken;
  feed->taken += 1;
  return QP_OK;
}

qp_status qp_feed_release(qp_feed* feed, int32_t group) {
  if (feed == nullptr || group < 0) return QP_ERR_INVALID_ARG;
  std::lock_guard<std::mutex> lk(feed->mu);
  if (group >= feed->taken || group < feed->written - feed->n_slots) return QP_ERR_INVALID_ARG;
  const int slot = group % feed->n_slots;
  if (!feed->busy[slot]) return QP_ERR_INVALID_ARG;
  feed->busy[slot] = 0;
  feed->cv.notify_all();
  return QP_OK;
}

qp_status qp_feed_consume(qp_feed* feed, void* device_buf0, void* device_buf1, size_t buf_bytes, qp_group_fn fn,
                          void* user, void* hip_stream, qp_feed_stats* stats_or_null) {
  if (feed == nullptr || fn == nullptr || device_buf0 == nullptr || device_buf1 == nullptr || device_buf0 == device_buf1 ||
      buf_bytes == 0 || (((uintptr_t)device_buf0 | (uintptr_t)device_buf1) & 15u))
    return QP_ERR_INVALID_ARG;
  qp_status st = ensure_device_side(feed);
  if (st != QP_OK) return st;
  hipStream_t main = (hipStream_t)hip_stream;
  void* bufs[2] = {device_buf0, device_buf1};
  std::deque<int32_t> copying;  // groups whose host->device copy has been enqueued and whose slot is still held
  const Clock::time_point t0 = Clock::now();
  double waited = 0.0, first_wait = 0.0;
  int32_t n_done = 0;
  // hands back the slots whose copies have finished; with `block`, waits for the oldest one
  auto recycle = [&](bool block) -> qp_status {
    while (!copying.empty()) {
      const int32_t g = copying.front();
      hipEvent_t ev = feed->slot_done[g % feed->n_slots];
      hipError_t e = block ? hipEventSynchronize(ev) : hipEventQuery(ev);
      if (e == hipErrorNotReady) {
        (void)hipGetLastError();
        return QP_OK;
      }
      if (e != hipSuccess) return hip_failed(e);
      copying.pop_front();
      qp_status r = qp_feed_release(feed, g);
      if (r != QP_OK) return r;
      block = false;
    }
    return QP_OK;
  };
  qp_status result = QP_OK;
  for (;;) {
    const void* slot = nullptr;
    size_t bytes = 0;
    int32_t g = -1;
    const Clock::time_point tw = Clock::now();
    // The producer may be waiting for a slot that a finished copy still holds: while nothing is published, hand
    // back finished slots (waiting for the oldest copy if need be) before blocking on the producer.
    for (;;) {
      st = qp_feed_next(feed, 0, &slot, &bytes, &g);
      if (st != QP_FEED_TIMEOUT) break;
      if (!copying.empty()) {
        st = recycle(true);
        if (st != QP_OK) break;
        continue;
      }
      st = qp_feed_next(feed, -1, &slot, &bytes, &g);
      break;
    }
    const double w = ms_since(tw);
    waited += w;
    if (n_done == 0) first_wait = w;
    if (st == QP_FEED_END) break;
    if (st != QP_OK) {
      result = st;
      break;
    }
    if (bytes > buf_bytes) {
      (void)qp_feed_release(feed, g);
      result = QP_ERR_CAPACITY;
      break;
    }
    const int b = g & 1;
    hipError_t e = hipSuccess;
    // The compute that read this buffer (group g - 2) must be done before the copy overwrites it. The host waits
    // for it rather than the copy stream: group g - 1 is still queued or running, so the GPU stays busy, and no
    // stream sits on a long-lived cross-stream wait.
    if (g >= 2) e = hipEventSynchronize(feed->computed[b]);
    if (e == hipSuccess) e = hipMemcpyAsync(bufs[b], slot, bytes, hipMemcpyHostToDevice, feed->copy);
    if (e == hipSuccess) e = hipEventRecord(feed->copied[b], feed->copy);
    if (e == hipSuccess) e = hipEventRecord(feed->slot_done[g % feed->n_slots], feed->copy);
    if (e == hipSuccess) e = hipStreamWaitEvent(main, feed->copied[b], 0);
    if (e != hipSuccess) {
      (void)qp_feed_release(feed, g);
      result = hip_failed(e);
      break;
    }
    copying.push_back(g);
    result = fn(user, g, bufs[b], bytes, hip_stream);
    if (result != QP_OK) break;
    e = hipEventRecord(feed->computed[b], main);
    if (e != hipSuccess) {
      result = hip_failed(e);
      break;
    }
    n_done += 1;
    st = recycle(false);
    if (st != QP_OK) {
      result = st;
      break;
    }
  }
  // drain: the copies in flight finish (their slots go back), then the GPU work of the last groups
  hipError_t e = hipStreamSynchronize(feed->copy);
  if (e == hipSuccess) e = hipStreamSynchronize(main);
  if (e != hipSuccess && result == QP_OK) result = hip_failed(e);
  while (!copying.empty()) {
    (void)qp_feed_release(feed, copying.front());
    copying.pop_front();
  }
  // an early exit leaves groups nobody will take: a producer waiting for a free slot must not wait for ever
  if (result != QP_OK) (void)qp_feed_stop(feed);
  if (stats_or_null != nullptr) {
    stats_or_null->groups = n_done;
    stats_or_null->total_ms = ms_since(t0);
    stats_or_null->waited_ms = waited;
    stats_or_null->first_group_wait_ms = first_wait;
  }
  return result;
}

qp_status qp_feed_stub_producer(qp_feed* feed, const void* host_src, const size_t* bytes_per_group, int32_t n_groups,
                                int64_t first_latency_us, int64_t per_group_latency_us) {
  if (feed == nullptr || host_src == nullptr || bytes_per_group == nullptr || n_groups <= 0 || first_latency_us < 0 ||
      per_group_latency_us < 0 || feed->stub_started)
    return QP_ERR_INVALID_ARG;
  std::vector<size_t> sizes(bytes_per_group, bytes_per_group + n_groups);
  for (size_t s : sizes)
    if (s == 0 || s > feed->slot_bytes) return QP_ERR_CAPACITY;
  feed->stub_started = true;
  feed->stub = std::thread([feed, host_src, sizes, first_latency_us, per_group_latency_us] {
    const Clock::time_point t0 = Clock::now();
    size_t off = 0;
    for (size_t g = 0; g < sizes.size(); ++g) {
      void* slot = nullptr;
      if (qp_feed_begin_write(feed, &slot) != QP_OK) break;
      memcpy(slot, (const unsigned char*)host_src + off, sizes[g]);
      off += sizes[g];
      // group g is due first + g * per after the start; a full ring (slow consumer) delays it further
      std::this_thread::sleep_until(t0 + std::chrono::microseconds(first_latency_us + (int64_t)g * per_group_latency_us));
      if (qp_feed_publish(feed, sizes[g]) != QP_OK) break;
    }
    (void)qp_feed_close(feed);
    feed->stub_ms = ms_since(t0);
  });
  return QP_OK;
}

qp_status qp_feed_stub_join(qp_feed* feed, double* producer_ms_or_null) {
  if (feed == nullptr || !feed->stub_started) return QP_ERR_INVALID_ARG;
  if (feed->stub.joinable()) feed->stub.join();
  if (producer_ms_or_null != nullptr) *producer_ms_or_null = feed->stub_ms;
  return QP_OK;
}

}  // extern "C"
