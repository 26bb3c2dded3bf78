// The asynchronous swap planner (paper section 4.3): requests whose block moves are in flight wait,
// requests whose blocks have arrived are handed to the caller for the next compute batch.  Host logic
// only: the moves themselves are the pool's swap-out / swap-in on two streams of the planner.
#include <deque>
#include <mutex>
#include <new>

#include "flp_internal.h"
#include "flsched.h"

namespace {

struct Request {
  int64_t id;
  hipEvent_t done = nullptr;   // recorded on the in stream after the request's fetches (null: ready at once / manual)
  bool complete = false;       // manual mode, or no moves at all
};

}  // namespace

struct fls_sched {
  flp_pool* pool = nullptr;
  bool manual = false;
  hipStream_t s_in = nullptr, s_out = nullptr;
  hipEvent_t ev_compute = nullptr;   // last compute the caller announced
  bool have_compute = false;
  hipEvent_t ev_out = nullptr;       // last write-back issued
  bool have_out = false;
  std::deque<Request> waiting;       // in order of submission
  std::deque<hipEvent_t> spare;      // events of requests that have left
  fls_stats st{};
  mutable std::mutex mu;
};

namespace {

flp_status take_event(fls_sched* s, hipEvent_t* out) {
  if (!s->spare.empty()) {
    *out = s->spare.front();
    s->spare.pop_front();
    return FLP_OK;
  }
  FLP_TRY_HIP(hipEventCreateWithFlags(out, hipEventDisableTiming));
  return FLP_OK;
}

Request* find(fls_sched* s, int64_t id) {
  for (auto& r : s->waiting)
    if (r.id == id) return &r;
  return nullptr;
}

// true when the request's blocks are in the device tier
flp_status is_ready(const Request& r, bool* ready) {
  if (r.complete) {
    *ready = true;
    return FLP_OK;
  }
  if (!r.done) {
    *ready = false;             // manual mode, not completed yet
    return FLP_OK;
  }
  hipError_t q = hipEventQuery(r.done);
  if (q == hipSuccess) {
    *ready = true;
  } else if (q == hipErrorNotReady) {
    *ready = false;
  } else {
    flp_set_error("fls: hipEventQuery failed: %s", hipGetErrorString(q));
    return FLP_EHIP;
  }
  return FLP_OK;
}

}  // namespace

// The two move streams of a device, created when its first planner is and kept until the process ends; every
// planner on the device uses them.  The runtime binds a stream to one of a few hardware queues when the stream is
// made, by the load of the queues at that moment: streams made while a process holds only its first compute stream
// get queues of their own, streams made later (a second planner after the first was destroyed) have been seen to
// land on the compute stream's queue, where moves and compute take turns instead of overlapping (a step bound by
// its fetches: 9.2 ms instead of 8.0).  Both streams have the default priority.
static hipError_t move_streams(int pool_device, hipStream_t* s_in, hipStream_t* s_out) {
  constexpr int kMaxDevices = 64;
  static std::mutex mu;
  static hipStream_t streams[kMaxDevices][2];
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  // streams belong to the device that is current when they are made: it has to be the pool's
  if (dev < 0 || dev >= kMaxDevices || (pool_device >= 0 && dev != pool_device)) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lk(mu);
  for (int i = 0; i < 2; ++i)
    if (!streams[dev][i]) {
      e = hipStreamCreateWithFlags(&streams[dev][i], hipStreamNonBlocking);
      if (e != hipSuccess) {
        streams[dev][i] = nullptr;
        return e;
      }
    }
  *s_in = streams[dev][0];
  *s_out = streams[dev][1];
  return hipSuccess;
}

extern "C" flp_status fls_create(flp_pool* pool, int32_t manual, fls_sched** out) {
  if (!out || (!pool && !manual)) {
    flp_set_error("fls_create: null argument");
    return FLP_EINVAL;
  }
  *out = nullptr;
  fls_sched* s = new (std::nothrow) fls_sched();
  if (!s) {
    flp_set_error("fls_create: out of host memory");
    return FLP_ENOSPC;
  }
  s->pool = pool;
  s->manual = manual != 0;
  if (!s->manual) {
    hipError_t e = move_streams(pool->device, &s->s_in, &s->s_out);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&s->ev_compute, hipEventDisableTiming);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&s->ev_out, hipEventDisableTiming);
    if (e != hipSuccess) {
      flp_set_error("fls_create: %s", hipGetErrorString(e));
      fls_destroy(s);
      return FLP_EHIP;
    }
  }
  *out = s;
  return FLP_OK;
}

extern "C" flp_status fls_destroy(fls_sched* s) {
  if (!s) return FLP_OK;
  if (!s->manual) {
    if (s->s_in) (void)hipStreamSynchronize(s->s_in);
    if (s->s_out) (void)hipStreamSynchronize(s->s_out);
    for (auto& r : s->waiting)
      if (r.done) (void)hipEventDestroy(r.done);
    for (auto e : s->spare) (void)hipEventDestroy(e);
    if (s->ev_compute) (void)hipEventDestroy(s->ev_compute);
    if (s->ev_out) (void)hipEventDestroy(s->ev_out);
  }
  delete s;
  return FLP_OK;
}

extern "C" flp_status fls_submit(fls_sched* s, int64_t req_id, int32_t n_in, const int32_t* host_ids,
                                 const int32_t* dev_ids, int32_t n_out, const int32_t* out_dev_ids,
                                 const int32_t* out_host_ids, int32_t flags) {
  if (!s || n_in < 0 || n_out < 0 || (flags & ~(FLS_FETCH_INTO_RELEASED | FLS_UNHURRIED)) || (n_in > 0 && (!host_ids || !dev_ids)) || (n_out > 0 && (!out_dev_ids || !out_host_ids))) {
    flp_set_error("fls_submit: invalid argument");
    return FLP_EINVAL;
  }
  std::lock_guard<std::mutex> lk(s->mu);
  if (find(s, req_id)) {
    flp_set_error("fls_submit: request %lld is already waiting", (long long)req_id);
    return FLP_EINVAL;
  }
  Request r;
  r.id = req_id;
  if (s->manual) {
    r.complete = n_in == 0 && n_out == 0;
  } else if (n_in == 0 && n_out == 0) {
    r.complete = true;
  } else {
    // both lists are checked before anything is enqueued, so a refused request leaves no move behind
    FLP_TRY(flp_swap_check(s->pool, n_out, out_dev_ids, out_host_ids, 0, "fls_submit (write-backs)"));
    FLP_TRY(flp_swap_check(s->pool, n_in, host_ids, dev_ids, 1, "fls_submit (fetches)"));
    // a request that moves blocks both ways has its two kernels share the host link: the fetch, which the
    // request's compute waits for, is launched wider than the write-back
    const bool duplex = n_in > 0 && n_out > 0;
    const int width = (flags & FLS_UNHURRIED) ? FLP_WIDTH_NARROW : duplex ? FLP_WIDTH_DUPLEX : FLP_WIDTH_SINGLE;
    // fetches land in blocks that an earlier request's write-back may have released
    if (s->have_out) FLP_TRY_HIP(hipStreamWaitEvent(s->s_in, s->ev_out, 0));
    if (n_out > 0) {
      // the compute announced last may still append to the blocks that go out
      if (s->have_compute) FLP_TRY_HIP(hipStreamWaitEvent(s->s_out, s->ev_compute, 0));
      FLP_TRY(flp_swap_width(s->pool, n_out, out_dev_ids, out_host_ids, 0, s->s_out, width));
      FLP_TRY_HIP(hipEventRecord(s->ev_out, s->s_out));
      s->have_out = true;
      // ... or this request's own, when the caller says that they make the room
      if (flags & FLS_FETCH_INTO_RELEASED) FLP_TRY_HIP(hipStreamWaitEvent(s->s_in, s->ev_out, 0));
    }
    if (n_in > 0) FLP_TRY(flp_swap_width(s->pool, n_in, host_ids, dev_ids, 1, s->s_in, width));
    FLP_TRY(take_event(s, &r.done));
    FLP_TRY_HIP(hipEventRecord(r.done, s->s_in));
  }
  s->waiting.push_back(r);
  s->st.submitted++;
  s->st.blocks_in += n_in;
  s->st.blocks_out += n_out;
  return FLP_OK;
}

extern "C" flp_status fls_poll(fls_sched* s, int32_t max, int64_t* ready_ids, int32_t* n_ready) {
  if (!s || max < 0 || !n_ready || (max > 0 && !ready_ids)) {
    flp_set_error("fls_poll: invalid argument");
    return FLP_EINVAL;
  }
  std::lock_guard<std::mutex> lk(s->mu);
  int32_t n = 0;
  for (auto it = s->waiting.begin(); it != s->waiting.end() && n < max;) {
    bool ready = false;
    FLP_TRY(is_ready(*it, &ready));
    if (ready) {
      ready_ids[n++] = it->id;
      if (it->done) s->spare.push_back(it->done);
      it = s->waiting.erase(it);
    } else {
      ++it;                          // this one waits; a later request whose moves are done may still run
    }
  }
  *n_ready = n;
  s->st.polls++;
  if (n == 0) s->st.polls_empty++;
  s->st.ready_returned += n;
  return FLP_OK;
}

extern "C" flp_status fls_wait_next(fls_sched* s) {
  if (!s || s->manual) {
    flp_set_error("fls_wait_next: null planner, or a manual one (nothing to wait on)");
    return FLP_EINVAL;
  }
  hipEvent_t ev = nullptr;
  {
    std::lock_guard<std::mutex> lk(s->mu);
    if (s->waiting.empty() || s->waiting.front().complete) return FLP_OK;
    ev = s->waiting.front().done;
  }
  FLP_TRY_HIP(hipEventSynchronize(ev));    // outside the lock: other threads may submit meanwhile
  return FLP_OK;
}

extern "C" flp_status fls_stream_wait(fls_sched* s, int64_t req_id, void* compute_stream) {
  if (!s || s->manual) {
    flp_set_error("fls_stream_wait: null planner, or a manual one");
    return FLP_EINVAL;
  }
  std::lock_guard<std::mutex> lk(s->mu);
  for (auto it = s->waiting.begin(); it != s->waiting.end(); ++it) {
    if (it->id != req_id) continue;
    if (it->done) {
      FLP_TRY_HIP(hipStreamWaitEvent((hipStream_t)compute_stream, it->done, 0));
      s->spare.push_back(it->done);   // re-recorded only by a later submit, which is ordered after this wait call
    }
    s->waiting.erase(it);
    s->st.ready_returned++;
    return FLP_OK;
  }
  flp_set_error("fls_stream_wait: request %lld is not waiting", (long long)req_id);
  return FLP_EINVAL;
}

extern "C" flp_status fls_compute_enqueued(fls_sched* s, void* compute_stream) {
  if (!s) {
    flp_set_error("fls_compute_enqueued: null planner");
    return FLP_EINVAL;
  }
  std::lock_guard<std::mutex> lk(s->mu);
  if (s->manual) return FLP_OK;
  FLP_TRY_HIP(hipEventRecord(s->ev_compute, (hipStream_t)compute_stream));
  s->have_compute = true;
  return FLP_OK;
}

extern "C" flp_status fls_complete(fls_sched* s, int64_t req_id) {
  if (!s || !s->manual) {
    flp_set_error("fls_complete: null planner, or not a manual one");
    return FLP_EINVAL;
  }
  std::lock_guard<std::mutex> lk(s->mu);
  Request* r = find(s, req_id);
  if (!r) {
    flp_set_error("fls_complete: request %lld is not waiting", (long long)req_id);
    return FLP_EINVAL;
  }
  r->complete = true;
  return FLP_OK;
}

extern "C" flp_status fls_get_stats(const fls_sched* s, fls_stats* out) {
  if (!s || !out) {
    flp_set_error("fls_get_stats: null argument");
    return FLP_EINVAL;
  }
  std::lock_guard<std::mutex> lk(s->mu);
  *out = s->st;
  out->waiting = (int64_t)s->waiting.size();
  return FLP_OK;
}
