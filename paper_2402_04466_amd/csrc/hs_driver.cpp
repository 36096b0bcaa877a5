// Native stream driver: feeds several applications concurrently, one submitting thread each,
// the way the paper runs one process per application instance (Section V-B), at a fixed frame
// rate with absolute deadlines or back to back.  It sits on top of the public calls only
// (hs_submit_* / hs_poll_* / hs_wait_*), so what it measures is what any caller of the library
// gets -- without an interpreter between the frames.  Also here, on the same footing: the
// per-stream front of a batched application (hs_mux).
#include <pthread.h>
#include <sched.h>
#include <sys/prctl.h>
#include <time.h>

#include <cerrno>
#include <algorithm>
#include <chrono>
#include <condition_variable>
#include <cstring>
#include <deque>
#include <mutex>
#include <new>
#include <string>
#include <thread>
#include <vector>

#include "hs.h"
#include "hs_internal.h"

static inline uint64_t now_ns() {
  timespec ts;
  clock_gettime(CLOCK_MONOTONIC, &ts);
  return (uint64_t)ts.tv_sec * 1000000000ull + (uint64_t)ts.tv_nsec;
}

// ---- per-stream front of a batched application --------------------------------------------------
// The streams of the batch hand over their frames one by one, each with its own arrival stamp;
// the batch is submitted when its last frame arrives, and every stream collects its own result.
struct hs_mux {
  hs_app* app = nullptr;
  int batch = 0;
  std::mutex mu;
  std::condition_variable cv;
  // the batch being assembled
  std::vector<const uint8_t*> frames;
  std::vector<uint8_t*> outs;
  std::vector<uint64_t> ids, t_submit;
  std::vector<char> have;
  int n_have = 0;
  uint64_t n_batches = 0;
  // per submitted batch, in submit order: what to restore in its results
  struct Rec { std::vector<uint64_t> ids, t_submit; };
  std::deque<Rec> in_flight;
  // finished batches not yet collected by every stream, oldest first
  struct Done { std::vector<hs_result> r; std::vector<char> taken; int n_taken = 0; };
  std::deque<Done> done;
  bool draining = false;   // a thread is blocked in hs_wait_batch on behalf of all
  std::vector<hs_result> tmp;
};

// Files the batch the application has just delivered into m->tmp (mux lock held).
static void mux_file(hs_mux* m) {
  hs_mux::Done d;
  d.r = m->tmp;
  d.taken.assign((size_t)m->batch, 0);
  if (!m->in_flight.empty()) {
    const hs_mux::Rec& rec = m->in_flight.front();
    for (int j = 0; j < m->batch; ++j) {
      d.r[(size_t)j].frame_id = rec.ids[(size_t)j];
      d.r[(size_t)j].t_submit_ns = rec.t_submit[(size_t)j];   // the stream's own arrival
    }
    m->in_flight.pop_front();
  }
  m->done.push_back(std::move(d));
}

// Oldest finished result of `stream`, if any (mux lock held).
static bool mux_take(hs_mux* m, int stream, hs_result* out) {
  for (hs_mux::Done& d : m->done) {
    if (d.taken[(size_t)stream]) continue;
    *out = d.r[(size_t)stream];
    out->t_observed_ns = now_ns();
    d.taken[(size_t)stream] = 1;
    ++d.n_taken;
    while (!m->done.empty() && m->done.front().n_taken == m->batch) m->done.pop_front();
    return true;
  }
  return false;
}

extern "C" hs_status hs_create_mux(hs_app* app, int batch, hs_mux** out) {
  using hs::set_error;
  if (!app || !out || batch < 1 || batch > 16) { set_error("hs_create_mux: bad argument"); return HS_E_INVAL; }
  // the batch buffers below are handed to hs_submit_batch / hs_poll_batch, which move exactly
  // the application's batch of entries
  if (batch != hs_internal_app_batch(app)) {
    set_error("hs_create_mux: batch %d given, the application batches %d streams", batch,
              hs_internal_app_batch(app));
    return HS_E_INVAL;
  }
  if (hs_internal_app_grouped(app)) {
    set_error("hs_create_mux: the application is a member of a group");
    return HS_E_STATE;
  }
  try {
    hs_mux* m = new hs_mux();
    m->app = app;
    m->batch = batch;
    m->frames.assign((size_t)batch, nullptr);
    m->outs.assign((size_t)batch, nullptr);
    m->ids.assign((size_t)batch, 0);
    m->t_submit.assign((size_t)batch, 0);
    m->have.assign((size_t)batch, 0);
    m->tmp.resize((size_t)batch);
    *out = m;
    return HS_OK;
  } catch (const std::exception& e) {
    set_error("hs_create_mux: %s", e.what());
    return HS_E_NOMEM;
  }
}

extern "C" hs_status hs_destroy_mux(hs_mux* mux) {
  if (!mux) { hs::set_error("hs_destroy_mux: NULL"); return HS_E_INVAL; }
  delete mux;
  return HS_OK;
}

extern "C" hs_status hs_mux_submit(hs_mux* m, int stream, const uint8_t* d_frame,
                                   uint8_t* d_overlay_out, uint64_t frame_id) {
  using hs::set_error;
  const uint64_t t_arrival = now_ns();
  if (!m || stream < 0 || stream >= m->batch || !d_frame || !d_overlay_out) {
    set_error("hs_mux_submit: bad argument");
    return HS_E_INVAL;
  }
  try {
    std::lock_guard<std::mutex> lk(m->mu);
    const size_t j = (size_t)stream;
    if (m->have[j]) {
      set_error("hs_mux_submit: stream %d already has a frame waiting for its batch", stream);
      return HS_E_QUEUE_FULL;
    }
    m->frames[j] = d_frame; m->outs[j] = d_overlay_out; m->ids[j] = frame_id;
    m->t_submit[j] = t_arrival;
    if (m->n_have + 1 < m->batch) {
      m->have[j] = 1;
      ++m->n_have;
      return HS_OK;
    }
    // the last frame of the batch: hand the batch to the application
    const hs_status st = hs_submit_batch(m->app, m->frames.data(), m->outs.data(), m->n_batches);
    if (st != HS_OK) return st;   // this frame was not taken; the others keep waiting
    m->in_flight.push_back(hs_mux::Rec{m->ids, m->t_submit});
    ++m->n_batches;
    std::fill(m->have.begin(), m->have.end(), 0);
    m->n_have = 0;
    return HS_OK;
  } catch (const std::exception& e) {
    set_error("hs_mux_submit: %s", e.what());
    return HS_E_NOMEM;
  }
}

extern "C" hs_status hs_mux_poll(hs_mux* m, int stream, hs_result* out) {
  using hs::set_error;
  if (!m || !out || stream < 0 || stream >= m->batch) { set_error("hs_mux_poll: bad argument"); return HS_E_INVAL; }
  try {
    std::lock_guard<std::mutex> lk(m->mu);
    for (;;) {
      if (mux_take(m, stream, out)) return HS_OK;
      if (m->draining) break;   // another thread is fetching: it will file what it gets
      const hs_status st = hs_poll_batch(m->app, m->tmp.data());
      if (st == HS_E_NOT_READY) break;
      if (st != HS_OK) return st;
      mux_file(m);
    }
    set_error("hs_mux_poll: no finished frame for stream %d", stream);
    return HS_E_NOT_READY;
  } catch (const std::exception& e) {
    set_error("hs_mux_poll: %s", e.what());
    return HS_E_NOMEM;
  }
}

extern "C" hs_status hs_mux_wait(hs_mux* m, int stream, hs_result* out, uint64_t timeout_ns) {
  using hs::set_error;
  if (!m || !out || stream < 0 || stream >= m->batch) { set_error("hs_mux_wait: bad argument"); return HS_E_INVAL; }
  try {
    const auto deadline = std::chrono::steady_clock::now() + std::chrono::nanoseconds(timeout_ns);
    std::unique_lock<std::mutex> lk(m->mu);
    for (;;) {
      if (mux_take(m, stream, out)) return HS_OK;
      const auto left = std::chrono::duration_cast<std::chrono::nanoseconds>(
                            deadline - std::chrono::steady_clock::now()).count();
      if (left <= 0) { set_error("hs_mux_wait: timed out"); return HS_E_NOT_READY; }
      if (m->draining) {   // another thread is fetching the next batch for everybody
        m->cv.wait_for(lk, std::chrono::nanoseconds(std::min<int64_t>(left, 20000000)));
        continue;
      }
      // fetch the next finished batch on behalf of every stream; one thread at a time talks to
      // the application, so batches are filed in the order they are delivered
      hs_status st = hs_poll_batch(m->app, m->tmp.data());
      if (st == HS_E_NOT_READY) {
        m->draining = true;
        lk.unlock();
        std::vector<hs_result> got((size_t)m->batch);
        st = hs_wait_batch(m->app, got.data(), (uint64_t)std::min<int64_t>(left, 20000000));
        lk.lock();
        m->draining = false;
        if (st == HS_OK) m->tmp = got;
        m->cv.notify_all();
      }
      if (st == HS_OK) mux_file(m);
      else if (st != HS_E_NOT_READY) return st;
    }
  } catch (const std::exception& e) {
    set_error("hs_mux_wait: %s", e.what());
    return HS_E_NOMEM;
  }
}

namespace {

struct Worker {
  const hs_feed* feed = nullptr;
  int per_frame = 1;              // results per frame (batch streams or group members)
  hs_result* results = nullptr;   // [n_frames][per_frame]
  int64_t* lateness = nullptr;    // [n_frames] or NULL
  int n_frames = 0;
  uint64_t t0 = 0, period = 0;    // period 0: back to back
  int dropped = 0;
  hs_status status = HS_OK;
  std::string error;
};

hs_status feed_submit(const hs_feed* f, int k) {
  const uint8_t* const* fr = f->d_frames + (size_t)(k % f->n_frames) * f->batch;
  uint8_t* const* ou = f->d_outs + (size_t)(k % f->n_outs) * f->batch;
  if (f->mux) return hs_mux_submit(f->mux, f->mux_stream, fr[0], ou[0], (uint64_t)k);
  if (f->group) return hs_submit_group(f->group, fr[0], ou[0], (uint64_t)k);
  return hs_submit_batch(f->app, fr, ou, (uint64_t)k);
}

hs_status feed_poll(const hs_feed* f, hs_result* out) {
  if (f->mux) return hs_mux_poll(f->mux, f->mux_stream, out);
  return f->group ? hs_poll_group(f->group, out) : hs_poll_batch(f->app, out);
}

hs_status feed_wait(const hs_feed* f, hs_result* out) {
  const uint64_t ten_s = 10000000000ull;
  if (f->mux) return hs_mux_wait(f->mux, f->mux_stream, out, ten_s);
  return f->group ? hs_wait_group(f->group, out, ten_s) : hs_wait_batch(f->app, out, ten_s);
}

void worker_main(Worker* w) {
  const hs_feed* f = w->feed;
  if (f->cpu >= 0) {   // paper Section IV-C: the application's thread on a core of its own
    cpu_set_t set;
    CPU_ZERO(&set);
    CPU_SET(f->cpu, &set);
    (void)pthread_setaffinity_np(pthread_self(), sizeof(set), &set);
  }
  if (w->period) (void)prctl(PR_SET_TIMERSLACK, 1000UL);   // wake within 1 us of a deadline, not 50
  int got = 0;   // frames whose results have been collected, in order
  auto fail = [&](hs_status st) {
    w->status = st;
    w->error = hs_last_error();
  };
  auto slot = [&](int i) { return w->results + (size_t)i * w->per_frame; };
  for (int k = 0; k < w->n_frames; ++k) {
    for (;;) {   // collect whatever has finished
      const hs_status st = feed_poll(f, slot(got));
      if (st == HS_E_NOT_READY) break;
      if (st != HS_OK) return fail(st);
      ++got;
    }
    if (w->period) {
      const uint64_t deadline = w->t0 + (uint64_t)k * w->period;
      timespec ts;
      ts.tv_sec = (time_t)(deadline / 1000000000ull);
      ts.tv_nsec = (long)(deadline % 1000000000ull);
      while (clock_nanosleep(CLOCK_MONOTONIC, TIMER_ABSTIME, &ts, nullptr) == EINTR) {}
      if (w->lateness) w->lateness[k] = (int64_t)(now_ns() - deadline);
    }
    for (;;) {
      const hs_status st = feed_submit(f, k);
      if (st == HS_OK) break;
      if (st != HS_E_QUEUE_FULL) return fail(st);
      if (w->period) {   // a paced source does not wait: the frame is lost
        ++w->dropped;
        break;
      }
      const hs_status sw = feed_wait(f, slot(got));   // back to back: make room, try again
      if (sw != HS_OK) return fail(sw);
      ++got;
    }
  }
  while (got + w->dropped < w->n_frames) {
    const hs_status st = feed_wait(f, slot(got));
    if (st != HS_OK) return fail(st);
    ++got;
  }
}

}  // namespace

extern "C" hs_status hs_run_feeds(const hs_feed* feeds, int n_feeds, double fps, int n_frames,
                                  hs_result* const* results, int* dropped,
                                  int64_t* const* lateness_ns, double* elapsed_s) {
  using hs::set_error;
  if (!feeds || !results || n_feeds < 1 || n_frames < 1 || !(fps >= 0.0)) {
    set_error("hs_run_feeds: bad argument");
    return HS_E_INVAL;
  }
  for (int i = 0; i < n_feeds; ++i) {
    const hs_feed& f = feeds[i];
    if ((!f.app && !f.group && !f.mux) || ((f.group || f.mux) && f.batch != 1) || !f.d_frames || !f.d_outs || f.n_frames < 1 || f.n_outs < 1 ||
        f.batch < 1 || f.results_per_frame < 1 || !results[i]) {
      set_error("hs_run_feeds: feed %d is incomplete", i);
      return HS_E_INVAL;
    }
  }
  try {
    std::vector<Worker> workers((size_t)n_feeds);
    std::vector<std::thread> threads;
    const uint64_t t0 = now_ns() + 20000000ull;   // first deadline 20 ms from now
    for (int i = 0; i < n_feeds; ++i) {
      Worker& w = workers[(size_t)i];
      w.feed = &feeds[i];
      w.per_frame = feeds[i].results_per_frame;
      w.results = results[i];
      w.lateness = lateness_ns ? lateness_ns[i] : nullptr;
      w.n_frames = n_frames;
      w.t0 = t0;
      w.period = fps > 0.0 ? (uint64_t)(1e9 / fps) : 0;
    }
    const uint64_t t_begin = now_ns();
    for (int i = 0; i < n_feeds; ++i) threads.emplace_back(worker_main, &workers[(size_t)i]);
    for (std::thread& t : threads) t.join();
    if (elapsed_s) *elapsed_s = (double)(now_ns() - t_begin) * 1e-9;
    hs_status st = HS_OK;
    for (int i = 0; i < n_feeds; ++i) {
      if (dropped) dropped[i] = workers[(size_t)i].dropped;
      if (st == HS_OK && workers[(size_t)i].status != HS_OK) {
        st = workers[(size_t)i].status;
        set_error("hs_run_feeds: feed %d: %s", i, workers[(size_t)i].error.c_str());
      }
    }
    return st;
  } catch (const std::exception& e) {
    set_error("hs_run_feeds: %s", e.what());
    return HS_E_NOMEM;
  }
}
