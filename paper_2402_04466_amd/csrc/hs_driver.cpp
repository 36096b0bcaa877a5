// Native stream driver: feeds several applications concurrently, one submitting thread each,
// the way the paper runs one process per application instance (Section V-B), at a fixed frame
// rate with absolute deadlines or back to back.  It sits on top of the public calls only
// (hs_submit_* / hs_poll_* / hs_wait_*), so what it measures is what any caller of the library
// gets -- without an interpreter between the frames.
#include <pthread.h>
#include <sched.h>
#include <sys/prctl.h>
#include <time.h>

#include <cerrno>
#include <cstring>
#include <new>
#include <string>
#include <thread>
#include <vector>

#include "hs.h"
#include "hs_internal.h"

namespace {

inline uint64_t now_ns() {
  timespec ts;
  clock_gettime(CLOCK_MONOTONIC, &ts);
  return (uint64_t)ts.tv_sec * 1000000000ull + (uint64_t)ts.tv_nsec;
}

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
  if (f->group) return hs_submit_group(f->group, fr[0], ou[0], (uint64_t)k);
  return hs_submit_batch(f->app, fr, ou, (uint64_t)k);
}

hs_status feed_poll(const hs_feed* f, hs_result* out) {
  return f->group ? hs_poll_group(f->group, out) : hs_poll_batch(f->app, out);
}

hs_status feed_wait(const hs_feed* f, hs_result* out) {
  const uint64_t ten_s = 10000000000ull;
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
    if ((!f.app && !f.group) || !f.d_frames || !f.d_outs || f.n_frames < 1 || f.n_outs < 1 ||
        f.batch < 1 || f.results_per_frame < 1 || !results[i] || (f.group && f.batch != 1)) {
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
