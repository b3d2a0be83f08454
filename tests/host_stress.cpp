// Stress driver for the host runtime, linked with mw_host.cpp and the byte-less device double and
// built with sanitizers by tests/test_host_sanitizers.py.  No payload exists: buffers are fake
// addresses.  Mode "single": one thread, random posts of all eight operations, aborts, ring and
// handle exhaustion, completion in random order; invariants are checked at the end.  Mode "threads":
// several posting threads with their own worlds, a completion thread, heartbeats and the watchdog
// thread, all through the one library lock.
#include <atomic>
#include <chrono>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <random>
#include <thread>
#include <vector>

#include "../include/mw.h"

extern "C" {
int mwt_complete(int n, int from_back);
int mwt_pending(void);
int mwt_launch_count(void);
int mwt_fail_next_launch(void);
}

#define CHECK(c) do { if (!(c)) { std::fprintf(stderr, "CHECK failed: %s (line %d)\n", #c, __LINE__); std::exit(1); } } while (0)

static int single(unsigned seed) {
  std::mt19937 rng(seed);
  auto pick = [&](int n) { return (int)(rng() % (unsigned)n); };
  CHECK(mw_config_set("ring_depth", 4) == MW_OK);
  CHECK(mw_config_set("max_rings", 12) == MW_OK);
  CHECK(mw_config_set("handle_capacity", 512) == MW_OK);
  CHECK(mw_init(0, 16) == MW_OK);
  struct W { int id; int n; bool alive; };
  std::vector<W> worlds;
  int next_id = 0;
  std::vector<mw_handle> handles;
  long posted = 0, refused = 0;
  for (int step = 0; step < 60000; ++step) {
    int r = pick(100);
    if (r < 3 || worlds.empty()) {  // create a world (may hit the ring limit)
      int n = 2 + pick(3);
      int ids[4];
      int base = pick(16);
      for (int i = 0; i < n; ++i) ids[i] = (base + i * 3) % 16;
      int rc = mw_world_create(next_id, ids, n);
      CHECK(rc == MW_OK || rc == MW_ENOMEM || rc == MW_EINVAL);
      if (rc == MW_OK) worlds.push_back(W{next_id, n, true});
      ++next_id;
    } else if (r < 5) {
      W& w = worlds[(size_t)pick((int)worlds.size())];
      CHECK(mw_world_abort(w.id) == MW_OK);
      w.alive = false;
    } else if (r < 6) {
      int k = pick(16);
      CHECK(mw_worker_abort(k) == MW_OK);
      for (W& w : worlds) w.alive = mw_world_state(w.id) == MW_ALIVE;
    } else if (r < 20) {
      mwt_complete(1 + pick(6), pick(2));
    } else if (r < 30) {
      int rc = mw_flush();
      CHECK(rc == MW_OK || rc == MW_EHIP);
    } else if (r < 31) {
      mwt_fail_next_launch();
    } else if (r < 45 && !handles.empty()) {
      for (int k = 0; k < 8; ++k) {
        int st = mw_poll(handles[(size_t)pick((int)handles.size())]);
        CHECK(st == MW_DONE || st == MW_PENDING || st == MW_BROKEN || st == MW_EMISMATCH || st == MW_EBADHANDLE ||
              st == MW_EHIP);
      }
    } else {
      W& w = worlds[(size_t)pick((int)worlds.size())];
      mw_handle h = 0;
      void* buf = (void*)(uintptr_t)(0x10000 + 64 * pick(1000));
      void* buf2 = (void*)(uintptr_t)(0x900000 + 64 * pick(1000));
      size_t count = (size_t)pick(3) * 100;
      mw_dtype dt = pick(2) ? MW_F32 : MW_BF16;
      int a = pick(w.n), b = pick(w.n), rc;
      switch (pick(8)) {
        case 0: rc = mw_send(w.id, a, b, buf, count, dt, MW_STREAM_NONE, &h); break;
        case 1: rc = mw_recv(w.id, a, b, buf, count, dt, MW_STREAM_NONE, &h); break;
        case 2: rc = mw_broadcast(w.id, a, b, buf, count, dt, MW_STREAM_NONE, &h); break;
        case 3: rc = mw_allreduce_sum(w.id, a, buf, count, dt, MW_STREAM_NONE, &h); break;
        case 4: rc = mw_reduce_sum(w.id, a, b, buf, count, dt, MW_STREAM_NONE, &h); break;
        case 5: rc = mw_all_gather(w.id, a, buf, buf2, count, dt, MW_STREAM_NONE, &h); break;
        case 6: rc = mw_gather(w.id, a, b, buf, buf2, count, dt, MW_STREAM_NONE, &h); break;
        default: rc = mw_scatter(w.id, a, b, buf, buf2, count, dt, MW_STREAM_NONE, &h); break;
      }
      CHECK(rc == MW_OK || rc == MW_EBROKEN || rc == MW_EINVAL || rc == MW_ENOMEM);
      if (rc == MW_OK) {
        CHECK(h != 0);
        handles.push_back(h);
        ++posted;
      } else {
        ++refused;
        if (rc == MW_EBROKEN) CHECK(mw_world_state(w.id) == MW_BROKEN);
      }
      if (handles.size() > 300) handles.erase(handles.begin(), handles.begin() + 150);
    }
  }
  // drain: launch and complete everything, then break every world; nothing may stay matched-but-unfinished
  for (int i = 0; i < 1000 && (mw_pending_ops() > 0); ++i) {
    mw_flush();
    mwt_complete(1000, 0);
    for (mw_handle h : handles) mw_poll(h);
    for (W& w : worlds) mw_world_state(w.id);
  }
  for (W& w : worlds) CHECK(mw_world_abort(w.id) == MW_OK);
  mwt_complete(100000, 0);
  for (mw_handle h : handles) {
    int st = mw_poll(h);
    CHECK(st == MW_DONE || st == MW_BROKEN || st == MW_EMISMATCH || st == MW_EBADHANDLE);
  }
  CHECK(mw_pending_ops() == 0);
  std::printf("single: %ld posts accepted, %ld refused, %d worlds, %d launches\n", posted, refused, next_id,
              mwt_launch_count());
  CHECK(mw_shutdown() == MW_OK);
  return 0;
}

static int threads() {
  CHECK(mw_config_set("ring_depth", 16) == MW_OK);
  CHECK(mw_config_set("max_rings", 64) == MW_OK);
  CHECK(mw_config_set("handle_capacity", 4096) == MW_OK);
  const int T = 4;
  CHECK(mw_init(0, 3 * T) == MW_OK);
  for (int t = 0; t < T; ++t) {
    int a[2] = {3 * t, 3 * t + 1}, b[3] = {3 * t, 3 * t + 1, 3 * t + 2};
    CHECK(mw_world_create(10 * t, a, 2) == MW_OK);
    CHECK(mw_world_create(10 * t + 1, b, 3) == MW_OK);
  }
  CHECK(mw_watchdog_start(0.25, 0.01) == MW_OK);
  std::atomic<bool> stop{false}, all_done{false};
  std::atomic<int> finished{0};
  std::atomic<long> done{0}, broken{0};
  std::thread completer([&] {
    while (!stop.load()) {
      mwt_complete(8, 0);
      std::this_thread::sleep_for(std::chrono::microseconds(50));
    }
  });
  std::vector<std::thread> posters;
  for (int t = 0; t < T; ++t) {
    posters.emplace_back([&, t] {
      std::mt19937 rng(100 + (unsigned)t);
      for (int it = 0; it < 3000; ++it) {
        // worker 3t+2 of the last thread stops reporting half way: its 3-rank world breaks
        for (int k = 0; k < 3; ++k)
          if (!(t == T - 1 && k == 2 && it > 1500)) mw_heartbeat(3 * t + k);
        mw_handle h[5] = {0, 0, 0, 0, 0};
        int rc = mw_send(10 * t, 0, 1, (void*)0x1000, 16, MW_F32, MW_STREAM_NONE, &h[0]);
        CHECK(rc == MW_OK);
        rc = mw_recv(10 * t, 0, 1, (void*)0x2000, 16, MW_F32, MW_STREAM_NONE, &h[1]);
        CHECK(rc == MW_OK);
        int n_coll = 0;
        for (int r = 0; r < 3; ++r) {
          rc = mw_allreduce_sum(10 * t + 1, r, (void*)(uintptr_t)(0x3000 + 0x100 * r), 16, MW_F32, MW_STREAM_NONE, &h[2 + r]);
          CHECK(rc == MW_OK || rc == MW_EBROKEN);
          n_coll += rc == MW_OK;
        }
        mw_flush();
        for (int spins = 0;; ++spins) {
          int pend = 0;
          for (int k = 0; k < 5; ++k) {
            if (!h[k]) continue;
            int st = mw_poll(h[k]);
            CHECK(st == MW_DONE || st == MW_PENDING || st == MW_BROKEN);
            pend += st == MW_PENDING;
            if (st != MW_PENDING) {
              (st == MW_DONE ? done : broken) += 1;
              h[k] = 0;
            }
          }
          if (!pend) break;
          CHECK(spins < 2000000);
          if ((rng() & 15) == 0) std::this_thread::yield();
        }
      }
      finished += 1;
      while (!all_done.load()) {  // stay alive until everybody is through: only the silent worker may time out
        for (int k = 0; k < 3; ++k)
          if (!(t == T - 1 && k == 2)) mw_heartbeat(3 * t + k);
        std::this_thread::sleep_for(std::chrono::milliseconds(1));
      }
    });
  }
  for (int waited = 0; finished.load() < T || mw_world_state(10 * (T - 1) + 1) == MW_ALIVE; ++waited) {
    CHECK(waited < 60000);
    std::this_thread::sleep_for(std::chrono::milliseconds(1));
  }
  CHECK(mw_watchdog_stop() == MW_OK);
  all_done.store(true);
  for (auto& p : posters) p.join();
  stop.store(true);
  completer.join();
  CHECK(mw_world_state(10 * (T - 1) + 1) == MW_BROKEN);  // the silent worker's world
  CHECK(mw_world_state(10 * (T - 1)) == MW_ALIVE);       // its neighbours' two-rank world is untouched
  for (int t = 0; t + 1 < T; ++t) CHECK(mw_world_state(10 * t + 1) == MW_ALIVE);
  CHECK(mw_worker_state(3 * (T - 1) + 2) == MW_BROKEN);
  std::printf("threads: %ld handles done, %ld broken\n", done.load(), broken.load());
  CHECK(mw_watchdog_stop() == MW_OK);
  CHECK(mw_shutdown() == MW_OK);
  return 0;
}

int main(int argc, char** argv) {
  if (argc > 1 && !std::strcmp(argv[1], "threads")) return threads();
  for (unsigned seed = 1; seed <= 3; ++seed)
    if (single(seed)) return 1;
  return 0;
}
