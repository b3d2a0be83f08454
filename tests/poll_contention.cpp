// How much one mw_poll costs when many host threads busy-poll at once (Sec. 3.3: every worker's communicator
// busy-waits on the status of its operations, one core each).  Linked with mw_host.cpp and the byte-less device
// double.  T poller threads each own a world and spin on mw_poll of an operation that is in flight (the double
// never completes it), while the main thread keeps posting, flushing and polling in a world of its own; printed:
// nanoseconds per poll as seen by the pollers, and per post + flush + poll round of the main thread.
#include <atomic>
#include <chrono>
#include <cstdio>
#include <cstdlib>
#include <thread>
#include <vector>

#include "../include/mw.h"

extern "C" int mwt_complete(int n, int from_back);

#define CHECK(c) do { if (!(c)) { std::fprintf(stderr, "CHECK failed: %s (line %d)\n", #c, __LINE__); std::exit(1); } } while (0)

static double now() { return std::chrono::duration<double>(std::chrono::steady_clock::now().time_since_epoch()).count(); }

int main(int argc, char** argv) {
  const double seconds = argc > 1 ? std::atof(argv[1]) : 0.3;
  for (int T : {1, 8, 16, 32}) {
    CHECK(mw_init(0, 2 * T + 2) == MW_OK);
    std::vector<mw_handle> spin((size_t)T);
    for (int t = 0; t < T; ++t) {
      int ids[2] = {2 * t, 2 * t + 1};
      CHECK(mw_world_create(t, ids, 2) == MW_OK);
      mw_handle hs;
      CHECK(mw_send(t, 0, 1, (void*)0x1000, 16, MW_F32, MW_STREAM_NONE, &hs) == MW_OK);
      CHECK(mw_recv(t, 0, 1, (void*)0x2000, 16, MW_F32, MW_STREAM_NONE, &spin[(size_t)t]) == MW_OK);
    }
    int ids[2] = {2 * T, 2 * T + 1};
    CHECK(mw_world_create(T, ids, 2) == MW_OK);
    CHECK(mw_flush() == MW_OK);  // the pollers' operations are in flight from here on and stay there
    std::atomic<bool> go{false}, stop{false};
    std::vector<long> polls((size_t)T, 0);
    std::vector<std::thread> th;
    for (int t = 0; t < T; ++t)
      th.emplace_back([&, t] {
        while (!go.load()) {}
        long n = 0;
        while (!stop.load(std::memory_order_relaxed)) {
          CHECK(mw_poll(spin[(size_t)t]) == MW_PENDING);
          ++n;
        }
        polls[(size_t)t] = n;
      });
    go.store(true);
    const double t0 = now();
    long rounds = 0;
    while (now() - t0 < seconds) {  // the worker that makes progress: post, launch, see it complete
      mw_handle a, b;
      CHECK(mw_send(T, 0, 1, (void*)0x3000, 16, MW_F32, MW_STREAM_NONE, &a) == MW_OK);
      CHECK(mw_recv(T, 0, 1, (void*)0x4000, 16, MW_F32, MW_STREAM_NONE, &b) == MW_OK);
      CHECK(mw_flush() == MW_OK);
      CHECK(mwt_complete(1, 1) == 1);  // the newest launched operation: this one
      CHECK(mw_poll(b) == MW_DONE && mw_poll(a) == MW_DONE);
      ++rounds;
    }
    const double dt = now() - t0;
    stop.store(true);
    for (auto& x : th) x.join();
    long total = 0;
    for (long n : polls) total += n;
    std::printf("threads %2d: %8.1f ns per poll (per polling thread), %8.1f ns per post+flush+poll round of the posting thread\n", T,
                dt * 1e9 * T / (double)total, dt * 1e9 / (double)rounds);
    std::fflush(stdout);
    CHECK(mw_shutdown() == MW_OK);
  }
  return 0;
}
