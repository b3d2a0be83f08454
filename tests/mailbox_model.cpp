// The mailbox protocol on the CPU: the library's own host side (mb::MailboxHost from csrc/mw_mailbox.hpp) against
// threads that play the resident kernel -- one leader, W workers per epoch, epochs one after the other as on a
// stream -- with short idle and life times so that kernels close and reopen all the time while the host keeps
// submitting, asks for stops at random and looks after orphaned tickets only when it "polls".  Checked: every chunk
// of every ticket is executed exactly once, by the worker that owns it, inside an epoch that admitted it; every
// kernel thread ends; nothing is served from a queue slot that has been rewritten.  Run plain and under TSan.
#include <atomic>
#include <chrono>
#include <condition_variable>
#include <cstdio>
#include <cstdlib>
#include <deque>
#include <mutex>
#include <random>
#include <thread>
#include <vector>

#include "../paper_2407_08980_amd/csrc/mw_mailbox.hpp"

using namespace mw::mb;
#define CHECK(c) do { if (!(c)) { std::fprintf(stderr, "CHECK failed: %s (line %d)\n", #c, __LINE__); std::abort(); } } while (0)
static double now() { return std::chrono::duration<double>(std::chrono::steady_clock::now().time_since_epoch()).count(); }

struct Model {
  // "device memory"
  std::atomic<uint32_t> tail{0}, stop{0};
  Desc q[kQueueDepth];
  std::atomic<uint32_t> q_ticket[kQueueDepth];  // which ticket's descriptor the slot holds (model-only bookkeeping)
  std::atomic<uint64_t> admit{0};
  std::atomic<uint64_t> closed_word{0};
  // what was executed
  std::vector<std::atomic<uint32_t>> done;   // per ticket: chunks executed
  std::vector<std::atomic<uint8_t>> once;    // per (ticket, chunk) in a flat table of max_chunks per ticket
  static constexpr uint32_t kMaxChunks = 40;
  int W;
  double idle_s, life_s;
  std::atomic<int> live_threads{0};
  std::atomic<long> epochs{0}, closes_idle{0}, closes_stop{0}, closes_life{0};
  // the "stream": kernels run one after the other
  std::mutex mu;
  std::condition_variable cv;
  std::deque<std::pair<uint32_t, uint32_t>> launches;
  bool quit = false;
  std::thread stream;

  Model(int w, size_t max_tickets, double idle, double life) : done(max_tickets + 2), once((max_tickets + 2) * kMaxChunks), W(w), idle_s(idle), life_s(life) {
    for (auto& x : q_ticket) x.store(0);
    stream = std::thread([this] { run_stream(); });
  }
  ~Model() {
    { std::lock_guard<std::mutex> g(mu); quit = true; }
    cv.notify_all();
    stream.join();
  }
  void run_stream() {
    for (;;) {
      std::pair<uint32_t, uint32_t> l;
      {
        std::unique_lock<std::mutex> g(mu);
        cv.wait(g, [this] { return quit || !launches.empty(); });
        if (launches.empty()) return;
        l = launches.front();
        launches.pop_front();
      }
      kernel(l.first, l.second);
    }
  }
  void kernel(uint32_t epoch, uint32_t first) {
    epochs += 1;
    // the leader's word is NOT initialised: it still holds the previous kernel's closing word, as on the device
    std::vector<std::thread> th;
    live_threads += W + 1;
    th.emplace_back([=] { leader(epoch, first); live_threads -= 1; });
    for (int w = 0; w < W; ++w) th.emplace_back([=] { worker(epoch, first, (uint32_t)w); live_threads -= 1; });
    for (auto& t : th) t.join();
  }
  void leader(uint32_t epoch, uint32_t first) {
    uint32_t go = first - 1;
    const double t0 = now();
    double t_last = t0;
    for (;;) {
      const uint32_t t = tail.load(std::memory_order_acquire), s = stop.load(std::memory_order_acquire);
      if (t != go && before(go, t) && t - first < kEpochTickets) {
        go = t;
        admit.store(make_admit(go, 0), std::memory_order_release);
        t_last = now();
        continue;
      }
      const double n = now();
      const bool by_stop = s == epoch, by_idle = n - t_last > idle_s, by_life = n - t0 > life_s;
      if (by_stop || by_idle || by_life) {
        (by_stop ? closes_stop : by_idle ? closes_idle : closes_life) += 1;
        admit.store(make_admit(go, epoch), std::memory_order_release);
        closed_word.store(make_closed(epoch, go), std::memory_order_release);
        return;
      }
    }
  }
  void worker(uint32_t epoch, uint32_t first, uint32_t w) {
    uint32_t next = first;
    const double t0 = now();
    for (;;) {
      const uint64_t a = admit.load(std::memory_order_acquire);
      const uint32_t go = (uint32_t)a;
      const bool closing = closing_epoch(a) == epoch;
      while (before(next - 1, go)) {
        CHECK(q_ticket[next % kQueueDepth].load(std::memory_order_acquire) == next);  // the slot still holds OUR ticket
        const Desc d = q[next % kQueueDepth];
        CHECK(d.gen == next && d.n_chunks >= 1 && d.n_chunks <= kMaxChunks);
        for (uint32_t c = 0; c < d.n_chunks; ++c) {
          if (owner(d.start, c, (uint32_t)W) != w) continue;
          CHECK(once[(size_t)next * kMaxChunks + c].fetch_add(1) == 0);  // never twice
          done[next].fetch_add(1);
        }
        CHECK(q_ticket[next % kQueueDepth].load(std::memory_order_acquire) == next);  // ... and was not rewritten meanwhile
        ++next;
      }
      if (closing && next - 1 == go) return;
      CHECK(now() - t0 < 20.0);  // the safety net must never be what ends a worker
    }
  }
  // Port
  void write_desc(uint32_t index, const Desc& d) {
    q_ticket[index].store(0, std::memory_order_release);
    q[index] = d;
    q_ticket[index].store(d.gen, std::memory_order_release);
  }
  void ring(uint32_t t) { tail.store(t, std::memory_order_release); }
  void ask_stop(uint32_t epoch) { stop.store(epoch, std::memory_order_release); }
  uint64_t closed() { return closed_word.load(std::memory_order_acquire); }
  // A launch can fail (the runtime may refuse it): every `fail_every`-th does, when set.  Nothing is started then; the
  // descriptors stay queued and a later attend() must start the kernel.
  int fail_every = 0;
  long launch_calls = 0, failed_launches = 0;
  int launch(uint32_t epoch, uint32_t first) {
    if (fail_every && ++launch_calls % fail_every == 0) {
      ++failed_launches;
      return 1;
    }
    { std::lock_guard<std::mutex> g(mu); launches.emplace_back(epoch, first); }
    cv.notify_all();
    return 0;
  }
};

int main(int argc, char** argv) {
  const double seconds = argc > 1 ? std::atof(argv[1]) : 1.0;
  const size_t max_tickets = 3000000;
  long total_epochs = 0, total_tickets = 0, refused = 0;
  for (unsigned seed = 1; seed <= 3; ++seed) {
    const int W = seed == 1 ? 3 : seed == 2 ? 7 : 5;
    Model m(W, max_tickets, /*idle*/ seed == 1 ? 30e-6 : 2e-3, /*life*/ seed == 2 ? 200e-6 : 5e-3);
    if (seed == 3) m.fail_every = 7;
    MailboxHost<Model> host(&m);
    std::mt19937 rng(seed);
    std::vector<uint32_t> chunks(max_tickets + 2, 0);
    uint32_t issued = 0, verified = 0;
    const double t_end = now() + seconds / 3;
    std::vector<Desc> batch;
    while (now() < t_end && issued + 400 < max_tickets) {
      const unsigned r = rng() % 100;
      if (r < 55) {  // a flush: a window of small operations
        uint32_t n = 1 + rng() % (r < 5 ? 300 : 20);
        if (host.room() < n) {  // this epoch's tickets are used up: the library launches these the ordinary way
          host.stop();
          ++refused;
        } else {
          batch.clear();
          for (uint32_t i = 0; i < n; ++i) {
            Desc d{};
            d.gen = issued + 1 + i;  // model-only: the descriptor names its ticket
            d.n_chunks = 1 + rng() % (rng() % 4 == 0 ? Model::kMaxChunks : 3);
            chunks[issued + 1 + i] = d.n_chunks;
            batch.push_back(d);
          }
          uint32_t first = 0;
          const int rc = host.submit(batch.data(), n, &first);  // (a failed launch leaves the descriptors queued)
          CHECK((rc == 0 || m.fail_every) && first == issued + 1);
          issued += n;
        }
      } else if (r < 60) {
        if (seed != 2 || rng() % 64 == 0) host.stop();  // a bulk launch is coming (rarely with seed 2: its kernels end by lifetime)
      } else if (r < 90) {  // a poll: look after orphans, see what is complete
        if (host.needs_attention()) CHECK(host.attend() == 0 || m.fail_every);
        while (verified < issued && m.done[verified + 1].load() == chunks[verified + 1]) ++verified;
      } else {
        std::this_thread::sleep_for(std::chrono::microseconds(rng() % 120));  // long enough for the kernel to idle out
      }
    }
    const double t_drain = now();
    while (verified < issued) {  // the worker polls until everything is complete
      if (host.needs_attention()) CHECK(host.attend() == 0 || m.fail_every);
      while (verified < issued && m.done[verified + 1].load() == chunks[verified + 1]) ++verified;
      CHECK(now() - t_drain < 20.0);
    }
    host.stop();
    const double t_stop = now();
    while (host.running()) CHECK(now() - t_stop < 20.0);  // every kernel ends
    while (m.live_threads.load() != 0) CHECK(now() - t_stop < 20.0);
    for (uint32_t t = 1; t <= issued; ++t) {
      CHECK(m.done[t].load() == chunks[t]);
      for (uint32_t c = 0; c < chunks[t]; ++c) CHECK(m.once[(size_t)t * Model::kMaxChunks + c].load() == 1);
    }
    std::printf("seed %u: workers %d, tickets %u, epochs %ld (closed by idle %ld, by stop %ld, by life %ld)\n", seed, W, issued,
                m.epochs.load(), m.closes_idle.load(), m.closes_stop.load(), m.closes_life.load());
    if (m.fail_every) std::printf("        %ld of %ld launches refused, every descriptor served all the same\n", m.failed_launches, m.launch_calls);
    total_epochs += m.epochs.load();
    total_tickets += issued;
  }
  std::printf("mailbox model: %ld tickets over %ld epochs, %ld windows refused for lack of room, all chunks executed exactly once\n", total_tickets,
              total_epochs, refused);
  return 0;
}
