// Test double of the device backend.  It moves NO payload bytes and is never part
// of the product library: it is linked with mw_host.cpp into libmw_hostcheck.so so
// that the host state machine (matching, handles, ring slots, abort, deferred ring
// release) can be exercised on a machine without a GPU.  "Launches" are recorded;
// the test decides when the recorded operations complete.
#include <atomic>
#include <cstring>
#include <deque>
#include <mutex>
#include <vector>

#include "../../include/mw.h"
#include "mw_internal.hpp"

namespace mw {
namespace {

struct Recorded {
  LaunchOp op;
  int launch_id;
};

struct NullState {
  std::vector<uint32_t> flags;
  std::vector<RingHeader> headers;
  std::deque<Recorded> pending;       // launched, not yet completed by the test
  std::vector<Recorded> log;          // everything ever launched
  std::vector<int> launch_sizes;      // operations per launch
  std::vector<int> launch_streams;    // distinct streams waited on per launch
  int marks = 0;
  bool fail_next_launch = false;
  std::atomic<bool> attention{false};  // "queued work wants a kernel started"
  std::atomic<int> attends{0};         // how often the host runtime looked after it
  std::mutex mu;  // the test hooks may run on another thread than the library calls
};
NullState* g_null = nullptr;

class NullDevice : public Device {
 public:
  int init(int, const DeviceConfig& cfg) override {
    st_.flags.assign(cfg.total_slots, 0);
    st_.headers.assign(cfg.total_rings, RingHeader{});
    g_null = &st_;
    return MW_OK;
  }
  void shutdown() override { g_null = nullptr; }
  void set_config(const DeviceConfig&) override {}
  int launch(const LaunchOp* ops, const OpDeps* deps, int n, uint8_t* launched) override {
    std::lock_guard<std::mutex> g(st_.mu);
    if (st_.fail_next_launch) {
      st_.fail_next_launch = false;
      return MW_EHIP;
    }
    std::vector<void*> distinct;
    for (int i = 0; i < n; ++i)
      for (int k = 0; k < deps[i].n; ++k) {
        bool seen = false;
        for (void* t : distinct) seen |= t == deps[i].stream[k];
        if (!seen) distinct.push_back(deps[i].stream[k]);
      }
    const int n_streams = (int)distinct.size();
    int id = (int)st_.launch_sizes.size();
    st_.launch_sizes.push_back(n);
    st_.launch_streams.push_back(n_streams);
    for (int i = 0; i < n; ++i) {
      st_.pending.push_back(Recorded{ops[i], id});
      st_.log.push_back(Recorded{ops[i], id});
      launched[i] = 1;
    }
    return MW_OK;
  }
  int launch_static(const LaunchOp* ops, int n, void*) override {
    std::lock_guard<std::mutex> g(st_.mu);
    int id = (int)st_.launch_sizes.size();
    st_.launch_sizes.push_back(n);
    st_.launch_streams.push_back(1);
    for (int i = 0; i < n; ++i) st_.log.push_back(Recorded{ops[i], id});  // complete by stream order: never pending
    return MW_OK;
  }
  // The double has no resident kernel; a test can make it say that queued work wants a kernel started (as the product's
  // backend does when its kernel closed with descriptors left) and count how often the host runtime then looks after it.
  bool needs_attention() override { return st_.attention.load(std::memory_order_acquire); }
  int attend() override {
    if (st_.attention.exchange(false)) st_.attends.fetch_add(1);
    return MW_OK;
  }
  void mailbox_state(uint32_t* epoch, uint32_t* open, uint32_t* tail) override { *epoch = *open = *tail = 0; }
  int mark_world(uint32_t ring_index, const RingHeader& h) override {
    std::lock_guard<std::mutex> g(st_.mu);
    st_.headers[ring_index] = h;
    st_.marks += 1;
    return MW_OK;
  }
  uint32_t flag(uint32_t slot) override { return __atomic_load_n(&st_.flags[slot], __ATOMIC_ACQUIRE); }
  int read_ring(uint32_t ring_index, uint32_t, uint32_t depth, void* out) override {
    std::lock_guard<std::mutex> g(st_.mu);
    std::memcpy(out, &st_.headers[ring_index], sizeof(RingHeader));
    std::memset(reinterpret_cast<char*>(out) + sizeof(RingHeader), 0, (size_t)depth * kSlotBytes);
    return MW_OK;
  }
  int sync() override { return MW_OK; }
  int last_hip_error() override { return 0; }
  int profile_enable(int) override { return MW_OK; }
  int profile_read(int, uint64_t* l, double* ms, uint64_t* b) override {
    *l = 0;
    *ms = 0;
    *b = 0;
    return MW_OK;
  }

 private:
  NullState st_;
};

}  // namespace

Device* make_device() { return new NullDevice(); }

}  // namespace mw

using namespace mw;

// Hooks for the host-logic tests.
extern "C" {

int mwt_launch_count(void) {
  if (!g_null) return -1;
  std::lock_guard<std::mutex> g(g_null->mu);
  return (int)g_null->launch_sizes.size();
}
int mwt_launch_size(int id) { return g_null && id >= 0 && id < (int)g_null->launch_sizes.size() ? g_null->launch_sizes[id] : -1; }
int mwt_launch_streams(int id) { return g_null && id >= 0 && id < (int)g_null->launch_streams.size() ? g_null->launch_streams[id] : -1; }
int mwt_pending(void) {
  if (!g_null) return -1;
  std::lock_guard<std::mutex> g(g_null->mu);
  return (int)g_null->pending.size();
}
int mwt_marks(void) { return g_null ? g_null->marks : -1; }
int mwt_log_size(void) { return g_null ? (int)g_null->log.size() : -1; }

// Fields of the i-th operation ever launched: out[0..7] = buffers 0..7, out[8] = nbytes, out[9] = kind,
// out[10] = dtype, out[11] = nbuf, out[12] = slot, out[13] = gen, out[14] = world id, out[15] = epoch,
// out[16] = launch id, out[17] = root, out[18..25] = buffers 8..15.
int mwt_log_entry(int i, uint64_t* out) {
  if (!g_null || i < 0 || i >= (int)g_null->log.size()) return -1;
  const Recorded& r = g_null->log[i];
  for (int k = 0; k < kMaxBufs; ++k) out[k] = r.op.buf[k];
  out[8] = r.op.nbytes;
  out[9] = r.op.kind;
  out[10] = r.op.dtype;
  out[11] = r.op.nbuf;
  out[12] = r.op.slot;
  out[13] = r.op.gen;
  out[14] = r.op.world_id;
  out[15] = r.op.world_epoch;
  out[16] = (uint64_t)r.launch_id;
  out[17] = r.op.root;
  for (int k = 0; k < kMaxBufs; ++k) out[18 + k] = r.op.buf[kMaxBufs + k];
  return 0;
}

// Let the oldest n launched operations complete (newest first if from_back != 0).
int mwt_complete(int n, int from_back) {
  if (!g_null) return -1;
  std::lock_guard<std::mutex> g(g_null->mu);
  int done = 0;
  while (done < n && !g_null->pending.empty()) {
    Recorded r = from_back ? g_null->pending.back() : g_null->pending.front();
    if (from_back) g_null->pending.pop_back(); else g_null->pending.pop_front();
    __atomic_store_n(&g_null->flags[r.op.slot], r.op.gen, __ATOMIC_RELEASE);
    ++done;
  }
  return done;
}

// Make needs_attention() true until the host runtime calls attend(); mwt_attends() counts those calls.
int mwt_want_attention(void) {
  if (!g_null) return -1;
  g_null->attention.store(true, std::memory_order_release);
  return 0;
}
int mwt_attends(void) { return g_null ? g_null->attends.load() : -1; }

int mwt_fail_next_launch(void) {
  if (!g_null) return -1;
  g_null->fail_next_launch = true;
  return 0;
}

}  // extern "C"
