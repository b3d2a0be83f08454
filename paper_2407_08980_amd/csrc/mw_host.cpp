// Host runtime of the multi-world data plane: world table, matching of posted
// sides, handles, ring-slot bookkeeping, abort and deferred ring release.
//
// Paper anchors (arXiv 2407.08980): worlds as fault domains and a worker in
// many worlds (Sec. 3.1); non-blocking operations with polled status so that a
// pending operation in one world never holds up another (Sec. 3.2); per-world
// state kept side by side and looked up by key instead of being swapped in and
// out (Sec. 3.2 "State management for multiple worlds"); fencing a broken world,
// aborting its pending operations and raising to the caller (Sec. 3.3 "World
// Manager").
//
// Nothing here touches payload bytes: all data movement is in the device backend.

#include "../../include/mw.h"
#include "mw_internal.hpp"

#include <atomic>
#include <chrono>
#include <climits>
#include <cstdint>
#include <cstring>
#include <deque>
#include <memory>
#include <mutex>
#include <thread>
#include <unordered_map>
#include <vector>

namespace mw {
namespace {

constexpr uint32_t kNone = 0xFFFFFFFFu;

struct Post {  // one posted side that has not met its peers yet
  uint32_t hslot;
  uint64_t buf;
  uint64_t count;
  uint32_t dtype;
  void* stream;
  uint64_t buf2;  // second buffer of all-gather / gather / scatter posts
};

struct PairQ {
  std::deque<Post> sends, recvs;
};

struct Coll {  // a collective some ranks have posted
  int nposted = 0;
  bool have[kMaxBufs] = {};
  uint32_t kind[kMaxBufs] = {};
  int root[kMaxBufs] = {};
  Post post[kMaxBufs] = {};
};

struct World {
  int id = 0;
  std::vector<int> members;
  int state = MW_ALIVE;
  uint32_t epoch = 0;
  uint32_t ring_index = kNone;
  uint32_t first_slot = 0;
  uint32_t depth = 0;
  uint64_t free_mask[kMaxRingDepth / 64] = {};  // bit i set: ring slot i is free
  uint32_t n_free = 0;
  uint32_t queued = 0;     // operations with all sides posted, not launched yet
  std::vector<uint32_t> inflight;  // op records launched and not yet seen complete
  std::unordered_map<uint32_t, PairQ> pairs;  // key = src * MW_MAX_RANKS + dst
  std::deque<Coll> coll;                      // coll[0] has sequence number coll_base
  uint32_t coll_base = 0;
  std::vector<uint32_t> coll_next;            // per rank: sequence number of its next collective
  bool ring_released = false;
};

enum OpState : uint8_t { kOpFree = 0, kOpQueued = 1, kOpInflight = 2 };

struct OpRec {  // an operation all of whose sides have been posted
  LaunchOp l;
  void* streams[kMaxBufs];
  int n_streams;
  uint32_t handles[kMaxBufs];
  int n_handles;
  uint32_t world;  // index into worlds
  uint8_t state;
};

// One entry of the handle table.  Every field is written under the library lock; mw_poll also reads them WITHOUT
// the lock (poll_fast), as a sequence lock on `gen`: an entry is recycled by gen = 0, new fields, gen = new.
struct HandleEnt {
  std::atomic<uint32_t> gen{0};
  std::atomic<int32_t> status{MW_DONE};   // a never-used entry counts as terminal: it can be allocated
  std::atomic<uint32_t> op{kNone};        // record of the matched operation, kNone while waiting for a peer
  std::atomic<uint32_t> flag_slot{kNone}; // once launched: the ring slot whose completion word ...
  std::atomic<uint32_t> flag_gen{0};      // ... reaching this generation means the operation is complete
};

struct Context {
  std::unique_ptr<Device> dev;
  int n_workers = 0;
  DeviceConfig cfg{};
  uint32_t max_rings = 1024;
  uint32_t ring_depth = kDefaultRingDepth;

  std::vector<std::unique_ptr<World>> worlds;
  std::unordered_map<int, uint32_t> world_of_id;  // the key-value store of per-world state
  std::vector<std::vector<uint32_t>> worlds_of_worker;
  std::vector<uint32_t> free_rings;
  std::vector<uint32_t> slot_gen;  // per arena slot: last generation handed out

  std::vector<OpRec> ops;
  std::vector<uint32_t> free_ops;
  std::deque<uint32_t> ready;  // op records waiting for a launch, in match order
  std::deque<uint32_t> deferred;  // flush_locked's scratch: operations whose ring is full

  std::unique_ptr<HandleEnt[]> handles;  // fixed size: entries are read without the lock
  uint32_t n_handles = 0;
  uint32_t last_handle_gen = 0;  // generations are unique across the table, so a recycled entry never repeats one
  uint32_t handle_cursor = 0;

  // watchdog (Sec. 3.3): per-worker heartbeat epochs and times
  std::vector<uint64_t> beat_epoch;  // heartbeats received from each worker
  std::vector<double> last_beat;     // time of the latest one (seconds, caller's or the steady clock)
  std::vector<uint8_t> beating;      // worker has sent at least one heartbeat: it is being watched
  std::vector<uint8_t> failed;       // the watchdog has declared the worker failed

  uint32_t noalloc_gen = 0;  // generation of the latest mw_post_many_noalloc call

  std::vector<LaunchOp> launch_buf;
  std::vector<OpDeps> deps_buf;
  std::vector<uint32_t> launched_buf;
  std::vector<uint8_t> launched_flags;
};

std::mutex g_lock;
std::unique_ptr<Context> g_ctx;
// Lock-free polls: g_fast is the context while it may be read without the lock.  A poll counts itself in around
// its reads and mw_shutdown clears g_fast, then waits for the counts to drain before it frees anything (store then
// load on one side, add then load on the other, all sequentially consistent: either the poll sees no context or the
// shutdown sees the poll).  The count is striped over cache lines by thread so that busy-polling threads do not
// pass one line around (one shared counter: 870 ns per poll with 8 threads polling; striped: see tests/poll_contention.cpp).
std::atomic<Context*> g_fast{nullptr};
constexpr int kReaderStripes = 64;
struct alignas(64) ReaderStripe {
  std::atomic<int> n{0};
};
ReaderStripe g_fast_readers[kReaderStripes];
std::atomic<unsigned> g_next_stripe{0};

inline ReaderStripe& my_stripe() {
  thread_local unsigned mine = g_next_stripe.fetch_add(1, std::memory_order_relaxed) % kReaderStripes;
  return g_fast_readers[mine];
}

struct FastRead {  // RAII: the context for one lock-free read, or nullptr
  ReaderStripe& stripe;
  Context* c;
  FastRead() : stripe(my_stripe()) {
    stripe.n.fetch_add(1, std::memory_order_seq_cst);
    c = g_fast.load(std::memory_order_seq_cst);
  }
  ~FastRead() { stripe.n.fetch_sub(1, std::memory_order_release); }
};
// watchdog thread: wakes every period, takes g_lock, inspects the heartbeat table
std::thread g_wd_thread;
std::mutex g_wd_mu;  // guards g_wd_thread / g_wd_running
std::atomic<bool> g_wd_stop{false};
bool g_wd_running = false;
long g_cfg_chunk = 0, g_cfg_depth = kDefaultRingDepth, g_cfg_lds = 0, g_cfg_rings = 1024, g_cfg_handles = 1 << 20;
long g_cfg_mailbox = 1, g_cfg_mailbox_workers = 255, g_cfg_mailbox_idle_us = 300;

inline mw_handle make_handle(uint32_t slot, uint32_t gen) { return ((uint64_t)gen << 32) | slot; }

// ---- handles ---------------------------------------------------------------------------------
int alloc_handle(Context& c, uint32_t* out) {
  const uint32_t cap = c.n_handles;
  for (uint32_t tries = 0; tries < cap; ++tries) {
    uint32_t s = c.handle_cursor;
    c.handle_cursor = (s + 1 == cap) ? 0 : s + 1;
    HandleEnt& e = c.handles[s];
    if (e.status.load(std::memory_order_relaxed) == MW_PENDING) continue;  // still live: never recycle
    uint32_t g = e.gen.load(std::memory_order_relaxed) + 1;
    if (g == 0) g = 1;
    e.gen.store(0, std::memory_order_relaxed);  // lock-free readers of the old handle back off from here on
    std::atomic_thread_fence(std::memory_order_release);
    e.status.store(MW_PENDING, std::memory_order_relaxed);
    e.op.store(kNone, std::memory_order_relaxed);
    e.flag_slot.store(kNone, std::memory_order_relaxed);
    e.gen.store(g, std::memory_order_release);
    *out = s;
    return MW_OK;
  }
  return MW_ENOMEM;
}

inline void finish_handle(Context& c, uint32_t hslot, int status) {
  HandleEnt& e = c.handles[hslot];
  e.status.store(status, std::memory_order_release);
  e.op.store(kNone, std::memory_order_relaxed);
}

// ---- ring slots --------------------------------------------------------------------------------
inline void slot_release(World& w, uint32_t bit) {
  w.free_mask[bit >> 6] |= 1ull << (bit & 63);
  w.n_free += 1;
}

inline uint32_t slot_take(World& w) {  // caller checked n_free > 0
  for (uint32_t k = 0; k < kMaxRingDepth / 64; ++k) {
    if (w.free_mask[k]) {
      uint32_t b = (uint32_t)__builtin_ctzll(w.free_mask[k]);
      w.free_mask[k] &= ~(1ull << b);
      w.n_free -= 1;
      return k * 64 + b;
    }
  }
  return 0;
}

void release_ring_if_idle(Context& c, World& w) {
  if (w.state == MW_BROKEN && !w.ring_released && w.queued == 0 && w.inflight.empty()) {
    c.free_rings.push_back(w.ring_index);
    w.ring_released = true;
  }
}

void complete_op(Context& c, uint32_t opi) {
  OpRec& op = c.ops[opi];
  World& w = *c.worlds[op.world];
  for (int i = 0; i < op.n_handles; ++i) finish_handle(c, op.handles[i], MW_DONE);
  slot_release(w, op.l.slot - w.first_slot);
  op.state = kOpFree;
  c.free_ops.push_back(opi);
}

// Look at the completion words of a world's in-flight operations; retire the finished ones.
void retire_world(Context& c, World& w) {
  size_t k = 0;
  for (size_t i = 0; i < w.inflight.size(); ++i) {
    uint32_t opi = w.inflight[i];
    OpRec& op = c.ops[opi];
    if (c.dev->flag(op.l.slot) == op.l.gen) {
      complete_op(c, opi);
    } else {
      w.inflight[k++] = opi;
    }
  }
  w.inflight.resize(k);
  release_ring_if_idle(c, w);
}

void retire_one(Context& c, uint32_t opi) {
  OpRec& op = c.ops[opi];
  World& w = *c.worlds[op.world];
  for (size_t i = 0; i < w.inflight.size(); ++i) {
    if (w.inflight[i] == opi) {
      w.inflight[i] = w.inflight.back();
      w.inflight.pop_back();
      break;
    }
  }
  complete_op(c, opi);
  release_ring_if_idle(c, w);
}

// ---- launching ---------------------------------------------------------------------------------
int flush_locked(Context& c) {
  if (c.dev->needs_attention()) {  // operations queued for the resident kernel that closed as they came in
    int rc = c.dev->attend();
    if (rc != MW_OK) return rc;
  }
  if (c.ready.empty()) return MW_OK;
  c.launch_buf.clear();
  c.deps_buf.clear();
  c.launched_buf.clear();
  std::deque<uint32_t>& deferred = c.deferred;  // (a member: building a deque allocates)
  deferred.clear();
  while (!c.ready.empty()) {
    uint32_t opi = c.ready.front();
    c.ready.pop_front();
    OpRec& op = c.ops[opi];
    World& w = *c.worlds[op.world];
    if (w.n_free == 0) retire_world(c, w);
    if (w.n_free == 0) {  // ring full: stays queued until earlier operations retire
      deferred.push_back(opi);
      continue;
    }
    uint32_t bit = slot_take(w);
    uint32_t slot = w.first_slot + bit;
    uint32_t gen = c.slot_gen[slot] + 1;
    if (gen == 0) gen = 1;
    c.slot_gen[slot] = gen;
    op.l.slot = slot;
    op.l.gen = gen;
    op.l.world_epoch = w.epoch;
    c.launch_buf.push_back(op.l);
    c.launched_buf.push_back(opi);
    OpDeps d{};
    d.n = op.n_streams;
    for (int i = 0; i < op.n_streams; ++i) d.stream[i] = op.streams[i];
    c.deps_buf.push_back(d);
  }
  c.ready.swap(deferred);
  if (c.launch_buf.empty()) return MW_OK;
  c.launched_flags.assign(c.launch_buf.size(), 0);
  int rc = c.dev->launch(c.launch_buf.data(), c.deps_buf.data(), (int)c.launch_buf.size(), c.launched_flags.data());
  // Operations the device took are in flight; on a failure the others go back to the queue, slots freed.
  for (size_t i = c.launched_buf.size(); i-- > 0;) {
    uint32_t opi = c.launched_buf[i];
    OpRec& op = c.ops[opi];
    World& w = *c.worlds[op.world];
    if (c.launched_flags[i]) {
      op.state = kOpInflight;
      w.queued -= 1;
      w.inflight.push_back(opi);
      for (int k = 0; k < op.n_handles; ++k) {  // from here on a poll of these handles needs no lock until the flag flips
        HandleEnt& e = c.handles[op.handles[k]];
        e.flag_gen.store(op.l.gen, std::memory_order_relaxed);
        e.flag_slot.store(op.l.slot, std::memory_order_release);
      }
    } else {
      slot_release(w, op.l.slot - w.first_slot);
      c.ready.push_front(opi);
    }
  }
  return rc;
}

// An operation with all sides present: give it a record and queue it for the next launch.  `l` has
// kind, dtype, nbytes, nbuf, root and the buffers filled in; `posts` are its sides (handles, streams).
int enqueue_op(Context& c, uint32_t wi, const LaunchOp& l, const Post* posts, int n_posts) {
  uint32_t opi;
  if (!c.free_ops.empty()) {
    opi = c.free_ops.back();
    c.free_ops.pop_back();
  } else {
    opi = (uint32_t)c.ops.size();
    c.ops.emplace_back();
  }
  OpRec& op = c.ops[opi];
  std::memset(&op, 0, sizeof(op));
  op.world = wi;
  op.state = kOpQueued;
  op.l = l;
  op.l.world_id = (uint32_t)c.worlds[wi]->id;
  for (int i = 0; i < n_posts; ++i) {
    const Post& p = posts[i];
    op.handles[op.n_handles++] = p.hslot;
    c.handles[p.hslot].op.store(opi, std::memory_order_release);
    if (p.stream != MW_STREAM_NONE) {
      bool seen = false;
      for (int k = 0; k < op.n_streams; ++k) seen |= (op.streams[k] == p.stream);
      if (!seen) op.streams[op.n_streams++] = p.stream;
    }
  }
  c.worlds[wi]->queued += 1;
  c.ready.push_back(opi);
  return MW_OK;
}

inline uint64_t item_size(uint32_t dtype) { return dtype == MW_F32 ? 4 : 2; }

// ---- posting -----------------------------------------------------------------------------------
int post_p2p_locked(Context& c, bool is_send, int world_id, int src, int dst, const void* buf, size_t count,
                    mw_dtype dtype, void* stream, mw_handle* out) {
  if (!out || (dtype != MW_F32 && dtype != MW_BF16)) return MW_EINVAL;
  auto it = c.world_of_id.find(world_id);
  if (it == c.world_of_id.end()) return MW_ENOWORLD;
  World& w = *c.worlds[it->second];
  const int n = (int)w.members.size();
  if (src < 0 || dst < 0 || src >= n || dst >= n || src == dst) return MW_EINVAL;
  if (count > 0 && !buf) return MW_EINVAL;
  if (count > (SIZE_MAX >> 3)) return MW_EINVAL;
  if (w.state == MW_BROKEN) return MW_EBROKEN;
  uint32_t hs;
  int rc = alloc_handle(c, &hs);
  if (rc != MW_OK) return rc;
  *out = make_handle(hs, c.handles[hs].gen.load(std::memory_order_relaxed));
  Post me{hs, (uint64_t)(uintptr_t)buf, (uint64_t)count, (uint32_t)dtype, stream, 0};
  PairQ& q = w.pairs[(uint32_t)src * MW_MAX_RANKS + (uint32_t)dst];
  std::deque<Post>& theirs = is_send ? q.recvs : q.sends;
  if (theirs.empty()) {
    (is_send ? q.sends : q.recvs).push_back(me);
    return MW_OK;
  }
  Post other = theirs.front();
  theirs.pop_front();
  if (other.count != me.count || other.dtype != me.dtype) {
    finish_handle(c, hs, MW_EMISMATCH);
    finish_handle(c, other.hslot, MW_EMISMATCH);
    return MW_OK;
  }
  if (count == 0) {
    finish_handle(c, hs, MW_DONE);
    finish_handle(c, other.hslot, MW_DONE);
    return MW_OK;
  }
  Post pair[2] = {is_send ? me : other, is_send ? other : me};  // {send side, recv side}
  LaunchOp l{};
  l.kind = opCopy;
  l.dtype = (uint32_t)dtype;
  l.nbytes = count * item_size(dtype);
  l.nbuf = 2;
  l.buf[0] = pair[0].buf;
  l.buf[1] = pair[1].buf;
  return enqueue_op(c, it->second, l, pair, 2);
}

inline bool rooted(uint32_t kind) { return kind == opBcast || kind == opReduce || kind == opGather || kind == opScatter; }

// A collective all of whose n ranks have posted: check that the sides agree, then queue it (or complete it on the
// spot when there is nothing to move).
int run_collective(Context& c, uint32_t wi, const Coll& f, int n) {
  bool same = true;
  for (int r = 1; r < n; ++r) {
    same &= f.kind[r] == f.kind[0] && f.root[r] == f.root[0] && f.post[r].count == f.post[0].count &&
            f.post[r].dtype == f.post[0].dtype;
  }
  if (!same) {
    for (int r = 0; r < n; ++r) finish_handle(c, f.post[r].hslot, MW_EMISMATCH);
    return MW_OK;
  }
  const uint32_t k = f.kind[0];
  const int rt = f.root[0];
  const bool moves_alone = k == opAllGather || k == opGather || k == opScatter;  // a 1-rank world still copies
  if (f.post[0].count == 0 || (n == 1 && (!moves_alone || f.post[0].buf == f.post[0].buf2))) {
    for (int r = 0; r < n; ++r) finish_handle(c, f.post[r].hslot, MW_DONE);
    return MW_OK;
  }
  LaunchOp l{};
  l.kind = k;
  l.dtype = f.post[0].dtype;
  l.nbytes = f.post[0].count * item_size(f.post[0].dtype);
  l.nbuf = (uint32_t)n;
  l.root = (uint32_t)rt;
  switch (k) {
    case opBcast: {  // root first, then the other ranks ascending
      int at = 0;
      l.buf[at++] = f.post[rt].buf;
      for (int r = 0; r < n; ++r)
        if (r != rt) l.buf[at++] = f.post[r].buf;
      break;
    }
    case opAllReduce:
    case opReduce:
      for (int r = 0; r < n; ++r) l.buf[r] = f.post[r].buf;
      break;
    case opAllGather:
      for (int r = 0; r < n; ++r) {
        l.buf[r] = f.post[r].buf;
        l.buf[8 + r] = f.post[r].buf2;
      }
      break;
    case opGather:
      for (int r = 0; r < n; ++r) l.buf[r] = f.post[r].buf;
      l.buf[8] = f.post[rt].buf2;
      break;
    default:  // opScatter
      l.buf[0] = f.post[rt].buf;
      for (int r = 0; r < n; ++r) l.buf[8 + r] = f.post[r].buf2;
      break;
  }
  return enqueue_op(c, wi, l, f.post, n);
}

// kind is an OpKind other than opCopy.  buf / buf2 by kind:
//   broadcast, all-reduce, reduce: buf = the rank's tensor
//   all-gather: buf = source (count), buf2 = destination (n x count)
//   gather:     buf = source (count), buf2 = destination (n x count), used on the root only
//   scatter:    buf = source (n x count), used on the root only, buf2 = destination (count)
int post_coll_locked(Context& c, uint32_t kind, int world_id, int rank, int root, const void* buf, void* buf2,
                     size_t count, mw_dtype dtype, void* stream, mw_handle* out) {
  if (!out || (dtype != MW_F32 && dtype != MW_BF16)) return MW_EINVAL;
  auto it = c.world_of_id.find(world_id);
  if (it == c.world_of_id.end()) return MW_ENOWORLD;
  World& w = *c.worlds[it->second];
  const int n = (int)w.members.size();
  if (n > MW_MAX_COLL_RANKS) return MW_EINVAL;
  if (rank < 0 || rank >= n) return MW_EINVAL;
  if (rooted(kind) && (root < 0 || root >= n)) return MW_EINVAL;
  if (!rooted(kind)) root = 0;
  if (count > (SIZE_MAX >> 6)) return MW_EINVAL;
  if (count > 0) {
    const bool need1 = kind != opScatter || rank == root;
    const bool need2 = kind == opAllGather || kind == opScatter || (kind == opGather && rank == root);
    if ((need1 && !buf) || (need2 && !buf2)) return MW_EINVAL;
  }
  if ((kind == opAllReduce || kind == opReduce) && ((uintptr_t)buf % item_size(dtype)) != 0)
    return MW_EINVAL;  // elements are loaded whole
  if (w.state == MW_BROKEN) return MW_EBROKEN;
  uint32_t hs;
  int rc = alloc_handle(c, &hs);
  if (rc != MW_OK) return rc;
  *out = make_handle(hs, c.handles[hs].gen.load(std::memory_order_relaxed));
  uint32_t seq = w.coll_next[rank]++;
  uint32_t idx = seq - w.coll_base;
  while (w.coll.size() <= idx) w.coll.emplace_back();
  Coll& cl = w.coll[idx];
  cl.have[rank] = true;
  cl.kind[rank] = kind;
  cl.root[rank] = root;
  cl.post[rank] = Post{hs, (uint64_t)(uintptr_t)buf, (uint64_t)count, (uint32_t)dtype, stream, (uint64_t)(uintptr_t)buf2};
  cl.nposted += 1;
  // A world's collectives run in sequence order, each as soon as all its ranks have posted.
  while (!w.coll.empty() && w.coll.front().nposted == n) {
    rc = run_collective(c, it->second, w.coll.front(), n);
    w.coll.pop_front();
    w.coll_base += 1;
    if (rc != MW_OK) return rc;
  }
  return MW_OK;
}

int post_p2p(bool is_send, int world_id, int src, int dst, const void* buf, size_t count, mw_dtype dtype,
             void* stream, mw_handle* out) {
  std::lock_guard<std::mutex> g(g_lock);
  if (!g_ctx) return MW_ENOTINIT;
  return post_p2p_locked(*g_ctx, is_send, world_id, src, dst, buf, count, dtype, stream, out);
}

int post_coll(uint32_t kind, int world_id, int rank, int root, const void* buf, void* buf2, size_t count,
              mw_dtype dtype, void* stream, mw_handle* out) {
  std::lock_guard<std::mutex> g(g_lock);
  if (!g_ctx) return MW_ENOTINIT;
  return post_coll_locked(*g_ctx, kind, world_id, rank, root, buf, buf2, count, dtype, stream, out);
}

int abort_world_locked(Context& c, World& w) {
  if (w.state == MW_BROKEN) return MW_OK;
  w.state = MW_BROKEN;
  w.epoch += 1;
  for (auto& kv : w.pairs) {
    for (const Post& p : kv.second.sends) finish_handle(c, p.hslot, MW_BROKEN);
    for (const Post& p : kv.second.recvs) finish_handle(c, p.hslot, MW_BROKEN);
  }
  w.pairs.clear();
  for (const Coll& cl : w.coll)
    for (int r = 0; r < kMaxBufs; ++r)
      if (cl.have[r]) finish_handle(c, cl.post[r].hslot, MW_BROKEN);
  w.coll.clear();
  RingHeader h{};
  h.world_id = (uint32_t)w.id;
  h.state = MW_BROKEN;
  h.epoch = w.epoch;
  h.depth = w.depth;
  h.first_slot = w.first_slot;
  h.n_ranks = (uint32_t)w.members.size();
  int rc = c.dev->mark_world(w.ring_index, h);
  // Operations that already had all their sides are delivered: launch them now so that they retire.
  int rc2 = flush_locked(c);
  retire_world(c, w);
  return rc != MW_OK ? rc : rc2;
}

double steady_now() {
  return std::chrono::duration<double>(std::chrono::steady_clock::now().time_since_epoch()).count();
}

// One inspection of the heartbeat table at time `now`: every watched worker whose latest heartbeat is
// older than the timeout is declared failed and the worlds containing it are aborted.
int watchdog_check_locked(Context& c, double now, double timeout) {
  int newly = 0;
  for (size_t k = 0; k < c.beating.size(); ++k) {
    if (!c.beating[k] || c.failed[k] || !(now - c.last_beat[k] > timeout)) continue;
    c.failed[k] = 1;
    ++newly;
    for (uint32_t wi : c.worlds_of_worker[k]) abort_world_locked(c, *c.worlds[wi]);
  }
  return newly;
}

void stop_watchdog_thread() {  // called WITHOUT g_lock held
  std::thread t;
  {
    std::lock_guard<std::mutex> g(g_wd_mu);
    if (!g_wd_running) return;
    g_wd_stop.store(true);
    t = std::move(g_wd_thread);
    g_wd_running = false;
  }
  if (t.joinable()) t.join();
}

// A poll answered without the library lock: terminal states (they are sticky), operations still waiting for a
// peer, and -- the case every busy-waiting worker spins in (Sec. 3.3) -- operations in flight whose completion
// word has not flipped yet.  Everything that changes a table (launching a queued operation, retiring a completed
// one) and every error goes to the locked path.  Returns false if the locked path has to answer.
inline bool poll_fast(Context& c, mw_handle h, int* state) {
  const uint32_t slot = (uint32_t)(h & 0xFFFFFFFFu), gen = (uint32_t)(h >> 32);
  if (slot >= c.n_handles || gen == 0) return false;
  HandleEnt& e = c.handles[slot];
  if (e.gen.load(std::memory_order_acquire) != gen) return false;
  const int32_t st = e.status.load(std::memory_order_acquire);
  const uint32_t op = e.op.load(std::memory_order_relaxed);
  const uint32_t fs = e.flag_slot.load(std::memory_order_acquire);
  const uint32_t fg = e.flag_gen.load(std::memory_order_relaxed);
  std::atomic_thread_fence(std::memory_order_acquire);
  if (e.gen.load(std::memory_order_relaxed) != gen) return false;  // recycled while we looked
  if (st != MW_PENDING) {
    *state = st;
    return true;
  }
  if (op == kNone) {
    *state = MW_PENDING;
    return true;
  }
  if (fs != kNone && c.dev->flag(fs) != fg && !c.dev->needs_attention()) {
    *state = MW_PENDING;
    return true;
  }
  return false;
}

int poll_locked(Context& c, mw_handle h) {
  uint32_t slot = (uint32_t)(h & 0xFFFFFFFFu), gen = (uint32_t)(h >> 32);
  if (slot >= c.n_handles || gen == 0) return MW_EBADHANDLE;
  HandleEnt& e = c.handles[slot];
  if (e.gen.load(std::memory_order_relaxed) != gen) return MW_EBADHANDLE;
  const int32_t status = e.status.load(std::memory_order_relaxed);
  if (status != MW_PENDING) return status;
  if (e.op.load(std::memory_order_relaxed) == kNone) return MW_PENDING;  // still waiting for a peer
  uint32_t opi = e.op.load(std::memory_order_relaxed);
  if (c.ops[opi].state == kOpQueued) {
    int rc = flush_locked(c);
    if (rc != MW_OK) return rc;
  }
  OpRec& op = c.ops[opi];
  if (op.state == kOpInflight && c.dev->flag(op.l.slot) == op.l.gen) {
    retire_one(c, opi);
    return MW_DONE;
  }
  if (c.dev->needs_attention()) {  // it may sit in the resident kernel's queue with no kernel open: start one
    int rc = c.dev->attend();
    if (rc != MW_OK) return rc;
  }
  return MW_PENDING;
}

}  // namespace
}  // namespace mw

using namespace mw;

extern "C" {

int mw_init(int hip_device, int n_workers) {
  std::lock_guard<std::mutex> g(g_lock);
  if (g_ctx || n_workers < 1) return MW_EINVAL;
  std::unique_ptr<Context> c(new Context());
  c->n_workers = n_workers;
  c->max_rings = (uint32_t)g_cfg_rings;
  c->ring_depth = (uint32_t)g_cfg_depth;
  c->cfg.total_rings = c->max_rings;
  c->cfg.total_slots = c->max_rings * c->ring_depth;
  c->cfg.chunk_bytes = (uint32_t)g_cfg_chunk;
  c->cfg.reduce_lds = (uint32_t)g_cfg_lds;
  c->cfg.mailbox = (uint32_t)g_cfg_mailbox;
  c->cfg.mailbox_workers = (uint32_t)g_cfg_mailbox_workers;
  c->cfg.mailbox_idle_us = (uint32_t)g_cfg_mailbox_idle_us;
  c->dev.reset(make_device());
  int rc = c->dev->init(hip_device, c->cfg);
  if (rc != MW_OK) return rc;
  c->worlds_of_worker.resize((size_t)n_workers);
  c->beat_epoch.assign((size_t)n_workers, 0);
  c->last_beat.assign((size_t)n_workers, 0.0);
  c->beating.assign((size_t)n_workers, 0);
  c->failed.assign((size_t)n_workers, 0);
  c->slot_gen.assign(c->cfg.total_slots, 0);
  for (uint32_t r = c->max_rings; r-- > 0;) c->free_rings.push_back(r);
  c->handles.reset(new HandleEnt[(size_t)g_cfg_handles]);
  c->n_handles = (uint32_t)g_cfg_handles;
  g_ctx = std::move(c);
  g_fast.store(g_ctx.get(), std::memory_order_release);
  return MW_OK;
}

int mw_shutdown(void) {
  stop_watchdog_thread();
  std::lock_guard<std::mutex> g(g_lock);
  if (!g_ctx) return MW_ENOTINIT;
  g_fast.store(nullptr, std::memory_order_seq_cst);  // no new lock-free reader gets the context ...
  for (ReaderStripe& r : g_fast_readers)  // ... and the current ones leave
    while (r.n.load(std::memory_order_seq_cst) != 0) std::this_thread::yield();
  flush_locked(*g_ctx);
  g_ctx->dev->sync();
  g_ctx->dev->shutdown();
  g_ctx.reset();
  return MW_OK;
}

int mw_world_create(int world_id, const int* worker_ids, int n_ranks) {
  std::lock_guard<std::mutex> g(g_lock);
  if (!g_ctx) return MW_ENOTINIT;
  Context& c = *g_ctx;
  if (!worker_ids || n_ranks < 1 || n_ranks > MW_MAX_RANKS) return MW_EINVAL;
  for (int i = 0; i < n_ranks; ++i) {
    if (worker_ids[i] < 0 || worker_ids[i] >= c.n_workers) return MW_EINVAL;
    for (int j = 0; j < i; ++j)
      if (worker_ids[j] == worker_ids[i]) return MW_EINVAL;
  }
  for (int i = 0; i < n_ranks; ++i)
    if (c.failed[(size_t)worker_ids[i]]) return MW_EBROKEN;  // a failed worker is replaced by a NEW worker
  if (c.world_of_id.count(world_id)) return MW_EEXIST;
  if (c.free_rings.empty()) {  // rings of broken worlds come back once their operations retired
    for (auto& wp : c.worlds)
      if (wp->state == MW_BROKEN && !wp->ring_released) retire_world(c, *wp);
    if (c.free_rings.empty()) return MW_ENOMEM;
  }
  std::unique_ptr<World> w(new World());
  w->id = world_id;
  w->members.assign(worker_ids, worker_ids + n_ranks);
  w->ring_index = c.free_rings.back();
  c.free_rings.pop_back();
  w->depth = c.ring_depth;
  w->first_slot = w->ring_index * c.ring_depth;
  for (uint32_t b = 0; b < w->depth; ++b) slot_release(*w, b);
  w->coll_next.assign((size_t)n_ranks, 0);
  RingHeader h{};
  h.world_id = (uint32_t)world_id;
  h.state = MW_ALIVE;
  h.epoch = 0;
  h.depth = w->depth;
  h.first_slot = w->first_slot;
  h.n_ranks = (uint32_t)n_ranks;
  int rc = c.dev->mark_world(w->ring_index, h);
  if (rc != MW_OK) {
    c.free_rings.push_back(w->ring_index);
    return rc;
  }
  uint32_t wi = (uint32_t)c.worlds.size();
  for (int i = 0; i < n_ranks; ++i) {
    // A worker that keeps joining new worlds as old ones break (Sec. 3.1 recovery) must not pay for its
    // history on every abort: drop the broken worlds from its list before adding the new one.
    std::vector<uint32_t>& mine = c.worlds_of_worker[(size_t)worker_ids[i]];
    size_t k = 0;
    for (uint32_t x : mine)
      if (c.worlds[x]->state != MW_BROKEN) mine[k++] = x;
    mine.resize(k);
    mine.push_back(wi);
  }
  c.world_of_id.emplace(world_id, wi);
  c.worlds.push_back(std::move(w));
  return MW_OK;
}

int mw_world_abort(int world_id) {
  std::lock_guard<std::mutex> g(g_lock);
  if (!g_ctx) return MW_ENOTINIT;
  auto it = g_ctx->world_of_id.find(world_id);
  if (it == g_ctx->world_of_id.end()) return MW_ENOWORLD;
  return abort_world_locked(*g_ctx, *g_ctx->worlds[it->second]);
}

int mw_worker_abort(int worker_id) {
  std::lock_guard<std::mutex> g(g_lock);
  if (!g_ctx) return MW_ENOTINIT;
  Context& c = *g_ctx;
  if (worker_id < 0 || worker_id >= c.n_workers) return MW_EINVAL;
  int rc = MW_OK;
  for (uint32_t wi : c.worlds_of_worker[(size_t)worker_id]) {
    int r = abort_world_locked(c, *c.worlds[wi]);
    if (r != MW_OK) rc = r;
  }
  return rc;
}

int mw_heartbeat_at(int worker_id, double t) {
  std::lock_guard<std::mutex> g(g_lock);
  if (!g_ctx) return MW_ENOTINIT;
  Context& c = *g_ctx;
  if (worker_id < 0 || worker_id >= c.n_workers || !(t == t)) return MW_EINVAL;
  if (c.failed[(size_t)worker_id]) return MW_EBROKEN;
  if (!c.beating[(size_t)worker_id] || t > c.last_beat[(size_t)worker_id]) c.last_beat[(size_t)worker_id] = t;
  c.beating[(size_t)worker_id] = 1;
  c.beat_epoch[(size_t)worker_id] += 1;
  return MW_OK;
}

int mw_heartbeat(int worker_id) { return mw_heartbeat_at(worker_id, steady_now()); }

int mw_watchdog_check_at(double t, double timeout_s) {
  std::lock_guard<std::mutex> g(g_lock);
  if (!g_ctx) return MW_ENOTINIT;
  if (!(timeout_s >= 0) || !(t == t)) return MW_EINVAL;
  return watchdog_check_locked(*g_ctx, t, timeout_s);
}

int mw_watchdog_start(double timeout_s, double period_s) {
  if (!(timeout_s > 0) || !(period_s > 0)) return MW_EINVAL;
  {
    std::lock_guard<std::mutex> g(g_lock);
    if (!g_ctx) return MW_ENOTINIT;
  }
  std::lock_guard<std::mutex> g(g_wd_mu);
  if (g_wd_running) return MW_EINVAL;
  g_wd_stop.store(false);
  g_wd_running = true;
  g_wd_thread = std::thread([timeout_s, period_s] {
    while (!g_wd_stop.load()) {
      {
        std::lock_guard<std::mutex> g2(g_lock);
        if (g_ctx) watchdog_check_locked(*g_ctx, steady_now(), timeout_s);
      }
      // sleep one period in slices so that a stop request is honoured within ~10 ms
      for (double left = period_s; left > 0 && !g_wd_stop.load(); left -= 0.01)
        std::this_thread::sleep_for(std::chrono::duration<double>(left < 0.01 ? left : 0.01));
    }
  });
  return MW_OK;
}

int mw_watchdog_stop(void) {
  stop_watchdog_thread();
  return MW_OK;
}

int mw_worker_state(int worker_id) {
  std::lock_guard<std::mutex> g(g_lock);
  if (!g_ctx) return MW_ENOTINIT;
  if (worker_id < 0 || worker_id >= g_ctx->n_workers) return MW_EINVAL;
  return g_ctx->failed[(size_t)worker_id] ? MW_BROKEN : MW_ALIVE;
}

long mw_heartbeat_epoch(int worker_id) {
  std::lock_guard<std::mutex> g(g_lock);
  if (!g_ctx) return MW_ENOTINIT;
  if (worker_id < 0 || worker_id >= g_ctx->n_workers) return MW_EINVAL;
  return (long)g_ctx->beat_epoch[(size_t)worker_id];
}

int mw_world_state(int world_id) {
  std::lock_guard<std::mutex> g(g_lock);
  if (!g_ctx) return MW_ENOTINIT;
  auto it = g_ctx->world_of_id.find(world_id);
  if (it == g_ctx->world_of_id.end()) return MW_ENOWORLD;
  return g_ctx->worlds[it->second]->state;
}

int mw_send(int world_id, int src_rank, int dst_rank, const void* buf, size_t count, mw_dtype dtype,
            void* hip_stream, mw_handle* out) {
  return post_p2p(true, world_id, src_rank, dst_rank, buf, count, dtype, hip_stream, out);
}

int mw_recv(int world_id, int src_rank, int dst_rank, void* buf, size_t count, mw_dtype dtype, void* hip_stream,
            mw_handle* out) {
  return post_p2p(false, world_id, src_rank, dst_rank, buf, count, dtype, hip_stream, out);
}

int mw_broadcast(int world_id, int rank, int root_rank, void* buf, size_t count, mw_dtype dtype,
                 void* hip_stream, mw_handle* out) {
  return post_coll(opBcast, world_id, rank, root_rank, buf, nullptr, count, dtype, hip_stream, out);
}

int mw_allreduce_sum(int world_id, int rank, void* buf, size_t count, mw_dtype dtype, void* hip_stream,
                     mw_handle* out) {
  return post_coll(opAllReduce, world_id, rank, 0, buf, nullptr, count, dtype, hip_stream, out);
}

int mw_reduce_sum(int world_id, int rank, int root_rank, void* buf, size_t count, mw_dtype dtype, void* hip_stream,
                  mw_handle* out) {
  return post_coll(opReduce, world_id, rank, root_rank, buf, nullptr, count, dtype, hip_stream, out);
}

int mw_all_gather(int world_id, int rank, const void* sendbuf, void* recvbuf, size_t count, mw_dtype dtype,
                  void* hip_stream, mw_handle* out) {
  return post_coll(opAllGather, world_id, rank, 0, sendbuf, recvbuf, count, dtype, hip_stream, out);
}

int mw_gather(int world_id, int rank, int root_rank, const void* sendbuf, void* recvbuf, size_t count,
              mw_dtype dtype, void* hip_stream, mw_handle* out) {
  return post_coll(opGather, world_id, rank, root_rank, sendbuf, recvbuf, count, dtype, hip_stream, out);
}

int mw_scatter(int world_id, int rank, int root_rank, const void* sendbuf, void* recvbuf, size_t count,
               mw_dtype dtype, void* hip_stream, mw_handle* out) {
  return post_coll(opScatter, world_id, rank, root_rank, sendbuf, recvbuf, count, dtype, hip_stream, out);
}

int mw_post_many(const mw_post_desc* posts, int n, mw_handle* handles, int* results) {
  std::lock_guard<std::mutex> g(g_lock);
  if (!g_ctx) return MW_ENOTINIT;
  if (n < 0 || (n > 0 && (!posts || !handles))) return MW_EINVAL;
  int first_err = MW_OK;
  for (int i = 0; i < n; ++i) {
    const mw_post_desc& p = posts[i];
    handles[i] = 0;
    int rc;
    switch (p.kind) {
      case MW_POST_SEND:
        rc = post_p2p_locked(*g_ctx, true, p.world_id, p.a, p.b, p.buf, (size_t)p.count, (mw_dtype)p.dtype,
                             p.hip_stream, &handles[i]);
        break;
      case MW_POST_RECV:
        rc = post_p2p_locked(*g_ctx, false, p.world_id, p.a, p.b, p.buf, (size_t)p.count, (mw_dtype)p.dtype,
                             p.hip_stream, &handles[i]);
        break;
      case MW_POST_BROADCAST:
        rc = post_coll_locked(*g_ctx, opBcast, p.world_id, p.a, p.b, p.buf, nullptr, (size_t)p.count,
                              (mw_dtype)p.dtype, p.hip_stream, &handles[i]);
        break;
      case MW_POST_ALLREDUCE_SUM:
        rc = post_coll_locked(*g_ctx, opAllReduce, p.world_id, p.a, 0, p.buf, nullptr, (size_t)p.count,
                              (mw_dtype)p.dtype, p.hip_stream, &handles[i]);
        break;
      case MW_POST_REDUCE_SUM:
        rc = post_coll_locked(*g_ctx, opReduce, p.world_id, p.a, p.b, p.buf, nullptr, (size_t)p.count,
                              (mw_dtype)p.dtype, p.hip_stream, &handles[i]);
        break;
      case MW_POST_ALL_GATHER:
        rc = post_coll_locked(*g_ctx, opAllGather, p.world_id, p.a, 0, p.buf, p.buf2, (size_t)p.count,
                              (mw_dtype)p.dtype, p.hip_stream, &handles[i]);
        break;
      case MW_POST_GATHER:
        rc = post_coll_locked(*g_ctx, opGather, p.world_id, p.a, p.b, p.buf, p.buf2, (size_t)p.count,
                              (mw_dtype)p.dtype, p.hip_stream, &handles[i]);
        break;
      case MW_POST_SCATTER:
        rc = post_coll_locked(*g_ctx, opScatter, p.world_id, p.a, p.b, p.buf, p.buf2, (size_t)p.count,
                              (mw_dtype)p.dtype, p.hip_stream, &handles[i]);
        break;
      default:
        rc = MW_EINVAL;
    }
    if (rc != MW_OK) handles[i] = 0;
    if (results) results[i] = rc;
    if (rc != MW_OK && first_err == MW_OK) first_err = rc;
  }
  return first_err;
}

int mw_post_many_noalloc(const mw_post_desc* posts, int n, void* hip_stream) {
  std::lock_guard<std::mutex> g(g_lock);
  if (!g_ctx) return MW_ENOTINIT;
  Context& c = *g_ctx;
  if (n < 0 || n > MW_NOALLOC_MAX_POSTS || (n > 0 && !posts) || hip_stream == MW_STREAM_NONE) return MW_EINVAL;
  // Everything below lives on the stack: no table of the context is touched, nothing is allocated.
  LaunchOp ops[MW_NOALLOC_MAX_OPS];
  int n_ops = 0;
  bool used[MW_NOALLOC_MAX_POSTS] = {};
  const World* world_of[MW_NOALLOC_MAX_POSTS] = {};
  for (int i = 0; i < n; ++i) {  // validate every post as its posting call would
    const mw_post_desc& p = posts[i];
    if (p.kind < MW_POST_SEND || p.kind > MW_POST_SCATTER) return MW_EINVAL;
    if (p.dtype != MW_F32 && p.dtype != MW_BF16) return MW_EINVAL;
    auto it = c.world_of_id.find(p.world_id);
    if (it == c.world_of_id.end()) return MW_ENOWORLD;
    const World& w = *c.worlds[it->second];
    world_of[i] = &w;
    const int nr = (int)w.members.size();
    if (p.count > (SIZE_MAX >> 6)) return MW_EINVAL;
    if (p.kind <= MW_POST_RECV) {
      if (p.a < 0 || p.b < 0 || p.a >= nr || p.b >= nr || p.a == p.b) return MW_EINVAL;
      if (p.count > 0 && !p.buf) return MW_EINVAL;
    } else {
      const uint32_t k = (uint32_t)p.kind - MW_POST_BROADCAST + opBcast;  // the two enums run in the same order
      if (nr > MW_MAX_COLL_RANKS || p.a < 0 || p.a >= nr) return MW_EINVAL;
      if (rooted(k) && (p.b < 0 || p.b >= nr)) return MW_EINVAL;
      const int root = rooted(k) ? p.b : 0;
      if (p.count > 0) {
        const bool need1 = k != opScatter || p.a == root;
        const bool need2 = k == opAllGather || k == opScatter || (k == opGather && p.a == root);
        if ((need1 && !p.buf) || (need2 && !p.buf2)) return MW_EINVAL;
      }
      if ((k == opAllReduce || k == opReduce) && ((uintptr_t)p.buf % item_size((uint32_t)p.dtype)) != 0) return MW_EINVAL;
    }
    if (w.state == MW_BROKEN) return MW_EBROKEN;
  }
  for (int i = 0; i < n; ++i) {
    if (used[i]) continue;
    const mw_post_desc& p = posts[i];
    const World& w = *world_of[i];
    const int nr = (int)w.members.size();
    LaunchOp l{};
    l.dtype = (uint32_t)p.dtype;
    l.nbytes = p.count * item_size((uint32_t)p.dtype);
    l.world_id = (uint32_t)w.id;
    l.world_epoch = w.epoch;
    bool moves = p.count > 0;
    if (p.kind <= MW_POST_RECV) {
      // first in, first out per (world, src, dst): this side pairs with the earliest later side of the other kind
      // that no earlier side has taken
      int j = i + 1;
      while (j < n && !(!used[j] && posts[j].kind == 1 - p.kind && posts[j].world_id == p.world_id &&
                        posts[j].a == p.a && posts[j].b == p.b))
        ++j;
      if (j == n) return MW_EINVAL;  // a side without its peer: this call takes whole operations only
      used[i] = used[j] = true;
      if (posts[j].count != p.count || posts[j].dtype != p.dtype) return MW_EMISMATCH;
      const mw_post_desc& snd = p.kind == MW_POST_SEND ? p : posts[j];
      const mw_post_desc& rcv = p.kind == MW_POST_SEND ? posts[j] : p;
      l.kind = opCopy;
      l.nbuf = 2;
      l.buf[0] = (uint64_t)(uintptr_t)snd.buf;
      l.buf[1] = (uint64_t)(uintptr_t)rcv.buf;
    } else {
      const uint32_t k = (uint32_t)p.kind - MW_POST_BROADCAST + opBcast;
      const int root = rooted(k) ? p.b : 0;
      int side[kMaxBufs];
      for (int r = 0; r < nr; ++r) side[r] = -1;
      // the k-th collective a rank posts belongs to the world's k-th collective: with the earlier collectives
      // taken, that is every rank's first collective post that is still free
      for (int j = i; j < n; ++j)
        if (!used[j] && posts[j].kind > MW_POST_RECV && posts[j].world_id == p.world_id && side[posts[j].a] < 0)
          side[posts[j].a] = j;
      for (int r = 0; r < nr; ++r) {
        if (side[r] < 0) return MW_EINVAL;  // a rank did not post this collective
        used[side[r]] = true;
      }
      for (int r = 0; r < nr; ++r) {
        const mw_post_desc& q = posts[side[r]];
        const int qroot = rooted(k) ? q.b : 0;
        if (q.kind != p.kind || qroot != root || q.count != p.count || q.dtype != p.dtype) return MW_EMISMATCH;
      }
      l.kind = k;
      l.nbuf = (uint32_t)nr;
      l.root = (uint32_t)root;
      auto b1 = [&](int r) { return (uint64_t)(uintptr_t)posts[side[r]].buf; };
      auto b2 = [&](int r) { return (uint64_t)(uintptr_t)posts[side[r]].buf2; };
      switch (k) {
        case opBcast: {
          int at = 0;
          l.buf[at++] = b1(root);
          for (int r = 0; r < nr; ++r)
            if (r != root) l.buf[at++] = b1(r);
          break;
        }
        case opAllReduce:
        case opReduce:
          for (int r = 0; r < nr; ++r) l.buf[r] = b1(r);
          break;
        case opAllGather:
          for (int r = 0; r < nr; ++r) {
            l.buf[r] = b1(r);
            l.buf[8 + r] = b2(r);
          }
          break;
        case opGather:
          for (int r = 0; r < nr; ++r) l.buf[r] = b1(r);
          l.buf[8] = b2(root);
          break;
        default:  // opScatter
          l.buf[0] = b1(root);
          for (int r = 0; r < nr; ++r) l.buf[8 + r] = b2(r);
          break;
      }
      const bool moves_alone = k == opAllGather || k == opGather || k == opScatter;
      if (nr == 1 && (!moves_alone || p.buf == p.buf2)) moves = false;
    }
    if (!moves) continue;
    if (n_ops == MW_NOALLOC_MAX_OPS) return MW_EINVAL;
    l.slot = (uint32_t)n_ops;
    ops[n_ops++] = l;
  }
  // One generation per call, shared by its operations (their slots differ); never 0.
  c.noalloc_gen += 1;
  if (c.noalloc_gen == 0) c.noalloc_gen = 1;
  for (int i = 0; i < n_ops; ++i) ops[i].gen = c.noalloc_gen;
  return c.dev->launch_static(ops, n_ops, hip_stream);
}

int mw_poll(mw_handle h) {
  {
    FastRead r;
    int st;
    if (r.c && poll_fast(*r.c, h, &st)) return st;
  }
  std::lock_guard<std::mutex> g(g_lock);
  if (!g_ctx) return MW_ENOTINIT;
  return poll_locked(*g_ctx, h);
}

int mw_poll_many(const mw_handle* handles, int n, int* states) {
  if (n < 0 || (n > 0 && (!handles || !states))) return MW_EINVAL;
  int pending = 0, slow = 0;
  {
    FastRead r;
    if (r.c) {
      for (int i = 0; i < n; ++i) {
        if (poll_fast(*r.c, handles[i], &states[i])) {
          pending += states[i] == MW_PENDING;
        } else {
          states[i] = INT32_MIN;  // to be answered under the lock
          ++slow;
        }
      }
      if (!slow) return pending;
    }
  }
  std::lock_guard<std::mutex> g(g_lock);
  if (!g_ctx) return MW_ENOTINIT;
  for (int i = 0; i < n; ++i) {
    if (slow && states[i] != INT32_MIN) continue;
    states[i] = poll_locked(*g_ctx, handles[i]);
    pending += states[i] == MW_PENDING;
  }
  return pending;
}

int mw_pending_ops(void) {
  std::lock_guard<std::mutex> g(g_lock);
  if (!g_ctx) return MW_ENOTINIT;
  int n = 0;
  for (auto& w : g_ctx->worlds) n += (int)w->queued + (int)w->inflight.size();
  return n;
}

int mw_flush(void) {
  std::lock_guard<std::mutex> g(g_lock);
  if (!g_ctx) return MW_ENOTINIT;
  return flush_locked(*g_ctx);
}

int mw_config_set(const char* key, long value) {
  std::lock_guard<std::mutex> g(g_lock);
  if (!key) return MW_EINVAL;
  const bool live = (bool)g_ctx;
  if (!std::strcmp(key, "chunk_bytes")) {
    if (value != 0 && (value < 4096 || value > 4194304 || (value & (value - 1)))) return MW_EINVAL;
    g_cfg_chunk = value;
    if (live) {
      g_ctx->cfg.chunk_bytes = (uint32_t)value;
      g_ctx->dev->set_config(g_ctx->cfg);
    }
    return MW_OK;
  }
  if (!std::strcmp(key, "reduce_lds")) {
    if (value != 0 && value != 1) return MW_EINVAL;
    g_cfg_lds = value;
    if (live) {
      g_ctx->cfg.reduce_lds = (uint32_t)value;
      g_ctx->dev->set_config(g_ctx->cfg);
    }
    return MW_OK;
  }
  if (!std::strcmp(key, "mailbox")) {
    if (value != 0 && value != 1) return MW_EINVAL;
    g_cfg_mailbox = value;
    if (live) {
      g_ctx->cfg.mailbox = (uint32_t)value;
      g_ctx->dev->set_config(g_ctx->cfg);
    }
    return MW_OK;
  }
  if (!std::strcmp(key, "mailbox_idle_us")) {
    if (value < 10 || value > 50000) return MW_EINVAL;
    g_cfg_mailbox_idle_us = value;
    if (live) {
      g_ctx->cfg.mailbox_idle_us = (uint32_t)value;
      g_ctx->dev->set_config(g_ctx->cfg);
    }
    return MW_OK;
  }
  // geometry: only before mw_init
  if (live) return MW_EINVAL;
  if (!std::strcmp(key, "mailbox_workers")) {
    if (value < 1 || value > 1023) return MW_EINVAL;
    g_cfg_mailbox_workers = value;
    return MW_OK;
  }
  if (!std::strcmp(key, "ring_depth")) {
    if (value < 1 || value > kMaxRingDepth) return MW_EINVAL;
    g_cfg_depth = value;
    return MW_OK;
  }
  if (!std::strcmp(key, "max_rings")) {
    if (value < 1 || value > 65536) return MW_EINVAL;
    g_cfg_rings = value;
    return MW_OK;
  }
  if (!std::strcmp(key, "handle_capacity")) {
    if (value < 16 || value > (1l << 26)) return MW_EINVAL;
    g_cfg_handles = value;
    return MW_OK;
  }
  return MW_EINVAL;
}

long mw_config_get(const char* key) {
  std::lock_guard<std::mutex> g(g_lock);
  if (!key) return MW_EINVAL;
  if (!std::strcmp(key, "chunk_bytes")) return g_cfg_chunk;
  if (!std::strcmp(key, "reduce_lds")) return g_cfg_lds;
  if (!std::strcmp(key, "mailbox")) return g_cfg_mailbox;
  if (!std::strcmp(key, "mailbox_workers")) return g_cfg_mailbox_workers;
  if (!std::strcmp(key, "mailbox_idle_us")) return g_cfg_mailbox_idle_us;
  if (!std::strcmp(key, "ring_depth")) return g_cfg_depth;
  if (!std::strcmp(key, "max_rings")) return g_cfg_rings;
  if (!std::strcmp(key, "handle_capacity")) return g_cfg_handles;
  return MW_EINVAL;
}

int mw_handle_capacity(void) {
  std::lock_guard<std::mutex> g(g_lock);
  return g_ctx ? (int)g_ctx->n_handles : (int)g_cfg_handles;
}

int mw_last_hip_error(void) {
  std::lock_guard<std::mutex> g(g_lock);
  return g_ctx ? g_ctx->dev->last_hip_error() : 0;
}

#ifndef MW_BUILD_ID
#define MW_BUILD_ID "unknown"
#endif
const char* mw_build_id(void) { return MW_BUILD_ID; }

const char* mw_strerror(int err) {
  switch (err) {
    case MW_OK: return "ok";
    case MW_EINVAL: return "invalid argument";
    case MW_ENOWORLD: return "no such world";
    case MW_EBROKEN: return "world is broken";
    case MW_EEXIST: return "world id already used";
    case MW_EMISMATCH: return "sides of the operation disagree";
    case MW_ENOMEM: return "library table full";
    case MW_EBADHANDLE: return "bad or recycled handle";
    case MW_EHIP: return "HIP call failed";
    case MW_ENOTINIT: return "mw_init not called";
    default: return "unknown error";
  }
}

int mw_profile_enable(int on) {
  std::lock_guard<std::mutex> g(g_lock);
  if (!g_ctx) return MW_ENOTINIT;
  return g_ctx->dev->profile_enable(on);
}

int mw_profile_read(int kind, uint64_t* launches, double* total_ms, uint64_t* op_bytes) {
  std::lock_guard<std::mutex> g(g_lock);
  if (!g_ctx) return MW_ENOTINIT;
  if (kind < 0 || kind >= (int)kNumKinds || !launches || !total_ms || !op_bytes) return MW_EINVAL;
  return g_ctx->dev->profile_read(kind, launches, total_ms, op_bytes);
}

int mw_debug_mailbox(uint32_t* epoch, uint32_t* open, uint32_t* tail) {
  std::lock_guard<std::mutex> g(g_lock);
  if (!g_ctx) return MW_ENOTINIT;
  if (!epoch || !open || !tail) return MW_EINVAL;
  g_ctx->dev->mailbox_state(epoch, open, tail);
  return MW_OK;
}

long mw_debug_ring_read(int world_id, void* out, size_t cap) {
  std::lock_guard<std::mutex> g(g_lock);
  if (!g_ctx) return MW_ENOTINIT;
  Context& c = *g_ctx;
  auto it = c.world_of_id.find(world_id);
  if (it == c.world_of_id.end()) return MW_ENOWORLD;
  World& w = *c.worlds[it->second];
  size_t need = (size_t)kHeaderBytes + (size_t)w.depth * kSlotBytes;
  if (!out || cap < need) return MW_EINVAL;
  int rc = c.dev->read_ring(w.ring_index, w.first_slot, w.depth, out);
  return rc == MW_OK ? (long)need : rc;
}

int mw_debug_arena_hash(int except_world, uint64_t* hash) {
  std::lock_guard<std::mutex> g(g_lock);
  if (!g_ctx) return MW_ENOTINIT;
  Context& c = *g_ctx;
  if (!hash) return MW_EINVAL;
  uint32_t skip = kNone;
  if (except_world != -1) {
    auto it = c.world_of_id.find(except_world);
    if (it == c.world_of_id.end()) return MW_ENOWORLD;
    skip = c.worlds[it->second]->ring_index;
  }
  std::vector<unsigned char> tmp((size_t)kHeaderBytes + (size_t)c.ring_depth * kSlotBytes);
  uint64_t hsh = 1469598103934665603ull;
  for (uint32_t r = 0; r < c.max_rings; ++r) {
    if (r == skip) continue;
    int rc = c.dev->read_ring(r, r * c.ring_depth, c.ring_depth, tmp.data());
    if (rc != MW_OK) return rc;
    for (unsigned char b : tmp) {
      hsh ^= b;
      hsh *= 1099511628211ull;
    }
  }
  *hash = hsh;
  return MW_OK;
}

}  // extern "C"
