// The mailbox: a descriptor queue in device memory that the host writes and a resident kernel serves, so that a
// small operation does not pay a kernel launch (arXiv 2407.08980 Sec. 3.2 / 3.3: workers busy-wait on the status of
// their operations, so the latency of a small transfer is what a worker sees between posting and going on).
//
// This header holds what the host side, the resident kernel and the CPU model of the kernel (tests/mailbox_model.cpp)
// have in common: the layout of the queue, the rule that says which worker owns which chunk, and the host-side
// protocol (MailboxHost), which is written against a small `Port` so that the very same code runs against the GPU
// and against threads that play the kernel.
//
// Protocol.  Descriptors are numbered by *tickets* 1, 2, 3, ... (32 bits, compared modulo 2^32); ticket t lives in
// queue slot t % kQueueDepth.  The host writes descriptors, then the doorbell `tail` (the last ticket written).  The
// resident kernel has one *leader* and W *workers*:
//   - the leader is the only one who reads the doorbell.  It ADMITS tickets by publishing `admit` = last admitted
//     ticket (high half 0), and it decides when the kernel ends: when the host asks (stop word), when nothing new
//     has come for the idle time, or when the kernel's lifetime is up.  It then publishes admit with its epoch in
//     the high half and tells the host (`closed` = epoch << 32 | last admitted ticket).  Because one agent admits and closes, a
//     ticket is either admitted -- and then every worker serves it before it leaves -- or it is not, and then no
//     worker touches it: an operation is never served by a part of the workers only, and never twice.
//   - a worker serves the admitted tickets in order: of each it runs the chunks c with owner(start, c, W) == its
//     number.  It leaves when it has served every ticket up to a closing admit (or, as a safety net that no correct
//     run needs, when its own time limit is up).
//   - the host never waits for the kernel.  When it finds the kernel closed with tickets beyond the last admitted
//     one, it starts the next epoch at that ticket + 1, on the same stream, so the old kernel has ended before the
//     new one begins.  An epoch serves at most kQueueDepth tickets (see MailboxHost).
#pragma once

#include <atomic>
#include <cstdint>

#include "mw_internal.hpp"

namespace mw {
namespace mb {

constexpr uint32_t kQueueDepth = 4096;              // descriptors in the queue
constexpr uint32_t kEpochTickets = kQueueDepth / 2;  // tickets one epoch of the kernel serves at most (see MailboxHost)
constexpr uint32_t kKindCopy = 0, kKindBcast = 1, kKindReduce = 2;

// One queue entry: what one entry of a data kernel's argument block holds, 128 bytes.
struct Desc {
  uint64_t buf[kMaxBufs];  // copy: {source, destination}; fan-out: {root, destinations...}; reduce: all ranks
  uint64_t nbytes;
  uint32_t slot, gen, nbuf;
  uint32_t chunk_bytes;
  uint32_t world_id, world_epoch;  // journalled only
  uint32_t op_chunks, flags;       // as in the launched kernels' entries
  uint32_t target;                 // arrival count at which the operation is complete
  uint32_t kind;                   // kKindCopy / kKindBcast / kKindReduce
  uint32_t first_chunk;            // chunks of the same operation that earlier entries hold (0 for its first entry)
  uint32_t n_chunks;               // chunks of this entry
  uint32_t start;                  // chunks of all earlier tickets (mod 2^32; set by MailboxHost::submit): see owner()
  uint32_t pad;
};
static_assert(sizeof(Desc) == 128, "a descriptor is two cache lines");

// Device memory the HOST writes (through the PCIe aperture) and the kernel reads.
struct HostWritten {
  uint32_t tail;  // doorbell: last ticket whose descriptor is in the queue
  uint32_t stop;  // epoch the host asks to close (0 = none)
  uint32_t pad[30];
  Desc q[kQueueDepth];
};

// Device memory the LEADER writes and the workers read.
struct LeaderWritten {
  uint64_t admit;  // make_admit(): (closing epoch << 32) | last admitted ticket
  uint64_t pad[15];
};

#if defined(__HIP_DEVICE_COMPILE__) || defined(__HIPCC__)
#define MW_MB_HD __host__ __device__
#else
#define MW_MB_HD
#endif
// The leader's word: last admitted ticket, and in the high half the epoch of the kernel that is CLOSING with it (0
// while it is open).  The word is never reset between kernels: a worker of epoch e that still reads its
// predecessor's closing word sees a closing epoch that is not its own, and a last ticket that is its own first - 1.
MW_MB_HD inline uint64_t make_admit(uint32_t ticket, uint32_t closing_epoch) { return ((uint64_t)closing_epoch << 32) | ticket; }
MW_MB_HD inline uint32_t closing_epoch(uint64_t admit) { return (uint32_t)(admit >> 32); }
MW_MB_HD inline uint64_t make_closed(uint32_t epoch, uint32_t ticket) { return ((uint64_t)epoch << 32) | ticket; }

// Tickets are compared modulo 2^32: a is before b.
MW_MB_HD inline bool before(uint32_t a, uint32_t b) { return (int32_t)(a - b) < 0; }
// Which of W workers runs chunk c of a descriptor: chunks are dealt round-robin in the order they were queued
// (`start` counts the chunks of every earlier ticket), so a window of one-chunk messages and the chunks of a few
// larger operations both spread evenly over the workers.
MW_MB_HD inline uint32_t owner(uint32_t start, uint32_t chunk, uint32_t n_workers) {
  return (start % n_workers + chunk % n_workers) % n_workers;  // (no 32-bit wrap inside one descriptor)
}

// Host side.  Port provides:
//   void write_desc(uint32_t index, const Desc& d)   store a descriptor into queue slot `index`
//   void ring(uint32_t tail)                         make the descriptors visible, then the doorbell
//   void ask_stop(uint32_t epoch)                    write the stop word
//   uint64_t closed()                                what the last leader to close left: epoch << 32 | ticket (0: none yet)
//   int launch(uint32_t epoch, uint32_t first)       start a resident kernel that serves tickets from `first` on; 0 = ok
// All calls come from one thread at a time (the library lock), except needs_attention().
//
// Queue slots are recycled by EPOCH, never within one: a worker reads every descriptor of its epoch, also of
// operations it has no chunk of, and may lag behind operations that are long complete -- and when the leader has
// closed, its workers may still be draining.  So a kernel serves at most HALF the queue: the tickets of two
// consecutive epochs never share a slot, and the epoch before those two has ended for certain, because an epoch is
// only started after its predecessor's leader has closed, which it can only do after having run, which (same
// stream) is after the epoch before it has ended altogether.  When an epoch's tickets are used up the host asks that
// kernel to close and refuses descriptors until it has; the caller launches those operations the ordinary way.
template <class Port>
class MailboxHost {
 public:
  explicit MailboxHost(Port* port) : port_(port) {}

  // Forget everything (a new context: tickets, epochs and the memory behind the port start from zero).
  void reset() {
    tail_.store(0, std::memory_order_relaxed);
    epoch_.store(0, std::memory_order_relaxed);
    epoch_first_ = 1;
    chunk_cursor_ = 0;
  }

  // How many descriptors submit() would take now.
  uint32_t room() {
    const uint32_t tail = tail_.load(std::memory_order_relaxed);
    if (epoch_.load(std::memory_order_relaxed) == 0) return kEpochTickets - tail;  // nothing started yet: what is written opens epoch 1
    const bool open = running();
    const uint32_t last = (uint32_t)port_->closed();  // read after `open`: if it closed in between, `open` errs on the careful side
    if (!open && last == tail) return kEpochTickets;  // closed, nothing left over: a fresh epoch
    const uint32_t first = open ? epoch_first_ : last + 1u;  // closed with left-overs: they open the next epoch
    const uint32_t used = tail - first + 1u;
    return used >= kEpochTickets ? 0u : kEpochTickets - used;
  }

  // Queue n descriptors (n <= room()) as tickets first..first+n-1 and make sure a kernel will serve them.
  // Returns 0 or the launch's error; the descriptors stay queued either way (a later attend() retries the launch).
  int submit(const Desc* d, uint32_t n, uint32_t* first_ticket) {
    const uint32_t tail = tail_.load(std::memory_order_relaxed);
    *first_ticket = tail + 1;
    for (uint32_t i = 0; i < n; ++i) {
      Desc x = d[i];
      x.start = chunk_cursor_;
      chunk_cursor_ += x.n_chunks;
      port_->write_desc((tail + 1 + i) % kQueueDepth, x);
    }
    tail_.store(tail + n, std::memory_order_relaxed);
    port_->ring(tail + n);
    return attend();
  }

  // True when no kernel is open (none was ever started, or the last one has closed) and tickets wait that were not
  // admitted.  Reads one host word and two of this object's: polls call it without the lock, a stale answer only
  // delays the next look.
  bool needs_attention() const {
    const uint32_t tail = tail_.load(std::memory_order_relaxed), epoch = epoch_.load(std::memory_order_relaxed);
    if (tail == 0) return false;
    if (epoch == 0) return true;
    const uint64_t c = port_->closed();
    if ((uint32_t)(c >> 32) != epoch) return false;  // open: it will see them
    return (uint32_t)c != tail;
  }

  // Start the next epoch if tickets wait and no kernel is open.
  int attend() {
    if (!needs_attention()) return 0;
    const uint32_t epoch = epoch_.load(std::memory_order_relaxed);
    const uint32_t first = epoch == 0 ? 1u : (uint32_t)port_->closed() + 1u;
    int rc = port_->launch(epoch + 1, first);
    if (rc != 0) return rc;
    epoch_first_ = first;
    epoch_.store(epoch + 1, std::memory_order_relaxed);
    return 0;
  }

  // Ask the open kernel (if any) to close: when its tickets are used up, before bulk launches (which want the whole
  // chip) and at shutdown.
  void stop() {
    if (running()) port_->ask_stop(epoch_.load(std::memory_order_relaxed));
  }

  uint32_t tail() const { return tail_.load(std::memory_order_relaxed); }
  uint32_t epoch() const { return epoch_.load(std::memory_order_relaxed); }
  bool running() const {
    const uint32_t epoch = epoch_.load(std::memory_order_relaxed);
    return epoch != 0 && (uint32_t)(port_->closed() >> 32) != epoch;
  }

 private:
  Port* port_;
  std::atomic<uint32_t> tail_{0};    // last ticket written
  std::atomic<uint32_t> epoch_{0};   // epoch of the last kernel started (0 = none yet)
  uint32_t epoch_first_ = 1;      // first ticket of that epoch
  uint32_t chunk_cursor_ = 0;     // chunks queued so far
};

}  // namespace mb
}  // namespace mw
