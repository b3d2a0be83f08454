// Internal contract between the host runtime (mw_host.cpp) and a device backend.
//
// The host runtime owns the world table, matching, handles and ring-slot
// bookkeeping.  A backend owns device memory and launches.  The real backend
// is mw_device.hip; mw_device_null.cpp is a test double that moves no bytes
// and lets the host state machine be exercised without a GPU.
#pragma once

#include <cstddef>
#include <cstdint>

namespace mw {

constexpr int kMaxBufs = 8;          // buffers named by one descriptor (== MW_MAX_COLL_RANKS)
constexpr int kSlotBytes = 256;      // one ring slot in HBM
constexpr int kHeaderBytes = 256;    // one ring header in HBM
constexpr int kMaxRingDepth = 256;   // slots per world ring, at most
constexpr int kDefaultRingDepth = 128;

constexpr int kMaxOpBufs = 16;       // buffers one operation may name (all-gather: 8 sources + 8 destinations)

// Kernel kinds (one internal stream and one profile counter each).
enum Kind : uint32_t { kCopy = 0, kBcast = 1, kReduce = 2, kNumKinds = 3 };

// Operation kinds.  Gather and scatter run as copy segments, all-gather as fan-out segments,
// reduce as an all-reduce that stores to the root only.
enum OpKind : uint32_t {
  opCopy = 0, opBcast = 1, opAllReduce = 2, opReduce = 3, opAllGather = 4, opGather = 5, opScatter = 6, opNumKinds = 7
};

// Journal half of a ring slot (first 128 bytes): the descriptor of the operation
// occupying the slot, written by the GPU when the operation is dispatched.
struct SlotDesc {
  uint64_t buf[kMaxBufs];  // buffers of the operation's first kernel entry: copy {src, dst}; broadcast
                           // {root, dst...}; (all-)reduce: all ranks; gather / scatter / all-gather: the
                           // first segment's source and destination(s)
  uint64_t nbytes;         // bytes per rank
  uint32_t kind;           // OpKind
  uint32_t dtype;
  uint32_t nbuf;
  uint32_t world_id;
  uint32_t world_epoch;
  uint32_t gen;       // completion generation this operation publishes
  uint32_t nchunks;        // chunks of the whole operation (all its segments)
  uint32_t chunk_bytes;
  uint32_t pad[6];
};
static_assert(sizeof(SlotDesc) == 128, "journal half is 128 bytes");

// Sync half of a ring slot (second 128 bytes): touched only by device atomics.
struct SlotSync {
  uint32_t arrived;   // chunks retired so far; the last one resets it to 0
  uint32_t done_gen;  // generation of the last operation completed in this slot
  uint32_t pad[30];
};
static_assert(sizeof(SlotSync) == 128, "sync half is 128 bytes");

struct RingSlot {
  SlotDesc d;
  SlotSync s;
};
static_assert(sizeof(RingSlot) == kSlotBytes, "ring slot size");

// Ring header in HBM, written by the world-marker kernel at create and abort.
struct RingHeader {
  uint32_t world_id;
  uint32_t state;   // 0 alive, 2 broken
  uint32_t epoch;   // bumped by every marker write
  uint32_t depth;
  uint32_t first_slot;  // global index of the ring's first slot
  uint32_t n_ranks;
  uint32_t pad[58];
};
static_assert(sizeof(RingHeader) == kHeaderBytes, "ring header size");

// One operation handed to a launch.  Buffer layout by kind:
//   opCopy       buf[0] = source, buf[1] = destination                                  (nbuf = 2)
//   opBcast      buf[0] = root's buffer, buf[1..n-1] = the other ranks' in rank order   (nbuf = n)
//   opAllReduce  buf[r] = rank r's buffer                                               (nbuf = n)
//   opReduce     buf[r] = rank r's buffer; only buf[root] is written                    (nbuf = n)
//   opAllGather  buf[r] = rank r's source, buf[8 + r] = rank r's destination (n x nbytes)
//   opGather     buf[r] = rank r's source, buf[8] = the root's destination (n x nbytes)
//   opScatter    buf[0] = the root's source (n x nbytes), buf[8 + r] = rank r's destination
struct LaunchOp {
  uint64_t buf[kMaxOpBufs];
  uint64_t nbytes;  // bytes per rank
  uint32_t kind;    // OpKind
  uint32_t dtype;
  uint32_t nbuf;    // ranks taking part (2 for a copy)
  uint32_t root;
  uint32_t slot;    // global ring slot index
  uint32_t gen;
  uint32_t world_id;
  uint32_t world_epoch;
};

// The caller streams one operation is ordered after (hipStream_t as void*, NULL = the null stream;
// MW_STREAM_NONE never appears here).  At most one per posted side.
struct OpDeps {
  void* stream[kMaxBufs];
  int n;
};

struct DeviceConfig {
  uint32_t total_slots;   // ring slots in the arena
  uint32_t total_rings;   // ring headers in the arena
  uint32_t chunk_bytes;   // 0 = choose per launch
  uint32_t reduce_lds;    // stage all-reduce tiles through LDS
  uint32_t mailbox;       // serve small flushes through the resident mailbox kernel instead of launching
  uint32_t mailbox_workers;  // workgroups of the resident kernel that move data (1..1023)
  uint32_t mailbox_idle_us;  // the resident kernel ends after this long without a new descriptor
};

class Device {
 public:
  virtual ~Device() {}
  virtual int init(int hip_device, const DeviceConfig& cfg) = 0;
  virtual void shutdown() = 0;
  virtual void set_config(const DeviceConfig& cfg) = 0;
  // Launch `n` operations (any mix of kinds, any worlds); operation i is ordered after the work already
  // enqueued on each stream of deps[i], and on nothing else: an operation never waits for a stream that
  // only another operation named (Sec. 3.2: a pending operation in one world must not hold up another).
  // Returns 0 or MW_EHIP; launched[i] is set to 1 for every operation that was enqueued on the device (all
  // of them on success; on failure the others were not and may be retried).
  virtual int launch(const LaunchOp* ops, const OpDeps* deps, int n, uint8_t* launched) = 0;
  // Enqueue `n` <= MW_NOALLOC_MAX_OPS operations on the caller's stream with their completion state in the static
  // device scratch (slot = index of the operation); allocates nothing, publishes nothing to the host.
  virtual int launch_static(const LaunchOp* ops, int n, void* stream) = 0;
  // The mailbox (resident kernel): true when operations wait in its queue and no kernel is open to serve them
  // (it closed for lack of work just as they came in); cheap and callable without the lock.  attend() starts the
  // next kernel then.  mailbox_state: epoch of the last kernel started, whether it is still open, last ticket queued.
  virtual bool needs_attention() = 0;
  virtual int attend() = 0;
  virtual void mailbox_state(uint32_t* epoch, uint32_t* open, uint32_t* tail) = 0;
  // Write a ring header (world create / abort marker).  Asynchronous, on the library's stream.
  virtual int mark_world(uint32_t ring_index, const RingHeader& h) = 0;
  // Host-visible completion word of a slot (acquire load of the pinned mirror).
  virtual uint32_t flag(uint32_t slot) = 0;
  // Diagnostics: block until idle, then copy arena bytes to the host.
  virtual int read_ring(uint32_t ring_index, uint32_t first_slot, uint32_t depth, void* out) = 0;
  virtual int sync() = 0;
  virtual int last_hip_error() = 0;
  virtual int profile_enable(int on) = 0;
  virtual int profile_read(int kind, uint64_t* launches, double* ms, uint64_t* bytes) = 0;
};

Device* make_device();  // provided by exactly one backend per library

}  // namespace mw
