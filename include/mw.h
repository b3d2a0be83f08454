/*
 * mw.h -- C ABI of the multi-world tensor data plane for one AMD MI355X.
 *
 * Model (arXiv 2407.08980, "Enabling Elastic Model Serving with MultiWorld"):
 * a *world* is a process group with a fixed set of ranks and is one fault
 * domain; a worker may belong to many worlds at once; collective operations
 * name the world they run in; they never block, their status is polled; when
 * a worker fails only the worlds that contain it break, and every other world
 * keeps working (Sec. 3.1, 3.2, 3.3).
 *
 * Here the workers are *logical*: they all live in the calling process and
 * share one GPU, so a transfer is a device-local read and write.  Each rank
 * posts its own side of an operation (mw_send by the sender, mw_recv by the
 * receiver, one mw_broadcast / mw_allreduce_sum call per rank), because the
 * ranks stand for independent processes and "the other side never arrives"
 * must be expressible (Sec. 3.2).  An operation runs when its last side has
 * been posted; all data movement is done by GPU kernels of this library.
 *
 * Conventions for every function
 *   - returns MW_OK (0) or a negative mw_err; mw_poll / mw_world_state return a
 *     non-negative state or a negative mw_err.  Nothing throws, aborts or
 *     blocks on the device (mw_shutdown and the mw_debug_* calls excepted).
 *   - `buf` arguments are DEVICE pointers to caller-owned memory of the GPU
 *     passed to mw_init.  The library never frees or reallocates them.  Any
 *     alignment and any element count are accepted (16-byte aligned buffers
 *     take the fast path).
 *   - `hip_stream` is a hipStream_t passed as void* (NULL = the null stream).
 *     The operation is ordered after all work enqueued on that stream before
 *     the library launches it (at the latest: everything enqueued before the
 *     post).  MW_STREAM_NONE states that the buffer is already final and no
 *     ordering is needed.
 *   - From the post until mw_poll returns a terminal state the sender's buffer
 *     must not be written and the receiver's buffer must not be read or
 *     written by the caller.  After MW_DONE the data is visible to work
 *     enqueued afterwards on any stream and to host copies.
 *   - All calls are serialised by one internal lock; they may come from any
 *     host thread.
 */
#ifndef MW_H_
#define MW_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* mw_poll / mw_world_state results */
enum { MW_DONE = 0, MW_PENDING = 1, MW_BROKEN = 2, MW_ALIVE = 0 };

typedef enum {
  MW_OK = 0,
  MW_EINVAL = -1,     /* bad argument (rank out of range, src == dst, NULL buffer with count > 0, ...) */
  MW_ENOWORLD = -2,   /* no world with this id */
  MW_EBROKEN = -3,    /* post refused: the world is broken (Sec. 3.3, World Manager) */
  MW_EEXIST = -4,     /* world id already used (ids are never reused, recovery makes NEW worlds, Sec. 3.1) */
  MW_EMISMATCH = -5,  /* the sides of an operation disagree on count, dtype, kind or root */
  MW_ENOMEM = -6,     /* a library table is full (worlds, handles, ring arena) */
  MW_EBADHANDLE = -7, /* handle never issued, or its slot has been recycled */
  MW_EHIP = -8,       /* a HIP call failed; mw_last_hip_error() has the code */
  MW_ENOTINIT = -9    /* mw_init has not been called (or failed) */
} mw_err;

typedef enum { MW_F32 = 0, MW_BF16 = 1 } mw_dtype;

typedef uint64_t mw_handle; /* low 32 bits: table slot, high 32 bits: generation; 0 is never issued */

#define MW_STREAM_NONE ((void*)(intptr_t)-1)
#define MW_MAX_RANKS 64     /* ranks per world (point-to-point) */
#define MW_MAX_COLL_RANKS 8 /* ranks per world for broadcast / all-reduce */

/* ---- context --------------------------------------------------------------------------- */

/* Create the library context on HIP device `hip_device` for logical workers 0..n_workers-1.
 * Allocates (once) the ring arena in HBM, the device and host-pinned completion arrays and an
 * internal stream.  One context per process.  MW_EINVAL if already initialised or n_workers<1,
 * MW_EHIP if the device cannot be used. */
int mw_init(int hip_device, int n_workers);

/* Wait for in-flight operations, free everything.  Blocks.  Handles become invalid. */
int mw_shutdown(void);

/* ---- world manager (Sec. 3.3 "World Manager": initialize_world / remove_world) ---------- */

/* Create world `world_id` whose rank r is worker worker_ids[r] (host array, read during the
 * call).  Gives the world its own mailbox ring (a slice of the HBM arena).  Never disturbs
 * traffic of existing worlds: no device synchronisation, no allocation (online instantiation,
 * Sec. 3.1).  1 <= n_ranks <= MW_MAX_RANKS, workers distinct and < n_workers. */
int mw_world_create(int world_id, const int* worker_ids, int n_ranks);

/* Break a world: it is fenced off (later posts return MW_EBROKEN), every operation of it that is
 * still waiting for a peer becomes MW_BROKEN, operations that already had all their sides are
 * completed normally (what was sent before a failure is delivered, Sec. 4.1 / Fig. 4).  The
 * world's ring is released once its in-flight operations have retired.  No other world is
 * touched, stalled or synchronised.  Idempotent. */
int mw_world_abort(int world_id);

/* A worker failed: abort every world that contains it, and no other (Sec. 3.1, Fig. 2). */
int mw_worker_abort(int worker_id);

/* MW_ALIVE, MW_BROKEN or MW_ENOWORLD. */
int mw_world_state(int world_id);

/* ---- world communicator (Sec. 3.3 "World Communicator"), all non-blocking (Sec. 3.2) ----- */

/* Point-to-point.  Matching is first-in first-out per (world, src_rank, dst_rank), no tags: the
 * k-th send pairs with the k-th recv.  A send completes only when its recv has been posted and the
 * bytes are in the receiver's buffer.  `count` elements of `dtype`; the transfer is byte-exact.
 * On success *out is a handle for mw_poll.  Sides that disagree on count or dtype both poll as
 * MW_EMISMATCH and nothing is moved. */
int mw_send(int world_id, int src_rank, int dst_rank, const void* buf, size_t count, mw_dtype dtype,
            void* hip_stream, mw_handle* out);
int mw_recv(int world_id, int src_rank, int dst_rank, void* buf, size_t count, mw_dtype dtype,
            void* hip_stream, mw_handle* out);

/* Broadcast, posted once by every rank of the world with its own buffer: afterwards every rank's
 * buffer holds root_rank's bytes; the root's buffer is only read.  The k-th collective a rank posts
 * in a world belongs to that world's k-th collective; it runs when all ranks have posted it.
 * Worlds of at most MW_MAX_COLL_RANKS ranks. */
int mw_broadcast(int world_id, int rank, int root_rank, void* buf, size_t count, mw_dtype dtype,
                 void* hip_stream, mw_handle* out);

/* Sum all-reduce, in place, posted once by every rank: afterwards every rank's buffer holds the
 * element-wise sum over the ranks.  Accumulation is in fp32 in ascending rank order
 * ((x0 + x1) + x2) + ..., so results are deterministic and bit-identical on all ranks; bf16
 * results are rounded once, to nearest even.  Worlds of at most MW_MAX_COLL_RANKS ranks; `buf` must
 * be aligned to the element size (MW_EINVAL otherwise). */
int mw_allreduce_sum(int world_id, int rank, void* buf, size_t count, mw_dtype dtype, void* hip_stream,
                     mw_handle* out);

/* The communicator's other four collectives (Sec. 3.3 lists eight operations), posted once by every
 * rank like broadcast and all-reduce, sequenced and completed the same way, worlds of at most
 * MW_MAX_COLL_RANKS ranks.  n = ranks of the world, S = count elements of dtype.
 *
 * mw_reduce_sum: root_rank's buffer receives the element-wise sum over the ranks (fp32 accumulation in
 *   ascending rank order, as all-reduce); every other rank's buffer is only read.
 * mw_all_gather: every rank's recvbuf (n x S) receives the ranks' sendbufs (S each) concatenated in rank
 *   order.  A rank may contribute in place (sendbuf == recvbuf + rank x S bytes).
 * mw_gather: as all-gather, but only root_rank has a recvbuf (pass NULL elsewhere).
 * mw_scatter: rank r's recvbuf (S) receives slice r of root_rank's sendbuf (n x S); sendbuf is used on
 *   the root only (pass NULL elsewhere).
 * The copies are byte-exact. */
int mw_reduce_sum(int world_id, int rank, int root_rank, void* buf, size_t count, mw_dtype dtype, void* hip_stream,
                  mw_handle* out);
int mw_all_gather(int world_id, int rank, const void* sendbuf, void* recvbuf, size_t count, mw_dtype dtype,
                  void* hip_stream, mw_handle* out);
int mw_gather(int world_id, int rank, int root_rank, const void* sendbuf, void* recvbuf, size_t count,
              mw_dtype dtype, void* hip_stream, mw_handle* out);
int mw_scatter(int world_id, int rank, int root_rank, const void* sendbuf, void* recvbuf, size_t count,
               mw_dtype dtype, void* hip_stream, mw_handle* out);

/* Status of an operation: MW_DONE, MW_PENDING, MW_BROKEN, or MW_EMISMATCH / MW_EBADHANDLE.  Never
 * blocks and never synchronises the device: completion is read from a host-visible flag that the
 * GPU writes when the operation's last chunk has retired (Sec. 3.2: asynchronous operations need
 * their status polled).  Polling an operation that is complete on the host side but not yet
 * launched launches it.  Terminal states are sticky; a handle stays valid until its table slot is
 * reused (at least mw_handle_capacity() further posts). */
int mw_poll(mw_handle h);

/* ---- watchdog (Sec. 3.3 "Watchdog") ------------------------------------------------------------ */

/* Failures of workers that share a host are silent (Sec. 3.2 "Reliable fault detection"), so each
 * worker reports its health periodically and a watchdog declares a worker failed when its reports
 * have been missing for longer than a timeout (the paper's example is 3 seconds); the worlds containing it are then
 * aborted exactly as by mw_worker_abort, and no others.
 *
 * mw_heartbeat(worker): the worker is alive now (steady clock).  A worker is watched from its first
 *   heartbeat on; workers that never send one are never declared failed.  MW_EBROKEN once the worker
 *   has been declared failed (a failed worker does not come back: recovery uses a new worker id and
 *   new worlds, Sec. 3.1); mw_world_create refuses such a worker with MW_EBROKEN too.
 * mw_watchdog_start(timeout_s, period_s): start the library's watchdog thread, which inspects the
 *   heartbeat table every period_s seconds.  MW_EINVAL if it is already running.
 * mw_watchdog_stop(): stop and join it (mw_shutdown does this too).
 * mw_heartbeat_at / mw_watchdog_check_at: the same with the caller's clock (seconds, any origin) instead
 *   of the steady clock and the thread: one inspection at time t with the given timeout; returns the
 *   number of workers newly declared failed.  For callers that drive the check from their own polling
 *   loop, and for deterministic tests.
 * mw_worker_state: MW_ALIVE or MW_BROKEN (declared failed by the watchdog).
 * mw_heartbeat_epoch: heartbeats received from the worker so far. */
int mw_heartbeat(int worker_id);
int mw_heartbeat_at(int worker_id, double t);
int mw_watchdog_start(double timeout_s, double period_s);
int mw_watchdog_stop(void);
int mw_watchdog_check_at(double t, double timeout_s);
int mw_worker_state(int worker_id);
long mw_heartbeat_epoch(int worker_id);

/* ---- extensions ----------------------------------------------------------------------------- */

/* Launch every operation whose sides have all been posted (one batched launch per kernel kind,
 * covering operations of all worlds).  mw_poll does this on demand; calling it after a group of
 * posts batches them into one launch. */
int mw_flush(void);

/* Post many sides with one call (one lock acquisition): posts[i] is what the corresponding
 * mw_send / mw_recv / mw_broadcast / mw_allreduce_sum / mw_reduce_sum / mw_all_gather / mw_gather /
 * mw_scatter call would take -- `a`/`b` are src/dst rank for point-to-point, rank/root for the rooted
 * collectives, rank/unused otherwise; buf2 is the recvbuf of all-gather, gather and scatter (buf their
 * sendbuf).  Posts are processed in array
 * order and independently: handles[i] is the handle, or 0 if that post was refused; results[i] (may be
 * NULL) is its return code.  Returns MW_OK or the first refusal's code.  Host arrays, read/written
 * during the call. */
typedef enum {
  MW_POST_SEND = 0, MW_POST_RECV = 1, MW_POST_BROADCAST = 2, MW_POST_ALLREDUCE_SUM = 3,
  MW_POST_REDUCE_SUM = 4, MW_POST_ALL_GATHER = 5, MW_POST_GATHER = 6, MW_POST_SCATTER = 7
} mw_post_kind;
typedef struct {
  int32_t kind; /* mw_post_kind */
  int32_t world_id;
  int32_t a;
  int32_t b;
  void* buf;
  uint64_t count;
  int32_t dtype; /* mw_dtype */
  int32_t reserved;
  void* hip_stream;
  void* buf2;
} mw_post_desc;
int mw_post_many(const mw_post_desc* posts, int n, mw_handle* handles, int* results);

/* For callers that cannot allocate or wait on the host: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  A variant of mw_post_many that allocates nothing, on the device or on the
 * host, and hands out no handles: the array must hold WHOLE operations (every side of each), which are matched by
 * the same rules as everywhere else (first in, first out per (world, src, dst); the k-th collective a rank posts
 * in a world belongs to that world's k-th collective), independently of sides posted through the other calls,
 * whose queues are neither read nor changed.  All of them are enqueued on `hip_stream` (hipStream_t as void*,
 * NULL = the null stream; MW_STREAM_NONE is refused) behind whatever that stream already holds, and they are
 * complete when work enqueued on that stream afterwards runs: completion is by stream order, there is nothing to
 * poll.  The posts' own hip_stream fields are ignored.  The operations of one call run concurrently: apart from
 * buffers that are only read, they must not share bytes.
 *
 * The kernels are the ones every other call uses; their per-operation completion state (arrival counter,
 * completion word: device memory beyond the callers' buffers) lives in a static device array of
 * MW_NOALLOC_MAX_OPS slots (16.25 KiB per GPU, held until the process ends) instead of the ring arena, and is
 * re-armed by a small fill kernel at the start of every call (no memset node: the call may be recorded into a
 * graph).  Every call on a GPU shares that array: two calls whose kernels overlap in time on one GPU race on it --
 * issue them on one stream, or order them with events.
 *
 * At most MW_NOALLOC_MAX_POSTS posts forming at most MW_NOALLOC_MAX_OPS operations that move data: MW_EINVAL
 * beyond that, for a side whose peers are not all in the array, and for whatever the posting calls refuse;
 * MW_ENOWORLD / MW_EBROKEN for an unknown / broken world; MW_EMISMATCH if the sides of an operation disagree.  On
 * any error nothing has been enqueued.  Needs mw_init (which does allocate) to have been called. */
#define MW_NOALLOC_MAX_POSTS 128
#define MW_NOALLOC_MAX_OPS 64
int mw_post_many_noalloc(const mw_post_desc* posts, int n, void* hip_stream);

/* Number of operations that have all their sides posted and have not yet been seen complete by a
 * poll (queued for launch or in flight).  0 means every remaining MW_PENDING handle waits for a peer. */
int mw_pending_ops(void);

/* Poll n handles at once: states[i] = mw_poll(handles[i]).  Returns the number not yet terminal. */
int mw_poll_many(const mw_handle* handles, int n, int* states);

/* Tunables.  key: "chunk_bytes" (power of two, 4096..4194304; 0 = choose per launch), "reduce_lds" (0/1: stage
 * all-reduce tiles through LDS), "mailbox" (0/1, see below), "mailbox_idle_us" (10..50000, default 300) -- these four may be set at any time; "ring_depth" (1..256
 * slots per world, default 128), "max_rings", "handle_capacity", "mailbox_workers" (1..1023, default 255; never more than the GPU's compute units less one are used) -- only before
 * mw_init.  MW_EINVAL for unknown keys or bad values.
 *
 * "mailbox" = 1 (the default) turns on the resident mailbox kernel: a flush whose operations have final buffers (no busy caller
 * stream) and move at most 64 MiB together is not launched but written as descriptors into a queue in device memory
 * that a resident kernel serves (one leader that admits descriptors and decides when the kernel ends, and
 * mailbox_workers workgroups that move the data), so a small operation does not pay a kernel launch (Sec. 3.2 / 3.3:
 * a worker busy-waits on its operation, so that latency is what it sees).  Results, completion and polling are
 * the same as for launched operations.  The kernel is started on demand and never waited for; it ends by itself
 * when the host asks (a larger flush wants the whole chip; mw_shutdown), after mailbox_idle_us without work, and after 100 ms
 * at the latest; operations that arrive just as it ends are served by the next one, which the following mw_flush or
 * mw_poll starts.  While a kernel is open a device-wide synchronisation by the caller waits for it to end (at most the
 * idle time); stream-level synchronisation does not.  With 0 every flush is launched. */
int mw_config_set(const char* key, long value);
long mw_config_get(const char* key);

int mw_handle_capacity(void);
int mw_last_hip_error(void);
const char* mw_strerror(int err);

/* Identity of the sources this library was compiled from: the hex SHA-256 (first 16 digits) over the files
 * of csrc/ and this header, passed in by the build script; "unknown" for a build made by hand.  The Python
 * binding refuses a library whose identity is not that of the sources beside it.  Static storage. */
const char* mw_build_id(void);

/* Per-kernel timing with HIP events on the library's own stream.  mw_profile_enable(1) starts
 * bracketing every data-kernel launch with events; mw_profile_read sums the finished launches of
 * kernel kind `kind` (0 copy incl. gather / scatter segments, 1 fan-out: broadcast and all-gather, 2 reduce:
 * all-reduce and reduce): number of launches, total milliseconds
 * and total payload-descriptor bytes (sum of nbytes over operations).  Reading waits for the
 * recorded events (blocks); it is for benchmarks, not for the data path.  While timing is enabled every flush is
 * launched (work done by the resident mailbox kernel cannot be bracketed by events). */
int mw_profile_enable(int on);
int mw_profile_read(int kind, uint64_t* launches, double* total_ms, uint64_t* op_bytes);

/* Diagnostics (block until the library's stream is idle).
 * mw_debug_ring_read copies world `world_id`'s ring header and slots from HBM to `out` (host):
 * returns the number of bytes written, or a negative error; MW_EINVAL if cap is too small.
 * mw_debug_arena_hash returns an FNV-1a hash of every ring byte NOT belonging to `except_world`
 * (pass -1 to hash everything) so that tests can show a teardown touched nothing else. */
long mw_debug_ring_read(int world_id, void* out, size_t cap);
/* State of the resident mailbox kernel: epoch = how many have been started, open = 1 while the latest has not closed,
 * tail = descriptors queued so far. */
int mw_debug_mailbox(uint32_t* epoch, uint32_t* open, uint32_t* tail);
int mw_debug_arena_hash(int except_world, uint64_t* hash);

#ifdef __cplusplus
}
#endif
#endif /* MW_H_ */
