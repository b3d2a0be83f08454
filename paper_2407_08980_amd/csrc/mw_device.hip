// Device backend for gfx950 (MI355X): the kernels of the multi-world data plane
// and their launch logic.
//
//   mw_k_copy    batched point-to-point copy: one launch moves the matched
//                send/recv pairs of many worlds (the communicator's send/recv,
//                arXiv 2407.08980 Sec. 3.3)
//   mw_k_bcast   broadcast fan-out: the root's chunk is read once and written
//                to every other rank's buffer (Sec. 3.3)
//   mw_k_reduce  sum all-reduce among a world's logical ranks, in place, fp32
//                accumulation in ascending rank order (Sec. 3.3)
//   mw_k_mark    writes a world's ring header: alive at creation, broken with a
//                bumped epoch at abort (Sec. 3.3 "World Manager")
//
// Every data kernel ends with the completion protocol: the workgroup that
// retires the last chunk of an operation publishes the operation's generation
// to the ring slot in HBM and to a host-pinned word, which is what the host
// polls -- no HIP call, no device synchronisation (Sec. 3.2: asynchronous
// operations report no status by themselves, so it is polled).
//
// All of this is bandwidth-bound work: 128-bit coalesced raw-buffer accesses with streaming
// cache policies through hardware bounds-checked windows, no matrix instructions.

#include <hip/hip_runtime.h>
#include <immintrin.h>

#include <algorithm>
#include <cstdio>
#include <cstring>
#include <vector>

#include "../../include/mw.h"
#include "mw_internal.hpp"
#include "mw_mailbox.hpp"

// Scratch of the entry point that allocates nothing (mw_post_many_noalloc): ring slots (arrival counter and
// completion word per operation) followed by the completion words the kernels otherwise write to host-pinned
// memory.  One copy per GPU, held until the process ends; every call on a GPU shares it, so calls that overlap
// on one GPU race.  Host code never uses this name as an address: the per-device address comes from
// hipGetSymbolAddress at init (g_scratch_ptr).
static __device__ __align__(256) unsigned char scratch[MW_NOALLOC_MAX_OPS * (mw::kSlotBytes + 4)];
constexpr int kMaxHipDevices = 64;
static unsigned char* g_scratch_ptr[kMaxHipDevices] = {};  // device address of `scratch`, per HIP device

// The mailbox queue lives in fine-grained device memory, which the host writes through the PCIe aperture and the
// resident kernel polls at HBM speed (measured round trip host -> polling wave -> host: 2.0-2.1 us whatever the
// number of polling waves; through host-pinned memory the same round trip is 2.4 us with one poller and 25 us with
// 256, because every poll crosses the bus).  One block per GPU, allocated at the first mw_init on that GPU and kept
// until the process ends.
static mw::mb::HostWritten* g_mailbox_mem[kMaxHipDevices] = {};

namespace mw {
namespace {

constexpr int kStaticOps = MW_NOALLOC_MAX_OPS;

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kCopyWG = 1024;    // threads per workgroup, copy / broadcast
constexpr int kCopyU = 4;        // 16-byte vectors in flight per thread
constexpr int kReduceWG = 1024;  // threads per workgroup, (all-)reduce
constexpr int kCopyMax = 64;     // entries per copy launch (kernel arguments stay under 4 KiB)
constexpr int kCollMax = 35;     // entries per fan-out / reduce launch
// (All-)reduce, register path: 16-byte vectors per rank in flight per thread, by number of ranks.  Two ranks
// give a thread only two loads per vector; a second vector brings it to the four that the other counts have.
constexpr int reduce_u(int n) { return n == 2 ? 2 : 1; }
// (All-)reduce, LDS-staged path: vectors per rank in the tile for a given chunk size (host and device agree)
__host__ __device__ constexpr uint32_t lds_stride(uint32_t chunk_bytes) {
  return (chunk_bytes + 15) / 16 < (uint32_t)kReduceWG ? (chunk_bytes + 15) / 16 : (uint32_t)kReduceWG;
}

// An operation is one or more *entries* of one kernel: a copy is one copy entry, a gather or a
// scatter n copy entries, a broadcast one fan-out entry, an all-gather n (or more) fan-out entries,
// an (all-)reduce one reduce entry.  All entries of an operation share its ring slot; `op_chunks`
// is the chunk count of the whole operation, which is what the arrival counter runs up to.
// flags: bit 0 = this entry journals the descriptor; bits 1-7 = element type; bits 8-15 = OpKind;
// bits 16-23 = ranks of the operation; bits 24-31 = mask of the ranks whose buffer a reduce entry stores to.
struct CopyEnt {
  uint64_t src, dst, nbytes;
  uint32_t slot, gen;
  uint32_t world_id, world_epoch;  // journalled only
  uint32_t op_chunks, flags;
  uint32_t target, pad;  // the arrival count at which the operation is complete (see retire_chunk)
};
// The argument block travels by value in the kernel-argument segment, which the host fills through the PCIe
// aperture at launch: 4 KiB of it cost 1.5 us of host time per launch, so every kernel exists for three capacities
// and a launch takes the smallest that holds its entries.
template <int CAP>
struct CopyArgs {
  uint32_t n;
  uint32_t chunk_shift;
  uint32_t first_chunk[CAP + 1];  // first_chunk[i] = chunks before entry i; [n] = total
  uint32_t rotate;  // see chunk_of_workgroup
  CopyEnt e[CAP];
};
constexpr int kCopyCap[3] = {8, 24, kCopyMax};
static_assert(sizeof(CopyArgs<kCopyMax>) <= 4096, "kernel argument block");

struct CollEnt {
  uint64_t buf[kMaxBufs];
  uint64_t nbytes;
  uint32_t slot, gen, nbuf;
  uint32_t chunk_bytes;  // per entry: the best chunk of a reduce entry depends on its number of ranks
  uint32_t world_id, world_epoch;  // journalled only
  uint32_t op_chunks, flags;
  uint32_t target, pad;
};
template <int CAP>
struct CollArgs {
  uint32_t n;
  uint32_t rotate;  // see chunk_of_workgroup
  uint32_t first_chunk[CAP + 1];
  uint32_t pad;
  CollEnt e[CAP];
};
constexpr int kCollCap[3] = {4, 12, kCollMax};
static_assert(sizeof(CollArgs<kCollMax>) <= 4096, "kernel argument block");

// ------------------------------------------------------------------------------------------------
// device helpers
// ------------------------------------------------------------------------------------------------

// Workgroup -> chunk.  The hardware deals consecutive workgroups out to the 8 XCDs in turn, so with chunk = workgroup
// index XCD k would only ever touch addresses congruent to k x chunk modulo 8 x chunk: a fixed eighth of the address
// bits that select L2 and memory channels.  Rotating every full row of 8 workgroups by its row number lets each XCD
// sweep all residues.  Kernel time, 8 worlds, mean over 7-8 relative placements of the buffers (offsets of 0 B ... 2 MiB
// between consecutive buffers; a placement alone moves a figure by +-3 %), TB/s of algorithmic traffic:
//   copy, 64 KiB chunks        5.88 -> 6.32  (128 KiB chunks without rotation: 6.26)
//   broadcast, 4 ranks, 64 KiB  5.60 -> 6.14  (128 KiB without: 5.94)
//   reduce to a root, 4 ranks   6.15 (32 KiB) -> 6.35 (24 KiB)
//   all-reduce, 4 ranks, 12 KiB 6.09 (5.86-6.33 by placement) -> 6.03 (5.96-6.12): evens the placements out, gains nothing
// so copies, fan-outs and reductions to a root rotate, launches holding an all-reduce do not.  Adding further row bits
// to the rotation, or xor-ing instead, changed nothing.  The last, partial row keeps the identity: the map stays one to one.
__device__ __forceinline__ uint32_t chunk_of_workgroup(uint32_t b, uint32_t grid, uint32_t rotate) {
  if (!rotate || b >= (grid & ~7u)) return b;
  return (b & ~7u) | ((b + (b >> 3)) & 7u);
}

// Index of the operation that owns chunk c: the largest i with first_chunk[i] <= c.
__device__ __forceinline__ int find_op(const uint32_t* first_chunk, int n, uint32_t c) {
  int lo = 0, hi = n;
  while (hi - lo > 1) {
    int mid = (lo + hi) >> 1;
    if (first_chunk[mid] <= c) lo = mid; else hi = mid;
  }
  return lo;
}

// Payload is moved with raw buffer instructions through a *window*: a buffer resource that covers
// exactly the bytes of one chunk of one buffer.  The hardware checks every access against the
// window (a load outside it returns zero, a store outside it is dropped), offsets are 32-bit, and the
// compiler tracks the instructions' completion like any other load or store.
//
// Cache policy bits (gfx940 family: sc0 = 1, nt = 2, sc1 = 16).  Stores carry the system-scope bits
// and the streaming hint: they are written through to memory instead of staying dirty in the issuing
// XCD's L2, and they are acknowledged (vmcnt) only once they are performed at that scope.  This is
// what lets an operation be declared complete while the kernel that moved it is still running,
// without a per-chunk L2 write-back (measured: one `buffer_wbl2` per workgroup cost 40 % of the copy
// bandwidth, one per wave 90 %; write-through stores cost nothing).  Loads stream past the L2
// (sc1 nt): nothing here is read twice.
typedef __amdgpu_buffer_rsrc_t rsrc_t;
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
constexpr int kLoadPolicy = 16 | 2;
constexpr int kStorePolicy = 1 | 16 | 2;

__device__ __forceinline__ rsrc_t window(uint64_t base, uint64_t len) {
  return __builtin_amdgcn_make_buffer_rsrc(reinterpret_cast<void*>(base), 0, (int)len, 0x00020000);
}

template <typename T>
struct Io;
template <>
struct Io<u32x4> {
  static __device__ __forceinline__ u32x4 ld(rsrc_t r, uint32_t o) {
    return __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(r, o, 0, kLoadPolicy));
  }
  static __device__ __forceinline__ void st(rsrc_t r, uint32_t o, u32x4 v) {
    __builtin_amdgcn_raw_buffer_store_b128(v, r, o, 0, kStorePolicy);
  }
};
template <>
struct Io<u32x2> {
  static __device__ __forceinline__ u32x2 ld(rsrc_t r, uint32_t o) {
    return __builtin_bit_cast(u32x2, __builtin_amdgcn_raw_buffer_load_b64(r, o, 0, kLoadPolicy));
  }
  static __device__ __forceinline__ void st(rsrc_t r, uint32_t o, u32x2 v) {
    __builtin_amdgcn_raw_buffer_store_b64(v, r, o, 0, kStorePolicy);
  }
};
template <>
struct Io<uint32_t> {
  static __device__ __forceinline__ uint32_t ld(rsrc_t r, uint32_t o) {
    return __builtin_amdgcn_raw_buffer_load_b32(r, o, 0, kLoadPolicy);
  }
  static __device__ __forceinline__ void st(rsrc_t r, uint32_t o, uint32_t v) {
    __builtin_amdgcn_raw_buffer_store_b32(v, r, o, 0, kStorePolicy);
  }
};
template <>
struct Io<uint16_t> {
  static __device__ __forceinline__ uint16_t ld(rsrc_t r, uint32_t o) {
    return __builtin_amdgcn_raw_buffer_load_b16(r, o, 0, kLoadPolicy);
  }
  static __device__ __forceinline__ void st(rsrc_t r, uint32_t o, uint16_t v) {
    __builtin_amdgcn_raw_buffer_store_b16(v, r, o, 0, kStorePolicy);
  }
};
template <>
struct Io<unsigned char> {
  static __device__ __forceinline__ unsigned char ld(rsrc_t r, uint32_t o) {
    return __builtin_amdgcn_raw_buffer_load_b8(r, o, 0, kLoadPolicy);
  }
  static __device__ __forceinline__ void st(rsrc_t r, uint32_t o, unsigned char v) {
    __builtin_amdgcn_raw_buffer_store_b8(v, r, o, 0, kStorePolicy);
  }
};

// Completion protocol.  Every wave waits until its own write-through stores are acknowledged,
// the workgroup meets, then one thread counts the chunk in (device-scope atomic, performed at
// the memory side).  A slot's arrival counter only ever counts up: the host keeps the running total
// of chunks it has sent through the slot and hands every operation the count at which it is complete
// (`target`), so nothing has to be re-armed -- there is no store that a later operation in the same
// slot could overtake.  The workgroup that brings the count to `target` knows that every other chunk's
// stores were acknowledged before their count-in; it publishes the operation's generation in the ring
// slot (HBM, the journal) and in the host-pinned word the host polls.  An operation of a single chunk
// is complete when that chunk is: it skips the counter (and one memory round trip).
__device__ __forceinline__ void retire_chunk(RingSlot* slots, uint32_t* host_flags, uint32_t slot, uint32_t gen,
                                             uint32_t nchunks, uint32_t target) {
  __builtin_amdgcn_s_waitcnt(0);  // vmcnt(0) expcnt(0) lgkmcnt(0): all of this wave's stores are performed
  __syncthreads();
  if (threadIdx.x == 0) {
    SlotSync* s = &slots[slot].s;
    bool last = nchunks == 1;
    if (!last) last = __hip_atomic_fetch_add(&s->arrived, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) + 1 == target;
    if (last) {
      __hip_atomic_store(&s->done_gen, gen, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      __hip_atomic_store(&host_flags[slot], gen, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
    }
  }
}

// Copy the `len` bytes of window s to every window d[0..nd) with accesses of type T (every window's
// base is aligned to T).  Unrolled so that U loads are in flight per thread before the first store.
template <typename T, int WG, int U, int ND>
__device__ __forceinline__ void move_units(rsrc_t s, const rsrc_t* d, int nd, uint32_t len) {
  constexpr uint32_t B = sizeof(T);
  const uint32_t n = len / B;
  const uint32_t step = WG * U;
  const uint32_t full = n - n % step;
  uint32_t i = threadIdx.x;
  for (; i < full; i += step) {
    T v[U];
#pragma unroll
    for (int u = 0; u < U; ++u) v[u] = Io<T>::ld(s, (i + u * WG) * B);
    // vmcnt(0): drain before turning round.  The counter covers stores as well as loads, so a wave
    // alternates between one read burst (U x 1 KiB) and one write burst with nothing else of its own
    // in flight.  Measured on 8 x 512 MiB: 6.39-6.44 TB/s of traffic against 6.02 TB/s when the
    // compiler's finer-grained waits let stores trickle out between the loads.
    __builtin_amdgcn_s_waitcnt(0x0F70);
#pragma unroll
    for (int k = 0; k < ND; ++k) {
      if (k < nd) {
#pragma unroll
        for (int u = 0; u < U; ++u) Io<T>::st(d[k], (i + u * WG) * B, v[u]);
      }
    }
  }
  for (; i < n; i += WG) {
    T v = Io<T>::ld(s, i * B);
#pragma unroll
    for (int k = 0; k < ND; ++k)
      if (k < nd) Io<T>::st(d[k], i * B, v);
  }
  // bytes past the last whole unit
  for (uint32_t b = n * B + threadIdx.x; b < len; b += WG) {
    unsigned char v = Io<unsigned char>::ld(s, b);
#pragma unroll
    for (int k = 0; k < ND; ++k)
      if (k < nd) Io<unsigned char>::st(d[k], b, v);
  }
}

// Pick the widest access every buffer is aligned to (`align` = OR of all the base addresses).
template <int WG, int U, int ND>
__device__ __forceinline__ void move_any(uint64_t align, rsrc_t s, const rsrc_t* d, int nd, uint32_t len) {
  const uint32_t a = (uint32_t)align & 15u;
  if (a == 0) move_units<u32x4, WG, U, ND>(s, d, nd, len);
  else if ((a & 7) == 0) move_units<u32x2, WG, U, ND>(s, d, nd, len);
  else if ((a & 3) == 0) move_units<uint32_t, WG, U, ND>(s, d, nd, len);
  else if ((a & 1) == 0) move_units<uint16_t, WG, U, ND>(s, d, nd, len);
  else move_units<unsigned char, WG, U, ND>(s, d, nd, len);
}

// ------------------------------------------------------------------------------------------------
// K1: batched multi-world copy
// ------------------------------------------------------------------------------------------------
template <int CAP>
__global__ __launch_bounds__(kCopyWG) void mw_k_copy(const CopyArgs<CAP> a, RingSlot* __restrict__ slots,
                                                      uint32_t* __restrict__ host_flags) {
  const uint32_t c = chunk_of_workgroup(blockIdx.x, gridDim.x, a.rotate);
  const int op = find_op(a.first_chunk, (int)a.n, c);
  const uint64_t src = a.e[op].src, dst = a.e[op].dst, nbytes = a.e[op].nbytes;
  const uint32_t slot = a.e[op].slot, gen = a.e[op].gen;
  const uint32_t ci = c - a.first_chunk[op];
  const uint32_t nchunks = a.e[op].op_chunks, flags = a.e[op].flags;
  const uint64_t off = (uint64_t)ci << a.chunk_shift;
  const uint64_t chunk = 1ull << a.chunk_shift;
  const uint64_t len = (nbytes - off < chunk) ? nbytes - off : chunk;
  if (ci == 0 && threadIdx.x == 0 && (flags & 1u)) {  // journal the descriptor into the world's ring
    SlotDesc* d = &slots[slot].d;
    d->buf[0] = src;
    d->buf[1] = dst;
    d->nbytes = nbytes;
    d->kind = (flags >> 8) & 0xFFu;
    d->dtype = (flags >> 1) & 0x7Fu;
    d->nbuf = (flags >> 16) & 0xFFu;
    d->world_id = a.e[op].world_id;
    d->world_epoch = a.e[op].world_epoch;
    d->gen = gen;
    d->nchunks = nchunks;
    d->chunk_bytes = (uint32_t)chunk;
  }
  const rsrc_t dw[1] = {window(dst + off, len)};
  move_any<kCopyWG, kCopyU, 1>(src | dst, window(src + off, len), dw, 1, (uint32_t)len);
  retire_chunk(slots, host_flags, slot, gen, nchunks, a.e[op].target);
}

// ------------------------------------------------------------------------------------------------
// K2: broadcast fan-out
// ------------------------------------------------------------------------------------------------
template <int CAP>
__global__ __launch_bounds__(kCopyWG) void mw_k_bcast(const CollArgs<CAP> a, RingSlot* __restrict__ slots,
                                                       uint32_t* __restrict__ host_flags) {
  const uint32_t c = chunk_of_workgroup(blockIdx.x, gridDim.x, a.rotate);
  const int op = find_op(a.first_chunk, (int)a.n, c);
  const uint64_t nbytes = a.e[op].nbytes;
  const uint32_t slot = a.e[op].slot, gen = a.e[op].gen, nbuf = a.e[op].nbuf;
  const uint32_t ci = c - a.first_chunk[op];
  const uint32_t nchunks = a.e[op].op_chunks, flags = a.e[op].flags;
  const uint64_t chunk = a.e[op].chunk_bytes;
  const uint64_t off = (uint64_t)ci * chunk;
  const uint64_t len = (nbytes - off < chunk) ? nbytes - off : chunk;
  rsrc_t dw[kMaxBufs - 1];
  uint64_t align = a.e[op].buf[0];
#pragma unroll
  for (int k = 0; k < kMaxBufs - 1; ++k) {
    const bool used = k + 1 < (int)nbuf;
    dw[k] = window(used ? a.e[op].buf[k + 1] + off : 0, used ? len : 0);
    align |= used ? a.e[op].buf[k + 1] : 0;
  }
  if (ci == 0 && threadIdx.x == 0 && (flags & 1u)) {
    SlotDesc* d = &slots[slot].d;
#pragma unroll
    for (int k = 0; k < kMaxBufs; ++k) d->buf[k] = (k < (int)nbuf) ? a.e[op].buf[k] : 0;
    d->nbytes = nbytes;
    d->kind = (flags >> 8) & 0xFFu;
    d->dtype = (flags >> 1) & 0x7Fu;
    d->nbuf = (flags >> 16) & 0xFFu;
    d->world_id = a.e[op].world_id;
    d->world_epoch = a.e[op].world_epoch;
    d->gen = gen;
    d->nchunks = nchunks;
    d->chunk_bytes = (uint32_t)chunk;
  }
  move_any<kCopyWG, kCopyU, kMaxBufs - 1>(align, window(a.e[op].buf[0] + off, len), dw, (int)nbuf - 1, (uint32_t)len);
  retire_chunk(slots, host_flags, slot, gen, nchunks, a.e[op].target);
}

// ------------------------------------------------------------------------------------------------
// K3: sum all-reduce among logical ranks
// ------------------------------------------------------------------------------------------------
__device__ __forceinline__ float bf16_to_f32(uint32_t h) { return __uint_as_float(h << 16); }

// Round to nearest, ties to even; NaN stays a quiet NaN.
__device__ __forceinline__ uint32_t f32_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (u >> 16) | 0x40u;
  return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}

// One 16-byte vector per rank: acc = ((x0 + x1) + x2) + ...
template <bool BF16>
struct Acc;
template <>
struct Acc<false> {
  f32x4 v;
  __device__ __forceinline__ void init(u32x4 x) { v = __builtin_bit_cast(f32x4, x); }
  __device__ __forceinline__ void add(u32x4 x) { v = v + __builtin_bit_cast(f32x4, x); }
  __device__ __forceinline__ u32x4 out() const { return __builtin_bit_cast(u32x4, v); }
};
template <>
struct Acc<true> {
  float v[8];
  __device__ __forceinline__ void init(u32x4 x) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      v[2 * i] = bf16_to_f32(x[i] & 0xFFFFu);
      v[2 * i + 1] = bf16_to_f32(x[i] >> 16);
    }
  }
  __device__ __forceinline__ void add(u32x4 x) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      v[2 * i] += bf16_to_f32(x[i] & 0xFFFFu);
      v[2 * i + 1] += bf16_to_f32(x[i] >> 16);
    }
  }
  __device__ __forceinline__ u32x4 out() const {
    u32x4 r;
#pragma unroll
    for (int i = 0; i < 4; ++i) r[i] = f32_to_bf16(v[2 * i]) | (f32_to_bf16(v[2 * i + 1]) << 16);
    return r;
  }
};

// Register path, instantiated for the exact number of ranks N so that the loads of all ranks are
// issued back to back with no branch between them: every thread holds U vectors of every rank and
// folds them in, in rank order.  ALL: every rank receives the sum; otherwise only `root` does.
template <bool BF16, int N, bool ALL>
__device__ __forceinline__ void reduce_vectors(const uint64_t* buf, uint64_t off, uint32_t len, uint32_t root,
                                               uint32_t nvec) {
  constexpr int U = reduce_u(N);
  const uint32_t step = kReduceWG * U;
  rsrc_t w[N];
#pragma unroll
  for (int r = 0; r < N; ++r) w[r] = window(buf[r] + off, len);
  rsrc_t wroot = w[0];
  if (!ALL) {
#pragma unroll
    for (int r = 1; r < N; ++r)
      if ((uint32_t)r == root) wroot = w[r];
  }
  for (uint32_t i = threadIdx.x; i < nvec; i += step) {
    u32x4 x[N][U];
#pragma unroll
    for (int r = 0; r < N; ++r) {
#pragma unroll
      for (int u = 0; u < U; ++u) {
        uint32_t j = i + u * kReduceWG;
        if (j < nvec) x[r][u] = Io<u32x4>::ld(w[r], j * 16);
      }
    }
    u32x4 y[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      Acc<BF16> acc;
      acc.init(x[0][u]);
#pragma unroll
      for (int r = 1; r < N; ++r) acc.add(x[r][u]);
      y[u] = acc.out();
    }
    if (ALL) {
#pragma unroll
      for (int r = 0; r < N; ++r) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
          uint32_t j = i + u * kReduceWG;
          if (j < nvec) Io<u32x4>::st(w[r], j * 16, y[u]);
        }
      }
    } else {
#pragma unroll
      for (int u = 0; u < U; ++u) {
        uint32_t j = i + u * kReduceWG;
        if (j < nvec) Io<u32x4>::st(wroot, j * 16, y[u]);
      }
    }
  }
}

template <bool BF16, int N>
__device__ __forceinline__ void reduce_vectors_n(const uint64_t* buf, uint64_t off, uint32_t len, uint32_t wmask,
                                                 uint32_t nvec) {
  if (wmask == (1u << N) - 1) reduce_vectors<BF16, N, true>(buf, off, len, 0, nvec);
  else reduce_vectors<BF16, N, false>(buf, off, len, (uint32_t)__builtin_ctz(wmask), nvec);
}

template <bool BF16>
__device__ __forceinline__ void reduce_vectors_any(const uint64_t* buf, uint64_t off, uint32_t len, int nbuf,
                                                   uint32_t wmask, uint32_t nvec) {
  switch (nbuf) {
    case 2: reduce_vectors_n<BF16, 2>(buf, off, len, wmask, nvec); break;
    case 3: reduce_vectors_n<BF16, 3>(buf, off, len, wmask, nvec); break;
    case 4: reduce_vectors_n<BF16, 4>(buf, off, len, wmask, nvec); break;
    case 5: reduce_vectors_n<BF16, 5>(buf, off, len, wmask, nvec); break;
    case 6: reduce_vectors_n<BF16, 6>(buf, off, len, wmask, nvec); break;
    case 7: reduce_vectors_n<BF16, 7>(buf, off, len, wmask, nvec); break;
    default: reduce_vectors_n<BF16, 8>(buf, off, len, wmask, nvec); break;
  }
}

// LDS-staged path: the workgroup first lands one tile of every rank in LDS with wide loads,
// then each thread sums its column across the staged rank tiles and writes all ranks.  The
// staging decouples the (n x tile) read burst from the arithmetic and the write burst.
// `stride` = vectors per rank in the tile (the chunk's vectors, at most one per thread); the launch sizes
// the dynamic LDS to ranks x stride vectors, so small rank counts and small chunks leave room for a second
// workgroup on the CU.
template <bool BF16>
__device__ __forceinline__ void reduce_vectors_lds(const rsrc_t* w, int nbuf, uint32_t wmask, uint32_t nvec,
                                                   u32x4* tile, uint32_t stride) {
  for (uint32_t base = 0; base < nvec; base += stride) {
    const uint32_t j = base + threadIdx.x;
    const bool mine = threadIdx.x < stride && j < nvec;
#pragma unroll
    for (int r = 0; r < kMaxBufs; ++r) {
      if (r < nbuf && mine) tile[r * stride + threadIdx.x] = Io<u32x4>::ld(w[r], j * 16);
    }
    __syncthreads();
    if (mine) {
      Acc<BF16> acc;
      acc.init(tile[threadIdx.x]);
      for (int r = 1; r < nbuf; ++r) acc.add(tile[r * stride + threadIdx.x]);
      const u32x4 y = acc.out();
#pragma unroll
      for (int r = 0; r < kMaxBufs; ++r) {
        if (r < nbuf && ((wmask >> r) & 1u)) Io<u32x4>::st(w[r], j * 16, y);
      }
    }
    __syncthreads();
  }
}

// Element-wise path for tails and for buffers that are not 16-byte aligned.
template <bool BF16>
__device__ __forceinline__ void reduce_scalar(const rsrc_t* w, int nbuf, uint32_t wmask, uint32_t first,
                                              uint32_t nelem) {
  for (uint32_t i = first + threadIdx.x; i < nelem; i += kReduceWG) {
    float acc = 0.f;
    uint32_t out = 0;
#pragma unroll
    for (int r = 0; r < kMaxBufs; ++r) {
      if (r < nbuf) {
        const float x = BF16 ? bf16_to_f32(Io<uint16_t>::ld(w[r], i * 2)) : __uint_as_float(Io<uint32_t>::ld(w[r], i * 4));
        acc = r == 0 ? x : acc + x;
      }
    }
    out = BF16 ? f32_to_bf16(acc) : __float_as_uint(acc);
#pragma unroll
    for (int r = 0; r < kMaxBufs; ++r) {
      if (r < nbuf && ((wmask >> r) & 1u)) {
        if (BF16) Io<uint16_t>::st(w[r], i * 2, (uint16_t)out);
        else Io<uint32_t>::st(w[r], i * 4, out);
      }
    }
  }
}

template <bool LDS, int CAP>
__global__ __launch_bounds__(kReduceWG) void mw_k_reduce(const CollArgs<CAP> a, RingSlot* __restrict__ slots,
                                                          uint32_t* __restrict__ host_flags) {
  extern __shared__ u32x4 tile[];  // LDS-staged variant: ranks x stride vectors, sized by the launch
  const uint32_t c = chunk_of_workgroup(blockIdx.x, gridDim.x, a.rotate);
  const int op = find_op(a.first_chunk, (int)a.n, c);
  const uint64_t nbytes = a.e[op].nbytes;
  const uint32_t slot = a.e[op].slot, gen = a.e[op].gen, nbuf = a.e[op].nbuf;
  const uint32_t ci = c - a.first_chunk[op];
  const uint32_t nchunks = a.e[op].op_chunks, flags = a.e[op].flags;
  const uint32_t wmask = flags >> 24;  // ranks whose buffer receives the sum (all of them, or the root only)
  const uint32_t dtype = (flags >> 1) & 0x7Fu;
  const uint64_t chunk = a.e[op].chunk_bytes;
  const uint64_t off = (uint64_t)ci * chunk;
  const uint64_t len = (nbytes - off < chunk) ? nbytes - off : chunk;
  const uint64_t* buf = a.e[op].buf;  // unused entries are zero
  uint64_t align = 0;
#pragma unroll
  for (int k = 0; k < kMaxBufs; ++k) align |= buf[k];
  if (ci == 0 && threadIdx.x == 0 && (flags & 1u)) {
    SlotDesc* d = &slots[slot].d;
#pragma unroll
    for (int k = 0; k < kMaxBufs; ++k) d->buf[k] = buf[k];
    d->nbytes = nbytes;
    d->kind = (flags >> 8) & 0xFFu;
    d->dtype = dtype;
    d->nbuf = nbuf;
    d->world_id = a.e[op].world_id;
    d->world_epoch = a.e[op].world_epoch;
    d->gen = gen;
    d->nchunks = nchunks;
    d->chunk_bytes = (uint32_t)chunk;
  }
  rsrc_t w[kMaxBufs];
#pragma unroll
  for (int k = 0; k < kMaxBufs; ++k) w[k] = window(k < (int)nbuf ? buf[k] + off : 0, k < (int)nbuf ? len : 0);
  const bool bf16 = dtype == MW_BF16;
  const uint32_t isz = bf16 ? 2 : 4;
  const uint32_t nelem = (uint32_t)len / isz;
  uint32_t nvec = 0;
  if ((align & 15) == 0) {
    nvec = (uint32_t)len >> 4;
    if (LDS) {
      const uint32_t stride = lds_stride((uint32_t)chunk);
      if (bf16) reduce_vectors_lds<true>(w, (int)nbuf, wmask, nvec, tile, stride);
      else reduce_vectors_lds<false>(w, (int)nbuf, wmask, nvec, tile, stride);
    } else {
      if (bf16) reduce_vectors_any<true>(buf, off, (uint32_t)len, (int)nbuf, wmask, nvec);
      else reduce_vectors_any<false>(buf, off, (uint32_t)len, (int)nbuf, wmask, nvec);
    }
  }
  const uint32_t first = nvec * (16 / isz);
  if (first < nelem) {
    if (bf16) reduce_scalar<true>(w, (int)nbuf, wmask, first, nelem);
    else reduce_scalar<false>(w, (int)nbuf, wmask, first, nelem);
  }
  retire_chunk(slots, host_flags, slot, gen, nchunks, a.e[op].target);
}

// ------------------------------------------------------------------------------------------------
// The mailbox: a resident kernel that serves descriptors the host writes into device memory, so that a small
// operation does not pay a launch (protocol and its reasons: mw_mailbox.hpp).  Workgroup 0 is the leader (one
// thread), workgroups 1..W are the workers.  Every loop here ends by itself: the leader when the host asks, when
// nothing has come for `idle_ticks`, or at `life_ticks` at the latest; a worker when it has served everything up to
// the leader's closing word, or -- a safety net that no correct run needs -- at its own time limit.
// ------------------------------------------------------------------------------------------------
// (the builtin returns a signed int: widen through uint32_t, or a low word with bit 31 set smears into the high word)
__device__ __forceinline__ uint32_t uniform32(uint32_t v) { return (uint32_t)__builtin_amdgcn_readfirstlane(v); }
__device__ __forceinline__ uint64_t uniform64(uint64_t v) {
  return ((uint64_t)uniform32((uint32_t)(v >> 32)) << 32) | (uint64_t)uniform32((uint32_t)v);
}

// One chunk of one descriptor, by the whole workgroup: what one workgroup of mw_k_copy / mw_k_bcast /
// mw_k_reduce<false> does for one chunk of one entry, ending with the same completion protocol.
__device__ __forceinline__ void mailbox_chunk(const mb::Desc* d, uint32_t ci, RingSlot* slots, uint32_t* host_flags) {
  const uint64_t nbytes = uniform64(d->nbytes);
  const uint32_t slot = uniform32(d->slot), gen = uniform32(d->gen), nbuf = uniform32(d->nbuf), flags = uniform32(d->flags);
  const uint32_t kind = uniform32(d->kind), nchunks = uniform32(d->op_chunks), target = uniform32(d->target);
  const uint64_t chunk = uniform32(d->chunk_bytes);
  uint64_t buf[kMaxBufs];
#pragma unroll
  for (int k = 0; k < kMaxBufs; ++k) buf[k] = uniform64(d->buf[k]);
  const uint64_t off = (uint64_t)ci * chunk;
  const uint64_t len = (nbytes - off < chunk) ? nbytes - off : chunk;
  if (ci == 0 && threadIdx.x == 0 && (flags & 1u)) {  // journal the descriptor into the world's ring
    SlotDesc* j = &slots[slot].d;
#pragma unroll
    for (int k = 0; k < kMaxBufs; ++k) j->buf[k] = buf[k];
    j->nbytes = nbytes;
    j->kind = (flags >> 8) & 0xFFu;
    j->dtype = (flags >> 1) & 0x7Fu;
    j->nbuf = (flags >> 16) & 0xFFu;
    j->world_id = d->world_id;
    j->world_epoch = d->world_epoch;
    j->gen = gen;
    j->nchunks = nchunks;
    j->chunk_bytes = (uint32_t)chunk;
  }
  if (kind == mb::kKindCopy) {
    const rsrc_t dw[1] = {window(buf[1] + off, len)};
    move_any<kCopyWG, kCopyU, 1>(buf[0] | buf[1], window(buf[0] + off, len), dw, 1, (uint32_t)len);
  } else if (kind == mb::kKindBcast) {
    rsrc_t dw[kMaxBufs - 1];
    uint64_t align = buf[0];
#pragma unroll
    for (int k = 0; k < kMaxBufs - 1; ++k) {
      const bool used = k + 1 < (int)nbuf;
      dw[k] = window(used ? buf[k + 1] + off : 0, used ? len : 0);
      align |= used ? buf[k + 1] : 0;
    }
    move_any<kCopyWG, kCopyU, kMaxBufs - 1>(align, window(buf[0] + off, len), dw, (int)nbuf - 1, (uint32_t)len);
  } else {
    const uint32_t wmask = flags >> 24;
    const bool bf16 = ((flags >> 1) & 0x7Fu) == MW_BF16;
    const uint32_t isz = bf16 ? 2 : 4;
    uint64_t align = 0;
#pragma unroll
    for (int k = 0; k < kMaxBufs; ++k) align |= buf[k];
    rsrc_t w[kMaxBufs];
#pragma unroll
    for (int k = 0; k < kMaxBufs; ++k) w[k] = window(k < (int)nbuf ? buf[k] + off : 0, k < (int)nbuf ? len : 0);
    const uint32_t nelem = (uint32_t)len / isz;
    uint32_t nvec = 0;
    if ((align & 15) == 0) {
      nvec = (uint32_t)len >> 4;
      if (bf16) reduce_vectors_any<true>(buf, off, (uint32_t)len, (int)nbuf, wmask, nvec);
      else reduce_vectors_any<false>(buf, off, (uint32_t)len, (int)nbuf, wmask, nvec);
    }
    const uint32_t first = nvec * (16 / isz);
    if (first < nelem) {
      if (bf16) reduce_scalar<true>(w, (int)nbuf, wmask, first, nelem);
      else reduce_scalar<false>(w, (int)nbuf, wmask, first, nelem);
    }
  }
  retire_chunk(slots, host_flags, slot, gen, nchunks, target);
}

constexpr int kMailboxBatch = 64;  // descriptors a worker fetches at a time (16 lanes each, one round trip for all);
                                  // one wavefront then finds this worker's chunks among them, a lane per descriptor
static_assert(kMailboxBatch == 64 && kMailboxBatch * 16 <= kCopyWG, "one lane of the first wavefront per descriptor");

__global__ __launch_bounds__(kCopyWG) void mw_k_mailbox(const mb::HostWritten* __restrict__ hw, mb::LeaderWritten* __restrict__ lw,
                                                        uint64_t* __restrict__ closed_host, uint32_t epoch, uint32_t first,
                                                        uint32_t n_workers, uint64_t idle_ticks, uint64_t life_ticks,
                                                        RingSlot* __restrict__ slots, uint32_t* __restrict__ host_flags) {
  if (blockIdx.x == 0) {  // ---- the leader: the only reader of the doorbell, the only one who admits and closes
    if (threadIdx.x != 0) return;
    uint32_t go = first - 1;
    const uint64_t t0 = wall_clock64();
    uint64_t t_last = t0;
    for (;;) {
      // doorbell and stop word in one 8-byte load, past every cache: the host writes them through the PCIe aperture
      const uint64_t w = __hip_atomic_load(reinterpret_cast<const uint64_t*>(&hw->tail), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
      const uint32_t tail = (uint32_t)w, stop = (uint32_t)(w >> 32);
      const uint64_t now = wall_clock64();
      if (tail != go && mb::before(go, tail) && tail - first < mb::kEpochTickets) {
        go = tail;
        __hip_atomic_store(&lw->admit, mb::make_admit(go, 0), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        t_last = now;
        continue;
      }
      if (stop == epoch || now - t_last > idle_ticks || now - t0 > life_ticks) {
        __hip_atomic_store(&lw->admit, mb::make_admit(go, epoch), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __builtin_amdgcn_s_waitcnt(0);  // the workers' closing word is out before the host hears of it
        __hip_atomic_store(closed_host, mb::make_closed(epoch, go), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
        return;
      }
    }
  }
  // ---- a worker
  __shared__ uint64_t s_admit;
  __shared__ uint64_t s_mine;                 // which descriptors of the batch hold chunks of mine
  __shared__ uint32_t s_c0[kMailboxBatch];    // ... and my first chunk of each
  __shared__ __align__(16) mb::Desc s_desc[kMailboxBatch];
  const uint32_t me = blockIdx.x - 1;
  uint32_t next = first;
  const uint64_t t0 = wall_clock64();
  const uint64_t my_life = life_ticks + life_ticks / 2 + 50000000ull;  // the leader's life and half a second more
  for (;;) {
    if (threadIdx.x == 0) s_admit = __hip_atomic_load(&lw->admit, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __syncthreads();
    const uint64_t a = s_admit;
    __syncthreads();  // everybody has read it before thread 0 overwrites it in the next round
    const uint32_t go = (uint32_t)a;
    const bool closing = mb::closing_epoch(a) == epoch;
    while (mb::before(next - 1, go)) {
      const uint32_t batch = go - next + 1 < (uint32_t)kMailboxBatch ? go - next + 1 : (uint32_t)kMailboxBatch;
      if (threadIdx.x < batch * 16) {  // 16 lanes x 8 bytes per descriptor, past every cache (host-written memory)
        const uint32_t b = threadIdx.x / 16, k = threadIdx.x % 16;
        const uint64_t* src = reinterpret_cast<const uint64_t*>(&hw->q[(next + b) % mb::kQueueDepth]) + k;
        reinterpret_cast<uint64_t*>(&s_desc[b])[k] = __hip_atomic_load(src, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
      }
      __syncthreads();
      if (threadIdx.x < 64) {  // the first wavefront: lane b looks at descriptor b
        bool mine = false;
        if (threadIdx.x < batch) {
          // my chunks of it: owner(start, c, W) == me  <=>  c = (me - start) mod W, then every W-th
          const uint32_t c0 = (me + n_workers - s_desc[threadIdx.x].start % n_workers) % n_workers;
          s_c0[threadIdx.x] = c0;
          mine = c0 < s_desc[threadIdx.x].n_chunks;
        }
        const uint64_t m = __ballot(mine);
        if (threadIdx.x == 0) s_mine = m;
      }
      __syncthreads();
      uint64_t mine = uniform64(s_mine);
      while (mine) {
        const uint32_t b = (uint32_t)__builtin_ctzll(mine);
        mine &= mine - 1;
        const uint32_t n_chunks = uniform32(s_desc[b].n_chunks);
        for (uint32_t c = uniform32(s_c0[b]); c < n_chunks; c += n_workers) mailbox_chunk(&s_desc[b], c, slots, host_flags);
      }
      __syncthreads();  // the batch is overwritten next
      next += batch;
    }
    if (closing && next - 1 == go) return;
    if (wall_clock64() - t0 > my_life) return;  // safety net
  }
}

// ------------------------------------------------------------------------------------------------
// K5: world marker
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(64) void mw_k_mark(RingHeader* __restrict__ dst, const RingHeader h) {
  const uint32_t* w = reinterpret_cast<const uint32_t*>(&h);
  reinterpret_cast<uint32_t*>(dst)[threadIdx.x] = w[threadIdx.x];
}

// Re-arm the arrival counters of the first n static slots (the static array keeps the last call's contents).
__global__ __launch_bounds__(kStaticOps) void mw_k_clear(RingSlot* __restrict__ slots, uint32_t n) {
  if (threadIdx.x < n) __hip_atomic_store(&slots[threadIdx.x].s.arrived, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// ------------------------------------------------------------------------------------------------
// host side of the backend
// ------------------------------------------------------------------------------------------------
inline uint32_t floor_log2(uint64_t v) { return 63u - (uint32_t)__builtin_clzll(v | 1); }

class HipDevice : public Device {
 public:
  int init(int hip_device, const DeviceConfig& cfg) override {
    int rc = init_impl(hip_device, cfg);
    if (rc != MW_OK) release();  // nothing half-built survives a failed init
    return rc;
  }

  void shutdown() override {
    if (!ready_) return;
    (void)hipSetDevice(dev_);
    if (mb_hw_) mb_.stop();        // the resident kernel closes within microseconds of the stop word
    (void)hipDeviceSynchronize();  // operations behind a busy caller stream run on that stream
    release();
  }

  void set_config(const DeviceConfig& cfg) override {
    cfg_.chunk_bytes = cfg.chunk_bytes;
    cfg_.reduce_lds = cfg.reduce_lds;
    if (cfg_.mailbox && !cfg.mailbox) mb_.stop();
    cfg_.mailbox = cfg.mailbox;
    cfg_.mailbox_idle_us = std::min(50000u, std::max(10u, cfg.mailbox_idle_us));  // (takes effect with the next kernel)
  }

  int launch(const LaunchOp* ops, const OpDeps* deps, int n, uint8_t* launched) override {
    launched_ = launched;
    cur_slots_ = slots_;
    cur_flags_ = flags_dev_;
    counts_ = arena_counts_.data();
    host_flags_ok_ = true;
    if (chk(hipSetDevice(dev_))) return MW_EHIP;
    // Which caller streams still have work pending?  One query per distinct stream.  A stream with nothing
    // pending imposes no ordering: no event, no barrier packet.
    dep_streams_.clear();
    dep_busy_.clear();
    group_of_.assign((size_t)n, -1);
    bool any_dependent = false;
    for (int i = 0; i < n; ++i) {
      for (int k = 0; k < deps[i].n; ++k) {
        void* st = deps[i].stream[k];
        size_t j = 0;
        while (j < dep_streams_.size() && dep_streams_[j] != st) ++j;
        if (j == dep_streams_.size()) {
          hipError_t q = hipStreamQuery(reinterpret_cast<hipStream_t>(st));
          if (q != hipSuccess && q != hipErrorNotReady) {
            chk(q);
            return MW_EHIP;
          }
          dep_streams_.push_back(st);
          dep_busy_.push_back(q == hipErrorNotReady);
        }
        if (dep_busy_[j] && group_of_[(size_t)i] < 0) group_of_[(size_t)i] = (int)j;  // its first busy stream
      }
      any_dependent |= group_of_[(size_t)i] >= 0;
    }
    // Operations whose buffers are final go to the library's own lanes and wait for nothing.
    int rc = launch_group(ops, n, -1);
    if (rc != MW_OK || !any_dependent) return rc;
    // An operation behind a busy caller stream is enqueued ON that stream (behind its other busy streams
    // too, through events), so it is ordered by the stream itself and never stands in a lane in front of
    // operations of other worlds: a producer that is slow, or stuck, holds up only the operations that named
    // its stream (Sec. 3.2: a pending operation in one world must not hold up another).
    for (size_t g = 0; g < dep_streams_.size() && rc == MW_OK; ++g) {
      if (!dep_busy_[g]) continue;
      bool mine = false;
      for (int i = 0; i < n; ++i) mine |= group_of_[(size_t)i] == (int)g;
      if (!mine) continue;
      hipStream_t target = reinterpret_cast<hipStream_t>(dep_streams_[g]);
      waited_.clear();
      for (int i = 0; i < n; ++i) {
        if (group_of_[(size_t)i] != (int)g) continue;
        for (int k = 0; k < deps[i].n; ++k) {
          void* st = deps[i].stream[k];
          if (st == dep_streams_[g]) continue;
          size_t j = 0;
          while (dep_streams_[j] != st) ++j;
          if (!dep_busy_[j]) continue;
          bool seen = false;
          for (void* t : waited_) seen |= t == st;
          if (seen) continue;
          waited_.push_back(st);
          hipEvent_t ev = dep_events_[dep_cursor_];
          dep_cursor_ = (dep_cursor_ + 1) % kDepEvents;
          if (chk(hipEventRecord(ev, reinterpret_cast<hipStream_t>(st)))) return MW_EHIP;
          if (chk(hipStreamWaitEvent(target, ev, 0))) return MW_EHIP;
        }
      }
      for (uint32_t k = 0; k < kNumKinds; ++k) data_[k] = target;
      rc = launch_group(ops, n, (int)g);
    }
    return rc;
  }

  int launch_static(const LaunchOp* ops, int n, void* stream) override {
    if (n < 0 || n > kStaticOps) return fail_inval();
    if (chk(hipSetDevice(dev_))) return MW_EHIP;
    if (!static_base_) return fail_inval();
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    RingSlot* sslots = reinterpret_cast<RingSlot*>(static_base_);
    uint32_t* sflags = reinterpret_cast<uint32_t*>(static_base_ + (size_t)kStaticOps * sizeof(RingSlot));
    if (n == 0) return MW_OK;
    // The array keeps the previous call's contents: the arrival counters must start at zero.  A fill kernel,
    // not a memset node, so that the call may be recorded into a graph.
    hipLaunchKernelGGL(mw_k_clear, dim3(1), dim3(kStaticOps), 0, st, sslots, (uint32_t)n);
    if (chk(hipGetLastError())) return MW_EHIP;
    static_launched_.assign((size_t)n, 0);  // capacity reserved at init: no allocation
    launched_ = static_launched_.data();
    cur_slots_ = sslots;
    cur_flags_ = sflags;
    std::memset(static_counts_, 0, sizeof(static_counts_));  // the fill kernel above zeroes the device counters
    counts_ = static_counts_;
    host_flags_ok_ = false;
    group_of_.assign((size_t)n, -1);
    for (uint32_t k = 0; k < kNumKinds; ++k) data_[k] = st;
    return run_group(ops, n, -1);
  }

  int mark_world(uint32_t ring_index, const RingHeader& h) override {
    if (chk(hipSetDevice(dev_))) return MW_EHIP;
    hipLaunchKernelGGL(mw_k_mark, dim3(1), dim3(64), 0, ctl_, headers_ + ring_index, h);
    return chk(hipGetLastError()) ? MW_EHIP : MW_OK;
  }

  uint32_t flag(uint32_t slot) override { return __atomic_load_n(&flags_host_[slot], __ATOMIC_ACQUIRE); }

  int read_ring(uint32_t ring_index, uint32_t first_slot, uint32_t depth, void* out) override {
    int rc = sync();
    if (rc != MW_OK) return rc;
    if (chk(hipMemcpy(out, headers_ + ring_index, sizeof(RingHeader), hipMemcpyDeviceToHost))) return MW_EHIP;
    if (chk(hipMemcpy(reinterpret_cast<char*>(out) + sizeof(RingHeader), slots_ + first_slot,
                      (size_t)depth * sizeof(RingSlot), hipMemcpyDeviceToHost)))
      return MW_EHIP;
    return MW_OK;
  }

  int sync() override {
    if (chk(hipSetDevice(dev_))) return MW_EHIP;
    if (mb_hw_) {  // what is queued for the resident kernel is served, then it closes
      if (mb_.attend() != 0) return MW_EHIP;
      mb_.stop();
    }
    if (chk(hipDeviceSynchronize())) return MW_EHIP;  // the lanes, and the caller streams operations were put on
    return MW_OK;
  }

  int last_hip_error() override { return last_err_; }

  int profile_enable(int on) override {
    profiling_ = on != 0;
    return MW_OK;
  }

  int profile_read(int kind, uint64_t* launches, double* ms, uint64_t* bytes) override {
    if (chk(hipSetDevice(dev_))) return MW_EHIP;
    size_t k = 0;
    for (size_t i = 0; i < prof_.size(); ++i) {
      ProfRec& r = prof_[i];
      if ((int)r.kind != kind) {
        prof_[k++] = r;
        continue;
      }
      float t = 0.f;
      if (chk(hipEventSynchronize(r.stop)) || chk(hipEventElapsedTime(&t, r.start, r.stop))) return MW_EHIP;
      acc_[kind].launches += 1;
      acc_[kind].ms += t;
      acc_[kind].bytes += r.bytes;
      prof_free_.push_back(r.start);
      prof_free_.push_back(r.stop);
    }
    prof_.resize(k);
    *launches = acc_[kind].launches;
    *ms = acc_[kind].ms;
    *bytes = acc_[kind].bytes;
    acc_[kind] = ProfAcc{};
    return MW_OK;
  }

 private:
  static constexpr int kDepEvents = 256;

  struct ProfRec {
    uint32_t kind;
    hipEvent_t start, stop;
    uint64_t bytes;
  };
  struct ProfAcc {
    uint64_t launches = 0;
    double ms = 0;
    uint64_t bytes = 0;
  };

  int init_impl(int hip_device, const DeviceConfig& cfg) {
    cfg_ = cfg;
    dev_ = hip_device;
    int count = 0;
    if (chk(hipGetDeviceCount(&count)) || hip_device < 0 || hip_device >= count) return MW_EHIP;
    if (chk(hipSetDevice(dev_))) return MW_EHIP;
    const size_t hdr_bytes = (size_t)cfg.total_rings * sizeof(RingHeader);
    const size_t slot_bytes = (size_t)cfg.total_slots * sizeof(RingSlot);
    if (chk(hipMalloc(&arena_, hdr_bytes + slot_bytes))) return MW_EHIP;
    if (chk(hipMemset(arena_, 0, hdr_bytes + slot_bytes))) return MW_EHIP;
    headers_ = reinterpret_cast<RingHeader*>(arena_);
    slots_ = reinterpret_cast<RingSlot*>(reinterpret_cast<char*>(arena_) + hdr_bytes);
    if (chk(hipHostMalloc(&flags_host_, (size_t)cfg.total_slots * sizeof(uint32_t),
                          hipHostMallocMapped | hipHostMallocCoherent)))
      return MW_EHIP;
    std::memset(flags_host_, 0, (size_t)cfg.total_slots * sizeof(uint32_t));
    if (chk(hipHostGetDevicePointer(reinterpret_cast<void**>(&flags_dev_), flags_host_, 0))) return MW_EHIP;
    for (auto& kind : lanes_)
      for (auto& st : kind)
        if (chk(hipStreamCreateWithFlags(&st, hipStreamNonBlocking))) return MW_EHIP;
    if (chk(hipStreamCreateWithFlags(&ctl_, hipStreamNonBlocking))) return MW_EHIP;
    dep_events_.assign(kDepEvents, nullptr);
    for (auto& e : dep_events_)
      if (chk(hipEventCreateWithFlags(&e, hipEventDisableTiming))) return MW_EHIP;
    // the LDS-staged reduce kernel takes up to 8 ranks x 16 KiB of dynamic LDS, above the 64 KiB default limit
    const void* lds_kernels[3] = {reinterpret_cast<const void*>(&mw_k_reduce<true, kCollCap[0]>),
                                  reinterpret_cast<const void*>(&mw_k_reduce<true, kCollCap[1]>),
                                  reinterpret_cast<const void*>(&mw_k_reduce<true, kCollCap[2]>)};
    for (const void* f : lds_kernels)
      if (chk(hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, kMaxBufs * kReduceWG * 16))) return MW_EHIP;
    arena_counts_.assign(cfg.total_slots, 0);  // the arena was zeroed above
    // The static scratch of the entry point that allocates nothing: each GPU holds its own copy of the array at
    // its own address, looked up once per device with that device current.
    if (hip_device < kMaxHipDevices && g_scratch_ptr[hip_device]) {
      static_base_ = g_scratch_ptr[hip_device];
    } else {
      unsigned char* ptr = nullptr;
      if (chk(hipGetSymbolAddress(reinterpret_cast<void**>(&ptr), HIP_SYMBOL(scratch))) || !ptr) return MW_EHIP;
      if (hip_device < kMaxHipDevices) g_scratch_ptr[hip_device] = ptr;
      static_base_ = ptr;
    }
    // The mailbox: queue (process-lifetime, fine-grained), leader's word, closing word, stream.  A GPU that cannot
    // give host-writable device memory simply has no mailbox: every flush is launched.
    // One workgroup of the resident kernel per compute unit, the leader included: measured, a second 1024-thread
    // workgroup of it is never resident beside the first, and a worker that is not resident serves its chunks only
    // when the others have left (with 319 workers a tensor-parallel iteration took 107 us instead of 7.4).
    int n_cu = 0;
    if (hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, hip_device) != hipSuccess || n_cu < 2) {
      (void)hipGetLastError();
      n_cu = 2;
    }
    cfg_.mailbox_workers = std::min((uint32_t)n_cu - 1u, std::max(1u, cfg.mailbox_workers));
    cfg_.mailbox_idle_us = std::min(50000u, std::max(10u, cfg.mailbox_idle_us));
    mb_.reset();
    int large_bar = 0;  // the host writes the queue with plain stores: the whole device memory must be in its address space
    if (hipDeviceGetAttribute(&large_bar, hipDeviceAttributeIsLargeBar, hip_device) != hipSuccess) {
      (void)hipGetLastError();
      large_bar = 0;
    }
    if (hip_device < kMaxHipDevices && large_bar) {
      if (!g_mailbox_mem[hip_device]) {
        void* p = nullptr;
        if (hipExtMallocWithFlags(&p, sizeof(mb::HostWritten), hipDeviceMallocFinegrained) == hipSuccess) g_mailbox_mem[hip_device] = static_cast<mb::HostWritten*>(p);
        else (void)hipGetLastError();
      }
      mb_hw_ = g_mailbox_mem[hip_device];
    }
    if (mb_hw_) {
      if (chk(hipMemset(mb_hw_, 0, 128))) return MW_EHIP;  // doorbell and stop word
      // Do the host's stores arrive?  Write a pattern the way descriptors are written, read it back with a copy.
      uint32_t probe[4] = {0x6d61696cu, 0x626f7821u, (uint32_t)hip_device, 0x00c0ffeeu}, back[4] = {};
      _mm_stream_si128(reinterpret_cast<__m128i*>(&mb_hw_->pad[2]), _mm_loadu_si128(reinterpret_cast<const __m128i*>(probe)));
      _mm_sfence();
      if (chk(hipMemcpy(back, &mb_hw_->pad[2], sizeof(back), hipMemcpyDeviceToHost))) return MW_EHIP;
      if (std::memcmp(probe, back, sizeof(probe)) != 0) mb_hw_ = nullptr;  // no mailbox on this machine: every flush is launched
    }
    if (mb_hw_) {
      if (chk(hipMalloc(reinterpret_cast<void**>(&mb_lw_), sizeof(mb::LeaderWritten))) || chk(hipMemset(mb_lw_, 0, sizeof(mb::LeaderWritten)))) return MW_EHIP;
      if (chk(hipHostMalloc(reinterpret_cast<void**>(&mb_closed_), 64, hipHostMallocMapped | hipHostMallocCoherent))) return MW_EHIP;
      *mb_closed_ = 0;
      if (chk(hipHostGetDevicePointer(reinterpret_cast<void**>(&mb_closed_dev_), mb_closed_, 0))) return MW_EHIP;
      if (chk(hipStreamCreateWithFlags(&mb_stream_, hipStreamNonBlocking))) return MW_EHIP;
    }
    mb_descs_.reserve(512);
    // Host tables sized once, so that launching never grows them (the no-allocation entry point relies on it).
    ents_.reserve(512);
    one_.reserve(64);
    chunks_.reserve(512);
    op_chunks_.reserve(512);
    chunk_bytes_.reserve(512);
    targets_.reserve(512);
    first_chunk_.reserve(512);
    group_of_.reserve(4096);
    static_launched_.reserve(kStaticOps);
    if (chk(hipDeviceSynchronize())) return MW_EHIP;
    ready_ = true;
    return MW_OK;
  }

  // Free whatever exists (also after a partial init).
  void release() {
    for (auto& e : dep_events_)
      if (e) (void)hipEventDestroy(e);
    dep_events_.clear();
    for (auto& r : prof_) {
      (void)hipEventDestroy(r.start);
      (void)hipEventDestroy(r.stop);
    }
    prof_.clear();
    for (auto& e : prof_free_) (void)hipEventDestroy(e);
    prof_free_.clear();
    for (auto& kind : lanes_)
      for (auto& st : kind) {
        if (st) (void)hipStreamDestroy(st);
        st = nullptr;
      }
    if (ctl_) (void)hipStreamDestroy(ctl_);
    ctl_ = nullptr;
    if (mb_stream_) (void)hipStreamDestroy(mb_stream_);
    mb_stream_ = nullptr;
    if (mb_lw_) (void)hipFree(mb_lw_);
    mb_lw_ = nullptr;
    if (mb_closed_) (void)hipHostFree(mb_closed_);
    mb_closed_ = nullptr;
    mb_hw_ = nullptr;  // the queue itself stays with the process
    if (arena_) (void)hipFree(arena_);
    arena_ = nullptr;
    if (flags_host_) (void)hipHostFree(flags_host_);
    flags_host_ = nullptr;
    ready_ = false;
  }

  bool chk(hipError_t e) {
    if (e == hipSuccess) return false;
    last_err_ = (int)e;
    return true;
  }

  hipEvent_t prof_event() {
    if (!prof_free_.empty()) {
      hipEvent_t e = prof_free_.back();
      prof_free_.pop_back();
      return e;
    }
    hipEvent_t e = nullptr;
    chk(hipEventCreate(&e));
    return e;
  }

  // Chunk size of an entry with `nbuf` buffers in a launch of `total_bytes`: enough workgroups to fill
  // 256 CUs several times over, chunks large enough to amortise the per-chunk completion protocol.
  // With the workgroup -> chunk rotation (chunk_of_workgroup) the kernels peak where one workgroup reads about
  // 64 KiB in one burst (TB/s of algorithmic traffic, 8 worlds, kernel time, by chunk):
  //   copy 8 x 512 MiB        32 KiB 5.37, 48 KiB 5.87, 64 KiB 6.49, 80 KiB 6.12, 96 KiB 6.03, 128 KiB 6.32, 256 KiB 6.20
  //   broadcast, 4 ranks      32 KiB 5.61, 48 KiB 5.78, 64 KiB 6.25, 80 KiB 6.06, 96 KiB 5.83, 128 KiB 6.10
  //   broadcast, 64 KiB / 128 KiB:   2 ranks 6.44 / 6.33   3 ranks 6.40 / 6.21   5 ranks 6.10 / 5.99   8 ranks 5.91 / 5.80
  // All-reduce (not rotated) peaks where a workgroup's chunks of all ranks together come to 40-64 KiB, whatever the
  // number of ranks (by chunk per rank):
  //   2 ranks 3.1 (8 KiB) 5.3 (16) 6.2 (24) 6.1 (32)     3 ranks 4.4 (8) 6.0 (16) 5.9 (32)
  //   4 ranks 5.4 (8) 6.2 (12) 5.9 (16) 5.5 (32)          5 ranks 6.1 (8) 6.0 (12) 5.7 (16)
  //   6 ranks 6.5 (8) 5.6 (16)    7 ranks 6.4 (8) 5.3 (16)    8 ranks 5.1 (4) 5.9 (8) 5.1 (16)
  // A reduce to one root writes one buffer only and peaks where the ranks' chunks come to about 96 KiB:
  //   2 ranks 5.55 (24 KiB) 6.25 (32) 6.37 (48) 6.32 (64)    3 ranks 6.25 (24 KiB) 6.47 (32) 6.24 (48)
  //   4 ranks 5.59 (16 KiB) 6.43 (24) 6.17 (32)               5 ranks 6.05 (16 KiB) 6.31 (24) 6.06 (32)
  //   6 ranks 5.69 (12 KiB) 6.21 (16) 6.21 (24) 5.92 (32)     8 ranks 5.19 (8 KiB) 6.17 (12) 5.68 (16) 6.02 (24)
  uint32_t pick_chunk_bytes(uint32_t kind, uint64_t total_bytes, uint32_t nbuf, bool all_ranks_written) const {
    if (cfg_.chunk_bytes) return cfg_.chunk_bytes;
    // Smaller launches take smaller chunks, down to where the launch still has ~512 (copies, fan-outs) or
    // ~256 (reduce) workgroups.  Kernel time by chunk size, 8 equal messages per launch:
    //   copy, 32 MiB of payload      16 KiB 18.6 us, 32 KiB 16.8, 64 KiB 14.9, 128 KiB 15.0
    //   copy, 8 MiB                  16 KiB  7.2 us, 32 KiB  7.1, 64 KiB  7.4, 128 KiB  8.4
    //   all-reduce, 2 x 16 MiB       8 KiB 22.9 us, 16 KiB 17.6, 32 KiB 17.7
    //   all-reduce, 2 x 2 MiB        8 KiB  7.7 us, 16 KiB  8.3, 32 KiB  9.1
    const uint64_t groups = kind == kReduce ? 256 : 512;
    const uint32_t fill = 1u << std::min(30u, floor_log2(total_bytes / groups + 1));
    // Copies and fan-outs: never below 32 KiB, so that the small messages of latency-bound traffic are one chunk
    // each and complete without the arrival counter.
    if (kind != kReduce) return std::min(64u << 10, std::max(32u << 10, fill));
    static const uint32_t all_kib[kMaxBufs + 1] = {32, 32, 32, 16, 12, 8, 8, 8, 8};
    static const uint32_t root_kib[kMaxBufs + 1] = {48, 48, 48, 32, 24, 24, 16, 16, 12};
    const uint32_t best = (all_ranks_written ? all_kib : root_kib)[std::min<uint32_t>(nbuf, kMaxBufs)] << 10;
    return std::min(best, std::max(std::min(best, 8u << 10), fill));
  }

  struct Ent {  // one kernel entry of an operation
    uint64_t buf[kMaxBufs];
    uint64_t nbytes;
    uint32_t nbuf, dtype, slot, gen, world_id, world_epoch, flags, group;
  };

  static Kind kernel_of(uint32_t op_kind) {
    switch (op_kind) {
      case opCopy: case opGather: case opScatter: return kCopy;
      case opBcast: case opAllGather: return kBcast;
      default: return kReduce;
    }
  }

  void push_ent(const LaunchOp& o, uint32_t group, const uint64_t* bufs, uint32_t nbuf, uint32_t wmask) {
    Ent e{};
    for (uint32_t k = 0; k < nbuf; ++k) e.buf[k] = bufs[k];
    e.nbytes = o.nbytes;
    e.nbuf = nbuf;
    e.dtype = o.dtype;
    e.slot = o.slot;
    e.gen = o.gen;
    e.world_id = o.world_id;
    e.world_epoch = o.world_epoch;
    e.group = group;
    const bool first = ents_.empty() || ents_.back().group != group;
    e.flags = (first ? 1u : 0u) | ((o.dtype & 0x7Fu) << 1) | (o.kind << 8) | (o.nbuf << 16) | (wmask << 24);
    ents_.push_back(e);
  }

  // The kernel entries of one operation (see LaunchOp for the buffer layouts).
  void expand(const LaunchOp& o, uint32_t group) {
    const uint32_t n = o.nbuf;
    uint64_t b[kMaxBufs];
    switch (o.kind) {
      case opCopy:
        push_ent(o, group, o.buf, 2, 0);
        break;
      case opBcast:
        push_ent(o, group, o.buf, n, 0);
        break;
      case opAllReduce:
        push_ent(o, group, o.buf, n, (1u << n) - 1);
        break;
      case opReduce:
        push_ent(o, group, o.buf, n, 1u << o.root);
        break;
      case opGather:  // rank q's tensor -> slice q of the root's destination
        for (uint32_t q = 0; q < n; ++q) {
          b[0] = o.buf[q];
          b[1] = o.buf[8] + q * o.nbytes;
          if (b[0] != b[1]) push_ent(o, group, b, 2, 0);
        }
        break;
      case opScatter:  // slice r of the root's source -> rank r's tensor
        for (uint32_t r = 0; r < n; ++r) {
          b[0] = o.buf[0] + r * o.nbytes;
          b[1] = o.buf[8 + r];
          if (b[0] != b[1]) push_ent(o, group, b, 2, 0);
        }
        break;
      case opAllGather:  // rank q's tensor is read once and fanned out to slice q of every destination
        for (uint32_t q = 0; q < n; ++q) {
          uint32_t k = 1;
          b[0] = o.buf[q];
          for (uint32_t r = 0; r < n; ++r) {
            const uint64_t d = o.buf[8 + r] + q * o.nbytes;
            if (d == b[0]) continue;  // contribution already in place
            b[k++] = d;
            if (k == kMaxBufs) {
              push_ent(o, group, b, k, 0);
              k = 1;
            }
          }
          if (k > 1) push_ent(o, group, b, k, 0);
        }
        break;
      default:
        break;
    }
  }

  // The operations of the dependency-free group (-1), on the library's lanes.
  int launch_group(const LaunchOp* ops, int n, int group) {
    via_mailbox_ = false;
    if (group < 0) {
      // Each kernel kind has its own streams so that a copy, a broadcast and an all-reduce launch of one
      // flush overlap.
      uint64_t bytes[kNumKinds] = {};
      uint32_t n_mine = 0;
      for (int i = 0; i < n; ++i) {  // traffic: every buffer once, (all-)reduce reads and writes them
        if (group_of_[(size_t)i] >= 0) continue;
        const uint32_t k = kernel_of(ops[i].kind);
        bytes[k] += ops[i].nbytes * ops[i].nbuf * (k == kReduce ? 2 : 1);
        n_mine += 1;
      }
      if (cfg_.mailbox && mb_hw_ && n_mine && !profiling_) {  // (kernel timing brackets launches: while it is on, everything is launched)
        // A small flush goes to the resident kernel: no launch.  A larger one wants the whole chip: the resident
        // kernel is asked to close (it does within a microsecond or two; nobody waits for it).
        const uint64_t traffic = bytes[kCopy] + bytes[kBcast] + bytes[kReduce];
        if (traffic <= kMailboxMaxTraffic && mb_.room() >= kMaxOpBufs * n_mine) {
          via_mailbox_ = true;
        } else {
          mb_.stop();
        }
      }
      for (uint32_t k = 0; k < kNumKinds; ++k) {
        if (!bytes[k]) {
          data_[k] = lanes_[k][1];
          continue;
        }
        // a kernel of >~10 us: 64 MiB of copy traffic, 32 MiB of reduce traffic (its small-chunk launches run slower)
        const uint64_t medium = k == kReduce ? (32ull << 20) : (64ull << 20);
        if (bytes[k] >= kLargeLaunchBytes) data_[k] = lanes_[k][0];
        else if (bytes[k] >= medium) data_[k] = lanes_[k][1 + lane_cursor_[k]++ % (kLanes - 1)];
        else data_[k] = lanes_[k][1];
      }
    }
    return run_group(ops, n, group);
  }

  // Expand every operation of `group` into the entries of its kernel and launch them kind by kind on
  // data_[kind].  All entries of an operation stay in one launch (they share one arrival count).
  int run_group(const LaunchOp* ops, int n, int group) {
    int rc = MW_OK;
    for (uint32_t kind = 0; kind < kNumKinds && rc == MW_OK; ++kind) {
      const size_t cap = kind == kCopy ? kCopyMax : kCollMax;
      ents_.clear();
      for (int i = 0; i < n && rc == MW_OK; ++i) {
        if (group_of_[(size_t)i] != group || kernel_of(ops[i].kind) != kind) continue;
        const size_t before = ents_.size();
        expand(ops[i], (uint32_t)i);
        if (ents_.size() == before) {  // every segment already in place: nothing to move, complete now
          if (host_flags_ok_) __atomic_store_n(&flags_host_[ops[i].slot], ops[i].gen, __ATOMIC_RELEASE);
          launched_[i] = 1;
          continue;
        }
        if (ents_.size() > cap) {  // launch what was gathered before this operation, keep its entries
          one_.assign(ents_.begin() + (long)before, ents_.end());
          ents_.resize(before);
          rc = launch_entries(kind);
          ents_.swap(one_);
        }
      }
      if (rc == MW_OK && !ents_.empty()) rc = launch_entries(kind);
    }
    return rc;
  }

  // Launch the gathered entries (ents_) as one kernel of `kind`.
  int launch_entries(uint32_t kind) {
    const int n = (int)ents_.size();
    uint64_t total_bytes = 0;
    for (const Ent& e : ents_) total_bytes += e.nbytes;
    // chunks per entry, and per operation (= run of entries with the same group); copies and fan-outs use
    // one (power of two) size per launch
    const uint32_t launch_chunk = pick_chunk_bytes(kind, total_bytes, 2, true);
    chunks_.resize((size_t)n);
    chunk_bytes_.resize((size_t)n);
    uint64_t chunks = 0;
    for (int i = 0; i < n; ++i) {
      const Ent& e = ents_[(size_t)i];
      const bool all_written = (e.flags >> 24) == (1u << e.nbuf) - 1u;
      const uint32_t cb = kind == kReduce ? pick_chunk_bytes(kind, total_bytes, e.nbuf, all_written) : launch_chunk;
      chunk_bytes_[(size_t)i] = cb;
      chunks_[(size_t)i] = (uint32_t)((e.nbytes + cb - 1) / cb);
      chunks += chunks_[(size_t)i];
    }
    if (chunks == 0 || chunks > 0x7FFFFFFFull) return fail_inval();
    // Per operation: its chunk count, and the arrival count at which it is complete -- the slot's running total
    // (counts_) plus its chunks.  An operation of one chunk does not touch the counter.
    op_chunks_.resize((size_t)n);
    targets_.resize((size_t)n);
    first_chunk_.resize((size_t)n);
    for (int i = 0; i < n;) {
      int j = i;
      uint32_t sum = 0;
      while (j < n && ents_[(size_t)j].group == ents_[(size_t)i].group) {
        first_chunk_[(size_t)j] = sum;  // chunks of the same operation in earlier entries
        sum += chunks_[(size_t)j++];
      }
      const uint32_t target = counts_[ents_[(size_t)i].slot] + (sum > 1 ? sum : 0);
      for (int k = i; k < j; ++k) {
        op_chunks_[(size_t)k] = sum;
        targets_[(size_t)k] = target;
      }
      i = j;
    }
    if (via_mailbox_) {  // no launch: the entries become descriptors in the resident kernel's queue
      if (int rc = mailbox_entries(kind)) return rc;
      return entries_are_on_their_way();
    }
    hipEvent_t e0 = nullptr, e1 = nullptr;
    if (profiling_) {
      e0 = prof_event();
      e1 = prof_event();
      if (chk(hipEventRecord(e0, data_[kind]))) return MW_EHIP;
    }
    const int* caps = kind == kCopy ? kCopyCap : kCollCap;
    const int tier = n <= caps[0] ? 0 : n <= caps[1] ? 1 : 2;
    if (kind == kCopy) {
      const uint32_t shift = floor_log2(launch_chunk);
      if (tier == 0) launch_copy<kCopyCap[0]>(shift);
      else if (tier == 1) launch_copy<kCopyCap[1]>(shift);
      else launch_copy<kCopyCap[2]>(shift);
    } else {
      if (tier == 0) launch_coll<kCollCap[0]>(kind);
      else if (tier == 1) launch_coll<kCollCap[1]>(kind);
      else launch_coll<kCollCap[2]>(kind);
    }
    if (chk(hipGetLastError())) return MW_EHIP;
    if (profiling_) {
      if (chk(hipEventRecord(e1, data_[kind]))) return MW_EHIP;
      prof_.push_back(ProfRec{kind, e0, e1, total_bytes});
    }
    return entries_are_on_their_way();
  }

  // The gathered entries are enqueued (launched, or queued for the resident kernel): their chunks will be counted in.
  int entries_are_on_their_way() {
    for (size_t i = 0; i < ents_.size(); ++i) {
      const Ent& e = ents_[i];
      counts_[e.slot] = targets_[i];
      launched_[e.group] = 1;  // group = index of the operation in this launch call
    }
    ents_.clear();
    return MW_OK;
  }

  template <int CAP>
  void launch_copy(uint32_t shift) {
    static CopyArgs<CAP> a;  // launches are serialised by the library's lock
    const int n = (int)ents_.size();
    uint32_t at = 0;
    a.n = (uint32_t)n;
    a.chunk_shift = shift;
    a.rotate = 1;
    for (int i = 0; i < n; ++i) {
      const Ent& e = ents_[(size_t)i];
      a.first_chunk[i] = at;
      at += chunks_[(size_t)i];
      a.e[i] = CopyEnt{e.buf[0], e.buf[1], e.nbytes, e.slot, e.gen, e.world_id, e.world_epoch,
                       op_chunks_[(size_t)i], e.flags, targets_[(size_t)i], 0};
    }
    a.first_chunk[n] = at;
    hipLaunchKernelGGL(mw_k_copy<CAP>, dim3(at), dim3(kCopyWG), 0, data_[kCopy], a, cur_slots_, cur_flags_);
  }

  template <int CAP>
  void launch_coll(uint32_t kind) {
    static CollArgs<CAP> a;
    const int n = (int)ents_.size();
    uint32_t at = 0;
    a.n = (uint32_t)n;
    a.rotate = 1;
    for (const Ent& e : ents_) a.rotate &= kind == kBcast || (e.flags >> 24) != (1u << e.nbuf) - 1u;
    for (int i = 0; i < n; ++i) {
      const Ent& e = ents_[(size_t)i];
      a.first_chunk[i] = at;
      at += chunks_[(size_t)i];
      CollEnt& c = a.e[i];
      for (int k = 0; k < kMaxBufs; ++k) c.buf[k] = e.buf[k];
      c.nbytes = e.nbytes;
      c.slot = e.slot;
      c.gen = e.gen;
      c.nbuf = e.nbuf;
      c.chunk_bytes = chunk_bytes_[(size_t)i];
      c.world_id = e.world_id;
      c.world_epoch = e.world_epoch;
      c.op_chunks = op_chunks_[(size_t)i];
      c.flags = e.flags;
      c.target = targets_[(size_t)i];
      c.pad = 0;
    }
    a.first_chunk[n] = at;
    if (kind == kBcast) {
      hipLaunchKernelGGL(mw_k_bcast<CAP>, dim3(at), dim3(kCopyWG), 0, data_[kind], a, cur_slots_, cur_flags_);
    } else if (cfg_.reduce_lds) {
      uint32_t lds = 0;
      for (int i = 0; i < n; ++i) lds = std::max(lds, a.e[i].nbuf * lds_stride(a.e[i].chunk_bytes) * 16u);
      hipLaunchKernelGGL((mw_k_reduce<true, CAP>), dim3(at), dim3(kReduceWG), lds, data_[kind], a, cur_slots_, cur_flags_);
    } else {
      hipLaunchKernelGGL((mw_k_reduce<false, CAP>), dim3(at), dim3(kReduceWG), 0, data_[kind], a, cur_slots_, cur_flags_);
    }
  }

  // The gathered entries (ents_, with chunks_ / chunk_bytes_ / op_chunks_ / targets_ / first_chunk_ filled in) as
  // descriptors for the resident kernel.  They stay queued whether or not a kernel could be started for them now
  // (the next flush or poll tries again), so the caller books them as on their way either way.
  int mailbox_entries(uint32_t kind) {
    const size_t n = ents_.size();
    mb_descs_.resize(n);
    for (size_t k = 0; k < n; ++k) {
      const Ent& e = ents_[k];
      mb::Desc& d = mb_descs_[k];
      std::memset(&d, 0, sizeof(d));
      for (int b = 0; b < kMaxBufs; ++b) d.buf[b] = e.buf[b];
      d.nbytes = e.nbytes;
      d.slot = e.slot;
      d.gen = e.gen;
      d.nbuf = e.nbuf;
      d.chunk_bytes = chunk_bytes_[k];
      d.world_id = e.world_id;
      d.world_epoch = e.world_epoch;
      d.op_chunks = op_chunks_[k];
      d.flags = e.flags;
      d.target = targets_[k];
      d.kind = kind == kCopy ? mb::kKindCopy : kind == kBcast ? mb::kKindBcast : mb::kKindReduce;
      d.first_chunk = first_chunk_[k];
      d.n_chunks = chunks_[k];
    }
    uint32_t first_ticket = 0;
    if (mb_.submit(mb_descs_.data(), (uint32_t)n, &first_ticket) != 0) {
      (void)entries_are_on_their_way();
      return MW_EHIP;
    }
    return MW_OK;
  }

 public:
  // ---- what mb::MailboxHost needs of the device (its Port)
  void write_desc(uint32_t index, const mb::Desc& d) {
    // write-combined memory: whole 16-byte stores, no read-modify-write
    const __m128i* src = reinterpret_cast<const __m128i*>(&d);
    __m128i* dst = reinterpret_cast<__m128i*>(&mb_hw_->q[index]);
    for (int k = 0; k < (int)(sizeof(mb::Desc) / 16); ++k) _mm_stream_si128(dst + k, _mm_loadu_si128(src + k));
  }
  void ring(uint32_t tail) {
    _mm_sfence();  // the descriptors leave the core's write-combining buffers before the doorbell does
    *reinterpret_cast<volatile uint32_t*>(&mb_hw_->tail) = tail;
    _mm_sfence();
  }
  void ask_stop(uint32_t epoch) {
    *reinterpret_cast<volatile uint32_t*>(&mb_hw_->stop) = epoch;
    _mm_sfence();
  }
  uint64_t closed() { return __atomic_load_n(mb_closed_, __ATOMIC_ACQUIRE); }
  int launch(uint32_t epoch, uint32_t first) {
    if (chk(hipSetDevice(dev_))) return MW_EHIP;
    hipLaunchKernelGGL(mw_k_mailbox, dim3(cfg_.mailbox_workers + 1), dim3(kCopyWG), 0, mb_stream_, mb_hw_, mb_lw_, mb_closed_dev_, epoch,
                       first, cfg_.mailbox_workers, (uint64_t)cfg_.mailbox_idle_us * kTicksPerUs, kMailboxLifeTicks, slots_, flags_dev_);
    return chk(hipGetLastError()) ? MW_EHIP : MW_OK;
  }
  bool needs_attention() override { return mb_hw_ && mb_.needs_attention(); }
  int attend() override { return mb_hw_ ? (mb_.attend() == 0 ? MW_OK : MW_EHIP) : MW_OK; }
  void mailbox_state(uint32_t* epoch, uint32_t* open, uint32_t* tail) override {
    *epoch = mb_.epoch();
    *open = mb_hw_ && mb_.running() ? 1u : 0u;
    *tail = mb_.tail();
  }

 private:
  // A flush of at most this much traffic goes to the mailbox (the all-reduce iteration of the tensor-parallel
  // workload is 36 MiB); above it the launch overhead no longer matters and the whole chip is wanted.
  static constexpr uint64_t kMailboxMaxTraffic = 64ull << 20;
  // wall_clock64() ticks at 100 MHz: the resident kernel closes after mailbox_idle_us without work (300 us unless
  // configured) and lives 100 ms at most
  static constexpr uint64_t kTicksPerUs = 100, kMailboxLifeTicks = 10000000;
  mb::HostWritten* mb_hw_ = nullptr;         // the queue (fine-grained device memory, host-writable)
  mb::LeaderWritten* mb_lw_ = nullptr;       // the leader's word (device memory)
  uint64_t* mb_closed_ = nullptr;            // what the last leader to close left (host-pinned) ...
  uint64_t* mb_closed_dev_ = nullptr;        // ... and its device address
  hipStream_t mb_stream_ = nullptr;          // resident kernels run one after the other on it
  mb::MailboxHost<HipDevice> mb_{this};
  std::vector<mb::Desc> mb_descs_;
  std::vector<uint32_t> first_chunk_;  // per entry: chunks of the same operation in earlier entries
  bool via_mailbox_ = false;                 // the current launch_group() call hands its entries to the mailbox

  int fail_inval() {
    last_err_ = (int)hipErrorInvalidValue;
    return MW_EHIP;
  }

  DeviceConfig cfg_{};
  int dev_ = 0;
  bool ready_ = false;
  int last_err_ = 0;
  void* arena_ = nullptr;
  RingHeader* headers_ = nullptr;
  RingSlot* slots_ = nullptr;
  uint32_t* flags_host_ = nullptr;
  uint32_t* flags_dev_ = nullptr;
  // kLanes streams per kernel kind.  Back-to-back kernels on one stream are separated by ~6 us of
  // release / acquire and dispatch; a launch on a stream that has gone idle costs ~10 us to get going.
  // So: large launches (>= 4 GiB of traffic, kernels of >~0.7 ms) go one after the other on lane 0 (two
  // bandwidth-bound kernels side by side measured -1 %, more than the boundary costs them; at 0.8 GiB per
  // launch it is the other way round: two worlds streaming 4 MB tensors together moved 2.91 TB/s one after
  // the other and 3.15 alternating); medium launches alternate between lanes 1 and 2, so that the
  // boundary of one is hidden behind the other (the 4 x 4-rank all-reduce iteration went from 19.2 to
  // 12.4 us, windows of 4 MB messages gained 8 %); small launches (kernels of a few us) stay on lane 1,
  // where alternating measured 15-25 % slower.
  static constexpr int kLanes = 4;
  static constexpr uint64_t kLargeLaunchBytes = 4096ull << 20;  // of traffic (bytes x buffers) per launch
  hipStream_t lanes_[kNumKinds][kLanes] = {};
  uint32_t lane_cursor_[kNumKinds] = {};
  hipStream_t data_[kNumKinds] = {};  // the lane each kind uses in the current launch() call
  hipStream_t ctl_ = nullptr;         // ring-header writes
  std::vector<hipEvent_t> dep_events_;
  int dep_cursor_ = 0;
  bool profiling_ = false;
  std::vector<ProfRec> prof_;
  std::vector<hipEvent_t> prof_free_;
  ProfAcc acc_[kNumKinds];
  std::vector<Ent> ents_, one_;
  uint8_t* launched_ = nullptr;  // the current launch() call's per-operation result array
  RingSlot* cur_slots_ = nullptr;   // where the current launch's kernels count chunks in and publish completion:
  uint32_t* cur_flags_ = nullptr;   // the arena and the host-pinned words, or the static scratch
  bool host_flags_ok_ = true;       // the current launch publishes to the host-pinned words
  unsigned char* static_base_ = nullptr;  // device address of `scratch` on dev_
  std::vector<uint8_t> static_launched_;
  std::vector<void*> dep_streams_, waited_;  // distinct caller streams of the current launch() call
  std::vector<uint8_t> dep_busy_;            // ... and whether each still had work pending
  std::vector<int> group_of_;                // per operation: index of its first busy stream, or -1
  std::vector<uint32_t> chunks_, op_chunks_, chunk_bytes_, targets_;
  std::vector<uint32_t> arena_counts_;          // per arena slot: chunks counted in so far (what the device counter will reach)
  uint32_t static_counts_[kStaticOps] = {};     // the same for the static scratch, whose counters every call zeroes
  uint32_t* counts_ = nullptr;                  // the one the current launch uses
};

}  // namespace

Device* make_device() { return new HipDevice(); }

}  // namespace mw
