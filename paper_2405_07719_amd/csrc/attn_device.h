// Device-side helpers shared by the attention kernels (forward and backward): vector types for the MFMA
// operands, 32-bit position descriptors, bf16 packing and the half-wave combine.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>
#include <functional>
#include <mutex>
#include <thread>
#include <unordered_map>

namespace usp {
namespace dev {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

// Position descriptor narrowed to 32 bits (the host checks L < 2^31): fewer registers in the mask path.
// fourth word of a raw (unstructured, bounds-checked by byte extent) buffer descriptor on gfx9-family chips:
// 32-bit data format, everything else zero
constexpr int kRawBufferFlags = 0x00020000;

struct PosDesc32 { int start0, len0, start1, len1; };
__device__ inline int pos_of(const PosDesc32& d, int i) { return i < d.len0 ? d.start0 + i : d.start1 + (i - d.len0); }
__device__ inline int pos_min(const PosDesc32& d, int a, int b) {
  int m = INT32_MAX;
  if (a < d.len0) m = d.start0 + a;
  if (b > d.len0) m = min(m, d.start1 + (max(a, d.len0) - d.len0));
  return m;
}
__device__ inline int pos_max(const PosDesc32& d, int a, int b) {
  int m = INT32_MIN;
  if (a < d.len0) m = d.start0 + min(b, d.len0) - 1;
  if (b > d.len0) m = max(m, d.start1 + (b - 1 - d.len0));
  return m;
}

// Tiles of a local index range that can hold a visible (query, key) pair: [a0,a1) then [b0,b1) (b may be empty).
struct TileRanges { int a0, a1, b0, b1; };

// Key tiles (of KT keys) visible to the query rows [row_lo, row_hi): under the causal rule kpos <= qpos the
// visible keys of each ascending run form a prefix of that run.
template <int KT>
__device__ inline TileRanges visible_key_tiles(int causal, const PosDesc32& qpos, const PosDesc32& kpos, int Lk,
                                               int row_lo, int row_hi) {
  TileRanges t;
  if (!causal) {
    t.a0 = 0; t.a1 = (Lk + KT - 1) / KT; t.b0 = t.b1 = t.a1;
    return t;
  }
  const int64_t qmax = pos_max(qpos, row_lo, row_hi);
  int64_t c0 = qmax - kpos.start0 + 1; c0 = c0 < 0 ? 0 : (c0 > kpos.len0 ? kpos.len0 : c0);
  int64_t c1 = qmax - kpos.start1 + 1; c1 = c1 < 0 ? 0 : (c1 > kpos.len1 ? kpos.len1 : c1);
  t.a0 = 0;
  t.a1 = (int)((c0 + KT - 1) / KT);
  if (c1 > 0) {
    t.b0 = (int)(kpos.len0 / KT);
    t.b1 = (int)(((int64_t)kpos.len0 + c1 + KT - 1) / KT);
    if (t.b0 < t.a1) t.b0 = t.a1;
    if (t.b1 < t.b0) t.b1 = t.b0;
  } else {
    t.b0 = t.b1 = t.a1;
  }
  return t;
}

// Query tiles (of QT rows) that see at least one key of [key_lo, key_hi): the rows of each ascending run
// with qpos >= the smallest key position form a suffix of that run.
template <int QT>
__device__ inline TileRanges visible_query_tiles(int causal, const PosDesc32& qpos, const PosDesc32& kpos, int Lq,
                                                 int key_lo, int key_hi) {
  TileRanges t;
  if (!causal) {
    t.a0 = 0; t.a1 = (Lq + QT - 1) / QT; t.b0 = t.b1 = t.a1;
    return t;
  }
  const int64_t kmin = pos_min(kpos, key_lo, key_hi);
  int64_t f0 = kmin - qpos.start0; f0 = f0 < 0 ? 0 : (f0 > qpos.len0 ? qpos.len0 : f0);   // first visible row of run 0
  int64_t f1 = kmin - qpos.start1; f1 = f1 < 0 ? 0 : (f1 > qpos.len1 ? qpos.len1 : f1);
  if (f0 < qpos.len0) {
    t.a0 = (int)(f0 / QT);
    t.a1 = (int)((qpos.len0 + QT - 1) / QT);
  } else {
    t.a0 = t.a1 = 0;
  }
  if (f1 < qpos.len1) {
    t.b0 = (int)((qpos.len0 + f1) / QT);
    t.b1 = (int)(((int64_t)qpos.len0 + qpos.len1 + QT - 1) / QT);
    if (t.b0 < t.a1) t.b0 = t.a1;
    if (t.b1 < t.b0) t.b1 = t.b0;
  } else {
    t.b0 = t.b1 = t.a1;
  }
  return t;
}

// Make a value that was loaded BEFORE a loop "arrive" here: the empty asm reads and redefines the register, so
// the compiler waits for the load at this point.  Without it the wait-count pass keeps the pre-loop load pending at
// the loop header and places its s_waitcnt vmcnt(n) at the first use INSIDE the loop, where, from the second trip
// on, it waits for that trip's freshly issued prefetch loads instead (the counter only knows "all but n").
__device__ inline void settle(bf16x8& x) {
  u32x4 t = __builtin_bit_cast(u32x4, x);
  asm volatile("" : "+v"(t));
  x = __builtin_bit_cast(bf16x8, t);
}
__device__ inline void settle(float& x) { asm volatile("" : "+v"(x)); }

__device__ inline uint32_t pack_bf16(float lo, float hi) {
  f32x2 f = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, bf16x2));
}

// Combine the two lane halves (lanes l and l ^ 32 hold the same query).  v_permlane32_swap(a, b) returns
// {a.lower | b.lower, a.upper | b.upper}; with a = b = x that is x of the lower half and x of the upper
// half, each broadcast to both halves.  (The two results are copied to scalars before the bit cast:
// a bit cast applied directly to a vector element reads element 0.)
__device__ inline float both_halves_max(float x) {
  const uint32_t xi = __builtin_bit_cast(uint32_t, x);
  const u32x2 r = __builtin_amdgcn_permlane32_swap(xi, xi, false, false);
  const uint32_t lo = r[0], hi = r[1];
  return fmaxf(__builtin_bit_cast(float, lo), __builtin_bit_cast(float, hi));
}
__device__ inline float both_halves_sum(float x) {
  const uint32_t xi = __builtin_bit_cast(uint32_t, x);
  const u32x2 r = __builtin_amdgcn_permlane32_swap(xi, xi, false, false);
  const uint32_t lo = r[0], hi = r[1];
  return __builtin_bit_cast(float, lo) + __builtin_bit_cast(float, hi);
}

// ---- persistent workgroups that draw their work items from counters ------------------------------------------
// The hardware deals the workgroups of a grid to the eight XCDs round robin, i.e. every XCD gets the same share,
// but the XCDs do not run at one speed (each settles at its own clock under the power limit: per-tile times
// differ by 4-8 % between the XCDs of one chip), and a CU whose workgroup has ended waits tens of microseconds
// for the dispatcher to start the next one.  So the attention kernels launch one workgroup per CU, and each
// draws work items, in heavy-first order, from counters in device memory until the items run out.
//
// The kernels number their items with the KV head (times batch: `n_groups` values) fastest.  The CUs of one XCD
// share an L2, and workgroups that read the same K/V walk its tiles at about the same time: with eight KV heads
// mixed on an XCD the L2 serves four CUs per tile instead of thirty-two, which costs more than an idle tail does.
// So the items are dealt to n_queues = gcd(8, n_groups) queues (item w to queue w mod n_queues: a queue holds the
// same KV heads throughout; ONE queue when there is one KV head, eight when there are eight), a workgroup on XCD x
// draws from queue x mod n_queues while that has items, and from the next queues round the ring after that.  It
// ends when it has found all queues empty.
//
// Every launch uses one of kTicketSlots sets of counters: one per queue, and one that counts the workgroups that
// have left.  A workgroup leaves when it finds no item, and says so; the one that leaves last (nobody draws after it)
// puts the whole set back to zero, so it is zero again at the next launch, graph replays included.  Two launches may
// share a set only if they do not execute at the same time: the host gives every stream (and every graph capture) a
// set of its own, see ticket_slot_for().
constexpr int kTicketSlots = 4096;      // 256 KiB of counters per kernel file
constexpr int kTicketKeyed = 3840;      // sets that belong to one stream (or one graph capture) each; the rest rotate
constexpr int kMaxItemQueues = 8;
constexpr int kSlotStride = 16;          // counters per set: eight queues, "left", padding to 64 bytes
constexpr unsigned kNoDraw = ~0u;
constexpr int kFirstRun = 8;            // see ItemQueues::first_item
static __device__ __attribute__((aligned(64))) unsigned g_work_ticket[kTicketSlots * kSlotStride];   // a set = one 64-byte line

// the XCD (accelerator complex die) this wave runs on, 0..7
__device__ inline int xcd_id() { return (int)(__builtin_amdgcn_s_getreg((3 << 11) | 20) & 7u); }   // XCC_ID[3:0]

// What a launch's workgroups need to draw items (all of it workgroup-uniform).  Every function here is for ONE
// thread of the workgroup; `empty` is that thread's record (one bit per queue) of the queues it has found empty.
struct ItemQueues {
  int slot, n_items, n_wgs, n_queues;
  __device__ unsigned* counter(int q) const { return &g_work_ticket[slot * kSlotStride + q]; }
  __device__ unsigned* left() const { return &g_work_ticket[slot * kSlotStride + kMaxItemQueues]; }
  // Queue q holds items q, q + n_queues, ...  The first n_wgs items of the launch are not drawn but given: that
  // saves every launch the latency of a first draw.  Draw number t from queue q is therefore item
  // q + n_queues (given(q) + t).  Which workgroup is given which item: see first_item().
  __device__ unsigned given(int q) const { return (unsigned)(max(0, n_wgs - q + n_queues - 1) / n_queues); }
  // The item workgroup b starts with: one of the first n_wgs items, each exactly once.  The hardware puts workgroup
  // b on XCD b mod 8, so item b would be one of its own queue, but would give the 32 CUs of an XCD 32 different
  // weights: they would finish their first items one by one, 15 us apart, start their second items one by one, and
  // such a train of CUs that walk the same K/V a few tiles behind one another is longer than the L2 holds: every
  // one of them fetches every tile again (five times the fabric traffic, measured).  Instead the XCDs that share a
  // queue take its given items in runs of kFirstRun: eight CUs of an XCD hold neighbouring weights, finish together
  // and start their next items together, in step like the first ones.  (Whole XCDs of neighbouring weights would
  // share even more, but then each XCD's CUs pair their items among themselves and a slow XCD is not helped.)
  __device__ int first_item(int b) const {
    if (n_wgs % kMaxItemQueues) return b;   // fewer workgroups than CUs: one item each, nothing to arrange
    const int x = b % kMaxItemQueues, j = b / kMaxItemQueues, per_xcd = n_wgs / kMaxItemQueues;
    const int q = x % n_queues, sharers = kMaxItemQueues / n_queues, rank = x / n_queues;
    const int run = per_xcd % kFirstRun ? per_xcd : kFirstRun;
    return q + n_queues * (((j / run) * sharers + rank) * run + j % run);
  }
  __device__ unsigned items_of(int q) const {
    return (unsigned)(max(0, n_items - q + n_queues - 1) / n_queues) - given(q);   // n_wgs <= n_items: never negative
  }
  __device__ int item(int q, unsigned t) const { return q + n_queues * (int)(given(q) + t); }
  __device__ int own() const { return xcd_id() % n_queues; }
  __device__ static unsigned add1(unsigned* c) { return __hip_atomic_fetch_add(c, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }

  // First half of a draw: asks the workgroup's own queue, unless that is known to be empty.  The answer is only
  // needed in finish(), so the caller can put work between the two.
  __device__ unsigned begin(unsigned empty) const {
    const int q = own();
    return ((empty >> q) & 1u) ? kNoDraw : add1(counter(q));
  }
  // Second half: the next item, or n_items when none is left.
  __device__ int finish(unsigned own_ticket, unsigned& empty) const {
    const int q0 = own();
    if (own_ticket != kNoDraw) {
      if (own_ticket < items_of(q0)) return item(q0, own_ticket);
      empty |= 1u << q0;
    }
    while (n_queues > 1) {
      // a look at the other queues (a hint; the draw decides): the first one round the ring that still has items
      // The eight counters of the set lie in 32 bytes: two 16-byte loads that go past the caches, as an atomic load
      // of agent scope does (cache policy sc1), bring them all in one round trip to memory.  (One atomic load per
      // queue, each waited for before the next, cost a workgroup that finds everything empty, as each one does at
      // the end of a launch, 8 us; eight independent atomic loads cost the memory channel that holds the line more
      // than they saved when many workgroups ran out of items together.)
      const __amdgpu_buffer_rsrc_t set = __builtin_amdgcn_make_buffer_rsrc((void*)counter(0), 0, kMaxItemQueues * 4, kRawBufferFlags);
      constexpr int kPastCaches = 16;   // sc1
      const u32x4 d0 = __builtin_amdgcn_raw_buffer_load_b128(set, 0, 0, kPastCaches);
      const u32x4 d1 = __builtin_amdgcn_raw_buffer_load_b128(set, 16, 0, kPastCaches);
      const unsigned drawn[kMaxItemQueues] = {d0[0], d0[1], d0[2], d0[3], d1[0], d1[1], d1[2], d1[3]};
      int best = -1, best_away = kMaxItemQueues;
#pragma unroll
      for (int q = 0; q < kMaxItemQueues; ++q) {
        if (q >= n_queues || ((empty >> q) & 1u)) continue;
        const int away = (q - q0 + n_queues) % n_queues;
        if (drawn[q] < items_of(q) && away < best_away) { best = q; best_away = away; }
      }
      if (best < 0) break;
      const unsigned t = add1(counter(best));
      if (t < items_of(best)) return item(best, t);
      empty |= 1u << best;
    }
    return n_items;
  }
  // The workgroup has found no item and ends.  Its draws are complete (their answers were read) before this count,
  // all of them go to the same place (agent-scope atomics), so whoever counts last also writes last.
  __device__ void leave() const {
    if (add1(left()) == (unsigned)n_wgs - 1u) {
#pragma unroll
      for (int q = 0; q <= kMaxItemQueues; ++q)
        __hip_atomic_store(&g_work_ticket[slot * kSlotStride + q], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
  }
};

}  // namespace dev

// host side: CUs of the current device, and the counter the next launch uses
inline int compute_units() {
  static std::atomic<int> known[64];   // per device, asked once: later calls may come during stream capture
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
  int n = known[dev].load(std::memory_order_relaxed);
  if (n == 0) {
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n < 1) n = 256;
    known[dev].store(n, std::memory_order_relaxed);
  }
  return n;
}
// The set of counters a launch uses.  Two launches may share a set only if they never execute at the same time.
// Launches on ONE stream never do, so a set belongs to a stream: the first kTicketKeyed - 1 distinct streams seen by
// the process each get a set of their own, for good (stream handles of destroyed streams come back, and so do their
// sets).  A launch recorded into a graph executes whenever and wherever the graph is replayed, so a capture gets a
// set of its own too (keyed by the capture's id and the stream being captured); the per-thread default stream is a
// different stream in every thread and is keyed by the thread as well.  What can still collide: two executable
// graphs instantiated from one capture replayed at the same time, and, once more than kTicketKeyed - 1 streams and
// captures have been seen, the later ones, which share the last kTicketSlots - kTicketKeyed sets in rotation as all
// launches once did (two of THOSE collide only if they execute at the same time and are fewer than that many
// launches apart).
inline int ticket_slot_for(hipStream_t stream) {
  struct Key {
    const void* stream;
    unsigned long long capture;
    size_t thread;
    bool operator==(const Key& o) const { return stream == o.stream && capture == o.capture && thread == o.thread; }
  };
  struct KeyHash {
    size_t operator()(const Key& k) const {
      return std::hash<const void*>()(k.stream) ^ (std::hash<unsigned long long>()(k.capture) * 0x9E3779B97F4A7C15ull) ^
             (k.thread * 0xC2B2AE3D27D4EB4Full);
    }
  };
  static std::mutex mu;
  static std::unordered_map<Key, int, KeyHash> slots;
  static std::atomic<unsigned> overflow{0};
  Key key{(const void*)stream, 0ull, 0};
  if (stream == hipStreamPerThread) key.thread = std::hash<std::thread::id>()(std::this_thread::get_id()) | 1u;
  hipStreamCaptureStatus status = hipStreamCaptureStatusNone;
  unsigned long long id = 0;
  if (stream != nullptr && hipStreamGetCaptureInfo(stream, &status, &id) == hipSuccess) {
    if (status == hipStreamCaptureStatusActive) key.capture = id + 1;
  } else {
    (void)hipGetLastError();   // the legacy default stream cannot be captured; nothing to report
  }
  {
    std::lock_guard<std::mutex> lock(mu);
    auto it = slots.find(key);
    if (it != slots.end()) return it->second;
    if ((int)slots.size() < dev::kTicketKeyed) {
      const int slot = (int)slots.size();
      slots.emplace(key, slot);
      return slot;
    }
  }
  return dev::kTicketKeyed + (int)(overflow.fetch_add(1, std::memory_order_relaxed) % (dev::kTicketSlots - dev::kTicketKeyed));
}

}  // namespace usp
