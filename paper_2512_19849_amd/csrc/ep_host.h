// State shared by the two host translation units of libep.so: the per-thread proxy state, the handle,
// and small helpers.  proxy.cpp holds the CPU proxy threads (sender half + receiver half in one process,
// since the peer ranks are partitions of this GPU's memory); api.cpp holds set-up, tear-down and the C ABI.
#ifndef EP_HOST_H_
#define EP_HOST_H_
#include <hip/hip_runtime_api.h>
#include <fcntl.h>
#include <sys/mman.h>
#include <sys/stat.h>
#include <unistd.h>
#include <immintrin.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>
#include <time.h>

#include <atomic>
#include <deque>
#include <map>
#include <memory>
#include <mutex>
#include <new>
#include <thread>
#include <utility>
#include <vector>

#include "ep_internal.h"

namespace ep {

// Text of the most recent failure on this thread (ep_last_error).
extern thread_local char g_last_error[256];

bool hip_ok(hipError_t e, const char *what);
#define HIP_OK(call) ::ep::hip_ok((call), #call)

inline uint64_t now_ns() {
  timespec ts;
  clock_gettime(CLOCK_MONOTONIC, &ts);
  return (uint64_t)ts.tv_sec * 1000000000ull + (uint64_t)ts.tv_nsec;
}

// splitmix64: the proxy's own generator for the delivery-reordering test hook.
inline uint64_t mix64(uint64_t &state) {
  uint64_t z = (state += 0x9E3779B97F4A7C15ull);
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}

// Statistics counters have one writer (the owning proxy thread): a plain add, no locked instruction.
inline void bump(std::atomic<uint64_t> &a, uint64_t v = 1) {
  a.store(a.load(std::memory_order_relaxed) + v, std::memory_order_relaxed);
}

// What travels from the sender half to the receiver half: the 32-bit immediate
// (Section 3.3) plus what the receiver knows from the connection it arrived on.
//   Write : [31]=0 [30:19] local expert [18:13] rows-1 [12:0] low bits of dst_off/16
//   Atomic: [31]=1 [30:19] local expert [18:0]  value
struct WireEvent {
  uint32_t imm;
  uint16_t src;       // connection = source rank
  uint8_t dst_rank;   // the receiving rank (whose proxy this event reaches)
  uint8_t ordered;    // 0 plain; 1 sequenced message of the chunked high-throughput mode;
                      // 2 / 3 ring-buffer channel, sender -> receiver / receiver -> sender
  uint16_t slice;     // ring-buffer channels: the token slice (part of the connection's identity)
};

// Messages of one sequenced channel that arrived ahead of their turn (the control buffer of Section 3.3,
// per channel).  Those within kWin numbers of the next expected one sit in a window indexed by number
// mod kWin - no allocation per message, which matters when most messages of a busy channel arrive
// early; anything further ahead (or behind: a protocol error that a Drain reports) goes to a map.
struct ReorderBuf {
  static constexpr uint32_t kWin = 256;
  struct Win {
    WireEvent ev[kWin];
    uint64_t have[kWin / 64] = {};
  };
  std::unique_ptr<Win> win;  // allocated with the first early message
  std::map<uint32_t, WireEvent> far;
  uint32_t count = 0;

  bool empty() const { return count == 0; }
  void put(uint32_t next, uint32_t seq, const WireEvent &e) {
    if (seq - next < kWin) {  // (unsigned: a number behind `next` is "far")
      if (!win) win.reset(new Win());
      const uint32_t i = seq % kWin;
      if (!((win->have[i / 64] >> (i % 64)) & 1)) ++count;
      win->ev[i] = e;
      win->have[i / 64] |= 1ull << (i % 64);
    } else if (far.emplace(seq, e).second) {
      ++count;
    }
  }
  // Removes the message numbered seq, if it is here.  seq is always the channel's next number, so a
  // window slot can only hold that very number (a later one with the same index was not yet within
  // kWin of the next number when it arrived, and went to the map).
  bool take(uint32_t seq, WireEvent &out) {
    if (count == 0) return false;
    const uint32_t i = seq % kWin;
    if (win && ((win->have[i / 64] >> (i % 64)) & 1)) {
      out = win->ev[i];
      win->have[i / 64] &= ~(1ull << (i % 64));
      --count;
      return true;
    }
    if (!far.empty()) {
      auto it = far.find(seq);
      if (it != far.end()) {
        out = it->second;
        far.erase(it);
        --count;
        return true;
      }
    }
    return false;
  }
};

// A message on its way out of the sender half: the notice the receiver will get, and (registered
// heaps) the copies that have to complete first.  Packed per-token Writes are one message with
// several source segments of one row each and one contiguous destination.
constexpr int kMaxPackRows = 16;
struct Outbound {
  WireEvent notice;
  uint32_t nseg = 0;          // 0: nothing to copy (the kernel placed the rows, or an Atomic)
  uint64_t seglen = 0, dof = 0;
  uint64_t so[kMaxPackRows];
  const char *sbase = nullptr;
  char *dbase = nullptr;
  uint32_t le = 0;            // packing: the open message's expert
  uint64_t opened_ns = 0;     // packing: when its first row was polled
};

struct alignas(64) ProxyThread {
  int tid = 0;
  // no pacing, packing, reordering transport, sender-side fence or event log configured: a Write whose
  // payload is already in place has nothing between its command and its arrival notice
  bool plain_writes = false;
  std::thread th;
  std::vector<int> channels;
  std::vector<uint64_t> head;  // consumer index per owned channel (private copy)
  // receiver half: rows seen and parked atomics per (source, global expert)
  std::vector<int32_t> seen;
  std::vector<std::deque<int32_t>> parked;  // the control buffer
  std::vector<std::deque<int32_t>> sender_parked;  // sender-side fence: atomics not yet sent, per (source, expert)
  std::vector<uint8_t> atomic_flying;              // ... and whether one of that expert is on its way
  std::vector<WireEvent> window;            // in-flight immediates (reordering hook)
  // proxy-performed peer writes (registered heaps): descriptors of the batch being filled, and the
  // batches in flight with the arrival notices they will release when their copy kernel is done
  static constexpr int kBatchSlots = 8;
  hipEvent_t events[kBatchSlots] = {};
  CopyDesc *descs = nullptr;    // pinned host [kBatchSlots][kCopyBatchMax]
  CopyDesc *d_descs = nullptr;  // the same memory as the device sees it
  CopyBatchArgs cur{};
  struct Batch {
    int slot;
    std::vector<WireEvent> notices;
  };
  std::deque<Batch> inflight;
  std::vector<WireEvent> cur_notices;
  int cur_slot = 0;
  bool gpu_ready = false;
  // ordered (high-throughput) channels: next sequence number and early arrivals per (source, destination rank)
  std::vector<uint32_t> next_seq;
  std::vector<ReorderBuf> early;
  // pacing: messages in flight per destination rank, and those waiting at the sender for room
  std::vector<int32_t> in_flight;
  std::vector<std::deque<Outbound>> held;
  size_t held_total = 0;
  // best-effort packing: the open (still growing) message per (source, global expert), -1 = none
  std::vector<int32_t> open_idx;
  std::vector<Outbound> open;
  std::vector<uint32_t> open_key;
  // ring-buffer channels: the same per (source, slice, destination rank, direction)
  std::vector<uint32_t> ring_next;
  std::vector<ReorderBuf> ring_early;
  uint64_t rng = 0;
  uint64_t applied_unpublished = 0;  // atomics applied but not yet added to `applied` (owner thread only)
  bool stamp_apply = false;          // last_apply_ns is due
  // What ep_wait spins on, in a cache line of its own: the waiting thread re-reads it all the time, and
  // anything the owner writes per command in the same line would miss on every write.
  alignas(64) std::atomic<uint64_t> applied{0}, drains{0};
  // statistics (written by the owner thread only, read racy-but-atomically)
  alignas(64) std::atomic<uint64_t> cmds{0}, writes{0}, atomics{0}, write_bytes{0}, write_rows{0}, deferred{0},
      rejected{0}, first_poll_ns{0}, last_apply_ns{0}, ordered_parked{0}, barriers{0}, copy_batches{0},
      copied_bytes{0}, write_msgs{0}, paced{0}, max_in_flight{0}, sender_held{0};
  std::mutex log_mu;
  std::vector<uint32_t> cmd_log, event_log;
};

}  // namespace ep

// The opaque handle of include/ep.h.
struct ep_handle {
  ep_config cfg{};
  ep::Tunables tune{};       // EP_* overrides, read once in ep_proxy_start
  bool cache_hints = false;  // EP_FLAG_CACHE_HINTS
  bool host_only = false;
  int E_loc = 0;
  uint64_t heap_bytes = 0;
  uint32_t entries = 0, log2_entries = 0;
  // pinned host (or plain host memory when host_only)
  uint64_t *slots = nullptr;  // 2 x uint64 per command
  uint64_t *head = nullptr;   // [C * kHeadStride]
  int32_t *recv_count = nullptr;
  int *recv_flag = nullptr;  // posted count + 1, cleared by the GPU-side wait
  int32_t *recv_tail = nullptr;  // [S, R] rows announced per communication channel (ordered mode)
  int32_t *ring_tail = nullptr, *ring_head = nullptr;  // [S, slices, R] rows announced / released per ring channel
  void *d_ring_tail = nullptr, *d_ring_head = nullptr;
  unsigned *ring_seq_fwd = nullptr, *ring_seq_rev = nullptr, *ring_cum_fwd = nullptr, *ring_cum_rev = nullptr;
  uint64_t ring_slot_bytes = 0, ring_total_bytes = 0;
  std::atomic<int64_t> expected_drains{0};
  // registered heaps (symmetric memory): when set, the proxy performs the Writes
  std::atomic<const char *> src_base{nullptr};
  std::atomic<char *> dst_base{nullptr};
  uint64_t src_bytes = 0, dst_bytes = 0;
  int device = 0;
  hipStream_t copy_stream = nullptr;  // the proxy's copy kernels (all threads; launches under copy_mu)
  std::mutex copy_mu;
  // Barrier: a counter and a generation shared by the peer processes of one node
  struct SharedBarrier {
    std::atomic<uint32_t> arrived;
    std::atomic<uint32_t> generation;
  };
  SharedBarrier *barrier = nullptr;
  SharedBarrier private_barrier{};
  bool barrier_is_shm = false;
  char barrier_path[64] = "";
  void *d_recv_flag = nullptr;
  int *dev_error = nullptr;
  void *d_recv_count = nullptr;
  // device state
  ep::RingDev ring{};
  int32_t *tile_hist = nullptr, *tile_base = nullptr, *chunk_cnt = nullptr, *expert_done = nullptr;
  unsigned *ticket = nullptr, *waves_done = nullptr, *ht_seq = nullptr;
  int ntiles_cap = 0, chunks_per_expert = 0;
  // host-only producer state
  std::atomic<uint64_t> host_tail[ep::kMaxChannels];
  std::atomic<uint64_t> host_stalls{0};
  // proxy
  std::atomic<bool> stop{false};
  std::atomic<int64_t> expected_atomics{0};
  // ep_profile: while on, ep_layout / ep_dispatch / ep_combine launch with a pair of events that receive their
  // kernels' own begin and end timestamps; ep_profile_read adds the pairs up
  bool profiling = false;
  std::vector<std::pair<hipEvent_t, hipEvent_t>> timed[3];
  std::vector<hipEvent_t> spare_events;  // made ahead of time (ep_profile) or handed back by ep_profile_read
  // what calls on capturing streams would have added to the two expected_* counts (ep_captured)
  std::atomic<int64_t> captured_atomics{0}, captured_drains{0};
  std::atomic<int> proxy_error{0};
  int nthreads = 0;
  ep::ProxyThread *threads = nullptr;
  // Only with EP_FLAG_CACHE_HINTS (the caller's promise that ep_combine reads the buffer ep_dispatch
  // wrote, with nothing but in-place work on it in between):
  // What the last launch of this handle wrote, if it was a bf16 ep_dispatch of all its rows: the
  // receive buffer, the token count and the stream.  An ep_combine that reads the same buffer for
  // the same tokens on the same stream directly afterwards knows which rows are still in the
  // memory-side cache (the last tokens') and reads those first, with cached loads.
  std::atomic<const void *> fresh_buf{nullptr};
  std::atomic<int32_t> fresh_T{0};
  std::atomic<void *> fresh_stream{nullptr};
  std::atomic<int32_t> fresh_reverse{0};  // ... and whether that dispatch took the tokens backwards
  // A dispatch into the buffer of the previous dispatch starts at the other end of the token range:
  // the rows touched last in the previous step (written last, then read through the cache by the
  // combine) are the ones the memory-side cache still holds, and they are overwritten in place
  // instead of being pushed out by the first rows of a dispatch that starts at the far end.
  std::atomic<const void *> last_recv{nullptr};
  std::atomic<int32_t> last_reverse{0};
  uint64_t timeout_ns = 0;
};

namespace ep {

inline int dev_err(const ep_handle *h) {
  return h->dev_error ? __atomic_load_n(h->dev_error, __ATOMIC_RELAXED) : 0;
}

// Body of one proxy thread: polls the FIFO channels it owns until the handle is stopped.
void proxy_main(ep_handle *h, ProxyThread *P);

}  // namespace ep
#endif  // EP_HOST_H_
