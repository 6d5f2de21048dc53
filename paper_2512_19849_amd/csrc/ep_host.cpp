// Host side of libep.so: the handle, the pinned-host FIFO channels, the
// multithreaded CPU proxy (sender half + receiver half in one process, since
// the peer ranks are partitions of this GPU's memory) and the C ABI.
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
#include <mutex>
#include <new>
#include <thread>
#include <vector>

#include "ep_internal.h"

namespace ep {
namespace {

// Text of the most recent failure on this thread (ep_last_error).
thread_local char g_last_error[256] = "";

bool hip_ok(hipError_t e, const char *what) {
  if (e == hipSuccess) return true;
  snprintf(g_last_error, sizeof(g_last_error), "%s: %s (%d)", what, hipGetErrorString(e), (int)e);
  return false;
}
#define HIP_OK(call) hip_ok((call), #call)

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
  std::vector<std::map<uint32_t, WireEvent>> early;
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
  std::vector<std::map<uint32_t, WireEvent>> ring_early;
  uint64_t rng = 0;
  // statistics (written by the owner thread only, read racy-but-atomically)
  std::atomic<uint64_t> cmds{0}, writes{0}, atomics{0}, drains{0}, write_bytes{0}, write_rows{0},
      applied{0}, deferred{0}, rejected{0}, first_poll_ns{0}, last_apply_ns{0}, ordered_parked{0}, barriers{0},
      copy_batches{0}, copied_bytes{0}, write_msgs{0}, paced{0}, max_in_flight{0}, sender_held{0};
  std::mutex log_mu;
  std::vector<uint32_t> cmd_log, event_log;
};

}  // namespace
}  // namespace ep

using namespace ep;

struct ep_handle {
  ep_config cfg{};
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
  RingDev ring{};
  int32_t *tile_hist = nullptr, *tile_base = nullptr, *chunk_cnt = nullptr, *expert_done = nullptr;
  unsigned *ticket = nullptr, *waves_done = nullptr, *ht_seq = nullptr;
  int ntiles_cap = 0, chunks_per_expert = 0;
  // host-only producer state
  std::atomic<uint64_t> host_tail[kMaxChannels];
  std::atomic<uint64_t> host_stalls{0};
  // proxy
  std::atomic<bool> stop{false};
  std::atomic<int64_t> expected_atomics{0};
  std::atomic<int> proxy_error{0};
  int nthreads = 0;
  ProxyThread *threads = nullptr;
  uint64_t timeout_ns = 0;
};

namespace {

inline int dev_err(const ep_handle *h) {
  return h->dev_error ? __atomic_load_n(h->dev_error, __ATOMIC_RELAXED) : 0;
}

void log_event(ep_handle *h, ProxyThread &P, uint32_t kind, uint32_t src, uint32_t e, uint32_t val) {
  if (!(h->cfg.flags & EP_FLAG_LOG_EVENTS)) return;
  std::lock_guard<std::mutex> g(P.log_mu);
  P.event_log.insert(P.event_log.end(), {kind | ((uint32_t)P.tid << 8), src, e, val});
}

void release_sender_parked(ep_handle *h, ProxyThread &P, uint32_t src, uint32_t dr, uint32_t le, size_t key);

void apply_atomic(ep_handle *h, ProxyThread &P, uint32_t src, uint32_t e, int32_t value) {
  const size_t key = (size_t)src * h->cfg.num_experts + e;
  P.seen[key] -= value;
  // completion counter in pinned host memory, visible to the GPU (Section 4.1)
  __atomic_store_n(&h->recv_count[key], value, __ATOMIC_RELEASE);
  __atomic_store_n(&h->recv_flag[key], value + 1, __ATOMIC_RELEASE);
  log_event(h, P, 3, src, e, (uint32_t)value);
  P.last_apply_ns.store(now_ns(), std::memory_order_relaxed);
  P.applied.store(P.applied.load(std::memory_order_relaxed) + 1, std::memory_order_release);
  if (!P.sender_parked.empty()) {  // sender-side fence: the next Atomic of this expert may go now
    P.atomic_flying[key] = 0;
    if (!P.sender_parked[key].empty())
      release_sender_parked(h, P, src, e / (uint32_t)h->E_loc, e % (uint32_t)h->E_loc, key);
  }
}

// Receiver half: interpret one immediate.  Writes have already landed; they
// only advance the per-(source, expert) arrival count.  An Atomic is applied
// only when that count has reached its value, otherwise it waits in the
// control buffer; arrivals for other experts never release it (Section 3.3,
// "partial completion fence").
void send_msg(ep_handle *h, ProxyThread &P, const Outbound &m);
void release_sender_parked(ep_handle *h, ProxyThread &P, uint32_t src, uint32_t dr, uint32_t le, size_t key);
void deliver_ordered(ep_handle *h, ProxyThread &P, const WireEvent &ev);
void deliver_ring(ep_handle *h, ProxyThread &P, const WireEvent &ev);

void deliver(ep_handle *h, ProxyThread &P, const WireEvent &ev) {
  --P.in_flight[ev.dst_rank];  // the message has arrived: room for the next one to this rank
  if (ev.ordered >= 2) {
    deliver_ring(h, P, ev);
    return;
  }
  if (ev.ordered) {
    deliver_ordered(h, P, ev);
    return;
  }
  const uint32_t le = (ev.imm >> 19) & 0xFFFu;
  const uint32_t e = (uint32_t)ev.dst_rank * h->E_loc + le;
  const size_t key = (size_t)ev.src * h->cfg.num_experts + e;
  if (!(ev.imm >> 31)) {
    const int32_t rows = (int32_t)((ev.imm >> 13) & 0x3Fu) + 1;
    P.seen[key] += rows;
    log_event(h, P, 1, ev.src, e, (uint32_t)rows);
    // sender-side fence: this arrival is also the completion the sender half was waiting for
    if (!P.sender_parked.empty() && !P.sender_parked[key].empty())
      release_sender_parked(h, P, ev.src, ev.dst_rank, le, key);
    std::deque<int32_t> &q = P.parked[key];
    while (!q.empty() && P.seen[key] >= q.front()) {
      const int32_t v = q.front();
      q.pop_front();
      apply_atomic(h, P, ev.src, e, v);
    }
  } else {
    const int32_t value = (int32_t)(ev.imm & 0x7FFFFu);
    log_event(h, P, 2, ev.src, e, (uint32_t)value);
    std::deque<int32_t> &q = P.parked[key];
    if (q.empty() && P.seen[key] >= value) {
      apply_atomic(h, P, ev.src, e, value);
    } else {
      q.push_back(value);
      bump(P.deferred, 1);
    }
  }
}

// Receiver half, sequenced messages (Section 3.3, "partial ordering"): the immediate carries the low
// 16 bits of the communication channel's sequence number,
//   [31] kind (0 Write, 1 Atomic)  [30:15] sequence & 0xFFFF  [14:0] rows (Write) / value (Atomic).
// A message whose number is not the next one of its channel waits in the control buffer; when the
// missing ones arrive, the buffered ones are applied one after the other, in sequence.  Order is
// kept per channel only: other channels never hold a message back.
void apply_ordered(ep_handle *h, ProxyThread &P, size_t chan, const WireEvent &ev, uint32_t seq) {
  const uint32_t value = ev.imm & 0x7FFFu;
  if (ev.imm >> 31) {
    const int32_t now = __atomic_load_n(&h->recv_tail[chan], __ATOMIC_RELAXED) + (int32_t)value;
    __atomic_store_n(&h->recv_tail[chan], now, __ATOMIC_RELEASE);
    log_event(h, P, 7, ev.src, ev.dst_rank, seq);
    P.last_apply_ns.store(now_ns(), std::memory_order_relaxed);
  } else {
    log_event(h, P, 6, ev.src, ev.dst_rank, seq);
  }
}

void deliver_ordered(ep_handle *h, ProxyThread &P, const WireEvent &ev) {
  const size_t chan = (size_t)ev.src * h->cfg.num_ranks + ev.dst_rank;
  uint32_t &next = P.next_seq[chan];
  // rebuild the full number from its low 16 bits: it lies within +-32768 of the next expected one
  uint32_t seq = (next & ~0xFFFFu) | ((ev.imm >> 15) & 0xFFFFu);
  if (seq + 0x8000u < next) seq += 0x10000u;
  else if (seq >= next + 0x8000u && seq >= 0x10000u) seq -= 0x10000u;
  log_event(h, P, (ev.imm >> 31) ? 5 : 4, ev.src, ev.dst_rank, seq);
  if (seq != next) {
    P.early[chan].emplace(seq, ev);
    bump(P.ordered_parked, 1);
    return;
  }
  apply_ordered(h, P, chan, ev, seq);
  ++next;
  std::map<uint32_t, WireEvent> &q = P.early[chan];
  for (auto it = q.find(next); it != q.end(); it = q.find(next)) {
    apply_ordered(h, P, chan, it->second, next);
    q.erase(it);
    ++next;
  }
}

// Ring-buffer channels (Section 3.3): the same in-sequence rule per channel (source, slice,
// destination rank) and direction.  A tail Atomic adds its rows to the counter the receiving kernel
// polls, a head Atomic to the one the sending kernel polls; a Write only takes its turn.
inline uint32_t rebuild_seq(uint32_t next, uint32_t low16) {
  uint32_t seq = (next & ~0xFFFFu) | low16;
  if (seq + 0x8000u < next) seq += 0x10000u;
  else if (seq >= next + 0x8000u && seq >= 0x10000u) seq -= 0x10000u;
  return seq;
}

void apply_ring(ep_handle *h, ProxyThread &P, size_t chan, const WireEvent &ev, uint32_t seq) {
  const uint32_t value = ev.imm & 0x7FFFu;
  const uint32_t where = ((uint32_t)ev.slice << 8) | ev.dst_rank;
  if (!(ev.imm >> 31)) {
    log_event(h, P, 11, ev.src, where, seq);
    return;
  }
  int32_t *ctr = (ev.ordered == 2 ? h->ring_tail : h->ring_head) + chan;
  __atomic_store_n(ctr, __atomic_load_n(ctr, __ATOMIC_RELAXED) + (int32_t)value, __ATOMIC_RELEASE);
  log_event(h, P, ev.ordered == 2 ? 12 : 13, ev.src, where, seq);
  P.last_apply_ns.store(now_ns(), std::memory_order_relaxed);
}

void deliver_ring(ep_handle *h, ProxyThread &P, const WireEvent &ev) {
  const ep_config &c = h->cfg;
  const size_t chan = ((size_t)ev.src * c.ht_slices + ev.slice) * c.num_ranks + ev.dst_rank;
  const size_t dir = chan * 2 + (ev.ordered == 3);
  uint32_t &next = P.ring_next[dir];
  const uint32_t seq = rebuild_seq(next, (ev.imm >> 15) & 0xFFFFu);
  const uint32_t where = ((uint32_t)ev.slice << 8) | ev.dst_rank;
  log_event(h, P, ev.ordered == 3 ? 10 : ((ev.imm >> 31) ? 9 : 8), ev.src, where, seq);
  if (seq != next) {
    P.ring_early[dir].emplace(seq, ev);
    bump(P.ordered_parked, 1);
    return;
  }
  apply_ring(h, P, chan, ev, seq);
  ++next;
  std::map<uint32_t, WireEvent> &q = P.ring_early[dir];
  for (auto it = q.find(next); it != q.end(); it = q.find(next)) {
    apply_ring(h, P, chan, it->second, next);
    q.erase(it);
    ++next;
  }
}

// The "network" between the two halves.  With reorder_window == 0 immediates
// arrive in the order they were sent; otherwise up to reorder_window of them
// are in flight and a seeded draw decides which arrives next (an unordered
// transport such as the one Section 2.4 describes).
void transmit(ep_handle *h, ProxyThread &P, const WireEvent &ev) {
  const int W = h->cfg.reorder_window;
  if (W <= 0) {
    deliver(h, P, ev);
    return;
  }
  P.window.push_back(ev);
  if ((int)P.window.size() > W) {
    const size_t i = (size_t)(mix64(P.rng) % P.window.size());
    const WireEvent out = P.window[i];
    P.window[i] = P.window.back();
    P.window.pop_back();
    deliver(h, P, out);
  }
}

void flush_window(ep_handle *h, ProxyThread &P) {
  while (!P.window.empty()) {
    const size_t i = (size_t)(mix64(P.rng) % P.window.size());
    const WireEvent out = P.window[i];
    P.window[i] = P.window.back();
    P.window.pop_back();
    deliver(h, P, out);
  }
}

// ---- peer writes performed by the proxy ------------------------------------------------------
void fail_hip(ep_handle *h) {
  int zero = 0;
  h->proxy_error.compare_exchange_strong(zero, EP_EHIP);
}

// Hands the batch being filled to the device: one copy kernel on this thread's stream, an event
// behind it.  Its notices stay with the batch until the event has fired.
void launch_batch(ep_handle *h, ProxyThread &P) {
  if (P.cur.n == 0) return;
  P.cur.descs = P.d_descs + (size_t)P.cur_slot * kCopyBatchMax;
  P.cur.host_descs = P.descs + (size_t)P.cur_slot * kCopyBatchMax;
  {
    std::lock_guard<std::mutex> g(h->copy_mu);  // launch and event stay adjacent in the shared stream
    if (launch_copy_batch(P.cur, h->copy_stream) != 0 ||
        hipEventRecord(P.events[P.cur_slot], h->copy_stream) != hipSuccess)
      fail_hip(h);
  }
  bump(P.copy_batches, 1);
  P.inflight.push_back(ProxyThread::Batch{P.cur_slot, std::move(P.cur_notices)});
  P.cur_notices.clear();
  P.cur.n = 0;
  P.cur.max_len16 = 0;
  P.cur_slot = (P.cur_slot + 1) % ProxyThread::kBatchSlots;
}

// Completion polling (the stand-in for polling the send completion queue): batches finish in
// order; a finished batch releases its arrival notices to the receiver half.
enum ReapMode { kReapReady, kReapOne, kReapAll };
void reap_batches(ep_handle *h, ProxyThread &P, ReapMode mode) {
  while (!P.inflight.empty()) {
    ProxyThread::Batch &b = P.inflight.front();
    hipError_t e = mode == kReapReady ? hipEventQuery(P.events[b.slot]) : hipEventSynchronize(P.events[b.slot]);
    if (e == hipErrorNotReady) return;
    if (e != hipSuccess) fail_hip(h);
    for (const WireEvent &ev : b.notices) transmit(h, P, ev);
    P.inflight.pop_front();
    if (mode == kReapOne) return;
  }
}

// Offsets and length are bytes relative to the registered heaps, multiples of 16 below 64 GiB.
void queue_copy(ep_handle *h, ProxyThread &P, const char *sbase, char *dbase, uint64_t so, uint64_t dof,
                uint64_t len, const WireEvent *notice) {
  if (P.cur.n && (P.cur.src_base != sbase || P.cur.dst_base != dbase)) launch_batch(h, P);  // re-registered
  // the event about to be used must not belong to a batch still in flight
  while (P.cur.n == 0 && (int)P.inflight.size() >= ProxyThread::kBatchSlots - 1) reap_batches(h, P, kReapOne);
  P.cur.src_base = sbase;
  P.cur.dst_base = dbase;
  P.descs[(size_t)P.cur_slot * kCopyBatchMax + P.cur.n] =
      CopyDesc{(unsigned)(so >> 4), (unsigned)(dof >> 4), (unsigned)(len >> 4)};
  if (notice) P.cur_notices.push_back(*notice);
  if ((unsigned)(len >> 4) > P.cur.max_len16) P.cur.max_len16 = (unsigned)(len >> 4);
  bump(P.copied_bytes, len);
  if (++P.cur.n == kCopyBatchMax) launch_batch(h, P);
}

// ---- pacing (Section 6, "Congestion control with CPU proxy") ------------------------------------
// The proxy tracks the requests it has outstanding per destination and keeps further ones at the
// sender until earlier ones have arrived, so that a burst cannot pile up at one receiver.
void launch_msg(ep_handle *h, ProxyThread &P, const Outbound &m) {
  const uint32_t dr = m.notice.dst_rank;
  const int32_t now = ++P.in_flight[dr];
  if ((uint64_t)now > P.max_in_flight.load(std::memory_order_relaxed)) P.max_in_flight.store((uint64_t)now);
  log_event(h, P, 14, m.notice.src, dr, (uint32_t)now);
  if (m.nseg == 0) {
    transmit(h, P, m.notice);
    return;
  }
  // the notice rides on the last segment's copy: a batch completes as a whole, in order
  for (uint32_t i = 0; i < m.nseg; ++i)
    queue_copy(h, P, m.sbase, m.dbase, m.so[i], m.dof + i * m.seglen, m.seglen, i + 1 == m.nseg ? &m.notice : nullptr);
}

void send_msg(ep_handle *h, ProxyThread &P, const Outbound &m) {
  const int limit = h->cfg.max_outstanding;
  const uint32_t dr = m.notice.dst_rank;
  if (limit > 0 && (P.in_flight[dr] >= limit || !P.held[dr].empty())) {
    P.held[dr].push_back(m);  // keeps the order of messages to one destination
    ++P.held_total;
    bump(P.paced, 1);
    return;
  }
  launch_msg(h, P, m);
}

// Sender-side fence (the alternative weighed in Section 3.3, "Where to enforce the delivery
// semantics"): a count Atomic leaves only when the rows it vouches for have completed.  Sender and
// receiver halves share the arrival counts, so "completed" is the arrival of the rows' notices.
void release_sender_parked(ep_handle *h, ProxyThread &P, uint32_t src, uint32_t dr, uint32_t le, size_t key) {
  std::deque<int32_t> &q = P.sender_parked[key];
  // one Atomic per expert on its way at a time: the next one's rows are counted after this one has
  // been applied (it takes its rows off the arrival count)
  if (q.empty() || P.atomic_flying[key] || P.seen[key] < q.front()) return;
  const int32_t value = q.front();
  q.pop_front();
  P.atomic_flying[key] = 1;
  Outbound m;
  m.notice = WireEvent{(1u << 31) | (le << 19) | (uint32_t)value, (uint16_t)src, (uint8_t)dr, 0};
  send_msg(h, P, m);
}

// Lets waiting messages go wherever arrivals have made room.
void pump_held(ep_handle *h, ProxyThread &P) {
  if (!P.held_total) return;
  const int limit = h->cfg.max_outstanding;
  for (size_t dr = 0; dr < P.held.size(); ++dr) {
    std::deque<Outbound> &q = P.held[dr];
    while (!q.empty() && P.in_flight[dr] < limit) {
      const Outbound m = q.front();
      q.pop_front();
      --P.held_total;
      launch_msg(h, P, m);
    }
  }
}

// ---- best-effort packing of per-token Writes (Section 6, "More efficient low-latency kernel") ---
void close_open(ep_handle *h, ProxyThread &P, size_t slot) {
  Outbound m = P.open[slot];
  const uint32_t key = P.open_key[slot];
  P.open_idx[key] = -1;
  if (slot + 1 != P.open.size()) {
    P.open[slot] = P.open.back();
    P.open_key[slot] = P.open_key.back();
    P.open_idx[P.open_key[slot]] = (int32_t)slot;
  }
  P.open.pop_back();
  P.open_key.pop_back();
  const uint32_t rows = m.nseg;
  m.notice.imm = (m.le << 19) | ((rows - 1) << 13) | (uint32_t)((m.dof >> 4) & 0x1FFFu);
  if (!m.dbase) m.nseg = 0;  // rows already placed by the kernel: only the notice travels
  bump(P.write_msgs, 1);
  send_msg(h, P, m);
}

void close_all_open(ep_handle *h, ProxyThread &P) {
  while (!P.open.empty()) close_open(h, P, P.open.size() - 1);
}

// End of a poll sweep: open messages leave, unless they may still wait for more rows.
void close_due_open(ep_handle *h, ProxyThread &P) {
  const uint64_t hold = (uint64_t)h->cfg.pack_hold_us * 1000ull;
  if (!hold) {
    close_all_open(h, P);
    return;
  }
  const uint64_t now = now_ns();
  for (size_t i = P.open.size(); i-- > 0;)
    if (now - P.open[i].opened_ns >= hold) close_open(h, P, i);
}

void reject(ep_handle *h, ProxyThread &P) {
  bump(P.rejected, 1);
  int zero = 0;
  h->proxy_error.compare_exchange_strong(zero, EP_EBOUNDS);
}

// Sender half: one polled command.  Offsets are relative to the registered
// heap; the proxy translates and bounds-checks them before acting
// (Section 3.2, "Symmetric memory").
void process_cmd(ep_handle *h, ProxyThread &P, int fifo, uint32_t w0, uint32_t w1, uint32_t w2, uint32_t w3) {
  const ep_config &c = h->cfg;
  const uint32_t op = (w0 >> 28) & 7u, src = (w0 >> 20) & 0xFFu, dr = (w0 >> 12) & 0xFFu, le = w0 & 0xFFFu;
  bump(P.cmds, 1);
  if (P.first_poll_ns.load(std::memory_order_relaxed) == 0)
    P.first_poll_ns.store(now_ns(), std::memory_order_relaxed);
  if (c.flags & EP_FLAG_LOG_CMDS) {  // as polled, lap-parity bits included
    std::lock_guard<std::mutex> g(P.log_mu);
    P.cmd_log.insert(P.cmd_log.end(), {w0, w1, w2, w3});
  }
  w3 &= 0x7FFFFFFFu;
  switch (op) {
    case EP_OP_WRITE: {
      const uint64_t len = (uint64_t)(w1 & 0x3FFFFFFu) << 4;
      const uint32_t rows = (w1 >> 26) + 1;
      const uint64_t so = (uint64_t)w2 << 4, dof = (uint64_t)(w3 & 0x7FFFFFFFu) << 4;
      char *const dbase = h->dst_base.load(std::memory_order_acquire);
      const char *const sbase = h->src_base.load(std::memory_order_relaxed);
      // without registered heaps the source side is the larger of the send buffer a source may own
      // (max_tokens rows, per-token commands) and the receive heap (chunk commands: same offset on both sides)
      const uint64_t own = (uint64_t)c.max_tokens * 2ull * (uint64_t)c.hidden;
      const uint64_t slimit = dbase ? h->src_bytes : (own > h->heap_bytes ? own : h->heap_bytes);
      const uint64_t dlimit = dbase ? h->dst_bytes : h->heap_bytes;
      if ((int)src >= c.num_src || (int)dr >= c.num_ranks || (int)le >= h->E_loc || len == 0 ||
          so + len > slimit || dof + len > dlimit) {
        reject(h, P);
        return;
      }
      bump(P.writes, 1);
      bump(P.write_bytes, len);
      bump(P.write_rows, rows);
      // Without registered heaps the payload already sits in the destination partition (the kernel
      // stored it) and what remains of the peer write is its arrival notice; with them this thread
      // performs the write and the notice follows its completion.
      Outbound m;
      m.notice = WireEvent{(le << 19) | ((rows - 1) << 13) | (uint32_t)((dof >> 4) & 0x1FFFu), (uint16_t)src,
                           (uint8_t)dr, 0};
      m.nseg = dbase ? 1 : 0;
      m.seglen = len;
      m.dof = dof;
      m.so[0] = so;
      m.sbase = sbase;
      m.dbase = dbase;
      m.le = le;
      if (c.pack_rows > 1 && rows == 1) {
        // one-row Write: extend the open message of its expert if it continues it, else open one
        const uint32_t key = src * (uint32_t)c.num_experts + dr * (uint32_t)h->E_loc + le;
        int32_t slot = P.open_idx[key];
        if (slot >= 0) {
          Outbound &o = P.open[slot];
          if (o.dof + (uint64_t)o.nseg * o.seglen == dof && o.seglen == len && o.sbase == sbase && o.dbase == dbase) {
            o.so[o.nseg++] = so;
            if ((int)o.nseg == c.pack_rows) close_open(h, P, (size_t)slot);
            break;
          }
          close_open(h, P, (size_t)slot);
        }
        m.nseg = 1;  // counts the rows while the message is open
        if (c.pack_hold_us) m.opened_ns = now_ns();
        P.open_idx[key] = (int32_t)P.open.size();
        P.open.push_back(m);
        P.open_key.push_back(key);
        break;
      }
      bump(P.write_msgs, 1);
      send_msg(h, P, m);
      break;
    }
    case EP_OP_ATOMIC: {
      const uint32_t counter = w3 & 0x7FFFFFFFu;
      if ((int)src >= c.num_src || (int)dr >= c.num_ranks || (int)le >= h->E_loc || w1 > 0x7FFFFu ||
          counter != src * (uint32_t)h->E_loc + le) {
        reject(h, P);
        return;
      }
      bump(P.atomics, 1);
      if (c.pack_rows > 1) {  // rows of this expert still being packed leave before their count does
        const int32_t slot = P.open_idx[src * (uint32_t)c.num_experts + dr * (uint32_t)h->E_loc + le];
        if (slot >= 0) close_open(h, P, (size_t)slot);
      }
      if (c.flags & EP_FLAG_SENDER_FENCE) {
        const size_t key = (size_t)src * c.num_experts + (size_t)dr * h->E_loc + le;
        std::deque<int32_t> &q = P.sender_parked[key];
        if (!q.empty() || P.atomic_flying[key] || P.seen[key] < (int32_t)w1) {
          // rows still outstanding (or an earlier Atomic of this expert not applied yet): it waits here
          bump(P.sender_held, 1);
          log_event(h, P, 15, src, dr * (uint32_t)h->E_loc + le, w1);
        }
        q.push_back((int32_t)w1);
        release_sender_parked(h, P, src, dr, le, key);
        break;
      }
      Outbound m;
      m.notice = WireEvent{(1u << 31) | (le << 19) | w1, (uint16_t)src, (uint8_t)dr, 0};
      send_msg(h, P, m);
      break;
    }
    case EP_OP_ORDERED_WRITE: {
      const uint64_t len = (uint64_t)(w1 & 0x3FFFFFFu) << 4;
      const uint32_t rows = (w1 >> 26) + 1;
      const uint64_t dof = (uint64_t)w3 << 4;
      char *const dbase = h->dst_base.load(std::memory_order_acquire);
      const char *const sbase = h->src_base.load(std::memory_order_relaxed);
      const uint64_t limit = dbase ? (h->src_bytes < h->dst_bytes ? h->src_bytes : h->dst_bytes) : h->heap_bytes;
      if ((int)src >= c.num_src || (int)dr >= c.num_ranks || (int)le >= h->E_loc || len == 0 ||
          dof + len > limit) {
        reject(h, P);
        return;
      }
      bump(P.writes, 1);
      bump(P.write_bytes, len);
      bump(P.write_rows, rows);
      Outbound m;
      m.notice = WireEvent{((w2 & 0xFFFFu) << 15) | rows, (uint16_t)src, (uint8_t)dr, 1};
      m.nseg = dbase ? 1 : 0;  // packed chunk: same offset on both sides
      m.seglen = len;
      m.dof = m.so[0] = dof;
      m.sbase = sbase;
      m.dbase = dbase;
      bump(P.write_msgs, 1);
      send_msg(h, P, m);
      break;
    }
    case EP_OP_ORDERED_ATOMIC: {
      if ((int)src >= c.num_src || (int)dr >= c.num_ranks || w1 > 0x7FFFu ||
          w3 != src * (uint32_t)c.num_ranks + dr) {
        reject(h, P);
        return;
      }
      bump(P.atomics, 1);
      Outbound m;
      m.notice = WireEvent{(1u << 31) | ((w2 & 0xFFFFu) << 15) | w1, (uint16_t)src, (uint8_t)dr, 1};
      send_msg(h, P, m);
      break;
    }
    case EP_OP_RING: {
      const uint32_t kind = w1 >> 30, slice = le;
      if (c.ht_slices <= 0 || (int)src >= c.num_src || (int)dr >= c.num_ranks || (int)slice >= c.ht_slices ||
          kind > EP_RING_HEAD) {
        reject(h, P);
        return;
      }
      if (kind == EP_RING_WRITE) {
        const uint32_t rows = ((w1 >> 24) & 0x3Fu) + 1;
        const uint64_t len = (uint64_t)(w1 & 0xFFFFFFu) << 4, dof = (uint64_t)w3 << 4;
        // the slot must be one of this channel's own, and the length what its rows need
        const uint64_t first = ((uint64_t)slice * c.num_ranks + dr) * c.ht_ring_slots * h->ring_slot_bytes;
        const uint64_t rb8 = ((uint64_t)c.hidden + (uint64_t)c.hidden / 32u + 15u) / 16u * 16u;  // an FP8 row
        if (rows > (uint32_t)kChunkRows ||
            (len != 128u + (uint64_t)rows * 2u * c.hidden && len != 128u + (uint64_t)rows * rb8) || dof < first ||
            dof >= first + (uint64_t)c.ht_ring_slots * h->ring_slot_bytes || (dof - first) % h->ring_slot_bytes ||
            dof + len > h->ring_total_bytes) {
          reject(h, P);
          return;
        }
        bump(P.writes, 1);
        bump(P.write_bytes, len);
        bump(P.write_rows, rows);
        Outbound m;
        m.notice = WireEvent{((w2 & 0xFFFFu) << 15) | rows, (uint16_t)src, (uint8_t)dr, 2, (uint16_t)slice};
        bump(P.write_msgs, 1);
        send_msg(h, P, m);
      } else {
        const uint32_t value = w1 & 0x3FFFFFFFu;
        if (value > 0x7FFFu) {
          reject(h, P);
          return;
        }
        bump(P.atomics, 1);
        Outbound m;
        m.notice = WireEvent{(1u << 31) | ((w2 & 0xFFFFu) << 15) | value, (uint16_t)src, (uint8_t)dr,
                             (uint8_t)(kind == EP_RING_TAIL ? 2 : 3), (uint16_t)slice};
        send_msg(h, P, m);
      }
      break;
    }
    case EP_OP_DRAIN: {
      // everything this thread has taken over must have left and arrived: open packed messages,
      // copies in flight, messages in the transport, and those waiting for the pacing limit
      close_all_open(h, P);
      do {
        launch_batch(h, P);
        reap_batches(h, P, kReapAll);
        flush_window(h, P);
        pump_held(h, P);
      } while (P.held_total || P.cur.n || !P.inflight.empty() || !P.window.empty());
      // communication channels that travel through this FIFO (destination rank mod C == fifo) must
      // have nothing left waiting: a leftover means a sequence number never arrived
      for (int ss = 0; ss < c.num_src; ++ss)
        for (int r = fifo; r < c.num_ranks; r += c.num_channels)
          if (!P.early[(size_t)ss * c.num_ranks + r].empty()) {
            int zero = 0;
            h->proxy_error.compare_exchange_strong(zero, EP_ESTATE);
          }
      // ... and the ring-buffer channels of this FIFO ((slice * R + rank) mod C == fifo), both directions
      for (size_t ch = 0, n = P.ring_early.size() / 2; ch < n; ++ch)
        if ((int)((ch % ((size_t)c.ht_slices * c.num_ranks)) % c.num_channels) == fifo &&
            (!P.ring_early[2 * ch].empty() || !P.ring_early[2 * ch + 1].empty())) {
          int zero = 0;
          h->proxy_error.compare_exchange_strong(zero, EP_ESTATE);
        }
      P.drains.store(P.drains.load(std::memory_order_relaxed) + 1, std::memory_order_release);
      break;
    }
    case EP_OP_BARRIER: {
      // All-peer barrier, intra-node level: peers meet at a counter in shared memory; the one that
      // completes the count opens the next generation.  The command is popped (and the GPU's
      // Check-completion turns true) only after the barrier is established.
      const uint32_t peers = c.barrier_peers > 1 ? (uint32_t)c.barrier_peers : 1u;
      ep_handle::SharedBarrier *b = h->barrier;
      const uint32_t gen = b->generation.load(std::memory_order_acquire);
      if (b->arrived.fetch_add(1, std::memory_order_acq_rel) + 1 == peers) {
        b->arrived.store(0, std::memory_order_relaxed);
        b->generation.fetch_add(1, std::memory_order_release);
      } else {
        const uint64_t t0 = now_ns();
        uint64_t spins = 0;
        while (b->generation.load(std::memory_order_acquire) == gen) {
          if ((++spins & 255) == 0) {
            if (now_ns() - t0 > h->timeout_ns || h->stop.load(std::memory_order_relaxed)) {
              int zero = 0;
              h->proxy_error.compare_exchange_strong(zero, EP_ETIMEOUT);
              break;
            }
            std::this_thread::yield();
          } else {
            _mm_pause();
          }
        }
      }
      bump(P.barriers, 1);
      break;
    }
    default:
      reject(h, P);
      break;
  }
}

void proxy_main(ep_handle *h, ProxyThread *Pp) {
  ProxyThread &P = *Pp;
  const uint32_t mask = h->entries - 1;
  if (!h->host_only && hipSetDevice(h->device) != hipSuccess) fail_hip(h);
  uint64_t idle = 0;
  uint64_t idle_since = 0;
  while (!h->stop.load(std::memory_order_acquire)) {
    bool any = false;
    for (size_t ci = 0; ci < P.channels.size(); ++ci) {
      const int ch = P.channels[ci];
      uint64_t hd = P.head[ci];
      int n = 0;
      while (n < 256) {
        // Poll: a slot is ready when both lap-parity bits match the lap we are on.
        const uint64_t *slot = h->slots + ((size_t)ch * h->entries + (hd & mask)) * 2;
        const uint64_t lo = __atomic_load_n(slot, __ATOMIC_ACQUIRE);
        const uint64_t hi = __atomic_load_n(slot + 1, __ATOMIC_ACQUIRE);
        const uint32_t gen = (((uint32_t)(hd >> h->log2_entries)) & 1u) ^ 1u;
        const uint32_t w0 = (uint32_t)lo, w3 = (uint32_t)(hi >> 32);
        if ((w0 >> 31) != gen || (w3 >> 31) != gen) break;
        process_cmd(h, P, ch, w0, (uint32_t)(lo >> 32), (uint32_t)hi, w3);
        ++hd;
        ++n;
      }
      if (n) {
        // Pop: publish the new head where the GPU can read it
        P.head[ci] = hd;
        __atomic_store_n(&h->head[(size_t)ch * kHeadStride], hd, __ATOMIC_RELEASE);
        any = true;
      }
    }
    // best-effort packing never keeps a Write beyond the sweep that polled it
    if (!P.open.empty()) {
      close_due_open(h, P);
      if (!P.open.empty()) any = true;  // keep sweeping: the open messages have a deadline
    }
    // What has been collected goes out as one batch of peer writes - at once when nothing new came in,
    // else when it is worth a launch of its own (launches on the shared stream run one after the other,
    // ~10 us apart: during a burst few large batches beat many small ones); finished batches release
    // their arrival notices.
    if (P.cur.n && (!any || P.cur.n >= 2048)) launch_batch(h, P);
    if (!P.inflight.empty()) {
      reap_batches(h, P, kReapReady);
      any = true;
    }
    if (P.held_total) {
      // messages wait for room: let what is in the transport arrive, then send what fits
      flush_window(h, P);
      pump_held(h, P);
    }
    if (any) {
      idle = 0;
      continue;
    }
    if (!P.window.empty()) flush_window(h, P);  // nothing new: let in-flight immediates land
    if (P.held_total) continue;
    if (++idle < 4096) {
      _mm_pause();
    } else if (idle == 4096) {
      idle_since = now_ns();
      std::this_thread::yield();
    } else if (now_ns() - idle_since < 20000000ull) {
      std::this_thread::yield();
    } else {
      timespec ts{0, 50000};
      nanosleep(&ts, nullptr);
    }
  }
}

bool is_pow2(uint32_t v) { return v && !(v & (v - 1)); }

int validate(const ep_config &c) {
  if (c.num_ranks < 1 || c.num_ranks > 256) return EP_EINVAL;
  if (c.num_experts < 1 || c.num_experts > kMaxExperts || c.num_experts % c.num_ranks) return EP_EINVAL;
  if (c.top_k < 1 || c.top_k > 64) return EP_EINVAL;
  if (c.hidden < 128 || c.hidden % 128 || c.hidden > 65536) return EP_EINVAL;
  if (c.max_tokens < 1 || c.max_tokens >= (1 << 19)) return EP_EINVAL;
  if (c.num_src < 1 || c.num_src > 256) return EP_EINVAL;
  if (c.self_rank < 0 || c.self_rank >= c.num_ranks) return EP_EINVAL;
  if (c.num_channels < 1 || c.num_channels > kMaxChannels) return EP_EINVAL;
  if (c.ring_entries < 2 || c.ring_entries > (1 << 20) || !is_pow2((uint32_t)c.ring_entries)) return EP_EINVAL;
  if (c.num_proxy_threads < 0 || c.num_proxy_threads > kMaxThreads) return EP_EINVAL;
  // sequenced messages carry 16 bits of their number: a message must not be overtaken by 32768 or
  // more of its own channel, which a window of this size cannot do
  if (c.reorder_window < 0 || c.reorder_window > 16384) return EP_EINVAL;
  if (c.spin_timeout_ms < 0 || c.spin_timeout_ms > 60000) return EP_EINVAL;
  if (c.heap_rows < 0) return EP_EINVAL;
  if (c.barrier_peers < 0 || c.barrier_peers > 1024) return EP_EINVAL;
  if (memchr(c.barrier_name, 0, sizeof(c.barrier_name)) == nullptr) return EP_EINVAL;
  for (const char *p = c.barrier_name; *p; ++p)
    if (*p == '/') return EP_EINVAL;
  if (c.barrier_peers > 1 && !c.barrier_name[0]) return EP_EINVAL;
  if (c.max_outstanding < 0 || c.max_outstanding > (1 << 20) || c.pack_rows < 0 || c.pack_rows > kMaxPackRows ||
      c.pack_hold_us < 0 || c.pack_hold_us > 1000)
    return EP_EINVAL;
  if (c.ht_slices < 0 || c.ht_slices > 4096 || c.ht_ring_slots < 0 || c.ht_ring_slots > 64) return EP_EINVAL;
  if ((c.ht_slices > 0) != (c.ht_ring_slots > 0)) return EP_EINVAL;
  if (c.ht_slices > 0 && ((int64_t)c.num_ranks * c.ht_ring_slots > 4096 || c.num_proxy_threads < 1)) return EP_EINVAL;
  return EP_OK;
}

void free_all(ep_handle *h) {
  if (!h) return;
  if (h->host_only) {
    free(h->slots);
    free(h->head);
    free(h->recv_count);
    free(h->recv_flag);
    free(h->recv_tail);
    free(h->ring_tail);
    free(h->ring_head);
    free(h->dev_error);
  } else {
    if (h->slots) (void)hipHostFree(h->slots);
    if (h->head) (void)hipHostFree(h->head);
    if (h->recv_count) (void)hipHostFree(h->recv_count);
    if (h->recv_flag) (void)hipHostFree(h->recv_flag);
    if (h->recv_tail) (void)hipHostFree(h->recv_tail);
    if (h->ring_tail) (void)hipHostFree(h->ring_tail);
    if (h->ring_head) (void)hipHostFree(h->ring_head);
    if (h->dev_error) (void)hipHostFree(h->dev_error);
    void *dev[] = {h->ring.tail, h->ring.cached_head, h->ring.stalls, h->ring.refresh_lock, h->tile_hist, h->tile_base,
                   h->chunk_cnt, h->expert_done, h->ticket, h->waves_done, h->ht_seq,
                   h->ring_seq_fwd, h->ring_seq_rev, h->ring_cum_fwd, h->ring_cum_rev};
    for (void *p : dev)
      if (p) (void)hipFree(p);
  }
  if (h->barrier_is_shm && h->barrier) {
    munmap(h->barrier, sizeof(ep_handle::SharedBarrier));
    shm_unlink(h->barrier_path);  // the name goes; peers that still map the segment keep it
  }
  delete[] h->threads;
  delete h;
}

template <class T>
int pinned_alloc(bool host_only, T **p, size_t bytes) {
  if (host_only) {
    *p = (T *)aligned_alloc(64, (bytes + 63) / 64 * 64);
    if (!*p) return EP_ENOMEM;
  } else {
    void *q = nullptr;
    if (!HIP_OK(hipHostMalloc(&q, bytes, hipHostMallocMapped | hipHostMallocCoherent))) return EP_ENOMEM;
    *p = (T *)q;
  }
  memset(*p, 0, bytes);
  return EP_OK;
}

template <class T>
int dev_alloc_zero(T **p, size_t bytes) {
  void *q = nullptr;
  if (!HIP_OK(hipMalloc(&q, bytes))) return EP_ENOMEM;
  if (!HIP_OK(hipMemset(q, 0, bytes))) return EP_EHIP;
  *p = (T *)q;
  return EP_OK;
}

}  // namespace

extern "C" {

int ep_proxy_start(const ep_config *cfg, ep_handle **out) {
  if (!cfg || !out) return EP_EINVAL;
  *out = nullptr;
  int rc = validate(*cfg);
  if (rc) return rc;
  ep_handle *h = new (std::nothrow) ep_handle();
  if (!h) return EP_ENOMEM;
  h->cfg = *cfg;
  h->host_only = (cfg->flags & EP_FLAG_HOST_ONLY) != 0;
  h->E_loc = cfg->num_experts / cfg->num_ranks;
  if (h->cfg.heap_rows == 0) h->cfg.heap_rows = (int64_t)cfg->num_src * cfg->max_tokens * cfg->top_k;
  h->heap_bytes = (uint64_t)h->cfg.heap_rows * 2ull * (uint64_t)cfg->hidden;
  if ((h->heap_bytes >> 4) >= (1ull << 31)) {
    delete h;
    return EP_EINVAL;  // destination offsets are 31 bits of 16-byte units
  }
  h->entries = (uint32_t)cfg->ring_entries;
  while ((1u << h->log2_entries) < h->entries) ++h->log2_entries;
  const int ms = cfg->spin_timeout_ms ? cfg->spin_timeout_ms : 5000;
  h->timeout_ns = (uint64_t)ms * 1000000ull;
  for (auto &t : h->host_tail) t.store(0);
  const int C = cfg->num_channels, S = cfg->num_src, E = cfg->num_experts;

  if (!h->host_only) {
    int ndev = 0;
    if (!HIP_OK(hipGetDeviceCount(&ndev)) || ndev < 1 || !HIP_OK(hipGetDevice(&h->device))) {
      delete h;
      return EP_EHIP;
    }
  }
  rc = pinned_alloc(h->host_only, &h->slots, (size_t)C * h->entries * 16);
  if (!rc) rc = pinned_alloc(h->host_only, &h->head, (size_t)C * kHeadStride * 8);
  if (!rc) rc = pinned_alloc(h->host_only, &h->recv_count, (size_t)S * E * 4);
  if (!rc) rc = pinned_alloc(h->host_only, &h->recv_flag, (size_t)S * E * 4);
  if (!rc) rc = pinned_alloc(h->host_only, &h->recv_tail, (size_t)S * cfg->num_ranks * 4);
  if (!rc) rc = pinned_alloc(h->host_only, &h->dev_error, 64);
  const size_t nring = (size_t)S * cfg->ht_slices * cfg->num_ranks;
  h->ring_slot_bytes = 128u + (uint64_t)kChunkRows * 2u * cfg->hidden;
  h->ring_total_bytes = (uint64_t)cfg->ht_slices * cfg->num_ranks * cfg->ht_ring_slots * h->ring_slot_bytes;
  if (!rc && nring) rc = pinned_alloc(h->host_only, &h->ring_tail, nring * 4);
  if (!rc && nring) rc = pinned_alloc(h->host_only, &h->ring_head, nring * 4);
  if (!rc && !h->host_only) {
    h->ntiles_cap = (cfg->max_tokens + kLayoutTile - 1) / kLayoutTile;
    h->chunks_per_expert = (cfg->max_tokens + kChunkRows - 1) / kChunkRows;
    const size_t hist = ((size_t)S * h->ntiles_cap + 1) * E * 4;
    rc = dev_alloc_zero(&h->ring.tail, (size_t)C * 8);
    if (!rc) rc = dev_alloc_zero(&h->ring.cached_head, (size_t)C * 8);
    if (!rc) rc = dev_alloc_zero(&h->ring.stalls, 8);
    if (!rc) rc = dev_alloc_zero(&h->ring.refresh_lock, (size_t)C * 4);
    if (!rc) rc = dev_alloc_zero(&h->tile_hist, hist);
    if (!rc) rc = dev_alloc_zero(&h->tile_base, hist);
    if (!rc) rc = dev_alloc_zero(&h->chunk_cnt, (size_t)E * h->chunks_per_expert * 4);
    if (!rc) rc = dev_alloc_zero(&h->expert_done, (size_t)E * 4);
    if (!rc) rc = dev_alloc_zero(&h->ticket, 4);
    if (!rc) rc = dev_alloc_zero(&h->waves_done, 4);
    if (!rc) rc = dev_alloc_zero(&h->ht_seq, (size_t)S * cfg->num_ranks * 4);
    if (nring) {
      if (!rc) rc = dev_alloc_zero(&h->ring_seq_fwd, nring * 4);
      if (!rc) rc = dev_alloc_zero(&h->ring_seq_rev, nring * 4);
      if (!rc) rc = dev_alloc_zero(&h->ring_cum_fwd, nring * 4);
      if (!rc) rc = dev_alloc_zero(&h->ring_cum_rev, nring * 4);
      if (!rc && !HIP_OK(hipHostGetDevicePointer(&h->d_ring_tail, h->ring_tail, 0))) rc = EP_EHIP;
      if (!rc && !HIP_OK(hipHostGetDevicePointer(&h->d_ring_head, h->ring_head, 0))) rc = EP_EHIP;
    }
    void *dp = nullptr;
    if (!rc && !HIP_OK(hipHostGetDevicePointer(&dp, h->slots, 0))) rc = EP_EHIP;
    h->ring.slots = dp;
    if (!rc && !HIP_OK(hipHostGetDevicePointer(&dp, h->head, 0))) rc = EP_EHIP;
    h->ring.head = (const unsigned long long *)dp;
    if (!rc && !HIP_OK(hipHostGetDevicePointer(&dp, h->dev_error, 0))) rc = EP_EHIP;
    h->ring.error = (int *)dp;
    if (!rc && !HIP_OK(hipHostGetDevicePointer(&h->d_recv_count, h->recv_count, 0))) rc = EP_EHIP;
    if (!rc && !HIP_OK(hipHostGetDevicePointer(&h->d_recv_flag, h->recv_flag, 0))) rc = EP_EHIP;
    h->ring.entries = h->entries;
    h->ring.log2_entries = h->log2_entries;
    h->ring.channels = (unsigned)C;
    h->ring.timeout_ticks = (unsigned long long)ms * 100000ull;  // wall_clock64 runs at 100 MHz
    if (!rc && !HIP_OK(hipDeviceSynchronize())) rc = EP_EHIP;
  }
  if (rc) {
    free_all(h);
    return rc;
  }

  h->barrier = &h->private_barrier;
  if (cfg->barrier_peers > 1) {
    snprintf(h->barrier_path, sizeof(h->barrier_path), "/ep_barrier_%s", cfg->barrier_name);
    const int fd = shm_open(h->barrier_path, O_CREAT | O_RDWR, 0600);
    void *m = MAP_FAILED;
    if (fd >= 0 && ftruncate(fd, 64) == 0)  // a fresh segment is zero-filled: count 0, generation 0
      m = mmap(nullptr, sizeof(ep_handle::SharedBarrier), PROT_READ | PROT_WRITE, MAP_SHARED, fd, 0);
    if (fd >= 0) close(fd);
    if (m == MAP_FAILED) {
      snprintf(g_last_error, sizeof(g_last_error), "shared-memory barrier %s could not be mapped", h->barrier_path);
      free_all(h);
      return EP_ENOMEM;
    }
    h->barrier = (ep_handle::SharedBarrier *)m;
    h->barrier_is_shm = true;
  }
  h->nthreads = cfg->num_proxy_threads;
  h->threads = new (std::nothrow) ProxyThread[h->nthreads > 0 ? h->nthreads : 1];
  if (!h->threads) {
    free_all(h);
    return EP_ENOMEM;
  }
  for (int i = 0; i < h->nthreads; ++i) {
    ProxyThread &P = h->threads[i];
    P.tid = i;
    for (int c = i; c < C; c += h->nthreads) {
      P.channels.push_back(c);
      P.head.push_back(0);
    }
    P.seen.assign((size_t)S * E, 0);
    P.parked.resize((size_t)S * E);
    if (cfg->flags & EP_FLAG_SENDER_FENCE) {
      P.sender_parked.resize((size_t)S * E);
      P.atomic_flying.assign((size_t)S * E, 0);
    }
    P.next_seq.assign((size_t)S * cfg->num_ranks, 0);
    P.early.resize((size_t)S * cfg->num_ranks);
    P.in_flight.assign((size_t)cfg->num_ranks, 0);
    P.held.resize((size_t)cfg->num_ranks);
    if (cfg->pack_rows > 1) P.open_idx.assign((size_t)S * E, -1);
    P.ring_next.assign(nring * 2, 0);
    P.ring_early.resize(nring * 2);
    P.rng = cfg->reorder_seed * 0x9E3779B97F4A7C15ull + (uint64_t)i;
  }
  for (int i = 0; i < h->nthreads; ++i) h->threads[i].th = std::thread(proxy_main, h, &h->threads[i]);
  *out = h;
  return EP_OK;
}

int ep_proxy_stop(ep_handle *h) {
  if (!h) return EP_EINVAL;
  int rc = EP_OK;
  if (!h->host_only && !HIP_OK(hipDeviceSynchronize())) rc = EP_EHIP;
  h->stop.store(true, std::memory_order_release);
  for (int i = 0; i < h->nthreads; ++i)
    if (h->threads[i].th.joinable()) h->threads[i].th.join();
  for (int i = 0; i < h->nthreads; ++i) {
    ProxyThread &P = h->threads[i];
    if (!P.gpu_ready) continue;
    for (hipEvent_t &e : P.events)
      if (e) (void)hipEventDestroy(e);
    if (P.descs) (void)hipHostFree(P.descs);
  }
  if (h->copy_stream) (void)hipStreamDestroy(h->copy_stream);
  free_all(h);
  return rc;
}

int ep_register_heaps(ep_handle *h, const void *d_src_base, int64_t src_bytes, void *d_dst_base,
                      int64_t dst_bytes) {
  if (!h) return EP_EINVAL;
  if (h->host_only) return EP_ESTATE;
  if (!d_src_base != !d_dst_base) return EP_EINVAL;
  if (!d_dst_base) {
    h->dst_base.store(nullptr, std::memory_order_release);
    h->src_base.store(nullptr, std::memory_order_release);
    return EP_OK;
  }
  if (src_bytes <= 0 || dst_bytes <= 0 || (((uintptr_t)d_src_base | (uintptr_t)d_dst_base) & 15)) return EP_EINVAL;
  if (src_bytes > (1ll << 36) || dst_bytes > (1ll << 36)) return EP_EINVAL;  // offsets travel as 32-bit counts of 16 bytes
  if (h->nthreads < 1) return EP_EINVAL;
  // What the proxy needs to issue the writes, made once, on first registration: ONE stream (default
  // priority) shared by all proxy threads, and completion events per thread.  One stream, because a
  // process has few hardware queues (4 here) and streams beyond that share one: a copy kernel queued
  // behind a dispatch kernel that is itself blocked on a Drain (which waits for that copy) would never
  // start.  The caller's stream and this one get queues of their own as long as the process keeps
  // fewer streams than hardware queues; if they ever do collide, the kernel's bounded wait reports
  // EP_ETIMEOUT.
  if (!h->copy_stream && !HIP_OK(hipStreamCreateWithFlags(&h->copy_stream, hipStreamNonBlocking))) return EP_EHIP;
  for (int i = 0; i < h->nthreads; ++i) {
    ProxyThread &P = h->threads[i];
    if (P.gpu_ready) continue;
    for (hipEvent_t &e : P.events)
      if (!HIP_OK(hipEventCreateWithFlags(&e, hipEventDisableTiming))) return EP_EHIP;
    void *q = nullptr, *dq = nullptr;
    if (!HIP_OK(hipHostMalloc(&q, sizeof(CopyDesc) * ProxyThread::kBatchSlots * kCopyBatchMax,
                              hipHostMallocMapped | hipHostMallocCoherent)))
      return EP_ENOMEM;
    P.descs = (CopyDesc *)q;
    if (!HIP_OK(hipHostGetDevicePointer(&dq, q, 0))) return EP_EHIP;
    P.d_descs = (CopyDesc *)dq;
    P.gpu_ready = true;
  }
  h->src_bytes = (uint64_t)src_bytes;
  h->dst_bytes = (uint64_t)dst_bytes;
  h->src_base.store((const char *)d_src_base, std::memory_order_release);
  h->dst_base.store((char *)d_dst_base, std::memory_order_release);
  return EP_OK;
}

int ep_layout(ep_handle *h, const int32_t *d_topk_idx, int32_t T, int32_t *d_count, int32_t *d_expert_total,
              int32_t *d_rank_total, int32_t *d_base, int32_t *d_expert_offset, int32_t *d_rank_offset,
              int32_t *d_slot, int32_t *d_dst_row, void *stream) {
  if (!h) return EP_EINVAL;
  if (h->host_only) return EP_ESTATE;
  if (T < 0 || T > h->cfg.max_tokens) return EP_EINVAL;
  if (!d_count || !d_expert_total || !d_rank_total || !d_base || !d_expert_offset || !d_rank_offset) return EP_EINVAL;
  if (T > 0 && (!d_topk_idx || !d_slot || !d_dst_row)) return EP_EINVAL;
  LayoutArgs a{};
  a.idx = d_topk_idx;
  a.S = h->cfg.num_src;
  a.T = T;
  a.K = h->cfg.top_k;
  a.E = h->cfg.num_experts;
  a.R = h->cfg.num_ranks;
  a.E_loc = h->E_loc;
  a.ntiles = (T + kLayoutTile - 1) / kLayoutTile;
  a.tile_hist = h->tile_hist;
  a.tile_base = h->tile_base;
  a.ticket = h->ticket;
  a.count = d_count;
  a.expert_total = d_expert_total;
  a.rank_total = d_rank_total;
  a.base = d_base;
  a.expert_offset = d_expert_offset;
  a.rank_offset = d_rank_offset;
  a.slot = d_slot;
  a.dst_row = d_dst_row;
  a.error = h->ring.error;
  return HIP_OK((hipError_t)launch_layout(a, stream)) ? EP_OK : EP_EHIP;
}

static uint32_t row_bytes_of(int H, int payload) {
  return payload == EP_BF16 ? 2u * (uint32_t)H : ((uint32_t)H + (uint32_t)H / 32u + 15u) / 16u * 16u;
}

int ep_dispatch(ep_handle *h, const void *d_x, const int32_t *d_topk_idx, const int32_t *d_dst_row,
                const int32_t *d_count, const int32_t *d_base, int32_t T, int32_t src_rank,
                int32_t dst_rank_filter, int32_t payload, int32_t cmd_mode, void *d_recv, float *d_recv_scale,
                int64_t recv_rows, void *stream) {
  if (!h) return EP_EINVAL;
  if (h->host_only) return EP_ESTATE;
  const ep_config &c = h->cfg;
  const int mode = cmd_mode & EP_CMD_MODE_MASK;
  if (T < 0 || T > c.max_tokens || src_rank < 0 || src_rank >= c.num_src) return EP_EINVAL;
  if (dst_rank_filter < -1 || dst_rank_filter >= c.num_ranks) return EP_EINVAL;
  if (payload != EP_BF16 && payload != EP_FP8_E4M3) return EP_EINVAL;
  if (mode != EP_CMD_PER_TOKEN && mode != EP_CMD_CHUNK32 && mode != EP_CMD_NONE && mode != EP_CMD_CHUNK32_ORDERED)
    return EP_EINVAL;
  if (mode == EP_CMD_CHUNK32_ORDERED) {
    if (cmd_mode & EP_CMD_ATOMICS_FIRST) return EP_EINVAL;
    cmd_mode |= EP_CMD_DRAIN;
  }
  if (cmd_mode & ~(EP_CMD_MODE_MASK | EP_CMD_ATOMICS_FIRST | EP_CMD_DRAIN | EP_CMD_NO_PLACEMENT)) return EP_EINVAL;
  if (const char *dbase = h->dst_base.load(std::memory_order_acquire)) {
    // the proxy performs the writes: rows travel as 16-bit words only, and the offsets the kernel
    // is about to put into its commands must be relative to the registered source heap
    if (mode != EP_CMD_NONE) {
      if (payload != EP_BF16) return EP_EINVAL;
      const bool chunked = mode != EP_CMD_PER_TOKEN;
      if (chunked && ((cmd_mode & EP_CMD_NO_PLACEMENT) || d_recv != (const void *)h->src_base.load())) return EP_EINVAL;
      if (!chunked && (!(cmd_mode & EP_CMD_NO_PLACEMENT) || d_x != (const void *)h->src_base.load())) return EP_EINVAL;
      if (!chunked && (uint64_t)recv_rows * 2u * (uint64_t)c.hidden > h->dst_bytes) return EP_EINVAL;
    }
    (void)dbase;
  } else if (cmd_mode & EP_CMD_NO_PLACEMENT) {
    return EP_EINVAL;
  }
  if (recv_rows < 0 || recv_rows > c.heap_rows) return EP_EINVAL;
  if (T > 0 && (!d_x || !d_topk_idx || !d_dst_row || !d_recv)) return EP_EINVAL;
  if ((payload == EP_FP8_E4M3) != (d_recv_scale != nullptr)) return EP_EINVAL;
  if (mode != EP_CMD_NONE) {
    if (h->nthreads < 1 || !d_count || !d_base) return EP_EINVAL;
    if (mode == EP_CMD_NONE && (cmd_mode & (EP_CMD_ATOMICS_FIRST | EP_CMD_DRAIN))) return EP_EINVAL;
  } else if (cmd_mode & (EP_CMD_ATOMICS_FIRST | EP_CMD_DRAIN)) {
    return EP_EINVAL;
  }
  if (((uintptr_t)d_x | (uintptr_t)d_recv) & 15) return EP_EINVAL;
  if (int e = dev_err(h)) return e;

  DispatchArgs a{};
  a.x = d_x;
  a.idx = d_topk_idx;
  a.dst_row = d_dst_row;
  a.count = d_count;
  a.base = d_base;
  a.recv = d_recv;
  a.recv_scale = d_recv_scale;
  a.recv_rows = recv_rows;
  a.T = T;
  a.K = c.top_k;
  a.H = c.hidden;
  a.E = c.num_experts;
  a.E_loc = h->E_loc;
  a.src = src_rank;
  a.filter = dst_rank_filter;
  a.cmd_mode = cmd_mode;
  a.row_bytes = row_bytes_of(c.hidden, payload);
  a.chunks_per_expert = h->chunks_per_expert;
  a.chunk_cnt = h->chunk_cnt;
  a.expert_done = h->expert_done;
  a.waves_done = h->waves_done;
  a.ht_seq = h->ht_seq;
  a.R = c.num_ranks;
  a.ring = h->ring;
  if (mode != EP_CMD_NONE) {
    if (((uint64_t)T * a.row_bytes) >> 4 > 0xFFFFFFFFull) return EP_EINVAL;
    if (mode == EP_CMD_CHUNK32_ORDERED)
      h->expected_drains.fetch_add(c.num_channels, std::memory_order_relaxed);
    else
      h->expected_atomics.fetch_add(dst_rank_filter < 0 ? c.num_experts : h->E_loc, std::memory_order_relaxed);
  }
  if (T == 0) {
    // nothing to launch; a ring-on dispatch of zero tokens still owes its (all zero) count atomics,
    // which only a kernel can push: run it with one idle workgroup
    if (mode == EP_CMD_NONE) return EP_OK;
    a.T = 0;
  }
  return HIP_OK((hipError_t)launch_dispatch(a, payload, stream)) ? EP_OK : EP_EHIP;
}

int ep_combine(ep_handle *h, const void *d_y, const float *d_topk_w, const int32_t *d_dst_row, int32_t T,
               int64_t y_rows, void *d_out, void *stream) {
  if (!h) return EP_EINVAL;
  if (h->host_only) return EP_ESTATE;
  if (T < 0 || T > h->cfg.max_tokens || y_rows < 0) return EP_EINVAL;
  if (T == 0) return EP_OK;
  if (!d_topk_w || !d_dst_row || !d_out || (y_rows > 0 && !d_y)) return EP_EINVAL;
  if (((uintptr_t)d_y | (uintptr_t)d_out) & 15) return EP_EINVAL;
  CombineArgs a{};
  a.y = d_y;
  a.w = d_topk_w;
  a.dst_row = d_dst_row;
  a.out = d_out;
  a.y_rows = y_rows;
  a.T = T;
  a.K = h->cfg.top_k;
  a.H = h->cfg.hidden;
  a.error = h->ring.error;
  return HIP_OK((hipError_t)launch_combine(a, stream)) ? EP_OK : EP_EHIP;
}

int ep_dedup(ep_handle *h, const int32_t *d_topk_idx, int32_t T, int32_t ranks_per_group, int32_t *d_group_idx,
             int32_t *d_first_k, void *stream) {
  if (!h) return EP_EINVAL;
  if (h->host_only) return EP_ESTATE;
  if (T < 0 || T > h->cfg.max_tokens) return EP_EINVAL;
  if (ranks_per_group < 1 || h->cfg.num_ranks % ranks_per_group) return EP_EINVAL;
  if (T > 0 && (!d_topk_idx || !d_group_idx || !d_first_k)) return EP_EINVAL;
  DedupArgs a{};
  a.idx = d_topk_idx;
  a.group_idx = d_group_idx;
  a.first_k = d_first_k;
  a.n_tokens = (long long)h->cfg.num_src * T;
  a.K = h->cfg.top_k;
  a.E = h->cfg.num_experts;
  a.E_loc = h->E_loc;
  a.ranks_per_group = ranks_per_group;
  a.error = h->ring.error;
  return HIP_OK((hipError_t)launch_dedup(a, stream)) ? EP_OK : EP_EHIP;
}

int ep_gather_index(ep_handle *h, const int32_t *d_dst_row, const int32_t *d_dst_row_g, const int32_t *d_first_k,
                    int32_t T, int64_t rows, int32_t *d_index, void *stream) {
  if (!h) return EP_EINVAL;
  if (h->host_only) return EP_ESTATE;
  if (T < 0 || T > h->cfg.max_tokens || rows < 0) return EP_EINVAL;
  if (T > 0 && (!d_dst_row || !d_dst_row_g || !d_first_k || !d_index)) return EP_EINVAL;
  GatherIndexArgs a{};
  a.dst_row = d_dst_row;
  a.dst_row_g = d_dst_row_g;
  a.first_k = d_first_k;
  a.index = d_index;
  a.rows = rows;
  a.T = T;
  a.K = h->cfg.top_k;
  a.error = h->ring.error;
  return HIP_OK((hipError_t)launch_gather_index(a, stream)) ? EP_OK : EP_EHIP;
}

int ep_combine_partial(ep_handle *h, const void *d_y, const float *d_topk_w, const int32_t *d_dst_row,
                       const int32_t *d_first_k, const int32_t *d_dst_row_g, int32_t T, int64_t y_rows,
                       int64_t rows_g, void *d_partial, void *stream) {
  if (!h) return EP_EINVAL;
  if (h->host_only) return EP_ESTATE;
  if (T < 0 || T > h->cfg.max_tokens || y_rows < 0 || rows_g < 0) return EP_EINVAL;
  if (T == 0) return EP_OK;
  if (!d_topk_w || !d_dst_row || !d_first_k || !d_dst_row_g || (y_rows > 0 && !d_y) || (rows_g > 0 && !d_partial))
    return EP_EINVAL;
  if (((uintptr_t)d_y | (uintptr_t)d_partial) & 15) return EP_EINVAL;
  CombinePartialArgs a{};
  a.y = d_y;
  a.w = d_topk_w;
  a.dst_row = d_dst_row;
  a.first_k = d_first_k;
  a.dst_row_g = d_dst_row_g;
  a.partial = d_partial;
  a.y_rows = y_rows;
  a.rows_g = rows_g;
  a.T = T;
  a.K = h->cfg.top_k;
  a.H = h->cfg.hidden;
  a.error = h->ring.error;
  return HIP_OK((hipError_t)launch_combine_partial(a, stream)) ? EP_OK : EP_EHIP;
}

int ep_barrier(ep_handle *h, void *stream) {
  if (!h) return EP_EINVAL;
  if (h->host_only) return EP_ESTATE;
  if (h->nthreads < 1) return EP_ESTATE;  // nobody would ever pop the command
  if (int e = dev_err(h)) return e;
  return HIP_OK((hipError_t)launch_barrier(h->ring, stream)) ? EP_OK : EP_EHIP;
}

int ep_fifo_stress(ep_handle *h, int32_t pushers, int32_t cmds_per_pusher, uint64_t *d_lat_sum, uint64_t *d_lat_max,
                   void *stream) {
  if (!h) return EP_EINVAL;
  if (h->host_only) return EP_ESTATE;
  if (h->nthreads < 1) return EP_ESTATE;  // nobody would ever pop a command
  if (pushers < 1 || pushers > 65536 || cmds_per_pusher < 1 || cmds_per_pusher > (1 << 20)) return EP_EINVAL;
  if (!d_lat_sum || !d_lat_max) return EP_EINVAL;
  if (int e = dev_err(h)) return e;
  h->expected_atomics.fetch_add((int64_t)pushers * cmds_per_pusher, std::memory_order_relaxed);
  return HIP_OK((hipError_t)launch_fifo_stress(h->ring, pushers, cmds_per_pusher, (unsigned long long *)d_lat_sum,
                                               (unsigned long long *)d_lat_max, stream))
             ? EP_OK
             : EP_EHIP;
}

int ep_recv_wait(ep_handle *h, int32_t src_rank, int32_t dst_rank_filter, int32_t *d_counts_out, void *stream) {
  if (!h) return EP_EINVAL;
  if (h->host_only) return EP_ESTATE;
  if (src_rank < 0 || src_rank >= h->cfg.num_src) return EP_EINVAL;
  if (dst_rank_filter < -1 || dst_rank_filter >= h->cfg.num_ranks) return EP_EINVAL;
  if (h->nthreads < 1) return EP_ESTATE;  // nobody would ever post a counter
  RecvWaitArgs a{};
  a.flags = (int *)h->d_recv_flag;
  a.out = d_counts_out;
  a.E = h->cfg.num_experts;
  a.E_loc = h->E_loc;
  a.src = src_rank;
  a.filter = dst_rank_filter;
  a.error = h->ring.error;
  a.timeout_ticks = h->ring.timeout_ticks;
  return HIP_OK((hipError_t)launch_recv_wait(a, stream)) ? EP_OK : EP_EHIP;
}

int ep_wait(ep_handle *h) {
  if (!h) return EP_EINVAL;
  const uint64_t t0 = now_ns();
  uint64_t spins = 0;
  for (;;) {
    if (int e = dev_err(h)) return e;
    if (int e = h->proxy_error.load(std::memory_order_relaxed)) return e;
    int64_t applied = 0, drained = 0;
    for (int i = 0; i < h->nthreads; ++i) {
      applied += (int64_t)h->threads[i].applied.load(std::memory_order_acquire);
      drained += (int64_t)h->threads[i].drains.load(std::memory_order_acquire);
    }
    if (applied >= h->expected_atomics.load(std::memory_order_relaxed) &&
        drained >= h->expected_drains.load(std::memory_order_relaxed)) {
      if (int e = h->proxy_error.load(std::memory_order_relaxed)) return e;
      return EP_OK;
    }
    if ((++spins & 1023) == 0) {
      if (now_ns() - t0 > h->timeout_ns) return EP_ETIMEOUT;
      std::this_thread::yield();
    } else {
      _mm_pause();
    }
  }
}

int ep_counters(ep_handle *h, const int32_t **recv_count, const int32_t **d_recv_count) {
  if (!h || !recv_count) return EP_EINVAL;
  *recv_count = h->recv_count;
  if (d_recv_count) *d_recv_count = (const int32_t *)h->d_recv_count;
  return EP_OK;
}

int ep_ring_counters(ep_handle *h, const int32_t **ring_tail, const int32_t **ring_head) {
  if (!h || !ring_tail || !ring_head) return EP_EINVAL;
  if (h->cfg.ht_slices <= 0) return EP_ESTATE;
  *ring_tail = h->ring_tail;
  *ring_head = h->ring_head;
  return EP_OK;
}

int ep_ht_dispatch(ep_handle *h, const void *d_x, const int32_t *d_topk_idx, const int32_t *d_dst_row, int32_t T,
                   int32_t src_rank, int32_t payload, void *d_ring, int64_t ring_bytes, void *d_recv,
                   float *d_recv_scale, int64_t recv_rows, void *stream) {
  if (!h) return EP_EINVAL;
  if (h->host_only || h->cfg.ht_slices <= 0) return EP_ESTATE;
  const ep_config &c = h->cfg;
  if (T < 0 || T > c.max_tokens || src_rank < 0 || src_rank >= c.num_src) return EP_EINVAL;
  if (recv_rows < 0 || recv_rows > c.heap_rows) return EP_EINVAL;
  if (payload != EP_BF16 && payload != EP_FP8_E4M3) return EP_EINVAL;
  if ((payload == EP_FP8_E4M3) != (d_recv_scale != nullptr)) return EP_EINVAL;
  if (!d_ring || ring_bytes < 0 || (uint64_t)ring_bytes < h->ring_total_bytes) return EP_EINVAL;
  if (T > 0 && (!d_x || !d_topk_idx || !d_dst_row || !d_recv)) return EP_EINVAL;
  if (((uintptr_t)d_x | (uintptr_t)d_recv | (uintptr_t)d_ring) & 15) return EP_EINVAL;
  if (h->ring_total_bytes >> 4 > 0x7FFFFFFFull) return EP_EINVAL;  // slot offsets travel as 31-bit counts of 16 bytes
  if (int e = dev_err(h)) return e;
  HtRingArgs a{};
  a.x = d_x;
  a.idx = d_topk_idx;
  a.dst_row = d_dst_row;
  a.ring_buf = d_ring;
  a.recv = d_recv;
  a.recv_scale = d_recv_scale;
  a.recv_rows = recv_rows;
  a.payload = payload;
  a.row_bytes = row_bytes_of(c.hidden, payload);
  a.T = T;
  a.K = c.top_k;
  a.H = c.hidden;
  a.E_loc = h->E_loc;
  a.R = c.num_ranks;
  a.src = src_rank;
  a.slices = c.ht_slices;
  a.slice_len = T > 0 ? (T + c.ht_slices - 1) / c.ht_slices : 1;
  a.W = c.ht_ring_slots;
  a.slot_bytes = (unsigned)h->ring_slot_bytes;
  const size_t first = (size_t)src_rank * c.ht_slices * c.num_ranks;
  a.tail = (const int32_t *)h->d_ring_tail + first;
  a.head = (const int32_t *)h->d_ring_head + first;
  a.seq_fwd = h->ring_seq_fwd + first;
  a.seq_rev = h->ring_seq_rev + first;
  a.cum_fwd = h->ring_cum_fwd + first;
  a.cum_rev = h->ring_cum_rev + first;
  a.waves_done = h->waves_done;
  a.fifo = h->ring;
  h->expected_drains.fetch_add(c.num_channels, std::memory_order_relaxed);
  return HIP_OK((hipError_t)launch_ht_ring(a, stream)) ? EP_OK : EP_EHIP;
}

int ep_tail_counters(ep_handle *h, const int32_t **recv_tail) {
  if (!h || !recv_tail) return EP_EINVAL;
  *recv_tail = h->recv_tail;
  return EP_OK;
}

int ep_stats(ep_handle *h, ep_stats_t *out) {
  if (!h || !out) return EP_EINVAL;
  memset(out, 0, sizeof(*out));
  for (int i = 0; i < h->nthreads; ++i) {
    ProxyThread &P = h->threads[i];
    const uint64_t n = P.cmds.load();
    out->cmds += n;
    if (i < 16) out->per_thread_cmds[i] = n;
    out->writes += P.writes.load();
    out->atomics += P.atomics.load();
    out->drains += P.drains.load();
    out->barriers += P.barriers.load();
    out->write_bytes += P.write_bytes.load();
    out->write_rows += P.write_rows.load();
    out->atomics_applied += P.applied.load();
    out->atomics_deferred += P.deferred.load();
    out->ordered_parked += P.ordered_parked.load();
    out->rejected += P.rejected.load();
    out->sender_held += P.sender_held.load();
    out->write_msgs += P.write_msgs.load();
    out->paced += P.paced.load();
    if (P.max_in_flight.load() > out->max_in_flight) out->max_in_flight = P.max_in_flight.load();
    out->copy_batches += P.copy_batches.load();
    out->copied_bytes += P.copied_bytes.load();
    const uint64_t f = P.first_poll_ns.load(), l = P.last_apply_ns.load();
    if (f && (!out->first_poll_ns || f < out->first_poll_ns)) out->first_poll_ns = f;
    if (l > out->last_apply_ns) out->last_apply_ns = l;
  }
  if (h->host_only) {
    out->gpu_ring_full = h->host_stalls.load();
  } else {
    unsigned long long st = 0;
    if (!HIP_OK(hipMemcpy(&st, h->ring.stalls, 8, hipMemcpyDeviceToHost))) return EP_EHIP;
    out->gpu_ring_full = st;
  }
  out->device_error = dev_err(h);
  out->proxy_error = h->proxy_error.load();
  return EP_OK;
}

int ep_reset_stats(ep_handle *h) {
  if (!h) return EP_EINVAL;
  int64_t applied = 0;
  for (int i = 0; i < h->nthreads; ++i) applied += (int64_t)h->threads[i].applied.load();
  if (applied != h->expected_atomics.load()) return EP_ESTATE;  // work in flight
  for (int i = 0; i < h->nthreads; ++i) {
    ProxyThread &P = h->threads[i];
    for (auto *a : {&P.cmds, &P.writes, &P.atomics, &P.drains, &P.write_bytes, &P.write_rows, &P.applied,
                    &P.deferred, &P.rejected, &P.first_poll_ns, &P.last_apply_ns, &P.ordered_parked, &P.barriers,
                    &P.copy_batches, &P.copied_bytes, &P.write_msgs, &P.paced, &P.max_in_flight,
                    &P.sender_held})
      a->store(0);
    std::lock_guard<std::mutex> g(P.log_mu);
    P.cmd_log.clear();
    P.event_log.clear();
  }
  h->expected_atomics.store(0);
  h->expected_drains.store(0);
  memset(h->recv_tail, 0, (size_t)h->cfg.num_src * h->cfg.num_ranks * 4);
  memset(h->recv_count, 0, (size_t)h->cfg.num_src * h->cfg.num_experts * 4);
  memset(h->recv_flag, 0, (size_t)h->cfg.num_src * h->cfg.num_experts * 4);
  if (h->host_only) {
    h->host_stalls.store(0);
  } else if (!HIP_OK(hipMemset(h->ring.stalls, 0, 8))) {
    return EP_EHIP;
  }
  return EP_OK;
}

static int copy_log(ep_handle *h, bool events, void *buf, size_t cap, size_t *n) {
  if (!h || !n) return EP_EINVAL;
  if (!(h->cfg.flags & (events ? EP_FLAG_LOG_EVENTS : EP_FLAG_LOG_CMDS))) return EP_ESTATE;
  size_t total = 0;
  uint32_t *dst = (uint32_t *)buf;
  for (int i = 0; i < h->nthreads; ++i) {
    ProxyThread &P = h->threads[i];
    std::lock_guard<std::mutex> g(P.log_mu);
    const std::vector<uint32_t> &v = events ? P.event_log : P.cmd_log;
    const size_t recs = v.size() / 4;
    for (size_t r = 0; r < recs; ++r, ++total)
      if (dst && total < cap) memcpy(dst + total * 4, v.data() + r * 4, 16);
  }
  *n = total;
  return EP_OK;
}

int ep_cmd_log(ep_handle *h, void *buf, size_t cap, size_t *n) { return copy_log(h, false, buf, cap, n); }
int ep_event_log(ep_handle *h, void *buf, size_t cap, size_t *n) { return copy_log(h, true, buf, cap, n); }

int ep_host_push(ep_handle *h, int32_t channel, uint32_t w0, uint32_t w1, uint32_t w2, uint32_t w3, uint64_t *idx) {
  if (!h || channel < 0 || channel >= h->cfg.num_channels) return EP_EINVAL;
  if (!h->host_only) return EP_ESTATE;
  const uint64_t i = h->host_tail[channel].fetch_add(1, std::memory_order_relaxed);
  const uint64_t *hp = &h->head[(size_t)channel * kHeadStride];
  if (i - __atomic_load_n(hp, __ATOMIC_ACQUIRE) >= h->entries) {
    h->host_stalls.fetch_add(1, std::memory_order_relaxed);
    const uint64_t t0 = now_ns();
    uint64_t spins = 0;
    while (i - __atomic_load_n(hp, __ATOMIC_ACQUIRE) >= h->entries) {
      if ((++spins & 255) == 0) {
        if (now_ns() - t0 > h->timeout_ns) {
          __atomic_store_n(h->dev_error, (int)EP_ETIMEOUT, __ATOMIC_RELAXED);
          return EP_ETIMEOUT;
        }
        std::this_thread::yield();
      } else {
        _mm_pause();
      }
    }
  }
  const uint32_t gen = (((uint32_t)(i >> h->log2_entries)) & 1u) ^ 1u;
  uint64_t *slot = h->slots + ((size_t)channel * h->entries + (i & (h->entries - 1))) * 2;
  const uint64_t lo = (uint64_t)((w0 & 0x7FFFFFFFu) | (gen << 31)) | ((uint64_t)w1 << 32);
  const uint64_t hi = (uint64_t)w2 | ((uint64_t)((w3 & 0x7FFFFFFFu) | (gen << 31)) << 32);
  __atomic_store_n(slot, lo, __ATOMIC_RELEASE);
  __atomic_store_n(slot + 1, hi, __ATOMIC_RELEASE);
  if (idx) *idx = i;
  return EP_OK;
}

int ep_host_check_completion(ep_handle *h, int32_t channel, uint64_t idx) {
  if (!h || channel < 0 || channel >= h->cfg.num_channels) return EP_EINVAL;
  return __atomic_load_n(&h->head[(size_t)channel * kHeadStride], __ATOMIC_ACQUIRE) > idx ? 1 : 0;
}

const char *ep_last_error(void) { return g_last_error; }

int ep_bw_probe(int32_t kind, const void *d_src, void *d_dst, int64_t bytes, void *stream) {
  if (kind < 0 || kind > 2 || bytes < 0 || (bytes & 15)) return EP_EINVAL;
  if (bytes >> 36) return EP_EINVAL;  // grid index range
  if ((kind != 1 && !d_src) || !d_dst) return EP_EINVAL;  // kind 0 uses d_dst as a 16-byte sink
  if (((uintptr_t)d_src | (uintptr_t)d_dst) & 15) return EP_EINVAL;
  return HIP_OK((hipError_t)launch_bw_probe(kind, d_src, d_dst, bytes, stream)) ? EP_OK : EP_EHIP;
}

int ep_host_expect_atomics(ep_handle *h, int32_t n) {
  if (!h || n < 0) return EP_EINVAL;
  h->expected_atomics.fetch_add(n, std::memory_order_relaxed);
  return EP_OK;
}

}  // extern "C"
