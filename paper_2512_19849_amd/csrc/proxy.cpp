// The CPU proxy of libep.so (Section 3.1-3.4): each thread polls its FIFO channels, translates and checks
// the offsets of every command, performs or forwards the write, and applies immediates at the receiving
// half under the completion fence / the per-channel ordering rules.
#include "ep_host.h"

namespace ep {
namespace {

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
  ++P.applied_unpublished;  // (ep_wait's counter and the clock are brought up to date once per polled batch)
  P.stamp_apply = true;
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
    P.stamp_apply = true;
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
  ReorderBuf &q = P.early[chan];
  if (seq != next) {
    q.put(next, seq, ev);
    bump(P.ordered_parked, 1);
    return;
  }
  apply_ordered(h, P, chan, ev, seq);
  ++next;
  for (WireEvent held; q.take(next, held); ++next) apply_ordered(h, P, chan, held, next);
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
  P.stamp_apply = true;
}

void deliver_ring(ep_handle *h, ProxyThread &P, const WireEvent &ev) {
  const ep_config &c = h->cfg;
  const size_t chan = ((size_t)ev.src * c.ht_slices + ev.slice) * c.num_ranks + ev.dst_rank;
  const size_t dir = chan * 2 + (ev.ordered == 3);
  uint32_t &next = P.ring_next[dir];
  const uint32_t seq = rebuild_seq(next, (ev.imm >> 15) & 0xFFFFu);
  const uint32_t where = ((uint32_t)ev.slice << 8) | ev.dst_rank;
  log_event(h, P, ev.ordered == 3 ? 10 : ((ev.imm >> 31) ? 9 : 8), ev.src, where, seq);
  ReorderBuf &q = P.ring_early[dir];
  if (seq != next) {
    q.put(next, seq, ev);
    bump(P.ordered_parked, 1);
    return;
  }
  apply_ring(h, P, chan, ev, seq);
  ++next;
  for (WireEvent held; q.take(next, held); ++next) apply_ring(h, P, chan, held, next);
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

// A notice that needs no copy before it: with nothing configured between the two halves it is
// delivered on the spot, else it takes the general way out (pacing, transport, ...).
inline void send_notice(ep_handle *h, ProxyThread &P, const WireEvent &ev) {
  if (P.plain_writes) {
    ++P.in_flight[ev.dst_rank];  // (deliver takes it off again)
    if (P.max_in_flight.load(std::memory_order_relaxed) == 0) P.max_in_flight.store(1, std::memory_order_relaxed);
    deliver(h, P, ev);
    return;
  }
  Outbound m;
  m.notice = ev;
  send_msg(h, P, m);
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
      if (P.plain_writes && !dbase) {
        // The common case, taken out of the general path below (which does the same in more steps):
        // the payload is in place, nothing is configured between the sender half and the receiver
        // half, so the Write's arrival is counted here and now, and count Atomics that were waiting
        // for it are applied.
        bump(P.write_msgs, 1);
        if (P.max_in_flight.load(std::memory_order_relaxed) == 0) P.max_in_flight.store(1, std::memory_order_relaxed);
        const uint32_t e = dr * (uint32_t)h->E_loc + le;
        const size_t key = (size_t)src * c.num_experts + e;
        P.seen[key] += (int32_t)rows;
        std::deque<int32_t> &q = P.parked[key];
        while (!q.empty() && P.seen[key] >= q.front()) {
          const int32_t v = q.front();
          q.pop_front();
          apply_atomic(h, P, src, e, v);
        }
        break;
      }
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
      send_notice(h, P, WireEvent{(1u << 31) | (le << 19) | w1, (uint16_t)src, (uint8_t)dr, 0});
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
      if (!dbase) {  // the kernel placed the rows: only the notice travels
        bump(P.write_msgs, 1);
        send_notice(h, P, WireEvent{((w2 & 0xFFFFu) << 15) | rows, (uint16_t)src, (uint8_t)dr, 1});
        break;
      }
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
      send_notice(h, P, WireEvent{(1u << 31) | ((w2 & 0xFFFFu) << 15) | w1, (uint16_t)src, (uint8_t)dr, 1});
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
        bump(P.write_msgs, 1);
        send_notice(h, P, WireEvent{((w2 & 0xFFFFu) << 15) | rows, (uint16_t)src, (uint8_t)dr, 2, (uint16_t)slice});
      } else {
        const uint32_t value = w1 & 0x3FFFFFFFu;
        if (value > 0x7FFFu) {
          reject(h, P);
          return;
        }
        bump(P.atomics, 1);
        send_notice(h, P, WireEvent{(1u << 31) | ((w2 & 0xFFFFu) << 15) | value, (uint16_t)src, (uint8_t)dr,
                                    (uint8_t)(kind == EP_RING_TAIL ? 2 : 3), (uint16_t)slice});
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
}  // namespace

// The atomics applied since the last call become visible to ep_wait, and the statistics' clock of
// the last application is set.  Once per polled batch rather than per atomic: the counter's cache
// line is in the waiting thread's hands most of the time, and every store to it has to fetch it back.
static inline void publish_applied(ProxyThread &P) {
  if (P.stamp_apply) {
    P.stamp_apply = false;
    P.last_apply_ns.store(now_ns(), std::memory_order_relaxed);
  }
  if (P.applied_unpublished) {
    P.applied.store(P.applied.load(std::memory_order_relaxed) + P.applied_unpublished, std::memory_order_release);
    P.applied_unpublished = 0;
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
        publish_applied(P);
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
    publish_applied(P);  // (what arrivals from the transport or finished copies have released)
    if (any) {
      idle = 0;
      continue;
    }
    if (!P.window.empty()) {  // nothing new: let in-flight immediates land
      flush_window(h, P);
      publish_applied(P);
    }
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

}  // namespace ep
