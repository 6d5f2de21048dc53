// Stand-alone driver for the host side of the library (ring + proxy threads) with several
// producer threads, built with ThreadSanitizer / AddressSanitizer by tests/test_host_sanitizers.py.
// The kernel launchers are stubbed: a host-only handle never calls them.
#include "../../include/ep.h"
#include "../../paper_2512_19849_amd/csrc/ep_internal.h"
#include <cstdio>
#include <string>
#include <thread>
#include <vector>
namespace ep {
int launch_layout(const LayoutArgs&, const Tunables&, void*, const LaunchTiming*) { return 0; }
int launch_dispatch(const DispatchArgs&, int, const Tunables&, void*, const LaunchTiming*) { return 0; }
int launch_combine(const CombineArgs&, const Tunables&, void*, const LaunchTiming*) { return 0; }
int launch_fill_u32(uint32_t*, uint32_t, long long, void*) { return 0; }
int launch_fp8_unpack(const void*, long long, int, unsigned, void*, float*, void*) { return 0; }
int static_layout_scratch(LayoutArgs*) { return 0; }
int launch_recv_wait(const RecvWaitArgs&, void*) { return 0; }
int launch_barrier(const RingDev&, void*) { return 0; }
int launch_dedup(const DedupArgs&, void*) { return 0; }
int launch_gather_index(const GatherIndexArgs&, void*) { return 0; }
int launch_combine_partial(const CombinePartialArgs&, void*) { return 0; }
int launch_bw_probe(int, const void*, void*, long long, void*) { return 0; }
int launch_copy_batch(const CopyBatchArgs&, void*) { return 0; }
int launch_row_probe(int, const int32_t*, int, long long, int, long long, void*, void*, void*) { return 0; }
int launch_ht_ring(const HtRingArgs&, const Tunables&, void*) { return 0; }
int launch_fifo_stress(const RingDev&, int, int, unsigned long long*, unsigned long long*, void*) { return 0; }
}
static uint32_t w0(uint32_t op, uint32_t src, uint32_t dr, uint32_t le) { return (op << 28) | (src << 20) | (dr << 12) | le; }
int main(int argc, char **argv) {
  // "policies": the same traffic with the proxy's options on - pacing, best-effort packing, the fence at
  // the sender - plus ring-buffer channel messages pushed by two threads
  const bool policies = argc > 1 && std::string(argv[1]) == "policies";
  ep_config c{}; c.num_ranks = 4; c.num_experts = 16; c.top_k = 2; c.hidden = 1024; c.max_tokens = 4096; c.num_src = 1;
  c.num_channels = 4; c.ring_entries = 16; c.num_proxy_threads = 2; c.reorder_window = 8; c.reorder_seed = 3;
  c.spin_timeout_ms = 5000; c.flags = EP_FLAG_HOST_ONLY | EP_FLAG_LOG_CMDS | EP_FLAG_LOG_EVENTS;
  if (policies) {
    c.max_outstanding = 5; c.pack_rows = 4; c.pack_hold_us = 20; c.ht_slices = 2; c.ht_ring_slots = 2;
    c.flags |= EP_FLAG_SENDER_FENCE;
  }
  ep_handle* h = nullptr;
  if (ep_proxy_start(&c, &h)) { printf("start failed\n"); return 1; }
  const int per = 500;
  for (int rep = 0; rep < 3; ++rep) {
    ep_host_expect_atomics(h, 16);
    std::vector<std::thread> ts;
    for (int p = 0; p < 4; ++p) ts.emplace_back([&, p] {
      for (int e = p; e < 16; e += 4) {
        uint32_t dr = e / 4, le = e % 4; uint64_t idx;
        ep_host_push(h, e % 4, w0(2, 0, dr, le), per, 0, le, &idx);
        for (int i = 0; i < per; ++i) ep_host_push(h, e % 4, w0(1, 0, dr, le), 2048 >> 4, 0, i * 128, &idx);
      }
    });
    for (auto& t : ts) t.join();
    // sequenced messages of one communication channel pushed by two threads in interleaved order
    std::thread o1([&] { for (uint32_t q = 0; q < 400; q += 4) { uint64_t i; ep_host_push(h, 1, w0(5, 0, 1, 0), 2048 >> 4, rep * 400 + q, 0, &i); ep_host_push(h, 1, w0(6, 0, 1, 0), 1, rep * 400 + q + 1, 1, &i); } });
    std::thread o2([&] { for (uint32_t q = 2; q < 400; q += 4) { uint64_t i; ep_host_push(h, 1, w0(5, 0, 1, 0), 2048 >> 4, rep * 400 + q, 0, &i); ep_host_push(h, 1, w0(6, 0, 1, 0), 1, rep * 400 + q + 1, 1, &i); } });
    o1.join(); o2.join();
    if (policies) {
      // one ring-buffer channel (slice 1, rank 2): a "sender" thread announces chunks, a "receiver" thread
      // releases them; both honour the counters the proxy posts
      const int32_t *tail = nullptr, *head = nullptr;
      ep_ring_counters(h, &tail, &head);
      const int chan = 1 * 4 + 2, fifo = chan % 4, chunks = 60;
      const uint32_t sb = 128 + 32 * 2048, base = rep * chunks;
      std::thread snd([&] {
        for (int n = 0; n < chunks; ++n) {
          while (n >= 2 && __atomic_load_n(&head[chan], __ATOMIC_ACQUIRE) < (int)(base + n - 1) * 32) std::this_thread::yield();
          uint64_t i;
          const uint32_t off = ((uint32_t)chan * 2 + n % 2) * sb;
          ep_host_push(h, fifo, w0(7, 0, 2, 1), (0u << 30) | (31u << 24) | ((128 + 32 * 2048) >> 4), 2 * (base + n), off >> 4, &i);
          ep_host_push(h, fifo, w0(7, 0, 2, 1), (1u << 30) | 32u, 2 * (base + n) + 1, 0, &i);
        }
      });
      std::thread rcv([&] {
        for (int n = 0; n < chunks; ++n) {
          while (__atomic_load_n(&tail[chan], __ATOMIC_ACQUIRE) < (int)(base + n + 1) * 32) std::this_thread::yield();
          uint64_t i;
          ep_host_push(h, fifo, w0(7, 0, 2, 1), (2u << 30) | 32u, base + n, 0, &i);
        }
      });
      snd.join(); rcv.join();
    }
    uint64_t di[4];
    for (int c2 = 0; c2 < 4; ++c2) ep_host_push(h, c2, w0(3, 0, 0, 0), 0, 0, 0, &di[c2]);
    uint64_t bi; ep_host_push(h, 0, w0(4, 0, 0, 0), 0, 0, 0, &bi);
    while (!ep_host_check_completion(h, 0, bi)) std::this_thread::yield();
    for (int c2 = 0; c2 < 4; ++c2) while (!ep_host_check_completion(h, c2, di[c2])) std::this_thread::yield();
    int rc = ep_wait(h);
    ep_stats_t st; ep_stats(h, &st);
    size_t n = 0; ep_cmd_log(h, nullptr, 0, &n);
    const int32_t *tails = nullptr; ep_tail_counters(h, &tails);
    printf("rep %d rc %d cmds %lu applied %lu deferred %lu parked %lu barriers %lu tail %d log %zu\n", rep, rc,
           (unsigned long)st.cmds, (unsigned long)st.atomics_applied, (unsigned long)st.atomics_deferred,
           (unsigned long)st.ordered_parked, (unsigned long)st.barriers, tails[1], n);
    if (rc != 0 || st.atomics_applied != 16 || tails[1] != 200 || st.proxy_error != 0) return 2;
    if (policies) {
      const int32_t *tail = nullptr, *head = nullptr;
      ep_ring_counters(h, &tail, &head);
      printf("   policies: msgs %lu of %lu writes, paced %lu, peak in flight %lu, sender held %lu, ring tail %d head %d\n",
             (unsigned long)st.write_msgs, (unsigned long)st.writes, (unsigned long)st.paced,
             (unsigned long)st.max_in_flight, (unsigned long)st.sender_held, tail[6], head[6]);
      if (st.max_in_flight > 5 || st.atomics_deferred != 0 || tail[6] != (rep + 1) * 60 * 32 || head[6] != tail[6] ||
          st.write_msgs >= st.writes)
        return 3;
    }
    ep_reset_stats(h);
  }
  ep_proxy_stop(h);
  return 0;
}
