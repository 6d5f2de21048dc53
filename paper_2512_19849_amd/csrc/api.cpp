// Set-up, tear-down and the C ABI of libep.so: argument checks, buffer allocation, kernel launches,
// statistics and logs.  Every entry point is declared in include/ep.h.
#include "ep_host.h"

namespace ep {

thread_local char g_last_error[256] = "";

bool hip_ok(hipError_t e, const char *what) {
  if (e == hipSuccess) return true;
  snprintf(g_last_error, sizeof(g_last_error), "%s: %s (%d)", what, hipGetErrorString(e), (int)e);
  return false;
}

}  // namespace ep

using namespace ep;

namespace {

bool is_pow2(uint32_t v) { return v && !(v & (v - 1)); }

int env_int(const char *name, int dflt) {
  const char *s = getenv(name);
  return (s && *s) ? atoi(s) : dflt;
}

// The EP_* launch-shape overrides, read once per handle; no launch looks at the environment.
Tunables read_tunables() {
  Tunables t;
  t.dispatch_vpl = env_int("EP_DISPATCH_VPL", t.dispatch_vpl);
  t.dispatch_fp8_vpl = env_int("EP_DISPATCH_FP8_VPL", t.dispatch_fp8_vpl);
  t.per_token_waves = env_int("EP_PER_TOKEN_WAVES", t.per_token_waves);
  t.dispatch_pipeline = env_int("EP_DISPATCH_PIPELINE", t.dispatch_pipeline);
  t.combine_vpl = env_int("EP_COMBINE_VPL", t.combine_vpl);
  t.layout_small = env_int("EP_LAYOUT_SMALL", t.layout_small);
  t.layout_tpb = env_int("EP_LAYOUT_TPB", t.layout_tpb);
  t.ht_threads = env_int("EP_HT_THREADS", t.ht_threads);
  const int mb = env_int("EP_COMBINE_FRESH_MB", t.combine_fresh_mb);
  t.combine_fresh_mb = mb < 0 ? 0 : (mb > 4096 ? 4096 : mb);
  return t;
}

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

// ep_profile: a fresh pair of events for one launch of call `which` (0 layout, 1 dispatch, 2 combine); false
// (and the launch goes untimed) when profiling is off, the stream is being captured, or no event can be made.
bool make_spare_events(ep_handle *h, size_t n) {
  while (h->spare_events.size() < n) {
    hipEvent_t e = nullptr;
    if (hipEventCreate(&e) != hipSuccess) {
      (void)hipGetLastError();
      return false;
    }
    h->spare_events.push_back(e);
  }
  return true;
}

bool timing_for(ep_handle *h, int which, void *stream, LaunchTiming *t) {
  if (!h->profiling || h->timed[which].size() >= 65536) return false;  // (never read: stop collecting)
  hipStreamCaptureStatus st = hipStreamCaptureStatusNone;
  if (hipStreamIsCapturing((hipStream_t)stream, &st) != hipSuccess) (void)hipGetLastError();
  if (st == hipStreamCaptureStatusActive) return false;
  if (h->spare_events.size() < 2 && !make_spare_events(h, 2)) return false;
  hipEvent_t a = h->spare_events.back();
  h->spare_events.pop_back();
  hipEvent_t b = h->spare_events.back();
  h->spare_events.pop_back();
  h->timed[which].emplace_back(a, b);
  t->start = a;
  t->stop = b;
  return true;
}

void drop_timed(ep_handle *h) {
  for (auto &v : h->timed) {
    for (auto &p : v) {
      (void)hipEventDestroy(p.first);
      (void)hipEventDestroy(p.second);
    }
    v.clear();
  }
  for (hipEvent_t e : h->spare_events) (void)hipEventDestroy(e);
  h->spare_events.clear();
}

// A launch entry point adds what its kernel will push to the counts ep_wait waits for - unless the
// stream is being captured into a graph: then nothing runs now, and the counts go to a ledger the
// caller reads with ep_captured and re-registers with ep_expect before every launch of the graph.
void expect_more(ep_handle *h, void *stream, int64_t atomics, int64_t drains) {
  hipStreamCaptureStatus st = hipStreamCaptureStatusNone;
  if (hipStreamIsCapturing((hipStream_t)stream, &st) != hipSuccess) {
    (void)hipGetLastError();  // (the legacy stream cannot be asked while another stream captures)
    st = hipStreamCaptureStatusNone;
  }
  if (st == hipStreamCaptureStatusActive) {
    h->captured_atomics.fetch_add(atomics, std::memory_order_relaxed);
    h->captured_drains.fetch_add(drains, std::memory_order_relaxed);
  } else {
    h->expected_atomics.fetch_add(atomics, std::memory_order_relaxed);
    h->expected_drains.fetch_add(drains, std::memory_order_relaxed);
  }
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
  h->tune = read_tunables();
  h->cache_hints = (cfg->flags & EP_FLAG_CACHE_HINTS) != 0;
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
    // grid-completion counters of the Drain epilogue: one per 64 workgroups (grids reach 2^19 workgroups) + 1
    if (!rc) rc = dev_alloc_zero(&h->waves_done, (size_t)(1 + (1 << 19) / 64 + 1) * 4);
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
    // (set-up is also where the static scratch of ep_layout_static gets its address looked up on this device)
    if (!rc && !HIP_OK((hipError_t)static_layout_scratch(nullptr))) rc = EP_EHIP;
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
    P.plain_writes = cfg->max_outstanding == 0 && cfg->pack_rows <= 1 && cfg->reorder_window == 0 &&
                     !(cfg->flags & (EP_FLAG_LOG_EVENTS | EP_FLAG_SENDER_FENCE));
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
  drop_timed(h);
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
  LaunchTiming tm{nullptr, nullptr};
  const bool timed = T > 0 && timing_for(h, 0, stream, &tm);
  return HIP_OK((hipError_t)launch_layout(a, h->tune, stream, timed ? &tm : nullptr)) ? EP_OK : EP_EHIP;
}

int ep_layout_static(const int32_t *d_topk_idx, int32_t S, int32_t T, int32_t K, int32_t E, int32_t R,
                     int32_t *d_count, int32_t *d_expert_total, int32_t *d_rank_total, int32_t *d_base,
                     int32_t *d_expert_offset, int32_t *d_rank_offset, int32_t *d_slot, int32_t *d_dst_row,
                     int32_t *d_status, void *stream) {
  if (R < 1 || R > 256 || E < 1 || E > kMaxExperts || E % R || K < 1 || K > 64 || S < 1 || S > 256) return EP_EINVAL;
  if (T < 0 || T >= (1 << 19)) return EP_EINVAL;
  if (!d_count || !d_expert_total || !d_rank_total || !d_base || !d_expert_offset || !d_rank_offset) return EP_EINVAL;
  if (T > 0 && (!d_topk_idx || !d_slot || !d_dst_row)) return EP_EINVAL;
  const int ntiles = (T + kLayoutTile - 1) / kLayoutTile;
  const long long entries = ((long long)S * ntiles + 1) * E;
  if (entries > kStaticLayoutEntries) {
    snprintf(g_last_error, sizeof(g_last_error),
             "ep_layout_static: (S * ceil(T/64) + 1) * E = %lld scratch entries, the static buffer holds %lld",
             entries, kStaticLayoutEntries);
    return EP_EINVAL;
  }
  LayoutArgs a{};
  a.idx = d_topk_idx;
  a.S = S;
  a.T = T;
  a.K = K;
  a.E = E;
  a.R = R;
  a.E_loc = E / R;
  a.ntiles = ntiles;
  a.count = d_count;
  a.expert_total = d_expert_total;
  a.rank_total = d_rank_total;
  a.base = d_base;
  a.expert_offset = d_expert_offset;
  a.rank_offset = d_rank_offset;
  a.slot = d_slot;
  a.dst_row = d_dst_row;
  a.error = d_status;  // null: errors go to a sink inside the static array
  if (!HIP_OK((hipError_t)static_layout_scratch(&a))) return EP_EHIP;
  // the array keeps what the last call left: the ticket has to start at zero (a fill kernel, not a memset
  // node, so that the call can be captured into a graph)
  if (!HIP_OK((hipError_t)launch_fill_u32(a.ticket, 0u, 1, stream))) return EP_EHIP;
  return HIP_OK((hipError_t)launch_layout(a, Tunables{}, stream, nullptr)) ? EP_OK : EP_EHIP;
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
  // With registered heaps and commands on, the proxy moves the rows.  FP8 rows then travel as one message
  // each (codes, scales, padding), so there is no separate scale array on the sending side.
  const char *const dbase = h->dst_base.load(std::memory_order_acquire);
  const bool proxy_moves = dbase != nullptr && mode != EP_CMD_NONE;
  const bool msg_rows = proxy_moves && payload == EP_FP8_E4M3;
  if (proxy_moves) {
    // the offsets the kernel is about to put into its commands must be relative to the registered heaps
    const uint64_t rb = row_bytes_of(c.hidden, payload);
    const void *sbase = (const void *)h->src_base.load();
    const bool chunked = mode != EP_CMD_PER_TOKEN;
    if (chunked) {  // the kernel packs a send heap laid out like the receive heap; chunks are forwarded
      if ((cmd_mode & EP_CMD_NO_PLACEMENT) || d_recv != sbase) return EP_EINVAL;
      if ((uint64_t)recv_rows * rb > h->src_bytes || (uint64_t)recv_rows * rb > h->dst_bytes) return EP_EINVAL;
    } else {        // every row is forwarded on its own, out of x (bf16) or out of one message per token (FP8)
      if (!(cmd_mode & EP_CMD_NO_PLACEMENT)) return EP_EINVAL;
      if (payload == EP_BF16 && d_x != sbase) return EP_EINVAL;
      if (payload == EP_FP8_E4M3 && (d_recv != sbase || (uint64_t)T * rb > h->src_bytes)) return EP_EINVAL;
      if ((uint64_t)recv_rows * rb > h->dst_bytes) return EP_EINVAL;
    }
    if (msg_rows && d_recv_scale) return EP_EINVAL;
  } else if (cmd_mode & EP_CMD_NO_PLACEMENT) {
    return EP_EINVAL;
  }
  if (recv_rows < 0 || recv_rows > c.heap_rows) return EP_EINVAL;
  if (T > 0 && (!d_x || !d_topk_idx || !d_dst_row || !d_recv)) return EP_EINVAL;
  if (!msg_rows && (payload == EP_FP8_E4M3) != (d_recv_scale != nullptr)) return EP_EINVAL;
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
  a.msg_rows = msg_rows ? (mode == EP_CMD_PER_TOKEN ? 2 : 1) : 0;
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
      expect_more(h, stream, 0, c.num_channels);
    else
      expect_more(h, stream, dst_rank_filter < 0 ? c.num_experts : h->E_loc, 0);
  }
  if (T == 0) {
    // nothing to launch; a ring-on dispatch of zero tokens still owes its (all zero) count atomics,
    // which only a kernel can push: run it with one idle workgroup
    if (mode == EP_CMD_NONE) return EP_OK;
    a.T = 0;
  }
  a.cache_hinted = h->cache_hints ? 1 : 0;
  if (h->cache_hints && T > 0 && !(cmd_mode & EP_CMD_NO_PLACEMENT)) {
    a.reverse = h->last_recv.load(std::memory_order_relaxed) == d_recv
                    ? !h->last_reverse.load(std::memory_order_relaxed)
                    : 0;
    h->last_recv.store(d_recv, std::memory_order_relaxed);
    h->last_reverse.store(a.reverse, std::memory_order_relaxed);
  }
  LaunchTiming tm{nullptr, nullptr};
  const bool timed = timing_for(h, 1, stream, &tm);
  const bool ok = HIP_OK((hipError_t)launch_dispatch(a, payload, h->tune, stream, timed ? &tm : nullptr));
  const bool all_rows = ok && h->cache_hints && payload == EP_BF16 && dst_rank_filter < 0 &&
                        !(cmd_mode & EP_CMD_NO_PLACEMENT) && T > 0;
  h->fresh_reverse.store(a.reverse, std::memory_order_relaxed);
  h->fresh_buf.store(all_rows ? d_recv : nullptr, std::memory_order_relaxed);
  h->fresh_T.store(T, std::memory_order_relaxed);
  h->fresh_stream.store(stream, std::memory_order_relaxed);
  return ok ? EP_OK : EP_EHIP;
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
  a.fresh_from = T;
  if (h->cache_hints && d_y && h->fresh_buf.exchange(nullptr, std::memory_order_relaxed) == d_y &&
      h->fresh_T.load(std::memory_order_relaxed) == T && h->fresh_stream.load(std::memory_order_relaxed) == stream) {
    // the dispatch kernel stored the tokens' rows in token order: the rows of the last tokens are what the
    // memory-side cache (256 MB) still holds
    const int64_t per_token = (int64_t)a.K * a.H * 2;
    const int64_t budget = (int64_t)h->tune.combine_fresh_mb << 20;
    const int64_t n = per_token > 0 ? budget / per_token : 0;
    a.fresh_from = n >= T ? 0 : T - (int32_t)n;
    a.fresh_head = h->fresh_reverse.load(std::memory_order_relaxed);
  }
  LaunchTiming tm{nullptr, nullptr};
  const bool timed = timing_for(h, 2, stream, &tm);
  return HIP_OK((hipError_t)launch_combine(a, h->tune, stream, timed ? &tm : nullptr)) ? EP_OK : EP_EHIP;
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
  h->fresh_buf.store(nullptr, std::memory_order_relaxed);
  return HIP_OK((hipError_t)launch_combine_partial(a, stream)) ? EP_OK : EP_EHIP;
}

int ep_fp8_unpack(ep_handle *h, const void *d_msgs, int64_t rows, void *d_recv, float *d_recv_scale, void *stream) {
  if (!h) return EP_EINVAL;
  if (h->host_only) return EP_ESTATE;
  if (rows < 0 || rows > h->cfg.heap_rows) return EP_EINVAL;
  if (rows == 0) return EP_OK;
  if (!d_msgs || !d_recv || !d_recv_scale) return EP_EINVAL;
  if (((uintptr_t)d_msgs | (uintptr_t)d_recv) & 15) return EP_EINVAL;
  return HIP_OK((hipError_t)launch_fp8_unpack(d_msgs, rows, h->cfg.hidden, row_bytes_of(h->cfg.hidden, EP_FP8_E4M3),
                                              d_recv, d_recv_scale, stream))
             ? EP_OK
             : EP_EHIP;
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
  expect_more(h, stream, (int64_t)pushers * cmds_per_pusher, 0);
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
  expect_more(h, stream, 0, c.num_channels);
  h->fresh_buf.store(nullptr, std::memory_order_relaxed);
  return HIP_OK((hipError_t)launch_ht_ring(a, h->tune, stream)) ? EP_OK : EP_EHIP;
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

int ep_row_probe(int32_t kind, const int32_t *d_rowmap, int32_t k, int64_t items, int32_t row_bytes, int64_t buf_rows,
                 void *d_buf, void *d_sink, void *stream) {
  if (kind < 0 || kind > 1 || !d_rowmap || !d_buf || !d_sink) return EP_EINVAL;
  if (k < 1 || k > 64 || items < 0 || items >= (1ll << 31) || buf_rows < 0) return EP_EINVAL;
  if (row_bytes < 16 || (row_bytes & 15) || row_bytes > (1 << 20)) return EP_EINVAL;
  if (((uintptr_t)d_buf | (uintptr_t)d_sink) & 15) return EP_EINVAL;
  if (items * (((int64_t)row_bytes / 16 + 63) / 64) >= (1ll << 33)) return EP_EINVAL;  // grid index range
  return HIP_OK((hipError_t)launch_row_probe(kind, d_rowmap, k, items, row_bytes, buf_rows, d_buf, d_sink, stream))
             ? EP_OK
             : EP_EHIP;
}

int ep_profile(ep_handle *h, int32_t on) {
  if (!h) return EP_EINVAL;
  if (h->host_only) return EP_ESTATE;
  if (on < 0 || on > 65536) return EP_EINVAL;
  // events are made here, ahead of the launches that use them (creating one costs microseconds)
  if (on > 0 && !make_spare_events(h, 2 * (size_t)on)) return EP_EHIP;
  h->profiling = on != 0;
  return EP_OK;
}

int ep_profile_read(ep_handle *h, int32_t call, double *total_ms, int32_t *launches, int32_t reset) {
  if (!h || call < 0 || call > 2 || !total_ms || !launches) return EP_EINVAL;
  if (h->host_only) return EP_ESTATE;
  double sum = 0.0;
  int n = 0;
  for (auto &p : h->timed[call]) {
    float ms = 0.0f;
    // the stop event completes with the launch's last kernel
    if (!HIP_OK(hipEventSynchronize(p.second)) || !HIP_OK(hipEventElapsedTime(&ms, p.first, p.second))) return EP_EHIP;
    sum += ms;
    ++n;
  }
  *total_ms = sum;
  *launches = n;
  if (reset) {
    for (auto &p : h->timed[call]) {
      h->spare_events.push_back(p.first);
      h->spare_events.push_back(p.second);
    }
    h->timed[call].clear();
  }
  return EP_OK;
}

int ep_captured(ep_handle *h, int64_t *atomics, int64_t *drains, int32_t reset) {
  if (!h || !atomics || !drains) return EP_EINVAL;
  if (reset) {
    *atomics = h->captured_atomics.exchange(0);
    *drains = h->captured_drains.exchange(0);
  } else {
    *atomics = h->captured_atomics.load();
    *drains = h->captured_drains.load();
  }
  return EP_OK;
}

int ep_expect(ep_handle *h, int64_t atomics, int64_t drains) {
  if (!h || atomics < 0 || drains < 0) return EP_EINVAL;
  h->expected_atomics.fetch_add(atomics, std::memory_order_relaxed);
  h->expected_drains.fetch_add(drains, std::memory_order_relaxed);
  return EP_OK;
}

int ep_host_expect_atomics(ep_handle *h, int32_t n) {
  if (!h || n < 0) return EP_EINVAL;
  h->expected_atomics.fetch_add(n, std::memory_order_relaxed);
  return EP_OK;
}

}  // extern "C"
