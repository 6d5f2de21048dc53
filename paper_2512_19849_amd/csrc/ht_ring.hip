// Ring-buffer communication channels of the high-throughput mode: one sender and one receiver workgroup per
// token slice, chunk slots reused under head/tail flow control.
#include "ep_device.h"

namespace ep {

// ------------------------------------------- ring-buffer channels (HT mode)
// Section 3.3 ("partial ordering"): tokens travel through rings of chunk slots; the sender may reuse
// a slot only after the receiver released it (head), the receiver may read it only after it was
// announced (tail); Write, tail Atomic and head Atomic are sequenced per channel and pass through the
// proxy.  A slice's sender and receiver workgroups are 8 apart in the grid (so that they become
// resident together); a workgroup depends on no workgroup but its partner.
// Every wait is bounded; after a timeout the workgroup's abort flag sends every wave to the exit.
constexpr int kHtMaxRanks = 256, kHtMaxSlots = 4096, kHtHeader = 128, kHtMaxOrder = 4096;

struct HtShared {
  int total[kHtMaxRanks];      // rows of channel (slice, r) in this dispatch
  int fill[kHtMaxRanks];       // sender: positions handed out; receiver: next chunk to consume
  unsigned seqb[kHtMaxRanks];  // the channel's sequence number before this dispatch
  unsigned cumb[kHtMaxRanks];  // rows the channel carried before this dispatch
  unsigned seen[kHtMaxRanks];  // sender: rows released so far (cached head); receiver: first chunk of this sweep
  int lock[kHtMaxRanks];       // sender: who refreshes the cached head; receiver: end chunk of this sweep
  int done[kHtMaxSlots];       // sender: rows stored per (r, slot)
  int order[kHtMaxOrder];      // sender: the slice's valid entries ((t - t0) * K + k), rank-major
  int start[kHtMaxRanks];      // sender: where rank r's entries begin in the order list
  int abort, remaining, progress, idle, sorted, nentries;
};

#define HT_LD(p) __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP)
#define HT_ST(p, v) __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP)

EP_DEV bool ht_valid(const HtRingArgs &a, int e, int row) {
  return e >= 0 && e / a.E_loc < a.R && row >= 0 && row < a.recv_rows;
}

// A wave moves a row in pieces of B KiB: B 16-byte loads per lane in flight, then B stores.
template <bool STREAM, int B>
EP_DEV void ht_load_piece(u32x4 (&r)[B], const u32x4 *src, int v0, int nvec) {
#pragma unroll
  for (int i = 0; i < B; ++i)
    if (v0 + i * 64 < nvec) r[i] = STREAM ? __builtin_nontemporal_load(src + v0 + i * 64) : src[v0 + i * 64];
}
template <bool THROUGH, int B>
EP_DEV void ht_store_piece(const u32x4 (&r)[B], u32x4 *dst, int v0, int nvec) {
#pragma unroll
  for (int i = 0; i < B; ++i)
    if (v0 + i * 64 < nvec) {
      if (THROUGH) store_payload(dst + v0 + i * 64, r[i]);
      else dst[v0 + i * 64] = r[i];
    }
}
template <bool STREAM, bool THROUGH, int B>
EP_DEV void ht_copy_row(u32x4 (&r)[B], u32x4 *dst, const u32x4 *src, int nvec, int lane) {
  for (int v0 = lane; v0 < nvec; v0 += 64 * B) {
    ht_load_piece<STREAM, B>(r, src, v0, nvec);
    ht_store_piece<THROUGH, B>(r, dst, v0, nvec);
  }
}

// Sender: wait until `need` rows of channel r have been released in this dispatch.
EP_DEV bool ht_wait_head(const HtRingArgs &a, HtShared &sh, int chan, int r, unsigned need, int lane) {
  const unsigned long long t0 = wall_clock64();
  for (;;) {
    if (HT_LD(&sh.abort)) return false;
    if (HT_LD(&sh.seen[r]) >= need) return true;
    if (lane == 0 && __hip_atomic_exchange(&sh.lock[r], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP) == 0) {
      // one PCIe read on behalf of every wave of the workgroup that waits for this channel
      const unsigned v =
          (unsigned)__hip_atomic_load(a.head + chan, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM) - sh.cumb[r];
      __hip_atomic_fetch_max(&sh.seen[r], v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
      HT_ST(&sh.lock[r], 0);
    }
    if (wall_clock64() - t0 > a.fifo.timeout_ticks) {
      dev_set_error(a.fifo.error, EP_ETIMEOUT);
      HT_ST(&sh.abort, 1);
      return false;
    }
    __builtin_amdgcn_s_sleep(32);
  }
}

// Sender bookkeeping for the rows a wave has stored but not yet counted: lane k keeps (rank, chunk)
// of the token's k-th entry.  After one wait for the wave's stores, every such lane adds its row to
// the chunk's count; the lane that completes a chunk announces it (Write, then the tail Atomic).
EP_DEV void ht_count_stored(const HtRingArgs &a, HtShared &sh, int c, bool mine, int r, int n) {
  wait_for_own_stores();
  if (!mine) return;
  const int w = n % a.W, sz = min(kChunkRows, sh.total[r] - (n << 5));
  const int old = __hip_atomic_fetch_add(&sh.done[r * a.W + w], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
  if (old + 1 != sz) return;
  HT_ST(&sh.done[r * a.W + w], 0);
  const int chan = c * a.R + r;
  const unsigned seq = sh.seqb[r] + 2u * (unsigned)n, fifo = (unsigned)chan % a.fifo.channels;
  const unsigned len = (unsigned)kHtHeader + (unsigned)sz * a.row_bytes;
  const unsigned w0 = cmd_w0(EP_OP_RING, a.src, (unsigned)r, (unsigned)c);
  ring_push(a.fifo, fifo, w0, ((unsigned)EP_RING_WRITE << 30) | ((unsigned)(sz - 1) << 24) | (len >> 4), seq,
            (unsigned)((((size_t)chan * a.W + w) * a.slot_bytes) >> 4));
  ring_push(a.fifo, fifo, w0, ((unsigned)EP_RING_TAIL << 30) | (unsigned)sz, seq + 1u, 0u);
}

// One (token, k) entry: claim the next position of its channel, wait for the slot if need be, store
// row and header.  Lane j of the wave remembers (rank, chunk) until the rows are counted.  Returns
// false when the workgroup is aborting.
struct HtPending {
  bool mine;
  int r, n;
};
EP_DEV bool ht_send_entry(const HtRingArgs &a, HtShared &sh, int c, int t, int k, int j, HtPending &pd, int lane) {
  const int e = a.idx[(size_t)t * a.K + k], row = a.dst_row[(size_t)t * a.K + k];
  if (!ht_valid(a, e, row)) return true;
  if (HT_LD(&sh.abort)) return false;
  const int nvec = a.H >> 3;
  const unsigned rb = a.row_bytes;
  const int r = e / a.E_loc, chan = c * a.R + r;
  // positions are handed out in arrival order
  int p = 0;
  if (lane == 0) p = __hip_atomic_fetch_add(&sh.fill[r], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
  p = __builtin_amdgcn_readfirstlane(p);
  const int n = p >> 5, slot_row = p & 31, w = n % a.W;
  if (n >= a.W && HT_LD(&sh.seen[r]) < 32u * (unsigned)(n - a.W + 1)) {
    // The slot is not known to be free.  Rows this wave has stored but not counted could be what
    // another wave's chunk is waiting for, so they are counted before this wave blocks: a waiting
    // wave then holds nothing but the position it waits for, and the rows of a channel's oldest
    // unreleased chunk can always be written.
    if (__any(pd.mine)) {
      ht_count_stored(a, sh, c, pd.mine, pd.r, pd.n);
      pd.mine = false;
    }
    if (!ht_wait_head(a, sh, chan, r, 32u * (unsigned)(n - a.W + 1), lane)) return false;
  }
  char *slot = (char *)a.ring_buf + ((size_t)chan * a.W + w) * a.slot_bytes;
  char *dst = slot + kHtHeader + (size_t)slot_row * rb;
  const u32x4 *xrow = (const u32x4 *)((const char *)a.x + (size_t)t * 2u * (unsigned)a.H);
  if (a.payload == EP_BF16) {
    u32x4 regs[8];  // cached loads: the token's row comes from HBM once and from a cache for its other k
    ht_copy_row<false, true, 8>(regs, (u32x4 *)dst, xrow, nvec, lane);
  } else {
    // FP8 message: the row's E4M3 codes, then one fp32 scale per 128 channels (Section 2.1: the ~7 KB token)
    const int npair = a.H >> 4;
    for (int p0 = 0; p0 < npair; p0 += 64) {
      const int p = p0 + lane;
      u32x4 lo = {0, 0, 0, 0}, hi = {0, 0, 0, 0}, q;
      float sc;
      if (p < npair) {
        lo = xrow[2 * p];
        hi = xrow[2 * p + 1];
      }
      quant16(lo, hi, q, sc);
      if (p < npair) {
        store_payload((u32x4 *)dst + p, q);
        if ((lane & 7) == 0)
          __hip_atomic_store((float *)(dst + a.H) + (p >> 3), sc, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
      }
    }
  }
  if (lane == 0) __hip_atomic_store((int *)slot + slot_row, row, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
  if (lane == j) {
    pd.mine = true;
    pd.r = r;
    pd.n = n;
  }
  return true;
}

EP_DEV void ht_sender(const HtRingArgs &a, HtShared &sh, int c, int t0, int t1) {
  const int lane = lane_id(), wave = threadIdx.x >> 6, nwaves = blockDim.x >> 6;
  HtPending pd{false, 0, 0};
  if (sh.sorted) {
    // Entries in rank-major order (the order list), dealt to the waves round-robin, 8 per wave between
    // two waits for its stores: the chunks of the first ranks are complete after the first round, so
    // the receiver works while the sender is still busy with the later ranks.
    constexpr int G = 8;
    const int total = sh.nentries;
    for (int first = 0; first < total; first += G * nwaves) {
      for (int j = 0; j < G; ++j) {
        const int i = first + j * nwaves + wave;
        if (i >= total) break;
        const int ent = sh.order[i];
        if (!ht_send_entry(a, sh, c, t0 + ent / a.K, ent % a.K, j, pd, lane)) return;
      }
      if (__any(pd.mine)) {
        ht_count_stored(a, sh, c, pd.mine, pd.r, pd.n);
        pd.mine = false;
      }
    }
    return;
  }
  // slices too long for the order list: token by token, all k of a token between two waits
  for (int t = t0 + wave; t < t1; t += nwaves) {
    for (int k = 0; k < a.K; ++k) {
      if (!ht_send_entry(a, sh, c, t, k, k & 63, pd, lane)) return;
      if (((k & 63) == 63 || k == a.K - 1) && __any(pd.mine)) {  // (top-k is at most 64: one entry per lane)
        ht_count_stored(a, sh, c, pd.mine, pd.r, pd.n);
        pd.mine = false;
      }
    }
    if (__any(pd.mine)) {
      ht_count_stored(a, sh, c, pd.mine, pd.r, pd.n);
      pd.mine = false;
    }
  }
}

EP_DEV void ht_receiver(const HtRingArgs &a, HtShared &sh, int c) {
  const int tid = threadIdx.x, lane = lane_id(), wave = tid >> 6, nwaves = blockDim.x >> 6;
  const bool fp8 = a.payload != EP_BF16;
  const int nvec = fp8 ? a.H >> 4 : a.H >> 3;  // 16-byte vectors of payload per row
  const unsigned rb = a.row_bytes;
  unsigned long long last = wall_clock64();
  for (;;) {
    // which chunks have been announced since the last sweep (at most W per channel)
    for (int r = tid; r < a.R; r += blockDim.x) {
      const int tot = sh.total[r], nch = (tot + 31) >> 5, n0 = sh.fill[r];
      int hi = n0;
      if (n0 < nch) {
        const unsigned avail =
            (unsigned)__hip_atomic_load(a.tail + c * a.R + r, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM) - sh.cumb[r];
        while (hi < nch && hi - n0 < a.W && avail >= (unsigned)min((hi + 1) << 5, tot)) ++hi;
      }
      sh.seen[r] = (unsigned)n0;
      sh.lock[r] = hi;
    }
    __syncthreads();
    // move their rows to where the header says; rows are dealt out to the waves round-robin
    int q = 0;
    for (int r = 0; r < a.R; ++r) {
      const int lo = (int)sh.seen[r], hi = sh.lock[r];
      for (int n = lo; n < hi; ++n) {
        if (q == 0) {
          // What the tails announced was written by another workgroup, possibly into lines an L2 still
          // holds from the slot's previous use: drop those before the first read of the sweep (the
          // acquire that pairs with the tail; not done on idle sweeps, it empties the XCD's L2).
          __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
        }
        const int sz = min(kChunkRows, sh.total[r] - (n << 5));
        const char *slot = (const char *)a.ring_buf + ((size_t)(c * a.R + r) * a.W + n % a.W) * a.slot_bytes;
        // this wave's rows of the chunk: j = first, first + nwaves, ... (rows are dealt round-robin over all chunks)
        const int first = (wave - q % nwaves + nwaves) % nwaves;
        q += sz;
        if (first >= sz) continue;
        // one load brings the destination rows of the whole chunk; the rows are then moved two at a
        // time so that the loads of both are in flight together
        const int hdr = lane < sz ? __builtin_nontemporal_load((const int *)slot + lane) : -1;
        const size_t out_stride = fp8 ? (size_t)a.H : (size_t)rb;
        for (int j = first; j < sz; j += 2 * nwaves) {
          const int j2 = j + nwaves;
          const int rowA = __builtin_amdgcn_readlane(hdr, __builtin_amdgcn_readfirstlane(j));
          const int rowB = j2 < sz ? __builtin_amdgcn_readlane(hdr, __builtin_amdgcn_readfirstlane(j2)) : -1;
          const bool okA = rowA >= 0 && rowA < a.recv_rows, okB = rowB >= 0 && rowB < a.recv_rows;
          if (!okA || (j2 < sz && !okB)) dev_set_error(a.fifo.error, EP_EBOUNDS);
          const char *srcA = slot + kHtHeader + (size_t)j * rb, *srcB = slot + kHtHeader + (size_t)j2 * rb;
          u32x4 *dstA = (u32x4 *)((char *)a.recv + (size_t)(okA ? rowA : 0) * out_stride);
          u32x4 *dstB = (u32x4 *)((char *)a.recv + (size_t)(okB ? rowB : 0) * out_stride);
          for (int v0 = lane; v0 < nvec; v0 += 64 * 8) {
            u32x4 ra[8], rb2[8];
            if (okA) ht_load_piece<true, 8>(ra, (const u32x4 *)srcA, v0, nvec);
            if (okB) ht_load_piece<true, 8>(rb2, (const u32x4 *)srcB, v0, nvec);
            if (okA) ht_store_piece<false, 8>(ra, dstA, v0, nvec);
            if (okB) ht_store_piece<false, 8>(rb2, dstB, v0, nvec);
          }
          if (fp8)  // the scales behind the codes go to their own array
            for (int b = lane; b < (a.H >> 7); b += 64) {
              if (okA) a.recv_scale[(size_t)rowA * (a.H >> 7) + b] = __builtin_nontemporal_load((const float *)(srcA + a.H) + b);
              if (okB) a.recv_scale[(size_t)rowB * (a.H >> 7) + b] = __builtin_nontemporal_load((const float *)(srcB + a.H) + b);
            }
        }
      }
    }
    wait_for_own_stores();  // every load of a slot has returned before the slot is released
    __syncthreads();
    // release the slots: one head Atomic per consumed chunk, numbered on the reverse channel
    for (int r = tid; r < a.R; r += blockDim.x) {
      const int lo = (int)sh.seen[r], hi = sh.lock[r];
      for (int n = lo; n < hi; ++n) {
        const int sz = min(kChunkRows, sh.total[r] - (n << 5));
        ring_push(a.fifo, (unsigned)(c * a.R + r) % a.fifo.channels, cmd_w0(EP_OP_RING, a.src, (unsigned)r, (unsigned)c),
                  ((unsigned)EP_RING_HEAD << 30) | (unsigned)sz, sh.seqb[r] + (unsigned)n, 0u);
      }
      if (hi > lo) {
        sh.fill[r] = hi;
        __hip_atomic_fetch_sub(&sh.remaining, hi - lo, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        HT_ST(&sh.progress, 1);
      }
    }
    __syncthreads();
    if (tid == 0) {
      const unsigned long long now = wall_clock64();
      const int progressed = HT_LD(&sh.progress);
      sh.idle = !progressed;
      if (HT_LD(&sh.remaining) <= 0) {
        sh.abort = 2;  // all chunks of the slice consumed
      } else if (progressed) {
        last = now;
        sh.progress = 0;
      } else if (now - last > a.fifo.timeout_ticks) {
        dev_set_error(a.fifo.error, EP_ETIMEOUT);
        sh.abort = 1;
      }
    }
    __syncthreads();
    if (sh.abort) break;
    if (sh.idle) __builtin_amdgcn_s_sleep(127);
  }
}

__global__ __launch_bounds__(1024) void ht_ring_kernel(HtRingArgs a) {
  __shared__ HtShared sh;
  // Workgroups are handed to the 8 XCDs round-robin.  In every run of 16 workgroups the first 8 are
  // the senders of 8 consecutive slices and the last 8 their receivers, so both roles are spread over
  // all XCDs (and their links to memory), and a slice's sender and receiver share an XCD and its L2.
  const int tid = threadIdx.x;
  const int c = ((blockIdx.x >> 4) << 3) | (blockIdx.x & 7);
  const bool sender = !(blockIdx.x & 8);
  const bool idle_wg = c >= a.slices;  // padding of the last run: takes part in nothing but the final count
  const int t0 = idle_wg ? 0 : min(a.T, c * a.slice_len), t1 = idle_wg ? 0 : min(a.T, t0 + a.slice_len);
  for (int r = tid; r < a.R; r += blockDim.x) {
    sh.total[r] = 0;
    sh.fill[r] = 0;
    sh.seen[r] = 0;
    sh.lock[r] = 0;
    sh.seqb[r] = idle_wg ? 0u : (sender ? a.seq_fwd : a.seq_rev)[c * a.R + r];
    sh.cumb[r] = idle_wg ? 0u : (sender ? a.cum_fwd : a.cum_rev)[c * a.R + r];
  }
  for (int i = tid; i < a.R * a.W; i += blockDim.x) sh.done[i] = 0;
  if (tid == 0) sh.abort = sh.remaining = sh.progress = sh.idle = 0;
  __syncthreads();
  // rows per channel of this slice: both sides count them from the routing table (the count
  // notification that precedes a high-throughput dispatch)
  for (int i = tid; i < (t1 - t0) * a.K; i += blockDim.x) {
    const int e = a.idx[(size_t)t0 * a.K + i], row = a.dst_row[(size_t)t0 * a.K + i];
    if (ht_valid(a, e, row))
      __hip_atomic_fetch_add(&sh.total[e / a.E_loc], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    else if (e >= 0)
      dev_set_error(a.fifo.error, EP_EBOUNDS);
  }
  __syncthreads();
  if (sender) {
    // rank-major list of the slice's entries, starting with rank c mod R so that the slices do not
    // all begin with the same destination
    if (tid == 0) {
      int acc = 0;
      for (int i = 0; i < a.R; ++i) {
        const int r = (c + i) % a.R;
        sh.start[r] = acc;
        acc += sh.total[r];
      }
      sh.nentries = acc;
      sh.sorted = (t1 - t0) * a.K <= kHtMaxOrder;
    }
    __syncthreads();
    if (sh.sorted)
      for (int i = tid; i < (t1 - t0) * a.K; i += blockDim.x) {
        const int e = a.idx[(size_t)t0 * a.K + i], row = a.dst_row[(size_t)t0 * a.K + i];
        if (ht_valid(a, e, row)) {
          const int r = e / a.E_loc;
          sh.order[sh.start[r] + __hip_atomic_fetch_add(&sh.lock[r], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP)] = i;
        }
      }
    __syncthreads();
    for (int r = tid; r < a.R; r += blockDim.x) sh.lock[r] = 0;  // from here on: the head-refresh locks
    __syncthreads();
    ht_sender(a, sh, c, t0, t1);
  } else {
    for (int r = tid; r < a.R; r += blockDim.x)
      __hip_atomic_fetch_add(&sh.remaining, (sh.total[r] + 31) >> 5, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    __syncthreads();
    ht_receiver(a, sh, c);
  }
  __syncthreads();
  // the channels' running sequence numbers and row totals, for the next dispatch
  for (int r = tid; r < a.R && !idle_wg; r += blockDim.x) {
    const unsigned nch = (unsigned)(sh.total[r] + 31) >> 5;
    if (sender) {
      a.seq_fwd[c * a.R + r] = sh.seqb[r] + 2u * nch;
      a.cum_fwd[c * a.R + r] = sh.cumb[r] + (unsigned)sh.total[r];
    } else {
      a.seq_rev[c * a.R + r] = sh.seqb[r] + nch;
      a.cum_rev[c * a.R + r] = sh.cumb[r] + (unsigned)sh.total[r];
    }
  }
  drain_all_channels(a.fifo, a.waves_done, (unsigned)a.src, lane_id());
}

int launch_ht_ring(const HtRingArgs &a, void *stream) {
  int threads = env_int("EP_HT_THREADS", 1024);
  if (threads < 64 || threads > 1024 || (threads & 63)) threads = 1024;
  hipLaunchKernelGGL(ht_ring_kernel, dim3(16u * (unsigned)((a.slices + 7) / 8)), dim3((unsigned)threads), 0, (hipStream_t)stream, a);
  return (int)hipGetLastError();
}

}  // namespace ep
