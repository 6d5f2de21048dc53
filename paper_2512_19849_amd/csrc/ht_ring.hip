// Ring-buffer communication channels of the high-throughput mode: one workgroup per token slice plays the
// sending and the receiving end in turns, chunk slots reused under head/tail flow control.
#include "ep_device.h"

namespace ep {

// ------------------------------------------- ring-buffer channels (HT mode)
// Section 3.3 ("partial ordering"): tokens travel through rings of chunk slots; the sender may reuse
// a slot only after the receiver released it (head), the receiver may read it only after it was
// announced (tail); Write, tail Atomic and head Atomic are sequenced per channel and pass through the
// proxy.
// One workgroup owns a token slice and plays both ends of the slice's channels in turns: a sending
// step (every wavefront takes a token, keeps its row in registers and stores it into the slot of
// each of its destinations that is known to be free, then announces the chunks it completed) and a
// receiving step (a sweep over the tails, the announced rows move to their final place, the slots
// are released).  Neither step waits for the other end: a wavefront whose slot is still occupied
// keeps its claimed position and tries again after the next sweep.  A workgroup therefore depends
// on nothing but the proxy, whatever the grid size and however many workgroups are resident, and
// every compute unit has rows to store all the time.
// On this hardware one counter tracks a wave's outstanding loads AND stores, so waiting for any load
// also waits for every store issued before it; the sending step is shaped around that: all of a
// token's metadata in one load, the row in one batch of loads, then nothing but stores.
// Every wait is bounded; without progress for the time limit the workgroup gives up with an error.
constexpr int kHtMaxRanks = 256, kHtMaxSlots = 4096, kHtHeader = 128;

struct HtShared {
  int total[kHtMaxRanks];      // rows of channel (slice, r) in this dispatch
  // sending end
  int fill[kHtMaxRanks];       // positions handed out
  unsigned seen[kHtMaxRanks];  // rows known to be released in this dispatch (cached head)
  int lock[kHtMaxRanks];       // who refreshes seen[r] over PCIe
  unsigned seqf[kHtMaxRanks];  // the channel's forward sequence number before this dispatch
  unsigned cumf[kHtMaxRanks];  // rows the channel carried before this dispatch (sender's count)
  int done[kHtMaxSlots];       // rows stored per (r, slot)
  // receiving end
  int next[kHtMaxRanks];       // next chunk to consume
  int lo[kHtMaxRanks], hi[kHtMaxRanks];  // chunks [lo, hi) are consumed in the current sweep
  unsigned seqr[kHtMaxRanks];  // the channel's reverse sequence number before this dispatch
  unsigned cumr[kHtMaxRanks];  // rows the channel carried before this dispatch (receiver's count)
  int abort, remaining, progress, idle;
};

#define HT_LD(p) __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP)
#define HT_ST(p, v) __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP)

EP_DEV bool ht_valid(const HtRingArgs &a, int e, int row) {
  return e >= 0 && e / a.E_loc < a.R && row >= 0 && row < a.recv_rows;
}

// B 16-byte vectors per lane of a row, starting at vector v0: loads in flight together, stores
// back to back.
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

// What a wave remembers of the token it is sending: lane k owns the token's k-th entry.
struct HtToken {
  unsigned long long pend;  // entries claimed but not stored yet (wave-uniform)
  int p;                    // lane k: the position claimed in its channel
};

// One token: claim a position per valid entry (unless the wave comes back to a token it could not
// finish), find the entries whose slot is free, load the row once and store it to each of them,
// write the headers, wait once for all the stores, count the rows and announce every chunk that
// became complete (Write, then the tail Atomic).  Returns true when the token is finished; false
// when some of its slots are still occupied (the wave has stored and counted what it could).
constexpr int kHtPiece = 16;  // vectors per lane held in registers (bf16 rows up to 8192 channels in one piece)
EP_DEV bool ht_send_token(const HtRingArgs &a, HtShared &sh, int c, int t, HtToken &tk) {
  const int lane = lane_id();
  int e = -1, row = -1;
  if (lane < a.K) {
    e = a.idx[(size_t)t * a.K + lane];
    row = a.dst_row[(size_t)t * a.K + lane];
  }
  const bool valid = lane < a.K && ht_valid(a, e, row);
  const int r = valid ? e / a.E_loc : 0, chan = c * a.R + r;
  if (tk.pend == 0ull) {  // a new token: positions are handed out in arrival order
    tk.p = valid ? __hip_atomic_fetch_add(&sh.fill[r], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP) : 0;
    tk.pend = __ballot(valid);
    if (tk.pend == 0ull) return true;
  }
  const bool mine = (tk.pend >> lane) & 1ull;
  const int n = tk.p >> 5, slot_row = tk.p & 31, w = n % a.W;
  bool occupied = false;
  if (mine && n >= a.W) {
    const unsigned need = 32u * (unsigned)(n - a.W + 1);
    if (HT_LD(&sh.seen[r]) < need) {
      // one PCIe read on behalf of every wave of the workgroup that needs this channel's head
      if (__hip_atomic_exchange(&sh.lock[r], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP) == 0) {
        const unsigned v =
            (unsigned)__hip_atomic_load(a.head + chan, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM) - sh.cumf[r];
        __hip_atomic_fetch_max(&sh.seen[r], v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        HT_ST(&sh.lock[r], 0);
      }
      occupied = HT_LD(&sh.seen[r]) < need;
    }
  }
  const bool go = mine && !occupied;
  const unsigned long long ready = __ballot(go);
  if (ready == 0ull) return false;
  // byte offset of the entry's row in the ring (slot header included), split for readlane
  const unsigned long long off =
      ((unsigned long long)chan * a.W + w) * a.slot_bytes + kHtHeader + (unsigned long long)slot_row * a.row_bytes;
  const unsigned off_lo = (unsigned)off, off_hi = (unsigned)(off >> 32);
  const u32x4 *xrow = (const u32x4 *)((const char *)a.x + (size_t)t * 2u * (unsigned)a.H);
  if (a.payload == EP_BF16) {
    const int nvec = a.H >> 3;
    for (int v0 = lane; v0 < nvec; v0 += 64 * kHtPiece) {
      u32x4 regs[kHtPiece];
      ht_load_piece<false, kHtPiece>(regs, xrow, v0, nvec);
      for (unsigned long long m = ready; m; m &= m - 1) {
        const int k = __builtin_ctzll(m);
        const unsigned long long o = ((unsigned long long)(unsigned)__builtin_amdgcn_readlane((int)off_hi, k) << 32) |
                                     (unsigned)__builtin_amdgcn_readlane((int)off_lo, k);
        ht_store_piece<true, kHtPiece>(regs, (u32x4 *)((char *)a.ring_buf + o), v0, nvec);
      }
    }
  } else {
    // FP8 message: the row's E4M3 codes, then one fp32 scale per 128 channels (Section 2.1: the ~7 KB
    // token); quantised once per token, stored to every destination
    constexpr int kPairs = 4;
    const int npair = a.H >> 4;
    for (int p0 = 0; p0 < npair; p0 += 64 * kPairs) {
      u32x4 q[kPairs];
      float sc[kPairs];
#pragma unroll
      for (int i = 0; i < kPairs; ++i) {
        const int p = p0 + i * 64 + lane;
        u32x4 lo = {0, 0, 0, 0}, hi = {0, 0, 0, 0};
        if (p < npair) {
          lo = xrow[2 * p];
          hi = xrow[2 * p + 1];
        }
        quant16(lo, hi, q[i], sc[i]);
      }
      for (unsigned long long m = ready; m; m &= m - 1) {
        const int k = __builtin_ctzll(m);
        const unsigned long long o = ((unsigned long long)(unsigned)__builtin_amdgcn_readlane((int)off_hi, k) << 32) |
                                     (unsigned)__builtin_amdgcn_readlane((int)off_lo, k);
        char *dst = (char *)a.ring_buf + o;
#pragma unroll
        for (int i = 0; i < kPairs; ++i) {
          const int p = p0 + i * 64 + lane;
          if (p < npair) {
            store_payload((u32x4 *)dst + p, q[i]);
            if ((lane & 7) == 0)
              __hip_atomic_store((float *)(dst + a.H) + (p >> 3), sc[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
          }
        }
      }
    }
  }
  if (go) {
    int *hdr = (int *)((char *)a.ring_buf + ((unsigned long long)chan * a.W + w) * a.slot_bytes);
    __hip_atomic_store(hdr + slot_row, row, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
  }
  wait_for_own_stores();
  if (go) {
    const int sz = min(kChunkRows, sh.total[r] - (n << 5));
    const int old = __hip_atomic_fetch_add(&sh.done[r * a.W + w], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    if (old + 1 == sz) {
      HT_ST(&sh.done[r * a.W + w], 0);
      const unsigned seq = sh.seqf[r] + 2u * (unsigned)n, fifo = (unsigned)chan % a.fifo.channels;
      const unsigned len = (unsigned)kHtHeader + (unsigned)sz * a.row_bytes;
      const unsigned w0 = cmd_w0(EP_OP_RING, a.src, (unsigned)r, (unsigned)c);
      ring_push(a.fifo, fifo, w0, ((unsigned)EP_RING_WRITE << 30) | ((unsigned)(sz - 1) << 24) | (len >> 4), seq,
                (unsigned)((((size_t)chan * a.W + w) * a.slot_bytes) >> 4));
      ring_push(a.fifo, fifo, w0, ((unsigned)EP_RING_TAIL << 30) | (unsigned)sz, seq + 1u, 0u);
    }
  }
  if (lane == 0) HT_ST(&sh.progress, 1);
  tk.pend &= ~ready;
  return tk.pend == 0ull;
}

// One sending step of a wavefront: the slice's tokens are dealt to the waves round-robin; a step
// takes about kHtStepRows rows' worth of them (q counts the wave's finished tokens).  Returns true
// when the wave has nothing left to send.
constexpr int kHtStepRows = 16;
EP_DEV bool ht_send_step(const HtRingArgs &a, HtShared &sh, int c, int t0, int ntok, int &q, HtToken &tk) {
  const int wave = threadIdx.x >> 6, nwaves = blockDim.x >> 6;
  const int budget = max(1, kHtStepRows / a.K);
  for (int j = 0; j < budget; ++j) {
    const int tt = wave + q * nwaves;
    if (tt >= ntok) return true;
    if (!ht_send_token(a, sh, c, t0 + tt, tk)) return false;
    ++q;
  }
  return false;
}

// One receiving step of the workgroup: a sweep over the slice's tails, the announced rows move to
// the rows their headers name, the consumed slots are released.  Called by every thread.
EP_DEV void ht_receive_step(const HtRingArgs &a, HtShared &sh, int c) {
  const int tid = threadIdx.x, lane = lane_id(), wave = tid >> 6, nwaves = blockDim.x >> 6;
  const bool fp8 = a.payload != EP_BF16;
  const int nvec = fp8 ? a.H >> 4 : a.H >> 3;  // 16-byte vectors of payload per row
  const unsigned rb = a.row_bytes;
  // which chunks have been announced since the last sweep (at most W per channel)
  for (int r = tid; r < a.R; r += blockDim.x) {
    const int tot = sh.total[r], nch = (tot + 31) >> 5, n0 = sh.next[r];
    int hi = n0;
    if (n0 < nch) {
      const unsigned avail =
          (unsigned)__hip_atomic_load(a.tail + c * a.R + r, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM) - sh.cumr[r];
      while (hi < nch && hi - n0 < a.W && avail >= (unsigned)min((hi + 1) << 5, tot)) ++hi;
    }
    sh.lo[r] = n0;
    sh.hi[r] = hi;
  }
  __syncthreads();
  // move their rows to where the header says; rows are dealt out to the waves round-robin
  int q = 0;
  for (int r = 0; r < a.R; ++r) {
    const int lo = sh.lo[r], hi = sh.hi[r];
    for (int n = lo; n < hi; ++n) {
      if (q == 0) {
        // What a tail announces reached memory from outside this compute unit's view (a network
        // adapter in the paper; here the sending step's write-through stores), possibly into lines
        // a cache still holds from the slot's previous use: drop those before the first read of
        // the sweep (the acquire that pairs with the tail; not done on idle sweeps, it empties
        // the XCD's L2).
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
    const int lo = sh.lo[r], hi = sh.hi[r];
    for (int n = lo; n < hi; ++n) {
      const int sz = min(kChunkRows, sh.total[r] - (n << 5));
      ring_push(a.fifo, (unsigned)(c * a.R + r) % a.fifo.channels, cmd_w0(EP_OP_RING, a.src, (unsigned)r, (unsigned)c),
                ((unsigned)EP_RING_HEAD << 30) | (unsigned)sz, sh.seqr[r] + (unsigned)n, 0u);
    }
    if (hi > lo) {
      sh.next[r] = hi;
      __hip_atomic_fetch_sub(&sh.remaining, hi - lo, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
      HT_ST(&sh.progress, 1);
    }
  }
}

__global__ __launch_bounds__(1024) void ht_ring_kernel(HtRingArgs a) {
  __shared__ HtShared sh;
  const int tid = threadIdx.x;
  const int c = blockIdx.x;  // the slice
  const int t0 = min(a.T, c * a.slice_len), t1 = min(a.T, t0 + a.slice_len);
  for (int r = tid; r < a.R; r += blockDim.x) {
    sh.total[r] = 0;
    sh.fill[r] = 0;
    sh.seen[r] = 0;
    sh.lock[r] = 0;
    sh.next[r] = 0;
    sh.seqf[r] = a.seq_fwd[c * a.R + r];
    sh.cumf[r] = a.cum_fwd[c * a.R + r];
    sh.seqr[r] = a.seq_rev[c * a.R + r];
    sh.cumr[r] = a.cum_rev[c * a.R + r];
  }
  for (int i = tid; i < a.R * a.W; i += blockDim.x) sh.done[i] = 0;
  if (tid == 0) sh.abort = sh.remaining = sh.progress = sh.idle = 0;
  __syncthreads();
  // rows per channel of this slice: both ends count them from the routing table (the count
  // notification that precedes a high-throughput dispatch)
  for (int i = tid; i < (t1 - t0) * a.K; i += blockDim.x) {
    const int e = a.idx[(size_t)t0 * a.K + i], row = a.dst_row[(size_t)t0 * a.K + i];
    if (ht_valid(a, e, row))
      __hip_atomic_fetch_add(&sh.total[e / a.E_loc], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    else if (e >= 0)
      dev_set_error(a.fifo.error, EP_EBOUNDS);
  }
  __syncthreads();
  if (tid == 0) {
    int chunks = 0;
    for (int r = 0; r < a.R; ++r) chunks += (sh.total[r] + 31) >> 5;
    sh.remaining = chunks;
  }
  __syncthreads();

  int q = 0;  // this wave has sent its first q tokens
  HtToken tk{0ull, 0};
  bool sent_all = false;
  unsigned long long last = wall_clock64();
  while (HT_LD(&sh.remaining) > 0) {  // (uniform: read between two barriers that no writer crosses)
    if (!sent_all) sent_all = ht_send_step(a, sh, c, t0, t1 - t0, q, tk);
    __syncthreads();
    ht_receive_step(a, sh, c);
    __syncthreads();
    if (tid == 0) {
      const unsigned long long now = wall_clock64();
      const int progressed = HT_LD(&sh.progress);
      sh.idle = !progressed;
      if (progressed) {
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
  __syncthreads();
  // the channels' running sequence numbers and row totals, for the next dispatch
  for (int r = tid; r < a.R; r += blockDim.x) {
    const unsigned nch = (unsigned)(sh.total[r] + 31) >> 5;
    a.seq_fwd[c * a.R + r] = sh.seqf[r] + 2u * nch;
    a.cum_fwd[c * a.R + r] = sh.cumf[r] + (unsigned)sh.total[r];
    a.seq_rev[c * a.R + r] = sh.seqr[r] + nch;
    a.cum_rev[c * a.R + r] = sh.cumr[r] + (unsigned)sh.total[r];
  }
  drain_all_channels(a.fifo, a.waves_done, (unsigned)a.src, lane_id());
}

int launch_ht_ring(const HtRingArgs &a, const Tunables &tune, void *stream) {
  int threads = tune.ht_threads;
  if (threads < 64 || threads > 1024 || (threads & 63)) threads = 1024;
  hipLaunchKernelGGL(ht_ring_kernel, dim3((unsigned)a.slices), dim3((unsigned)threads), 0, (hipStream_t)stream, a);
  return (int)hipGetLastError();
}

}  // namespace ep
