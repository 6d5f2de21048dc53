// HIP kernels for gfx950 (MI355X): layout, dispatch (bf16 / FP8 E4M3), combine,
// and the device side of the GPU->CPU FIFO channels.
//
// None of the work here is a dense contraction, so there is no MFMA: dispatch
// and combine are HBM-bound row copies / gathers done with 16-byte vector
// accesses, one wavefront (64 lanes) per token or per slice of a token; the
// layout is an integer counting sort built from LDS bit masks and popcounts.
#include <hip/hip_runtime.h>
#include <stdlib.h>

#include "ep_internal.h"

namespace ep {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

#define EP_DEV __device__ __forceinline__

// ---------------------------------------------------------------- utilities
EP_DEV void dev_set_error(int *err, int code) {
  // Sticky error word in pinned host memory; any failing lane may write it.
  __hip_atomic_store(err, code, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
}

EP_DEV int lane_id() { return threadIdx.x & 63; }

// ------------------------------------------------- FIFO channel, GPU side
// Push (Section 3.1, "Channel APIs"): reserve the next Idx of the channel with
// one device-scope atomic on the tail (which lives in device memory), wait for
// room using the device-resident cached copy of the head and re-reading the
// host copy over PCIe only when that cache says "full", then publish the
// 16-byte command with a single store.  Returns Idx, or ~0 after a timeout.
EP_DEV unsigned long long ring_push(const RingDev &r, unsigned c, unsigned w0, unsigned w1,
                                    unsigned w2, unsigned w3) {
  const unsigned long long idx =
      __hip_atomic_fetch_add(&r.tail[c], 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  const unsigned gen = (((unsigned)(idx >> r.log2_entries)) & 1u) ^ 1u;
  const u32x4 v = {w0 | (gen << 31), w1, w2, w3 | (gen << 31)};
  u32x4 *slot = (u32x4 *)r.slots + (size_t)c * r.entries + (size_t)(idx & (r.entries - 1));
  unsigned long long head =
      __hip_atomic_load(&r.cached_head[c], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  unsigned long long result = idx, t0 = 0;
  bool done = false, stalled = false;
  // Lanes of one wavefront push side by side, and the proxy consumes a channel in Idx order: a lane
  // whose Idx already fits must publish its command without waiting for a neighbour whose Idx does
  // not fit yet (that neighbour may be waiting for the very slot this lane has to fill).  So the
  // store sits INSIDE the wave-wide loop, and the loop ends when every active lane is done.
  do {
    if (!done) {
      if (idx - head < r.entries) {
        *(volatile __attribute__((address_space(1))) u32x4 *)slot = v;  // one 16-byte store straight to host memory (system scope)
        done = true;
      } else {
        // Full: wait for the proxy to pop.  Thousands of lanes can be waiting on one channel, and
        // each re-read of the head is a PCIe round trip, so only the lane that holds the channel's
        // refresh lock goes to host memory; everyone else watches the device-side copy it updates.
        if (!stalled) {
          stalled = true;
          t0 = wall_clock64();
          __hip_atomic_fetch_add(r.stalls, 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        if (__hip_atomic_exchange(&r.refresh_lock[c], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == 0u) {
          const unsigned long long h =
              __hip_atomic_load(&r.head[c * kHeadStride], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
          __hip_atomic_fetch_max(&r.cached_head[c], h, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          __hip_atomic_store(&r.refresh_lock[c], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        head = __hip_atomic_load(&r.cached_head[c], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (idx - head >= r.entries) {
          if (wall_clock64() - t0 > r.timeout_ticks) {
            dev_set_error(r.error, EP_ETIMEOUT);
            result = ~0ull;
            done = true;
          } else {
            __builtin_amdgcn_s_sleep(32);
          }
        }
      }
    }
  } while (__ballot(!done) != 0ull);
  return result;
}

// Check-completion(Idx): has the proxy popped command idx of channel c?
// Blocks (bounded) until it has; used after a Drain.
EP_DEV bool ring_wait_completion(const RingDev &r, unsigned c, unsigned long long idx) {
  const unsigned long long t0 = wall_clock64();
  for (;;) {
    unsigned long long head =
        __hip_atomic_load(&r.head[c * kHeadStride], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
    if (head > idx) return true;
    if (wall_clock64() - t0 > r.timeout_ticks) {
      dev_set_error(r.error, EP_ETIMEOUT);
      return false;
    }
    __builtin_amdgcn_s_sleep(32);
  }
}

// ------------------------------------------------------------------ layout
// The layout is a counting sort keyed by expert, stable in (source rank, token).
// Tokens are cut into tiles of 64 (one wavefront); f = s * ntiles + tile is the
// "flat" tile index, ascending in exactly the order rows are laid out inside an
// expert.  With hist[f][e] = entries of tile f that chose e,
//   P[f][e]  = sum_{f' < f} hist[f'][e]            (exclusive scan over flat tiles)
//   dst_row  = expert_offset[e] + P[f][e] + rank inside the tile
//   slot     = P[f][e] - P[s * ntiles][e] + rank
//   count[s][e] = P[(s+1) * ntiles][e] - P[s * ntiles][e],  base[s][e] = expert_offset[e] + P[s * ntiles][e].
//
// Kernel 1: one wavefront per tile.  Every lane owns a token and sets its bit in
// a 64-bit LDS mask per expert it chose (a token's experts are distinct, so one
// bit per (token, expert)).  The in-tile stable rank of an entry is the popcount
// of the mask below its lane; the tile histogram is the popcount of the whole
// mask.  The last workgroup to finish (ticket counter, nobody spins) scans the
// histograms (one thread per expert, a batch of flat tiles in registers at a
// time), then the expert totals (one wave scan), and writes every per-expert
// output.  Histograms cross workgroups through device-scope write-through stores
// and cache-bypassing loads, so the hand-over needs no L2 write-back/invalidate
// (measured: a device-scope fence here cost 7 us, mostly flushing other kernels'
// dirty lines).
EP_DEV int wave_inclusive_scan(int v, int lane) {
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    const int u = __shfl_up(v, d);
    if (lane >= d) v += u;
  }
  return v;
}

static int env_int(const char *name, int dflt);

constexpr int kScanBatch = 32;  // flat tiles a scanning thread holds in registers

__global__ __launch_bounds__(1024) void layout_count_kernel(LayoutArgs a) {
  extern __shared__ unsigned long long s_mask[];  // [waves][E]
  __shared__ int s_off[kMaxExperts + 1];
  __shared__ int s_part[1024];
  __shared__ int s_last;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int W = a.tiles_per_block;  // wavefronts that own a tile; the rest only help with the scan
  const int nblk = max(1, (a.ntiles + W - 1) / W);
  const int s = blockIdx.x / nblk;
  const int tile = wave < W ? (blockIdx.x % nblk) * W + wave : a.ntiles;
  const int E = a.E, K = a.K;
  const int F = a.S * a.ntiles;  // flat tiles

  for (int i = tid; i < W * E; i += blockDim.x) s_mask[i] = 0ull;
  __syncthreads();

  unsigned long long *m = s_mask + (size_t)(wave < W ? wave : 0) * E;
  const int t = tile * kLayoutTile + lane;
  const bool active = tile < a.ntiles && t < a.T;
  const size_t ebase = ((size_t)s * a.T + (active ? t : 0)) * K;
  const unsigned long long below = (1ull << lane) - 1ull;
  if (K <= 8) {  // the token's expert ids stay in registers across the barrier
    int ev[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) ev[k] = (active && k < K) ? a.idx[ebase + k] : -1;
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      const int e = ev[k];
      bool pend = e >= 0 && e < E;
      if (!pend && e != -1) dev_set_error(a.error, EP_EBOUNDS);
      // Skewed routing sends most lanes of a wave to the same few experts, and an LDS atomic
      // serialises lanes that hit one address.  Peel the two most common values first: their
      // lanes are found with a ballot and one lane writes the whole bit set.
#pragma unroll
      for (int round = 0; round < 2; ++round) {
        const unsigned long long pm = __ballot(pend);
        if (pm == 0) break;
        const int leader = __builtin_ctzll(pm);
        const int e0 = __builtin_amdgcn_readlane(e, leader);
        const unsigned long long same = __ballot(pend && e == e0);
        if (lane == leader) m[e0] |= same;
        pend = pend && e != e0;
      }
      if (pend) atomicOr(&m[e], 1ull << lane);
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < 8; ++k)
      if (active && k < K) a.slot[ebase + k] = (ev[k] >= 0 && ev[k] < E) ? __popcll(m[ev[k]] & below) : -1;
  } else {
    if (active) {
      for (int k = 0; k < K; ++k) {
        const int e = a.idx[ebase + k];
        if (e >= 0 && e < E)
          atomicOr(&m[e], 1ull << lane);
        else if (e != -1)
          dev_set_error(a.error, EP_EBOUNDS);
      }
    }
    __syncthreads();
    if (active) {
      for (int k = 0; k < K; ++k) {
        const int e = a.idx[ebase + k];
        a.slot[ebase + k] = (e >= 0 && e < E) ? __popcll(m[e] & below) : -1;
      }
    }
  }
  if (tile < a.ntiles) {
    int32_t *hist = a.tile_hist + ((size_t)s * a.ntiles + tile) * E;
    for (int e = lane; e < E; e += 64)
      __hip_atomic_store(hist + e, __popcll(m[e]), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }

  // ---- last workgroup to arrive does the scans
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");  // this wave's write-through stores are acknowledged
  __syncthreads();
  if (tid == 0) {
    const unsigned ticket = __hip_atomic_fetch_add(a.ticket, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    s_last = (ticket == gridDim.x - 1);
  }
  __syncthreads();
  if (!s_last) return;
  if (tid == 0) __hip_atomic_store(a.ticket, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);

  // P[*][e]: scan_split threads per expert, each owning a contiguous range of flat tiles
  // (thread = part * E + e, so a wavefront reads consecutive experts of one tile row).
  const int P = a.scan_split;
  const int len = (F + P - 1) / P;
  for (int e_base = 0; e_base < E; e_base += blockDim.x / P) {  // one pass unless E * P > workgroup size
    const int ne = min(E - e_base, (int)blockDim.x / P);
    const bool mine = tid < P * ne;
    const int part = mine ? tid / ne : 0;
    const int e = e_base + (mine ? tid - part * ne : 0);
    const int lo = min(F, part * len), hi = min(F, lo + len);
    int v[kScanBatch];
    int tot = 0;
    if (mine) {
      for (int f0 = lo; f0 < hi; f0 += kScanBatch) {
#pragma unroll
        for (int j = 0; j < kScanBatch; ++j)
          v[j] = (f0 + j < hi) ? __hip_atomic_load(a.tile_hist + (size_t)(f0 + j) * E + e, __ATOMIC_RELAXED,
                                                   __HIP_MEMORY_SCOPE_AGENT)
                               : 0;
#pragma unroll
        for (int j = 0; j < kScanBatch; ++j) tot += v[j];
      }
      s_part[tid] = tot;
    }
    __syncthreads();
    if (mine) {
      int carry = 0;
      for (int q = 0; q < part; ++q) carry += s_part[q * ne + (e - e_base)];
      for (int f0 = lo; f0 < hi; f0 += kScanBatch) {
        if (hi - lo > kScanBatch) {  // the range did not fit the registers: fetch the batch again
#pragma unroll
          for (int j = 0; j < kScanBatch; ++j)
            v[j] = (f0 + j < hi) ? __hip_atomic_load(a.tile_hist + (size_t)(f0 + j) * E + e, __ATOMIC_RELAXED,
                                                     __HIP_MEMORY_SCOPE_AGENT)
                                 : 0;
        }
#pragma unroll
        for (int j = 0; j < kScanBatch; ++j) {
          if (f0 + j < hi) a.tile_base[(size_t)(f0 + j) * E + e] = carry;
          carry += v[j];
        }
      }
      if (part == P - 1) {
        a.tile_base[(size_t)F * E + e] = carry;
        a.expert_total[e] = carry;
        s_off[e] = carry;
      }
    }
    __syncthreads();
  }
  __syncthreads();
  if (wave == 0) {  // exclusive scan over experts: 64 lanes x contiguous runs
    const int per = (E + 63) / 64;
    const int lo = min(E, lane * per), hi = min(E, lo + per);
    int sum = 0;
    for (int i = lo; i < hi; ++i) sum += s_off[i];
    const int incl = wave_inclusive_scan(sum, lane);
    int run = incl - sum;
    for (int i = lo; i < hi; ++i) {
      const int v = s_off[i];
      s_off[i] = run;
      a.expert_offset[i] = run;
      run += v;
    }
    if (lane == 63) {
      s_off[E] = incl;
      a.expert_offset[E] = incl;
    }
  }
  __syncthreads();
  for (int i = tid; i < a.S * E; i += blockDim.x) {
    const int ss = i / E, e = i - ss * E;
    const int lo = a.tile_base[(size_t)ss * a.ntiles * E + e], hi = a.tile_base[(size_t)(ss + 1) * a.ntiles * E + e];
    a.count[i] = hi - lo;
    a.base[i] = s_off[e] + lo;
  }
  for (int r = tid; r <= a.R; r += blockDim.x) {
    const int o = s_off[r * a.E_loc];  // r == R reads the end sentinel s_off[E]
    a.rank_offset[r] = o;
    if (r < a.R) a.rank_total[r] = s_off[(r + 1) * a.E_loc] - o;
  }
}

// Kernel 2: per entry, slot and dst_row from the tile prefix and the expert offset.
__global__ __launch_bounds__(256) void layout_finish_kernel(LayoutArgs a) {
  const long long n = (long long)a.S * a.T * a.K;
  const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
  if (i >= n) return;
  const int e = a.idx[i];
  if (e < 0 || e >= a.E) {
    a.slot[i] = -1;
    a.dst_row[i] = -1;
    return;
  }
  const long long tk = (long long)a.T * a.K;
  const int s = (int)(i / tk);
  const int t = (int)((i - (long long)s * tk) / a.K);
  const int before = a.tile_base[((size_t)s * a.ntiles + t / kLayoutTile) * a.E + e];
  const int first = a.tile_base[(size_t)s * a.ntiles * a.E + e];
  const int rank = a.slot[i];
  a.slot[i] = before - first + rank;
  a.dst_row[i] = a.expert_offset[e] + before + rank;
}

int launch_layout(const LayoutArgs &a, void *stream) {
  hipStream_t st = (hipStream_t)stream;
  // Workgroups are 1024 threads so that the last one has many hands for the scan, but only a few
  // wavefronts of each own a tile: the LDS atomics of one tile then compete with few others.
  const int kBlock = 1024;
  int W = env_int("EP_LAYOUT_TPB", 4);
  if (W != 1 && W != 2 && W != 4 && W != 8 && W != 16) W = 4;
  while (W > 1 && (size_t)W * a.E * sizeof(unsigned long long) > 65536 - 12288) W >>= 1;
  LayoutArgs b = a;
  b.tiles_per_block = W;
  b.scan_split = 1;  // threads per expert in the scan: a power of two, at most 16, all in one workgroup
  while (b.scan_split < 16 && b.scan_split * 2 * a.E <= kBlock) b.scan_split *= 2;
  const int nblk = (a.ntiles + W - 1) / W;
  const int grid1 = a.S * (nblk > 0 ? nblk : 1);
  const size_t lds = (size_t)W * a.E * sizeof(unsigned long long);
  hipLaunchKernelGGL(layout_count_kernel, dim3(grid1), dim3(kBlock), lds, st, b);
  hipError_t err = hipGetLastError();
  if (err != hipSuccess) return (int)err;
  const long long n = (long long)a.S * a.T * a.K;
  if (n > 0) {
    hipLaunchKernelGGL(layout_finish_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, a);
    err = hipGetLastError();
  }
  return (int)err;
}

// Payload rows are stored write-through at system scope (sc0 sc1): when such a store is
// acknowledged the bytes are in memory, visible to every XCD's L2 and to a PCIe reader, which is
// what a transfer command promises about the rows it names.  A wave therefore only has to wait
// for its own stores (vmcnt) before it touches a counter or pushes a command; no L2 write-back
// is needed, and the counters can be relaxed device-scope atomics.  Measured on MI355X the
// write-through stores stream as fast as non-temporal ones, whereas a device-scope release fence
// per wave (L2 write-back) made the dispatch 4-8x slower.
typedef __attribute__((address_space(1))) u32x4 global_u32x4;
EP_DEV void store_payload(u32x4 *p, const u32x4 &v) { *(volatile global_u32x4 *)p = v; }

// All stores of this wave are acknowledged after this (compiler and hardware barrier).
EP_DEV void wait_for_own_stores() { __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup"); }

// ------------------------------------------------- dispatch: command emission
struct TokenMeta {
  int e;       // expert of this lane's k (lane < K), -1 otherwise
  int row;     // destination row
  bool valid;  // this (t, k) is dispatched by this call
};

EP_DEV TokenMeta load_meta(const DispatchArgs &a, int t, int lane) {
  TokenMeta m{-1, -1, false};
  if (t < a.T && lane < a.K) {
    m.e = a.idx[(size_t)t * a.K + lane];
    m.row = a.dst_row[(size_t)t * a.K + lane];
    if (m.e >= 0) {
      if (m.e >= a.E || m.row < 0 || m.row >= a.recv_rows)
        dev_set_error(a.ring.error, EP_EBOUNDS);
      else if (a.filter < 0 || m.e / a.E_loc == a.filter)
        m.valid = true;
    } else if (m.e != -1) {
      dev_set_error(a.ring.error, EP_EBOUNDS);
    }
  }
  return m;
}

EP_DEV void push_count_atomic(const DispatchArgs &a, int e, int value) {
  const unsigned dr = (unsigned)(e / a.E_loc), le = (unsigned)(e - (int)dr * a.E_loc);
  ring_push(a.ring, (unsigned)e % a.ring.channels, cmd_w0(EP_OP_ATOMIC, a.src, dr, le), (unsigned)value, 0u,
            (unsigned)(a.src * a.E_loc) + le);
}

// Kernel prologue (workgroup 0, wavefront 0): the count Atomics that no row
// completion will trigger - experts with count 0, or all of them when the
// caller wants the atomics ahead of the writes.
EP_DEV void emit_leading_atomics(const DispatchArgs &a, int lane) {
  const bool first = (a.cmd_mode & EP_CMD_ATOMICS_FIRST) != 0;
  for (int e = lane; e < a.E; e += 64) {
    if (a.filter >= 0 && e / a.E_loc != a.filter) continue;
    const int c = a.count[e];
    if (first || c == 0) push_count_atomic(a, e, c);
  }
}

// Called by the lanes holding a dispatched (t,k) after the token's rows are
// stored and acknowledged (write-through, so they are in memory).  LL granularity: one Write per row.
// Chunk granularity: the lane that completes a run of <= 32 consecutive rows of
// an expert pushes the Write for the run.  Whoever completes the expert pushes
// its count Atomic (Section 3.3: the receiver holds it until that many rows
// arrived).  The scratch counters return to zero by themselves.
EP_DEV void emit_row_cmds(const DispatchArgs &a, const TokenMeta &m, int t) {
  const int e = m.e;
  const unsigned dr = (unsigned)(e / a.E_loc), le = (unsigned)(e - (int)dr * a.E_loc);
  // Everything for one destination expert goes through one FIFO (and therefore one proxy thread):
  // in-FIFO order is the only order the channel guarantees (Section 3.1, "GPU-side contention").
  const unsigned ch = (unsigned)e % a.ring.channels;
  const int c = a.count[e];
  const int mode = a.cmd_mode & EP_CMD_MODE_MASK;
  int finished_rows = 0;
  if (mode == EP_CMD_PER_TOKEN) {
    const unsigned long long so = (unsigned long long)t * a.row_bytes;
    const unsigned long long dof = (unsigned long long)m.row * a.row_bytes;
    ring_push(a.ring, ch, cmd_w0(EP_OP_WRITE, a.src, dr, le), a.row_bytes >> 4, (unsigned)(so >> 4),
              (unsigned)(dof >> 4));
    finished_rows = 1;
  } else {
    const int slot = m.row - a.base[e];
    const int j = slot >> 5;
    if (slot < 0 || j >= a.chunks_per_expert || slot >= c) {
      dev_set_error(a.ring.error, EP_EBOUNDS);
      return;
    }
    const int csize = min(kChunkRows, c - (j << 5));
    int *cnt = a.chunk_cnt + (size_t)e * a.chunks_per_expert + j;
    const int old = __hip_atomic_fetch_add(cnt, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (old + 1 == csize) {
      __hip_atomic_store(cnt, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      const unsigned long long off = (unsigned long long)(a.base[e] + (j << 5)) * a.row_bytes;
      const unsigned len = (unsigned)csize * a.row_bytes;
      if (mode == EP_CMD_CHUNK32_ORDERED) {
        // High-throughput style: the chunk's Write and the Atomic that advances the receiver's tail
        // take two consecutive sequence numbers of the communication channel (source, destination
        // rank) and travel through that channel's FIFO; the receiver re-establishes the order.
        const unsigned seq = __hip_atomic_fetch_add(a.ht_seq + (size_t)a.src * a.R + dr, 2u, __ATOMIC_RELAXED,
                                                    __HIP_MEMORY_SCOPE_AGENT);
        const unsigned och = dr % a.ring.channels;
        ring_push(a.ring, och, cmd_w0(EP_OP_ORDERED_WRITE, a.src, dr, le),
                  ((unsigned)(csize - 1) << 26) | (len >> 4), seq, (unsigned)(off >> 4));
        ring_push(a.ring, och, cmd_w0(EP_OP_ORDERED_ATOMIC, a.src, dr, 0), (unsigned)csize, seq + 1u,
                  (unsigned)(a.src * a.R) + dr);
        return;
      }
      ring_push(a.ring, ch, cmd_w0(EP_OP_WRITE, a.src, dr, le), ((unsigned)(csize - 1) << 26) | (len >> 4),
                (unsigned)(off >> 4), (unsigned)(off >> 4));
      finished_rows = csize;
    }
  }
  if (finished_rows) {
    const int done = __hip_atomic_fetch_add(a.expert_done + e, finished_rows, __ATOMIC_RELAXED,
                                            __HIP_MEMORY_SCOPE_AGENT) + finished_rows;
    if (done == c) {
      __hip_atomic_store(a.expert_done + e, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if (!(a.cmd_mode & EP_CMD_ATOMICS_FIRST)) push_count_atomic(a, e, c);
    }
  }
}

// Kernel epilogue with EP_CMD_DRAIN: the last wavefront of the grid pushes a
// Drain on every channel and blocks on Check-completion for each (Section 3.1:
// Drain and Barrier are blocking on the GPU side).
EP_DEV void drain_all_channels(const RingDev &ring, unsigned *waves_done, unsigned src, int lane) {
  const unsigned total = gridDim.x * (blockDim.x >> 6);
  unsigned done = 0;
  wait_for_own_stores();  // this wave's commands are in their rings before it reports done
  if (lane == 0)
    done = __hip_atomic_fetch_add(waves_done, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) + 1u;
  done = __builtin_amdgcn_readfirstlane(done);
  if (done != total) return;
  if (lane == 0) __hip_atomic_store(waves_done, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  for (unsigned c = lane; c < ring.channels; c += 64) {
    const unsigned long long idx = ring_push(ring, c, cmd_w0(EP_OP_DRAIN, src, 0, 0), 0u, 0u, 0u);
    if (idx != ~0ull) ring_wait_completion(ring, c, idx);
  }
}

EP_DEV void emit_drain(const DispatchArgs &a, int lane) {
  drain_all_channels(a.ring, a.waves_done, (unsigned)a.src, lane);
}

// ------------------------------------------------------------ dispatch bf16
// A token's row is H/8 16-byte vectors.  Wavefront (token, part) reads its
// slice of the row ONCE into registers (VPL vectors per lane) and stores it to
// every destination row; destination rows are wave-uniform and come from the
// lanes that hold the token's (expert, row) pairs.
template <int VPL>
__global__ void dispatch_bf16_kernel(DispatchArgs a) {
  const int wave = threadIdx.x >> 6, lane = lane_id();
  const int part = wave % a.parts;
  const int t = blockIdx.x * a.tokens_per_block + wave / a.parts;
  const bool ring_on = (a.cmd_mode & EP_CMD_MODE_MASK) != EP_CMD_NONE;
  const bool ordered = (a.cmd_mode & EP_CMD_MODE_MASK) == EP_CMD_CHUNK32_ORDERED;
  if (ring_on && !ordered && blockIdx.x == 0 && wave == 0) emit_leading_atomics(a, lane);

  const TokenMeta m = load_meta(a, t, lane);
  unsigned long long vmask = __ballot(m.valid);
  const int nvec = a.H >> 3;
  const int v0 = part * VPL * 64 + lane;
  if (vmask && !(a.cmd_mode & EP_CMD_NO_PLACEMENT)) {
    const u32x4 *src = (const u32x4 *)a.x + (size_t)t * nvec;
    u32x4 v[VPL];
#pragma unroll
    for (int i = 0; i < VPL; ++i)
      if (v0 + i * 64 < nvec) v[i] = __builtin_nontemporal_load(src + v0 + i * 64);
    unsigned long long mm = vmask;
    while (mm) {
      const int k = __builtin_ctzll(mm);
      mm &= mm - 1;
      const int row = __builtin_amdgcn_readlane(m.row, k);
      u32x4 *dst = (u32x4 *)a.recv + (size_t)row * nvec;
#pragma unroll
      for (int i = 0; i < VPL; ++i)
        if (v0 + i * 64 < nvec) store_payload(dst + v0 + i * 64, v[i]);
    }
  }
  if (!ring_on) return;
  wait_for_own_stores();  // the rows are in memory before a counter or command mentions them
  if (a.parts > 1) __syncthreads();
  if (part == 0 && m.valid) emit_row_cmds(a, m, t);
  if (a.cmd_mode & EP_CMD_DRAIN) emit_drain(a, lane);
}

// ------------------------------------------------------------- dispatch FP8
EP_DEV float bf16_lo(unsigned d) { return __uint_as_float(d << 16); }
EP_DEV float bf16_hi(unsigned d) { return __uint_as_float(d & 0xFFFF0000u); }

// Two floats -> two E4M3 codes (round to nearest even, saturate to +-448)
// in the low or high half of a dword.  The clamp is exact, so the hardware
// conversion never sees a value beyond the largest finite code.
template <bool HI>
EP_DEV unsigned cvt2_e4m3(float x, float y, unsigned old) {
  x = __builtin_amdgcn_fmed3f(x, 448.0f, -448.0f);
  y = __builtin_amdgcn_fmed3f(y, 448.0f, -448.0f);
  return (unsigned)__builtin_amdgcn_cvt_pk_fp8_f32(x, y, (int)old, HI);
}

// A lane owns 16 consecutive channels (two 16-byte loads, one 16-byte store of
// codes); 8 adjacent lanes own one 128-channel block and share its amax through
// three xor-shuffles.  scale = amax/448 and inv = 448/amax are IEEE divisions.
// Every lane of the wave must call this (lanes past the row's end with zeros).
EP_DEV void quant16(const u32x4 &lo, const u32x4 &hi, u32x4 &q, float &scale_out) {
  float f[16];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    f[2 * j] = bf16_lo(lo[j]);
    f[2 * j + 1] = bf16_hi(lo[j]);
    f[8 + 2 * j] = bf16_lo(hi[j]);
    f[8 + 2 * j + 1] = bf16_hi(hi[j]);
  }
  float amax = 0.0f;
#pragma unroll
  for (int j = 0; j < 16; ++j) amax = fmaxf(amax, fabsf(f[j]));
  amax = fmaxf(amax, __shfl_xor(amax, 1));
  amax = fmaxf(amax, __shfl_xor(amax, 2));
  amax = fmaxf(amax, __shfl_xor(amax, 4));
  float scale = 1.0f, inv = 1.0f;
  if (amax >= 0x1p-100f) {
    scale = amax / 448.0f;
    inv = 448.0f / amax;
  }
  scale_out = scale;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    unsigned d = cvt2_e4m3<false>(f[4 * j] * inv, f[4 * j + 1] * inv, 0u);
    q[j] = cvt2_e4m3<true>(f[4 * j + 2] * inv, f[4 * j + 3] * inv, d);
  }
}

template <int VPL>
__global__ void dispatch_fp8_kernel(DispatchArgs a) {
  const int wave = threadIdx.x >> 6, lane = lane_id();
  const int part = wave % a.parts;
  const int t = blockIdx.x * a.tokens_per_block + wave / a.parts;
  const bool ring_on = (a.cmd_mode & EP_CMD_MODE_MASK) != EP_CMD_NONE;
  const bool ordered = (a.cmd_mode & EP_CMD_MODE_MASK) == EP_CMD_CHUNK32_ORDERED;
  if (ring_on && !ordered && blockIdx.x == 0 && wave == 0) emit_leading_atomics(a, lane);

  const TokenMeta m = load_meta(a, t, lane);
  unsigned long long vmask = __ballot(m.valid);
  const int npair = a.H >> 4;  // 16-channel groups per row
  const int nblk = a.H >> 7;   // 128-channel blocks per row
  const int p0 = part * VPL * 64 + lane;
  if (vmask) {
    const u32x4 *src = (const u32x4 *)a.x + (size_t)t * npair * 2;
    u32x4 lo[VPL], hi[VPL], q[VPL];
    float sc[VPL];
#pragma unroll
    for (int i = 0; i < VPL; ++i)
      if (p0 + i * 64 < npair) {
        lo[i] = __builtin_nontemporal_load(src + 2 * (p0 + i * 64));
        hi[i] = __builtin_nontemporal_load(src + 2 * (p0 + i * 64) + 1);
      } else {
        lo[i] = u32x4{0, 0, 0, 0};
        hi[i] = u32x4{0, 0, 0, 0};
      }
#pragma unroll
    for (int i = 0; i < VPL; ++i) quant16(lo[i], hi[i], q[i], sc[i]);
    unsigned long long mm = vmask;
    while (mm) {
      const int k = __builtin_ctzll(mm);
      mm &= mm - 1;
      const int row = __builtin_amdgcn_readlane(m.row, k);
      u32x4 *dq = (u32x4 *)a.recv + (size_t)row * npair;
      float *ds = a.recv_scale + (size_t)row * nblk;
#pragma unroll
      for (int i = 0; i < VPL; ++i)
        if (p0 + i * 64 < npair) {
          store_payload(dq + p0 + i * 64, q[i]);
          if ((lane & 7) == 0)
            __hip_atomic_store(ds + ((p0 + i * 64) >> 3), sc[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
        }
    }
  }
  if (!ring_on) return;
  wait_for_own_stores();
  if (a.parts > 1) __syncthreads();
  if (part == 0 && m.valid) emit_row_cmds(a, m, t);
  if (a.cmd_mode & EP_CMD_DRAIN) emit_drain(a, lane);
}

static int env_int(const char *name, int dflt) {
  const char *s = getenv(name);
  return (s && *s) ? atoi(s) : dflt;
}

// units = 16-byte vectors (bf16) or 16-channel groups (FP8) per row; returns how many of them one
// lane carries.  The row then takes ceil(units / (64 * result)) waves, at most 16.
static int split_for(int units, int T, const int *cands, int ncand) {
  int best = cands[ncand - 1];
  for (int i = 0; i < ncand; ++i)
    if (cands[i] * 256 >= units) {
      best = cands[i];
      break;
    }
  for (int i = ncand - 1; i >= 0; --i) {
    if (cands[i] >= best) continue;
    const long long waves_now = (long long)T * ((units + best * 64 - 1) / (best * 64));
    if (waves_now >= 4096) break;
    if ((units + cands[i] * 64 - 1) / (cands[i] * 64) > 16) break;
    best = cands[i];
  }
  while ((units + best * 64 - 1) / (best * 64) > 16) {  // very wide rows: stay within 16 waves per token
    int next = best;
    for (int i = 0; i < ncand; ++i)
      if (cands[i] > best) {
        next = cands[i];
        break;
      }
    if (next == best) break;
    best = next;
  }
  return best;
}

int tuned_dispatch_vpl(int H, int T) {
  static const int c[] = {1, 2, 4, 7, 8, 14, 16};
  const int forced = env_int("EP_DISPATCH_VPL", 0);
  for (int v : c)
    if (v == forced) return v;
  // About four waves per token stream best (measured in the full path on 7168- and 4096-wide rows:
  // the command tail of one wave then overlaps the stores of the others); with few tokens the row
  // is split further until there are about 4096 waves (16 per compute unit).
  return split_for(H / 8, T, c, 7);
}

static int tuned_dispatch_fp8_vpl(int H, int T) {
  static const int c[] = {1, 2, 4};  // more than 4 groups per lane would spill at 128 VGPRs
  const int forced = env_int("EP_DISPATCH_FP8_VPL", 0);
  for (int v : c)
    if (v == forced) return v;
  return split_for(H / 16, T, c, 3);
}

int tuned_combine_vpl(int H) {
  static const int c[] = {1, 2, 4};
  const int forced = env_int("EP_COMBINE_VPL", 0);
  for (int v : c)
    if (v == forced) return v;
  (void)H;
  return 1;  // one 16-byte column slice per lane: fewest registers, most waves in flight (measured best)
}

template <int VPL>
static void launch_dispatch_bf16_t(DispatchArgs a, hipStream_t st) {
  const int nvec = a.H / 8;
  a.parts = (nvec + VPL * 64 - 1) / (VPL * 64);
  a.tokens_per_block = a.parts >= 4 ? 1 : 4 / a.parts;
  const int grid = max(1, (a.T + a.tokens_per_block - 1) / a.tokens_per_block);
  hipLaunchKernelGGL(dispatch_bf16_kernel<VPL>, dim3(grid), dim3(64 * a.parts * a.tokens_per_block), 0, st, a);
}

template <int VPL>
static void launch_dispatch_fp8_t(DispatchArgs a, hipStream_t st) {
  const int npair = a.H / 16;
  a.parts = (npair + VPL * 64 - 1) / (VPL * 64);
  a.tokens_per_block = a.parts >= 4 ? 1 : 4 / a.parts;
  const int grid = max(1, (a.T + a.tokens_per_block - 1) / a.tokens_per_block);
  hipLaunchKernelGGL(dispatch_fp8_kernel<VPL>, dim3(grid), dim3(64 * a.parts * a.tokens_per_block), 0, st, a);
}

int launch_dispatch(const DispatchArgs &a, int payload, void *stream) {
  hipStream_t st = (hipStream_t)stream;
  // T == 0 with the ring on still launches one (idle) workgroup: it owes the zero-count atomics
  if (a.T <= 0 && (a.cmd_mode & EP_CMD_MODE_MASK) == EP_CMD_NONE) return 0;
  if (payload == EP_BF16) {
    const int vpl = tuned_dispatch_vpl(a.H, a.T);
    if ((a.H / 8 + vpl * 64 - 1) / (vpl * 64) > 16) return (int)hipErrorInvalidValue;
    switch (vpl) {
      case 1: launch_dispatch_bf16_t<1>(a, st); break;
      case 2: launch_dispatch_bf16_t<2>(a, st); break;
      case 4: launch_dispatch_bf16_t<4>(a, st); break;
      case 7: launch_dispatch_bf16_t<7>(a, st); break;
      case 8: launch_dispatch_bf16_t<8>(a, st); break;
      case 14: launch_dispatch_bf16_t<14>(a, st); break;
      default: launch_dispatch_bf16_t<16>(a, st); break;
    }
  } else {
    const int vpl = tuned_dispatch_fp8_vpl(a.H, a.T);
    if ((a.H / 16 + vpl * 64 - 1) / (vpl * 64) > 16) return (int)hipErrorInvalidValue;
    switch (vpl) {
      case 1: launch_dispatch_fp8_t<1>(a, st); break;
      case 2: launch_dispatch_fp8_t<2>(a, st); break;
      default: launch_dispatch_fp8_t<4>(a, st); break;
    }
  }
  return (int)hipGetLastError();
}

// ---------------------------------------------------------------- combine
// out[t, 8 channels] = bf16( sum_k w[t,k] * y[row_k, 8 channels] ): per 16-byte
// column slice, K independent 16-byte loads are in flight per lane, then the
// fp32 fused multiply-add chain runs in ascending k from +0, and the result is
// rounded once (nearest even) to bf16.  Rows and weights are wave-uniform.
EP_DEV unsigned pack_bf16_rne(float a, float b) {
  unsigned ua = __float_as_uint(a), ub = __float_as_uint(b);
  ua = (ua + 0x7FFFu + ((ua >> 16) & 1u)) >> 16;
  ub = (ub + 0x7FFFu + ((ub >> 16) & 1u)) & 0xFFFF0000u;
  return ua | ub;
}

EP_DEV void fma8(float (&acc)[8], float w, const u32x4 &v) {
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    acc[2 * j] = __builtin_fmaf(w, bf16_lo(v[j]), acc[2 * j]);
    acc[2 * j + 1] = __builtin_fmaf(w, bf16_hi(v[j]), acc[2 * j + 1]);
  }
}

template <int VPL, int KT>
__global__ __launch_bounds__(256) void combine_kernel(CombineArgs a) {
  const int wave = threadIdx.x >> 6, lane = lane_id();
  const long long item = (long long)blockIdx.x * 4 + wave;
  const int t = (int)(item / a.parts), part = (int)(item % a.parts);
  if (t >= a.T) return;
  const int K = KT > 0 ? KT : a.K;
  int row = -1;
  float wt = 0.0f;
  if (lane < K) {
    row = a.dst_row[(size_t)t * K + lane];
    wt = a.w[(size_t)t * K + lane];
    if (row < -1 || row >= a.y_rows) {
      dev_set_error(a.error, EP_EBOUNDS);
      row = -1;
    }
  }
  const unsigned long long vmask = __ballot(row >= 0);
  const int nvec = a.H >> 3;
  const int v0 = part * VPL * 64 + lane;
  u32x4 *out = (u32x4 *)a.out + (size_t)t * nvec;
  if (vmask == 0) {  // every k masked: +0
#pragma unroll
    for (int i = 0; i < VPL; ++i)
      if (v0 + i * 64 < nvec) out[v0 + i * 64] = u32x4{0, 0, 0, 0};
    return;
  }
  const u32x4 *y = (const u32x4 *)a.y;
  if constexpr (KT > 0) {
    const int safe = __builtin_amdgcn_readlane(row, __builtin_ctzll(vmask));
    int rows[KT];
    float ws[KT];
#pragma unroll
    for (int k = 0; k < KT; ++k) {
      rows[k] = __builtin_amdgcn_readlane(row, k);
      ws[k] = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(wt), k));
    }
    u32x4 ld[VPL][KT];
#pragma unroll
    for (int i = 0; i < VPL; ++i)
      if (v0 + i * 64 < nvec) {
#pragma unroll
        for (int k = 0; k < KT; ++k)
          ld[i][k] = __builtin_nontemporal_load(y + (size_t)(rows[k] >= 0 ? rows[k] : safe) * nvec + v0 + i * 64);
      }
#pragma unroll
    for (int i = 0; i < VPL; ++i)
      if (v0 + i * 64 < nvec) {
        float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int k = 0; k < KT; ++k)
          if (rows[k] >= 0) fma8(acc, ws[k], ld[i][k]);
        u32x4 o = {pack_bf16_rne(acc[0], acc[1]), pack_bf16_rne(acc[2], acc[3]),
                   pack_bf16_rne(acc[4], acc[5]), pack_bf16_rne(acc[6], acc[7])};
        __builtin_nontemporal_store(o, out + v0 + i * 64);
      }
  } else {
#pragma unroll
    for (int i = 0; i < VPL; ++i)
      if (v0 + i * 64 < nvec) {
        float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        for (int k = 0; k < K; ++k) {
          const int r = __builtin_amdgcn_readlane(row, k);
          const float w = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(wt), k));
          if (r >= 0) fma8(acc, w, __builtin_nontemporal_load(y + (size_t)r * nvec + v0 + i * 64));
        }
        u32x4 o = {pack_bf16_rne(acc[0], acc[1]), pack_bf16_rne(acc[2], acc[3]),
                   pack_bf16_rne(acc[4], acc[5]), pack_bf16_rne(acc[6], acc[7])};
        __builtin_nontemporal_store(o, out + v0 + i * 64);
      }
  }
}

template <int VPL>
static void launch_combine_t(CombineArgs a, hipStream_t st) {
  const int nvec = a.H / 8;
  a.parts = (nvec + VPL * 64 - 1) / (VPL * 64);
  const long long items = (long long)a.T * a.parts;
  const unsigned grid = (unsigned)((items + 3) / 4);
  switch (a.K) {
    case 1: hipLaunchKernelGGL((combine_kernel<VPL, 1>), dim3(grid), dim3(256), 0, st, a); break;
    case 2: hipLaunchKernelGGL((combine_kernel<VPL, 2>), dim3(grid), dim3(256), 0, st, a); break;
    case 4: hipLaunchKernelGGL((combine_kernel<VPL, 4>), dim3(grid), dim3(256), 0, st, a); break;
    case 6: hipLaunchKernelGGL((combine_kernel<VPL, 6>), dim3(grid), dim3(256), 0, st, a); break;
    case 8: hipLaunchKernelGGL((combine_kernel<VPL, 8>), dim3(grid), dim3(256), 0, st, a); break;
    default: hipLaunchKernelGGL((combine_kernel<VPL, 0>), dim3(grid), dim3(256), 0, st, a); break;
  }
}

int launch_combine(const CombineArgs &a, void *stream) {
  hipStream_t st = (hipStream_t)stream;
  if (a.T <= 0) return 0;
  if ((a.H / 8 + 63) / 64 > 65535) return (int)hipErrorInvalidValue;
  switch (tuned_combine_vpl(a.H)) {
    case 2: launch_combine_t<2>(a, st); break;
    case 4: launch_combine_t<4>(a, st); break;
    default: launch_combine_t<1>(a, st); break;
  }
  return (int)hipGetLastError();
}

// -------------------------------------------------- high-throughput mode
// Dedup: one thread per token walks its K entries; an entry keeps its group if
// no earlier entry of the token named it.
__global__ __launch_bounds__(256) void dedup_kernel(DedupArgs a) {
  const long long t = (long long)blockIdx.x * 256 + threadIdx.x;
  if (t >= a.n_tokens) return;
  const int32_t *in = a.idx + t * a.K;
  for (int k = 0; k < a.K; ++k) {
    const int e = in[k];
    int g = -1, first = -1;
    if (e >= 0 && e < a.E) {
      g = (e / a.E_loc) / a.ranks_per_group;
      first = k;
      for (int j = 0; j < k; ++j) {
        const int ej = in[j];
        if (ej >= 0 && ej < a.E && (ej / a.E_loc) / a.ranks_per_group == g) {
          first = j;
          break;
        }
      }
      if (first != k) g = -1;
    } else if (e != -1) {
      dev_set_error(a.error, EP_EBOUNDS);
    }
    a.group_idx[t * a.K + k] = g;
    a.first_k[t * a.K + k] = first;
  }
}

int launch_dedup(const DedupArgs &a, void *stream) {
  if (a.n_tokens <= 0) return 0;
  hipLaunchKernelGGL(dedup_kernel, dim3((unsigned)((a.n_tokens + 255) / 256)), dim3(256), 0, (hipStream_t)stream, a);
  return (int)hipGetLastError();
}

__global__ __launch_bounds__(256) void gather_index_kernel(GatherIndexArgs a) {
  const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
  if (i >= (long long)a.T * a.K) return;
  const int r = a.dst_row[i];
  if (r < 0) return;
  const int fk = a.first_k[i];
  if (r >= a.rows || fk < 0 || fk >= a.K) {
    dev_set_error(a.error, EP_EBOUNDS);
    return;
  }
  a.index[r] = a.dst_row_g[i - (i % a.K) + fk];
}

int launch_gather_index(const GatherIndexArgs &a, void *stream) {
  const long long n = (long long)a.T * a.K;
  if (n <= 0) return 0;
  hipLaunchKernelGGL(gather_index_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, (hipStream_t)stream, a);
  return (int)hipGetLastError();
}

// First level of the hierarchical reduce: like the combine, but the K gathered
// rows of a token are summed per group and every group's sum is written to the
// group's own row.  Rows, weights and group leaders are wave-uniform.
template <int KT>
__global__ __launch_bounds__(256) void combine_partial_kernel(CombinePartialArgs a) {
  const int wave = threadIdx.x >> 6, lane = lane_id();
  const long long item = (long long)blockIdx.x * 4 + wave;
  const int t = (int)(item / a.parts), part = (int)(item % a.parts);
  if (t >= a.T) return;
  const int K = KT > 0 ? KT : a.K;
  int row = -1, fk = -1, prow = -1;
  float wt = 0.0f;
  if (lane < K) {
    row = a.dst_row[(size_t)t * K + lane];
    wt = a.w[(size_t)t * K + lane];
    fk = a.first_k[(size_t)t * K + lane];
    prow = a.dst_row_g[(size_t)t * K + lane];
    if (row < -1 || row >= a.y_rows || fk < -1 || fk >= K || (row >= 0 && fk < 0)) {
      dev_set_error(a.error, EP_EBOUNDS);
      row = -1;
    }
    if (row >= 0 && fk == lane && (prow < 0 || prow >= a.rows_g)) {
      dev_set_error(a.error, EP_EBOUNDS);
      row = -1;  // a leader without a valid row drops out; its followers find no open group below
    }
  }
  const unsigned long long vmask = __ballot(row >= 0);
  const unsigned long long leaders = __ballot(row >= 0 && fk == lane);
  if (vmask == 0) return;
  const int nvec = a.H >> 3;
  const int vi = part * 64 + lane;
  if (vi >= nvec) return;
  const u32x4 *y = (const u32x4 *)a.y;
  if constexpr (KT > 0) {
    int rows[KT], fks[KT];
    float ws[KT];
    u32x4 ld[KT];
    const int safe = __builtin_amdgcn_readlane(row, __builtin_ctzll(vmask));
#pragma unroll
    for (int k = 0; k < KT; ++k) {
      rows[k] = __builtin_amdgcn_readlane(row, k);
      fks[k] = __builtin_amdgcn_readlane(fk, k);
      ws[k] = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(wt), k));
      ld[k] = __builtin_nontemporal_load(y + (size_t)(rows[k] >= 0 ? rows[k] : safe) * nvec + vi);
    }
#pragma unroll
    for (int j = 0; j < KT; ++j) {
      if (!((leaders >> j) & 1)) continue;
      float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int k = 0; k < KT; ++k)
        if (rows[k] >= 0 && fks[k] == j) fma8(acc, ws[k], ld[k]);
      const int pr = __builtin_amdgcn_readlane(prow, j);
      u32x4 o = {pack_bf16_rne(acc[0], acc[1]), pack_bf16_rne(acc[2], acc[3]),
                 pack_bf16_rne(acc[4], acc[5]), pack_bf16_rne(acc[6], acc[7])};
      store_payload((u32x4 *)a.partial + (size_t)pr * nvec + vi, o);
    }
  } else {
    unsigned long long lm = leaders;
    while (lm) {
      const int j = __builtin_ctzll(lm);
      lm &= lm - 1;
      float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
      for (int k = 0; k < K; ++k) {
        const int r = __builtin_amdgcn_readlane(row, k);
        const int f = __builtin_amdgcn_readlane(fk, k);
        const float w = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(wt), k));
        if (r >= 0 && f == j) fma8(acc, w, __builtin_nontemporal_load(y + (size_t)r * nvec + vi));
      }
      const int pr = __builtin_amdgcn_readlane(prow, j);
      u32x4 o = {pack_bf16_rne(acc[0], acc[1]), pack_bf16_rne(acc[2], acc[3]),
                 pack_bf16_rne(acc[4], acc[5]), pack_bf16_rne(acc[6], acc[7])};
      store_payload((u32x4 *)a.partial + (size_t)pr * nvec + vi, o);
    }
  }
}

int launch_combine_partial(const CombinePartialArgs &a0, void *stream) {
  if (a0.T <= 0) return 0;
  CombinePartialArgs a = a0;
  const int nvec = a.H / 8;
  a.parts = (nvec + 63) / 64;
  const long long items = (long long)a.T * a.parts;
  const unsigned grid = (unsigned)((items + 3) / 4);
  hipStream_t st = (hipStream_t)stream;
  switch (a.K) {
    case 2: hipLaunchKernelGGL(combine_partial_kernel<2>, dim3(grid), dim3(256), 0, st, a); break;
    case 4: hipLaunchKernelGGL(combine_partial_kernel<4>, dim3(grid), dim3(256), 0, st, a); break;
    case 8: hipLaunchKernelGGL(combine_partial_kernel<8>, dim3(grid), dim3(256), 0, st, a); break;
    default: hipLaunchKernelGGL(combine_partial_kernel<0>, dim3(grid), dim3(256), 0, st, a); break;
  }
  return (int)hipGetLastError();
}

// ------------------------------------------------- proxy-issued peer writes
// blockIdx.y = descriptor, blockIdx.x strides over its 16-byte vectors.
__global__ __launch_bounds__(256) void copy_batch_kernel(const CopyBatchArgs b) {
  __shared__ unsigned sd[3 * kCopyGroup];
  const int g0 = blockIdx.y * kCopyGroup;
  const int mine = min(kCopyGroup, b.n - g0);
  if ((int)threadIdx.x < 3 * mine)
    sd[threadIdx.x] = __hip_atomic_load((const unsigned *)(b.descs + g0) + threadIdx.x, __ATOMIC_RELAXED,
                                        __HIP_MEMORY_SCOPE_SYSTEM);
  __syncthreads();
  for (int k = 0; k < mine; ++k) {
    const unsigned src16 = sd[3 * k], dst16 = sd[3 * k + 1], len16 = sd[3 * k + 2];
    const u32x4 *s = (const u32x4 *)b.src_base + src16;
    u32x4 *o = (u32x4 *)b.dst_base + dst16;
    for (unsigned i = blockIdx.x * 256 + threadIdx.x; i < len16; i += gridDim.x * 256)
      o[i] = __builtin_nontemporal_load(s + i);
  }
}

__global__ __launch_bounds__(256) void copy_large_kernel(const CopyArgBatch b) {
  const CopyDesc d = b.d[blockIdx.y];
  const u32x4 *s = (const u32x4 *)b.src_base + d.src16;
  u32x4 *o = (u32x4 *)b.dst_base + d.dst16;
  for (unsigned i = blockIdx.x * 256 + threadIdx.x; i < d.len16; i += gridDim.x * 256)
    o[i] = __builtin_nontemporal_load(s + i);
}

int launch_copy_batch(const CopyBatchArgs &b, void *stream) {
  if (b.n <= 0) return 0;
  unsigned gx = (b.max_len16 + 255) / 256;
  if (gx < 1) gx = 1;
  if (gx > 64) gx = 64;  // 64 x 4 KiB per pass and descriptor, grid-stride beyond
  if (b.max_len16 > 2048) {  // copies beyond 32 KiB: a workgroup per (copy, piece), descriptors as arguments
    CopyArgBatch a;
    a.src_base = b.src_base;
    a.dst_base = b.dst_base;
    for (int first = 0; first < b.n; first += kCopyArgMax) {
      const int m = b.n - first < kCopyArgMax ? b.n - first : kCopyArgMax;
      for (int i = 0; i < m; ++i) a.d[i] = b.host_descs[first + i];
      hipLaunchKernelGGL(copy_large_kernel, dim3(gx, (unsigned)m), dim3(256), 0, (hipStream_t)stream, a);
    }
    return (int)hipGetLastError();
  }
  hipLaunchKernelGGL(copy_batch_kernel, dim3(gx, (unsigned)((b.n + kCopyGroup - 1) / kCopyGroup)), dim3(256), 0,
                     (hipStream_t)stream, b);
  return (int)hipGetLastError();
}


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

// ---------------------------------------------------------------- barrier
// One lane pushes a Barrier on channel 0 and blocks on Check-completion: the proxy pops it only
// when every peer process has entered (Section 3.1: Barrier is blocking on the GPU side).
__global__ void barrier_kernel(RingDev ring) {
  if (threadIdx.x != 0) return;
  const unsigned long long idx = ring_push(ring, 0, cmd_w0(EP_OP_BARRIER, 0, 0, 0), 0u, 0u, 0u);
  if (idx != ~0ull) ring_wait_completion(ring, 0, idx);
}

int launch_barrier(const RingDev &ring, void *stream) {
  hipLaunchKernelGGL(barrier_kernel, dim3(1), dim3(64), 0, (hipStream_t)stream, ring);
  return (int)hipGetLastError();
}

// ------------------------------------------------------------- FIFO stress
// Closed loop: lane 0 of every wave pushes a command, waits until the proxy has popped it
// (Check-completion), and only then pushes the next one.
__global__ void fifo_stress_kernel(RingDev ring, int pushers, int per_pusher, unsigned long long *lat_sum,
                                   unsigned long long *lat_max) {
  const int p = (blockIdx.x * blockDim.x + threadIdx.x) >> 6;
  if (p >= pushers || lane_id() != 0) return;
  const unsigned ch = (unsigned)p % ring.channels;
  unsigned long long sum = 0, mx = 0;
  for (int i = 0; i < per_pusher; ++i) {
    const unsigned long long t0 = wall_clock64();
    const unsigned long long idx = ring_push(ring, ch, cmd_w0(EP_OP_ATOMIC, 0, 0, 0), 0u, 0u, 0u);
    if (idx == ~0ull || !ring_wait_completion(ring, ch, idx)) break;
    const unsigned long long dt = wall_clock64() - t0;
    sum += dt;
    mx = dt > mx ? dt : mx;
  }
  lat_sum[p] = sum;
  lat_max[p] = mx;
}

int launch_fifo_stress(const RingDev &ring, int pushers, int per_pusher, unsigned long long *lat_sum,
                       unsigned long long *lat_max, void *stream) {
  hipLaunchKernelGGL(fifo_stress_kernel, dim3((unsigned)((pushers + 3) / 4)), dim3(256), 0, (hipStream_t)stream, ring,
                     pushers, per_pusher, lat_sum, lat_max);
  return (int)hipGetLastError();
}

// ------------------------------------------------------------ receive wait
// One thread per expert polls its arrival flag in pinned host memory with
// system-scope loads (each poll is a PCIe read, so lanes sleep between polls),
// hands the posted count to the caller and clears the flag.  Every lane leaves
// the loop: either its flag arrived or the bound expired.
__global__ __launch_bounds__(1024) void recv_wait_kernel(RecvWaitArgs a) {
  for (int e = threadIdx.x; e < a.E; e += blockDim.x) {
    if (a.filter >= 0 && e / a.E_loc != a.filter) {
      if (a.out) a.out[e] = -1;
      continue;
    }
    int *flag = a.flags + (size_t)a.src * a.E + e;
    const unsigned long long t0 = wall_clock64();
    int v;
    for (;;) {
      v = __hip_atomic_load(flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
      if (v != 0) break;
      if (wall_clock64() - t0 > a.timeout_ticks) {
        dev_set_error(a.error, EP_ETIMEOUT);
        break;
      }
      __builtin_amdgcn_s_sleep(64);
    }
    if (v != 0) __hip_atomic_store(flag, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
    if (a.out) a.out[e] = v - 1;
  }
}

int launch_recv_wait(const RecvWaitArgs &a, void *stream) {
  const int threads = a.E < 64 ? 64 : (a.E > 1024 ? 1024 : (a.E + 63) / 64 * 64);
  hipLaunchKernelGGL(recv_wait_kernel, dim3(1), dim3(threads), 0, (hipStream_t)stream, a);
  return (int)hipGetLastError();
}

// ------------------------------------------------------------------- misc
__global__ void fill_u32_kernel(uint32_t *p, uint32_t v, long long n) {
  const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
  if (i < n) p[i] = v;
}

// Bandwidth probes: one 16-byte access per lane, one short wave per KiB (measured best shape).
__global__ __launch_bounds__(256) void bw_read_kernel(const u32x4 *p, long long n, u32x4 *sink) {
  const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
  if (i >= n) return;
  const u32x4 v = __builtin_nontemporal_load(p + i);
  if (v[0] == 0x9E3779B9u && v[1] == 0x7F4A7C15u && v[2] == 0xBF58476Du && v[3] == 0x1CE4E5B9u) *sink = v;
}
__global__ __launch_bounds__(256) void bw_write_kernel(u32x4 *p, long long n) {
  const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
  if (i < n) p[i] = u32x4{1u, 2u, 3u, (unsigned)i};
}
__global__ __launch_bounds__(256) void bw_copy_kernel(const u32x4 *s, u32x4 *d, long long n) {
  const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
  if (i < n) d[i] = __builtin_nontemporal_load(s + i);
}

int launch_bw_probe(int kind, const void *src, void *dst, long long bytes, void *stream) {
  const long long n = bytes / 16;
  if (n <= 0) return 0;
  const dim3 grid((unsigned)((n + 255) / 256)), block(256);
  hipStream_t st = (hipStream_t)stream;
  if (kind == 0) hipLaunchKernelGGL(bw_read_kernel, grid, block, 0, st, (const u32x4 *)src, n, (u32x4 *)dst);
  else if (kind == 1) hipLaunchKernelGGL(bw_write_kernel, grid, block, 0, st, (u32x4 *)dst, n);
  else hipLaunchKernelGGL(bw_copy_kernel, grid, block, 0, st, (const u32x4 *)src, (u32x4 *)dst, n);
  return (int)hipGetLastError();
}

int launch_fill_u32(uint32_t *p, uint32_t v, long long n, void *stream) {
  if (n <= 0) return 0;
  hipLaunchKernelGGL(fill_u32_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, (hipStream_t)stream, p, v, n);
  return (int)hipGetLastError();
}

}  // namespace ep
