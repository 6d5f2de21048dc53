// Dispatch (bf16 / FP8 E4M3) and the emission of transfer commands: HBM-bound row copies with 16-byte vector
// accesses, one wavefront per token or per slice of a token; no dense contraction, hence no MFMA.
#include "ep_device.h"

namespace ep {

// ------------------------------------------------- dispatch: command emission
struct TokenMeta {
  int e;       // expert of this lane's k (lane < K), -1 otherwise
  int row;     // destination row
  bool valid;  // this (t, k) is dispatched by this call
};

// Which group of tokens this workgroup takes: launch order, or the mirror image of it.
EP_DEV int token_block(const DispatchArgs &a) {
  return a.reverse ? (int)gridDim.x - 1 - (int)blockIdx.x : (int)blockIdx.x;
}

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
// `rows` more rows of expert e (c in all) have been handed to the channel; whoever hands over the
// last one pushes the expert's count Atomic.
EP_DEV void account_rows(const DispatchArgs &a, int e, int c, int rows) {
  const int done = __hip_atomic_fetch_add(a.expert_done + e, rows, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) + rows;
  if (done == c) {
    __hip_atomic_store(a.expert_done + e, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (!(a.cmd_mode & EP_CMD_ATOMICS_FIRST)) push_count_atomic(a, e, c);
  }
}

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
    ring_push_grouped(a.ring, ch, cmd_w0(EP_OP_WRITE, a.src, dr, le), a.row_bytes >> 4, (unsigned)(so >> 4),
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
  if (finished_rows) account_rows(a, e, c, finished_rows);
}

// One command per row, several tokens per workgroup: the tokens' (expert, row) pairs meet in LDS
// and the first wave pushes for all of them, sorted by channel, so that the commands of a channel
// leave as one run of consecutive slots written by neighbouring lanes (see ring_push_sorted).
EP_DEV void emit_block_cmds(const DispatchArgs &a, const TokenMeta &m, int part, int wave, int lane) {
  extern __shared__ u32x4 s_dyn[];
  int2 *s_pairs = (int2 *)s_dyn;  // [tokens_per_block][K], then the 2 KB of ring_push_sorted
  if (part == 0 && lane < a.K) s_pairs[(wave / a.parts) * a.K + lane] = make_int2(m.valid ? m.e : -1, m.row);
  __syncthreads();  // every wave has waited for its own stores before it came here
  if (wave != 0) return;
  const int n = a.tokens_per_block * a.K;
  u32x4 *scratch = (u32x4 *)(s_pairs + ((n + 1) & ~1));
  for (int i0 = 0; i0 < n; i0 += 64) {
    const int i = i0 + lane;
    const int2 p = i < n ? s_pairs[i] : make_int2(-1, -1);
    const bool active = p.x >= 0;
    const int e = active ? p.x : 0;
    const unsigned dr = (unsigned)(e / a.E_loc), le = (unsigned)(e - (int)dr * a.E_loc);
    const unsigned long long so = (unsigned long long)(token_block(a) * a.tokens_per_block + i / a.K) * a.row_bytes;
    const unsigned long long dof = (unsigned long long)p.y * a.row_bytes;
    ring_push_sorted(a.ring, active, (unsigned)e % a.ring.channels, cmd_w0(EP_OP_WRITE, a.src, dr, le),
                     a.row_bytes >> 4, (unsigned)(so >> 4), (unsigned)(dof >> 4), scratch);
    if (active) account_rows(a, e, a.count[e], 1);
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
// (The same placement as in dispatch_bf16_kernel below, as a function for the form with a command wave; the plain
// kernel keeps its own copy: with the body moved into a function the compiler allocated 61 instead of 46
// registers for it and spilled at 7 and 8 vectors per lane.)
template <int VPL>
EP_DEV void place_token_bf16(const DispatchArgs &a, const int row_of_lane, unsigned long long vmask, int t, int part,
                             int lane) {
  if (!vmask || (a.cmd_mode & EP_CMD_NO_PLACEMENT)) return;
  const int nvec = a.H >> 3;
  const int v0 = part * VPL * 64 + lane;
  const u32x4 *src = (const u32x4 *)a.x + (size_t)t * nvec;
  u32x4 v[VPL];
#pragma unroll
  for (int i = 0; i < VPL; ++i)
    if (v0 + i * 64 < nvec) v[i] = __builtin_nontemporal_load(src + v0 + i * 64);
  unsigned long long mm = vmask;
  while (mm) {
    const int k = __builtin_ctzll(mm);
    mm &= mm - 1;
    const int row = __builtin_amdgcn_readlane(row_of_lane, k);
    u32x4 *dst = (u32x4 *)a.recv + (size_t)row * nvec;
#pragma unroll
    for (int i = 0; i < VPL; ++i)
      if (v0 + i * 64 < nvec) store_payload(dst + v0 + i * 64, v[i]);
  }
}

template <int VPL>
__global__ void dispatch_bf16_kernel(DispatchArgs a) {
  const int wave = threadIdx.x >> 6, lane = lane_id();
  const int part = wave % a.parts;
  const int t = token_block(a) * a.tokens_per_block + wave / a.parts;
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
  if (a.block_cmds) {
    emit_block_cmds(a, m, part, wave, lane);
  } else {
    if (a.parts > 1) __syncthreads();
    if (part == 0 && m.valid) emit_row_cmds(a, m, t);
  }
  if (a.cmd_mode & EP_CMD_DRAIN) emit_drain(a, lane);
}

// ------------------------------------------------------------- dispatch FP8
template <int VPL>
EP_DEV void place_token_fp8(const DispatchArgs &a, const TokenMeta &m, unsigned long long vmask, int t, int part) {
  if (!vmask) return;
  const int lane = lane_id();
  const int npair = a.H >> 4;  // 16-channel groups per row
  const int nblk = a.H >> 7;   // 128-channel blocks per row
  const int p0 = part * VPL * 64 + lane;
  {
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
    // Where a row goes: into the two receive arrays (codes, scales), or - when the proxy moves the rows -
    // as ONE message of row_bytes bytes (the H codes, then the H/128 fp32 scales, padded to 16 bytes:
    // the ~7 KB token of Section 2.1) into the send heap: at its destination row for chunk commands
    // (the heap mirrors the receive heap), or once, at the token's own row, for per-token commands.
    unsigned long long mm = a.msg_rows == 2 ? 1ull : vmask;
    while (mm) {
      const int k = __builtin_ctzll(mm);
      mm &= mm - 1;
      const int row = a.msg_rows == 2 ? t : __builtin_amdgcn_readlane(m.row, k);
      u32x4 *dq;
      float *ds;
      if (a.msg_rows) {
        char *msg = (char *)a.recv + (size_t)row * a.row_bytes;
        dq = (u32x4 *)msg;
        ds = (float *)(msg + a.H);
      } else {
        dq = (u32x4 *)a.recv + (size_t)row * npair;
        ds = a.recv_scale + (size_t)row * nblk;
      }
#pragma unroll
      for (int i = 0; i < VPL; ++i)
        if (p0 + i * 64 < npair) {
          store_payload(dq + p0 + i * 64, q[i]);
          if ((lane & 7) == 0)
            __hip_atomic_store(ds + ((p0 + i * 64) >> 3), sc[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
        }
    }
  }
}

template <int VPL>
__global__ void dispatch_fp8_kernel(DispatchArgs a) {
  const int wave = threadIdx.x >> 6, lane = lane_id();
  const int part = wave % a.parts;
  const int t = token_block(a) * a.tokens_per_block + wave / a.parts;
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
    // Where a row goes: into the two receive arrays (codes, scales), or - when the proxy moves the rows -
    // as ONE message of row_bytes bytes (the H codes, then the H/128 fp32 scales, padded to 16 bytes:
    // the ~7 KB token of Section 2.1) into the send heap: at its destination row for chunk commands
    // (the heap mirrors the receive heap), or once, at the token's own row, for per-token commands.
    unsigned long long mm = a.msg_rows == 2 ? 1ull : vmask;
    while (mm) {
      const int k = __builtin_ctzll(mm);
      mm &= mm - 1;
      const int row = a.msg_rows == 2 ? t : __builtin_amdgcn_readlane(m.row, k);
      u32x4 *dq;
      float *ds;
      if (a.msg_rows) {
        char *msg = (char *)a.recv + (size_t)row * a.row_bytes;
        dq = (u32x4 *)msg;
        ds = (float *)(msg + a.H);
      } else {
        dq = (u32x4 *)a.recv + (size_t)row * npair;
        ds = a.recv_scale + (size_t)row * nblk;
      }
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
  if (a.block_cmds) {
    emit_block_cmds(a, m, part, wave, lane);
  } else {
    if (a.parts > 1) __syncthreads();
    if (part == 0 && m.valid) emit_row_cmds(a, m, t);
  }
  if (a.cmd_mode & EP_CMD_DRAIN) emit_drain(a, lane);
}

// ------------------------------------------- dispatch with a command wavefront
// Ring-on launches: persistent workgroups of D data waves and ONE command wave.  A data wave places its
// slice of a token, waits for its own stores, leaves the token's (expert, row) pairs in LDS and goes on
// to the workgroup's next batch of tokens; the command wave picks the batch up when all D waves have
// signed it off and does everything that needs a round trip through the L2 or a store to host memory -
// completion counting, Idx reservation, the Push itself, count Atomics - while the data waves are already
// storing the next batch.  Two batches of pairs fit the LDS, so the command wave may lag one batch behind.
// Waits between the waves are LDS polls, each bounded by the ring's time limit.
// Selected with EP_DISPATCH_PIPELINE=1 and off by default: measured on MI355X (4096 tokens x 7168, and 8192 x
// 4096) it is no faster than the plain form with chunk commands (111.9 vs 112.2 us, 125.6 vs 123.7 us) and
// slower with one command per row (121.8 vs 116.0 us, 158.9 vs 146.2 us).  Under a saturating store stream
// every round trip of the command wave (Idx reservation, head check, completion counting) queues behind the
// compute unit's own stores and takes microseconds, so one command wave per workgroup falls behind its data
// waves; and the row stores themselves run at the rate the memory system gives scattered rows whatever the
// kernel's shape, so hiding the commands' latency buys nothing there.
EP_DEV void pipe_wait_at_least(int *p, int want, const RingDev &r) {
  if (__hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP) >= want) return;
  const unsigned long long t0 = wall_clock64();
  while (__hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP) < want) {
    if (wall_clock64() - t0 > r.timeout_ticks) {
      dev_set_error(r.error, EP_ETIMEOUT);
      break;
    }
    __builtin_amdgcn_s_sleep(2);
  }
}

template <int VPL, bool FP8>
__global__ __launch_bounds__(1024) void dispatch_pipelined_kernel(DispatchArgs a) {
  extern __shared__ u32x4 s_dyn[];
  int *ctl = (int *)s_dyn;  // [0], [1]: sign-offs per slot (running totals); [2]: batches the command wave is through
  const int tpb = a.tokens_per_block, n = tpb * a.K, npad = (n + 1) & ~1;
  int2 *pairs = (int2 *)(ctl + 4);               // [2][npad]
  u32x4 *scratch = (u32x4 *)(pairs + 2 * npad);  // 2 KB for ring_push_sorted
  const int wave = threadIdx.x >> 6, lane = lane_id();
  const int D = a.parts * tpb;
  const int nb = (a.T + tpb - 1) / tpb;
  const int mode = a.cmd_mode & EP_CMD_MODE_MASK;
  if (threadIdx.x < 4) ctl[threadIdx.x] = 0;
  __syncthreads();
  if (wave < D) {
    const int part = wave % a.parts, tok = wave / a.parts;
    int it = 0;
#pragma nounroll
    for (int b = blockIdx.x; b < nb; b += gridDim.x, ++it) {
      const int t = (a.reverse ? nb - 1 - b : b) * tpb + tok;
      const TokenMeta m = load_meta(a, t, lane);
      const unsigned long long vmask = __ballot(m.valid);
      if (FP8) place_token_fp8<VPL>(a, m, vmask, t, part);
      else place_token_bf16<VPL>(a, m.row, vmask, t, part, lane);
      wait_for_own_stores();  // the rows are in memory before a counter or command mentions them
      const int slot = it & 1;
      if (it >= 2) pipe_wait_at_least(&ctl[2], it - 1, a.ring);  // the batch that used this slot last is through
      if (part == 0 && lane < a.K) pairs[slot * npad + tok * a.K + lane] = make_int2(m.valid ? m.e : -1, m.row);
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
      if (lane == 0) __hip_atomic_fetch_add(&ctl[slot], 1, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_WORKGROUP);
    }
  } else {
    if (mode != EP_CMD_CHUNK32_ORDERED && blockIdx.x == 0) emit_leading_atomics(a, lane);
    int it = 0;
#pragma nounroll
    for (int b = blockIdx.x; b < nb; b += gridDim.x, ++it) {
      const int t0 = (a.reverse ? nb - 1 - b : b) * tpb;
      const int slot = it & 1;
      pipe_wait_at_least(&ctl[slot], D * (it / 2 + 1), a.ring);
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
      const int2 *pp = pairs + slot * npad;
      for (int i0 = 0; i0 < n; i0 += 64) {
        const int i = i0 + lane;
        const int2 p = i < n ? pp[i] : make_int2(-1, -1);
        const bool active = p.x >= 0;
        const int t = t0 + i / a.K;
        if (mode == EP_CMD_PER_TOKEN) {  // one command per row, sorted by channel (see ring_push_sorted)
          const int e = active ? p.x : 0;
          const unsigned dr = (unsigned)(e / a.E_loc), le = (unsigned)(e - (int)dr * a.E_loc);
          const unsigned long long so = (unsigned long long)t * a.row_bytes;
          const unsigned long long dof = (unsigned long long)p.y * a.row_bytes;
          ring_push_sorted(a.ring, active, (unsigned)e % a.ring.channels, cmd_w0(EP_OP_WRITE, a.src, dr, le),
                           a.row_bytes >> 4, (unsigned)(so >> 4), (unsigned)(dof >> 4), scratch);
          if (active) account_rows(a, e, a.count[e], 1);
        } else if (active) {
          const TokenMeta m{p.x, p.y, true};
          emit_row_cmds(a, m, t);
        }
      }
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");  // the pairs have been read: the slot may be refilled
      if (lane == 0) __hip_atomic_store(&ctl[2], it + 1, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_WORKGROUP);
    }
  }
  if (a.cmd_mode & EP_CMD_DRAIN) emit_drain(a, lane);
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

static int tuned_dispatch_vpl(int H, int T, int forced) {
  static const int c[] = {1, 2, 4, 7, 8, 14, 16};
  for (int v : c)
    if (v == forced) return v;
  // About four waves per token stream best (measured in the full path on 7168- and 4096-wide rows:
  // the command tail of one wave then overlaps the stores of the others); with few tokens the row
  // is split further until there are about 4096 waves (16 per compute unit).
  return split_for(H / 8, T, c, 7);
}

static int tuned_dispatch_fp8_vpl(int H, int T, int forced) {
  static const int c[] = {1, 2, 4};  // more than 4 groups per lane would spill at 128 VGPRs
  for (int v : c)
    if (v == forced) return v;
  return split_for(H / 16, T, c, 3);
}

// One command per row: as many tokens per workgroup as 16 waves hold (their commands are pushed
// together, see emit_block_cmds).  Returns the dynamic LDS bytes of the launch.
static size_t block_cmds_setup(DispatchArgs &a, int waves) {
  a.block_cmds = 0;
  if ((a.cmd_mode & EP_CMD_MODE_MASK) != EP_CMD_PER_TOKEN) return 0;
  if (waves < 4 || waves > 16) waves = 16;  // (0 = not set)
  const int tpb = waves / a.parts;
  if (tpb < 2) return 0;
  a.tokens_per_block = tpb;
  a.block_cmds = 1;
  return (size_t)((tpb * a.K + 1) & ~1) * sizeof(int2) + 2048;
}

// Ring-on launches take the form with a command wave when it is switched on and the row needs at most 15 data
// waves: returns false when the launch has to take the plain form.
template <int VPL, bool FP8>
static bool launch_pipelined(DispatchArgs a, const Tunables &tune, hipStream_t st, const LaunchTiming *tm) {
  if ((a.cmd_mode & EP_CMD_MODE_MASK) == EP_CMD_NONE || !tune.dispatch_pipeline || a.parts > 15) return false;
  int want = tune.per_token_waves;  // data waves per workgroup, at most
  if (want < 1 || want > 15) want = 12;
  a.tokens_per_block = want / a.parts > 0 ? want / a.parts : 1;
  const int D = a.parts * a.tokens_per_block;
  const int nb = (a.T + a.tokens_per_block - 1) / a.tokens_per_block;
  const int n = a.tokens_per_block * a.K;
  const size_t lds = 16 + (size_t)((n + 1) & ~1) * 2 * sizeof(int2) + 2048;
  // two workgroups per compute unit (256 of them) keep the chip full; each walks its batches with stride gridDim
  const int grid = nb < 1 ? 1 : (nb < 512 ? nb : 512);
  launch_kernel(dispatch_pipelined_kernel<VPL, FP8>, dim3(grid), dim3(64 * (D + 1)), lds, st, tm ? tm->start : nullptr,
                tm ? tm->stop : nullptr, a);
  return true;
}

template <int VPL>
static void launch_dispatch_bf16_t(DispatchArgs a, const Tunables &tune, hipStream_t st, const LaunchTiming *tm) {
  const int nvec = a.H / 8;
  a.parts = (nvec + VPL * 64 - 1) / (VPL * 64);
  if (launch_pipelined<VPL, false>(a, tune, st, tm)) return;
  a.tokens_per_block = a.parts >= 4 ? 1 : 4 / a.parts;
  const size_t lds = block_cmds_setup(a, tune.per_token_waves);
  const int grid = max(1, (a.T + a.tokens_per_block - 1) / a.tokens_per_block);
  launch_kernel(dispatch_bf16_kernel<VPL>, dim3(grid), dim3(64 * a.parts * a.tokens_per_block), lds, st,
                tm ? tm->start : nullptr, tm ? tm->stop : nullptr, a);
}

template <int VPL>
static void launch_dispatch_fp8_t(DispatchArgs a, const Tunables &tune, hipStream_t st, const LaunchTiming *tm) {
  const int npair = a.H / 16;
  a.parts = (npair + VPL * 64 - 1) / (VPL * 64);
  if (launch_pipelined<VPL, true>(a, tune, st, tm)) return;
  a.tokens_per_block = a.parts >= 4 ? 1 : 4 / a.parts;
  const size_t lds = block_cmds_setup(a, tune.per_token_waves);
  const int grid = max(1, (a.T + a.tokens_per_block - 1) / a.tokens_per_block);
  launch_kernel(dispatch_fp8_kernel<VPL>, dim3(grid), dim3(64 * a.parts * a.tokens_per_block), lds, st,
                tm ? tm->start : nullptr, tm ? tm->stop : nullptr, a);
}

int launch_dispatch(const DispatchArgs &a, int payload, const Tunables &tune, void *stream,
                    const LaunchTiming *timing) {
  hipStream_t st = (hipStream_t)stream;
  // T == 0 with the ring on still launches one (idle) workgroup: it owes the zero-count atomics
  if (a.T <= 0 && (a.cmd_mode & EP_CMD_MODE_MASK) == EP_CMD_NONE) return 0;
  if (payload == EP_BF16) {
    int vpl = tuned_dispatch_vpl(a.H, a.T, tune.dispatch_vpl);
    const int cmds = a.cmd_mode & EP_CMD_MODE_MASK;
    const bool free_choice = !tune.dispatch_vpl && !tune.dispatch_pipeline;
    // One command per row: two 1 KiB slices per wave (rows of up to 8192 channels then still put two tokens
    // into a workgroup, whose first wave pushes for both) beat four by 3-9 us per dispatch, measured for
    // hidden 5120..8192 and 2048..8192 tokens.  The sequenced chunk mode gains 2-6 us from the same shape at
    // 4096 tokens (hidden 5120..8192) and nothing at 8192.
    if (free_choice && (cmds == EP_CMD_PER_TOKEN || cmds == EP_CMD_CHUNK32_ORDERED) &&
        !(a.cmd_mode & EP_CMD_NO_PLACEMENT) && vpl > 2 && (a.H / 8 + 127) / 128 <= 8)
      vpl = 2;
    // Ring off or plain chunk commands: rows that exceed the memory-side cache (256 MB) by half or more have to
    // stream to HBM while the kernel runs; then ONE slice per wave (many small waves, eight 1 KiB stores each)
    // is faster by 5-10 us per 450-900 MB than four slices per wave, which wins below that size by as much
    // (measured for 224 to 896 MiB of rows, hidden 4096..8192) - and also where the caller has said that the
    // rows are consumed in place, out of that cache.  (The sequenced chunk mode, bound by its hottest channel's
    // FIFO, was measured slower with one slice per wave on the skewed workload.)
    const long long rows_at_most = (long long)a.T * a.K < a.recv_rows ? (long long)a.T * a.K : a.recv_rows;
    if (free_choice && !a.cache_hinted && (cmds == EP_CMD_NONE || cmds == EP_CMD_CHUNK32) &&
        rows_at_most * a.H * 2 >= 384000000ll && (a.H / 8 + 63) / 64 <= 16)
      vpl = 1;
    // (7 and 8 vectors per lane make the compiler spill in the form with a command wave: rows that wide take 14 / 16)
    if ((a.cmd_mode & EP_CMD_MODE_MASK) != EP_CMD_NONE && tune.dispatch_pipeline && (vpl == 7 || vpl == 8)) vpl *= 2;
    if ((a.H / 8 + vpl * 64 - 1) / (vpl * 64) > 16) return (int)hipErrorInvalidValue;
    switch (vpl) {
      case 1: launch_dispatch_bf16_t<1>(a, tune, st, timing); break;
      case 2: launch_dispatch_bf16_t<2>(a, tune, st, timing); break;
      case 4: launch_dispatch_bf16_t<4>(a, tune, st, timing); break;
      case 7: launch_dispatch_bf16_t<7>(a, tune, st, timing); break;
      case 8: launch_dispatch_bf16_t<8>(a, tune, st, timing); break;
      case 14: launch_dispatch_bf16_t<14>(a, tune, st, timing); break;
      default: launch_dispatch_bf16_t<16>(a, tune, st, timing); break;
    }
  } else {
    const int vpl = tuned_dispatch_fp8_vpl(a.H, a.T, tune.dispatch_fp8_vpl);
    if ((a.H / 16 + vpl * 64 - 1) / (vpl * 64) > 16) return (int)hipErrorInvalidValue;
    switch (vpl) {
      case 1: launch_dispatch_fp8_t<1>(a, tune, st, timing); break;
      case 2: launch_dispatch_fp8_t<2>(a, tune, st, timing); break;
      default: launch_dispatch_fp8_t<4>(a, tune, st, timing); break;
    }
  }
  return (int)hipGetLastError();
}

}  // namespace ep
