// Device-side helpers shared by the HIP kernels of libep.so (gfx950): the GPU end of the GPU->CPU FIFO
// channels (Push, Check-completion, Drain), the payload store and its completion wait, the FP8
// quantiser, and small wave-level utilities.  Everything here is inlined into the kernels.
#ifndef EP_DEVICE_H_
#define EP_DEVICE_H_
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>

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
EP_DEV unsigned long long ring_publish(const RingDev &r, unsigned c, unsigned long long idx, unsigned w0, unsigned w1,
                                       unsigned w2, unsigned w3);
EP_DEV unsigned long long ring_push(const RingDev &r, unsigned c, unsigned w0, unsigned w1,
                                    unsigned w2, unsigned w3) {
  const unsigned long long idx =
      __hip_atomic_fetch_add(&r.tail[c], 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  return ring_publish(r, c, idx, w0, w1, w2, w3);
}

// Push for the case where many lanes of a wave push at once (one command per row): lanes that aim at
// the same channel share ONE atomic on its tail - the first of them reserves a run of Idx for all,
// the others take their place in the run.  Atomics on one address serialise in the L2, and a
// per-token dispatch sends tens of thousands of commands through a handful of tails.
EP_DEV unsigned long long ring_push_grouped(const RingDev &r, unsigned c, unsigned w0, unsigned w1, unsigned w2,
                                            unsigned w3) {
  const int me = lane_id();
  unsigned long long same = 0ull;
  for (unsigned long long m = __ballot(true); m; m &= m - 1) {
    const int j = __builtin_ctzll(m);
    if ((unsigned)__builtin_amdgcn_readlane((int)c, j) == c) same |= 1ull << j;
  }
  const int leader = __builtin_ctzll(same);
  unsigned long long base = 0ull;
  if (me == leader)
    base = __hip_atomic_fetch_add(&r.tail[c], (unsigned long long)__popcll(same), __ATOMIC_RELAXED,
                                  __HIP_MEMORY_SCOPE_AGENT);
  base = ((unsigned long long)(unsigned)__shfl((int)(base >> 32), leader) << 32) | (unsigned)__shfl((int)base, leader);
  return ring_publish(r, c, base + (unsigned long long)__popcll(same & ((1ull << me) - 1ull)), w0, w1, w2, w3);
}

// Push for a whole wave whose lanes hold one command each (or none: `active`), called by all 64
// lanes together.  Runs of Idx are reserved per channel as in ring_push_grouped; then the commands
// change lanes through LDS (`scratch`, 2 KB) so that lane order is (channel, Idx) order: neighbouring
// lanes store neighbouring slots, and the memory pipeline turns the slots of one 64-byte line into one
// write.  A line of host memory that the proxy is polling costs the PCIe root a round of coherence
// traffic per write that lands in it, whatever the size of the write.
EP_DEV void ring_push_sorted(const RingDev &r, bool active, unsigned c, unsigned w0, unsigned w1, unsigned w2,
                             unsigned w3, u32x4 *scratch) {
  const int me = lane_id();
  const unsigned long long act = __ballot(active);
  unsigned long long same = 0ull;
  int less = 0;
  for (unsigned long long m = act; m;) {  // once per distinct channel
    const unsigned cj = (unsigned)__builtin_amdgcn_readlane((int)c, __builtin_ctzll(m));
    const unsigned long long mj = __ballot(active && c == cj);
    if (cj == c) same = mj;
    if (cj < c) less += __popcll(mj);
    m &= ~mj;
  }
  const int leader = (active && same) ? __builtin_ctzll(same) : 0;
  const int before = __popcll(same & ((1ull << me) - 1ull));
  unsigned long long base = 0ull;
  if (active && me == leader)
    base = __hip_atomic_fetch_add(&r.tail[c], (unsigned long long)__popcll(same), __ATOMIC_RELAXED,
                                  __HIP_MEMORY_SCOPE_AGENT);
  base = ((unsigned long long)(unsigned)__shfl((int)(base >> 32), leader) << 32) | (unsigned)__shfl((int)base, leader);
  if (active) {
    const unsigned long long idx = base + (unsigned long long)before;
    scratch[less + before] = u32x4{w0, w1, w2, w3};
    scratch[64 + less + before] = u32x4{c, (unsigned)idx, (unsigned)(idx >> 32), 0u};
  }
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
  if (me < __popcll(act)) {
    const u32x4 w = scratch[me], q = scratch[64 + me];
    ring_publish(r, q.x, ((unsigned long long)q.z << 32) | q.y, w.x, w.y, w.z, w.w);
  }
  __builtin_amdgcn_wave_barrier();  // (the next round writes the scratch again)
}

// Second half of a Push: wait for room for the reserved Idx, then publish the command.
EP_DEV unsigned long long ring_publish(const RingDev &r, unsigned c, unsigned long long idx, unsigned w0, unsigned w1,
                                       unsigned w2, unsigned w3) {
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
        // one 16-byte store straight to host memory (system scope); not waited for here, see store_payload
        asm volatile("global_store_dwordx4 %0, %1, off sc0 sc1" ::"v"(slot), "v"(v) : "memory");
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
EP_DEV void wait_for_own_stores();
EP_DEV bool ring_wait_completion(const RingDev &r, unsigned c, unsigned long long idx) {
  // the command has to have left before it can be popped: a poll issued together with the Push store
  // only finds the old head, and the next poll comes a sleep and a PCIe round trip later
  wait_for_own_stores();
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

// Payload rows are stored write-through at system scope (sc0 sc1): when such a store is
// acknowledged the bytes are in memory, visible to every XCD's L2 and to a PCIe reader, which is
// what a transfer command promises about the rows it names.  A wave therefore only has to wait
// for its own stores (vmcnt) before it touches a counter or pushes a command; no L2 write-back
// is needed, and the counters can be relaxed device-scope atomics.  Measured on MI355X the
// write-through stores stream as fast as non-temporal ones, whereas a device-scope release fence
// per wave (L2 write-back) made the dispatch 4-8x slower.
// The store is written out as the instruction itself: the way to get these cache bits from C++ is
// a volatile access, and the compiler follows EVERY volatile store with a wait for all outstanding
// memory operations - a wave would then hand the memory system one kilobyte at a time (dispatch
// 91 -> 87 us without those waits).  The compiler does not count these stores, so the wait that
// orders them is explicit as well.
EP_DEV void store_payload(u32x4 *p, const u32x4 &v) {
  asm volatile("global_store_dwordx4 %0, %1, off sc0 sc1" ::"v"(p), "v"(v) : "memory");
}

// All stores of this wave are acknowledged after this (hardware wait, then a compiler barrier).
EP_DEV void wait_for_own_stores() {
  __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0); expcnt and lgkmcnt left alone
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
}

// Kernel epilogue with EP_CMD_DRAIN: the last workgroup of the grid to finish pushes a Drain on
// every channel and blocks on Check-completion for each (Section 3.1: Drain and Barrier are blocking
// on the GPU side).  Every wave of every workgroup must call this.
// "Last to finish" is counted per workgroup and in two levels (groups of kDrainGroup workgroups,
// then groups): atomics on ONE address serialise in the L2 at about 8 ns each, and one count per
// wave of a 32768-wave grid added 270 us to the kernel.  done_cnt: [1 + groups] scratch, zero
// between launches (the counters reset themselves).
constexpr unsigned kDrainGroup = 64;
EP_DEV void drain_all_channels(const RingDev &ring, unsigned *done_cnt, unsigned src, int lane) {
  wait_for_own_stores();  // this wave's commands are in their rings ...
  __syncthreads();        // ... and so are those of every wave of the workgroup
  if (threadIdx.x >= 64) return;
  unsigned last = 0;
  if (lane == 0) {
    const unsigned group = blockIdx.x / kDrainGroup, ngroups = (gridDim.x + kDrainGroup - 1) / kDrainGroup;
    const unsigned gsize = min(kDrainGroup, gridDim.x - group * kDrainGroup);
    if (__hip_atomic_fetch_add(&done_cnt[1 + group], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) + 1u == gsize) {
      __hip_atomic_store(&done_cnt[1 + group], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if (__hip_atomic_fetch_add(&done_cnt[0], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) + 1u == ngroups) {
        __hip_atomic_store(&done_cnt[0], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        last = 1;
      }
    }
  }
  if (!__builtin_amdgcn_readfirstlane(last)) return;
  for (unsigned c = lane; c < ring.channels; c += 64) {
    const unsigned long long idx = ring_push(ring, c, cmd_w0(EP_OP_DRAIN, src, 0, 0), 0u, 0u, 0u);
    if (idx != ~0ull) ring_wait_completion(ring, c, idx);
  }
}

// ---------------------------------------------------------- wave utilities
EP_DEV int wave_inclusive_scan(int v, int lane) {
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    const int u = __shfl_up(v, d);
    if (lane >= d) v += u;
  }
  return v;
}

// One launch, with the kernel's own begin / end timestamps delivered into the caller's events when asked for.
template <class Kernel, class Args>
static inline void launch_kernel(Kernel kernel, dim3 grid, dim3 block, size_t lds, hipStream_t st, void *ev_start,
                                 void *ev_stop, const Args &a) {
  if (ev_start || ev_stop)
    hipExtLaunchKernelGGL(kernel, grid, block, (unsigned)lds, st, (hipEvent_t)ev_start, (hipEvent_t)ev_stop, 0, a);
  else
    hipLaunchKernelGGL(kernel, grid, block, lds, st, a);
}

// ------------------------------------------------------------ FP8 quantiser
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

}  // namespace ep
#endif  // EP_DEVICE_H_
