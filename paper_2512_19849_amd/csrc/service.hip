// Service kernels: the copies the proxy issues when it performs the peer writes itself, Barrier, the FIFO
// stress test, the GPU-side wait for the completion counters, bandwidth probes, fill.
#include "ep_device.h"

namespace ep {

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

// Receiver side of FP8 rows that travelled as messages (codes, scales, padding): split them into the code and
// the scale array.  One wave per (row, 64 vectors of codes); the wave of a row's first slice also moves the scales.
__global__ __launch_bounds__(256) void fp8_unpack_kernel(const char *msgs, long long rows, int H, unsigned row_bytes,
                                                         u32x4 *q, float *scale) {
  const int lane = lane_id();
  const int nvec = H >> 4, parts = (nvec + 63) / 64, nblk = H >> 7;
  const long long w = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
  const long long row = w / parts;
  const int part = (int)(w % parts);
  if (row >= rows) return;
  const char *msg = msgs + (size_t)row * row_bytes;
  const int v = part * 64 + lane;
  if (v < nvec) q[(size_t)row * nvec + v] = __builtin_nontemporal_load((const u32x4 *)msg + v);
  if (part == 0)
    for (int b = lane; b < nblk; b += 64) scale[(size_t)row * nblk + b] = __builtin_nontemporal_load((const float *)(msg + H) + b);
}

int launch_fp8_unpack(const void *msgs, long long rows, int H, unsigned row_bytes, void *q, float *scale, void *stream) {
  const long long waves = rows * (((H >> 4) + 63) / 64);
  if (waves <= 0) return 0;
  if (waves >= (1ll << 33)) return (int)hipErrorInvalidValue;
  hipLaunchKernelGGL(fp8_unpack_kernel, dim3((unsigned)((waves + 3) / 4)), dim3(256), 0, (hipStream_t)stream,
                     (const char *)msgs, rows, H, row_bytes, (u32x4 *)q, scale);
  return (int)hipGetLastError();
}

// Row-pattern probes: the dispatch's stores without its loads (every item stores a constant to the slices of
// its k rows, write-through as the dispatch does), and the combine's loads without its stores (k streaming
// loads per lane, nothing written).  One wave per (item, 64-vector slice); rows outside the buffer are skipped.
template <bool WRITE>
__global__ __launch_bounds__(256) void row_probe_kernel(const int32_t *rowmap, int k, long long items, int nvec,
                                                        long long buf_rows, u32x4 *buf, u32x4 *sink) {
  const int lane = lane_id();
  const int parts = (nvec + 63) / 64;
  const long long w = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
  const long long item = w / parts;
  const int v = (int)(w % parts) * 64 + lane;
  if (item >= items) return;
  int row = lane < k ? rowmap[item * k + lane] : -1;
  if (row >= buf_rows) row = -1;
  u32x4 acc = {0u, 0u, 0u, 0u};
  for (int j = 0; j < k; ++j) {
    const int r = __builtin_amdgcn_readlane(row, j);
    if (r < 0 || v >= nvec) continue;
    u32x4 *p = buf + (size_t)r * nvec + v;
    if (WRITE) {
      store_payload(p, u32x4{1u, 2u, 3u, (unsigned)item});
    } else {
      const u32x4 x = __builtin_nontemporal_load(p);
      acc[0] ^= x[0], acc[1] ^= x[1], acc[2] ^= x[2], acc[3] ^= x[3];
    }
  }
  if (!WRITE && acc[0] == 0x9E3779B9u && acc[1] == 0x7F4A7C15u && acc[2] == 0xBF58476Du && acc[3] == 0x1CE4E5B9u) *sink = acc;
}

int launch_row_probe(int kind, const int32_t *rowmap, int k, long long items, int row_bytes, long long buf_rows,
                     void *buf, void *sink, void *stream) {
  const int nvec = row_bytes / 16;
  const long long waves = items * ((nvec + 63) / 64);
  if (waves <= 0) return 0;
  const dim3 grid((unsigned)((waves + 3) / 4)), block(256);
  if (kind == 0)
    hipLaunchKernelGGL(row_probe_kernel<true>, grid, block, 0, (hipStream_t)stream, rowmap, k, items, nvec, buf_rows,
                       (u32x4 *)buf, (u32x4 *)sink);
  else
    hipLaunchKernelGGL(row_probe_kernel<false>, grid, block, 0, (hipStream_t)stream, rowmap, k, items, nvec, buf_rows,
                       (u32x4 *)buf, (u32x4 *)sink);
  return (int)hipGetLastError();
}

int launch_fill_u32(uint32_t *p, uint32_t v, long long n, void *stream) {
  if (n <= 0) return 0;
  hipLaunchKernelGGL(fill_u32_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, (hipStream_t)stream, p, v, n);
  return (int)hipGetLastError();
}

}  // namespace ep
