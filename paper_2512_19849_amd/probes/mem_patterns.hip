// mem_patterns - what plain access patterns reach on one MI355X, as kernels with telling names, meant to be run
// under `rocprofv3 --kernel-trace --stats`: the averages per kernel name are the result.  No part of the
// dispatch/combine library; it exists to put numbers behind the library's design notes (which stores and loads
// run at the stream rate, which do not, and what each ingredient of the dispatch and combine kernels costs).
//
// Shapes are those of the 4096-token workload: rows of 14 KiB (hidden 7168, bf16), 8 rows per token, 448 MiB
// of rows, 56 MiB of token rows.  Every kernel is launched `reps` times back to back after 3 warm-up launches.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdio>
#include <cstdlib>
#include <numeric>
#include <random>
#include <vector>

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
#define CK(x)                                                                           \
  do {                                                                                  \
    hipError_t err_ = (x);                                                              \
    if (err_ != hipSuccess) {                                                           \
      printf("HIP error %s at line %d\n", hipGetErrorString(err_), __LINE__);           \
      exit(1);                                                                          \
    }                                                                                   \
  } while (0)
#define DEV __device__ __forceinline__

constexpr int T = 4096, K = 8, NV = 896;  // tokens, rows per token, 16-byte vectors per row
constexpr long long kRows = (long long)T * K, kVecs = kRows * NV, kBlocks = kVecs / 256;  // 4 KiB blocks

DEV void store_wt(u32x4 *p, const u32x4 &v) {  // write-through, system scope: the dispatch's kind of store
  asm volatile("global_store_dwordx4 %0, %1, off sc0 sc1" ::"v"(p), "v"(v) : "memory");
}
DEV void keep(const u32x4 &v, u32x4 *sink) {
  if (v[0] == 0x9E3779B9u && v[1] == 0x7F4A7C15u && v[2] == 0xBF58476Du && v[3] == 0x1CE4E5B9u) *sink = v;
}

// ---- write streams: one 16-byte store per lane, 1 KiB per wave, 4 KiB per workgroup
// (ALTERNATING only names the instance that is launched in turns with a read stream further down)
template <bool ALTERNATING>
__global__ __launch_bounds__(256) void write_stream_in_launch_order(u32x4 *p) {
  const long long j = (long long)blockIdx.x * 256 + threadIdx.x;
  store_wt(p + j, u32x4{1u, 2u, 3u, (unsigned)j});
}
// the same stores, but every wave first sleeps 0..15 x 64 clocks (pseudo-random): same addresses, scrambled timing
__global__ __launch_bounds__(256) void write_stream_with_jittered_timing(u32x4 *p) {
  const long long j = (long long)blockIdx.x * 256 + threadIdx.x;
  const unsigned w = (unsigned)(j >> 6) * 2654435761u;
  for (unsigned s = 0; s < ((w >> 20) & 15u); ++s) __builtin_amdgcn_s_sleep(1);
  store_wt(p + j, u32x4{1u, 2u, 3u, (unsigned)j});
}
// workgroup i writes block (i % G) * (blocks / G) + i / G: G sequential streams, visited in turns of 4 KiB
// (G = 8: one stream per XCD, since workgroups go to the XCDs round-robin)
template <int G>
__global__ __launch_bounds__(256) void write_interleaved_sequential_streams(u32x4 *p) {
  const unsigned i = blockIdx.x, blk = (i % G) * (unsigned)(kBlocks / G) + i / G;
  store_wt(p + (size_t)blk * 256 + threadIdx.x, u32x4{1u, 2u, 3u, blk});
}
// the launch-ordered stream (all 448 MiB) cut into chunks of CHUNK_KIB that sit at bit-reversed positions
// (inside each seventh of the buffer): inside a chunk the stores arrive in address order as in the plain
// stream, the chunks themselves are scattered; the position is computed, so no wave waits for a load before
// it stores
template <int CHUNK_KIB>
__global__ __launch_bounds__(256) void write_stream_in_scattered_chunks(u32x4 *p) {
  constexpr unsigned per = CHUNK_KIB / 4;     // 4 KiB blocks per chunk
  constexpr unsigned m = 16384u / per;        // chunks per seventh of the buffer (a power of two)
  const unsigned i = blockIdx.x, c = i / per, j = i % per;
  const unsigned q = c / m, r = c % m;
  const unsigned rr = m > 1 ? __brev(r) >> (32 - __builtin_ctz(m)) : 0u;
  const size_t blk = ((size_t)q * m + rr) * per + j;
  store_wt(p + blk * 256 + threadIdx.x, u32x4{1u, 2u, 3u, i});
}
// ---- rows
// one workgroup (14 waves) per row, rows in sequential order: globally the same sequential stream as above,
// but a wave first has to fetch its row number
__global__ __launch_bounds__(896) void write_rows_in_order_one_row_per_workgroup(u32x4 *p, const int *rowmap) {
  const int row = rowmap[blockIdx.x];
  store_wt(p + (size_t)row * NV + threadIdx.x, u32x4{1u, 2u, 3u, (unsigned)row});
}
// the dispatch's shape: 4 waves per token, each stores its 4 KiB slice to the token's 8 rows.
// SRC 0: a constant; 1: the slice is loaded (streaming) from the token's own row of x; 2: loaded with cached
// loads from one of 1024 token rows (16 MiB: stays in the memory-side cache)
// ZIPF only names the instance: destination rows in sequential order, or those of a Zipf routing
// (SRC 0 with the rows of a uniform routing over 8, 32 or 64 experts is launched under its own name below)
template <int SRC, bool ZIPF>
__global__ __launch_bounds__(256) void scatter_rows_dispatch_shape(const u32x4 *x, u32x4 *recv, const int *rowmap) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, t = blockIdx.x;
  const int row = lane < K ? rowmap[t * K + lane] : -1;
  const int v0 = wave * 256 + lane;
  u32x4 v[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    v[i] = u32x4{1u, 2u, 3u, (unsigned)t};
    if (v0 + i * 64 < NV) {
      if (SRC == 1) v[i] = __builtin_nontemporal_load(x + (size_t)t * NV + v0 + i * 64);
      if (SRC == 2) v[i] = x[(size_t)(t & 1023) * NV + v0 + i * 64];
    }
  }
#pragma unroll
  for (int k = 0; k < K; ++k) {
    u32x4 *dst = recv + (size_t)__builtin_amdgcn_readlane(row, k) * NV;
#pragma unroll
    for (int i = 0; i < 4; ++i)
      if (v0 + i * 64 < NV) store_wt(dst + v0 + i * 64, v[i]);
  }
}
// the same stores (constant data) when the tokens' 8 rows go to 8 distinct of E expert regions drawn uniformly:
// E sequential streams are being written at any time
template <int E>
__global__ __launch_bounds__(256) void scatter_rows_into_E_expert_regions(u32x4 *recv, const int *rowmap) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, t = blockIdx.x;
  const int row = lane < K ? rowmap[t * K + lane] : -1;
  const int v0 = wave * 256 + lane;
  const u32x4 v = {1u, 2u, 3u, (unsigned)t};
#pragma unroll
  for (int k = 0; k < K; ++k) {
    u32x4 *dst = recv + (size_t)__builtin_amdgcn_readlane(row, k) * NV;
#pragma unroll
    for (int i = 0; i < 4; ++i)
      if (v0 + i * 64 < NV) store_wt(dst + v0 + i * 64, v);
  }
}
// ---- reads
template <bool STREAMING, bool ALTERNATING>
__global__ __launch_bounds__(256) void read_stream(const u32x4 *p, u32x4 *sink) {
  const long long j = (long long)blockIdx.x * 256 + threadIdx.x;
  keep(STREAMING ? __builtin_nontemporal_load(p + j) : p[j], sink);
}
// the combine's shape: one wave per (token, 1 KiB slice), 8 streaming loads per lane from the token's 8 rows.
// OUT 0: nothing stored; 1: the sum goes to the token's row of `out` (streaming store); 2: to one of 16 rows of
// `out` (stays in the L2)
DEV float lo(unsigned d) { return __uint_as_float(d << 16); }
DEV float hi(unsigned d) { return __uint_as_float(d & 0xFFFF0000u); }
template <int OUT>
__global__ __launch_bounds__(256) void gather_rows_combine_shape(const u32x4 *y, const int *rowmap, u32x4 *out, u32x4 *sink) {
  const int lane = threadIdx.x & 63;
  const long long item = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
  const int t = (int)(item / 14), part = (int)(item % 14);
  const int row = lane < K ? rowmap[t * K + lane] : 0;
  u32x4 ld[K];
#pragma unroll
  for (int k = 0; k < K; ++k) ld[k] = __builtin_nontemporal_load(y + (size_t)__builtin_amdgcn_readlane(row, k) * NV + part * 64 + lane);
  float acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
  for (int k = 0; k < K; ++k)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      acc[2 * j] = __builtin_fmaf(0.125f, lo(ld[k][j]), acc[2 * j]);
      acc[2 * j + 1] = __builtin_fmaf(0.125f, hi(ld[k][j]), acc[2 * j + 1]);
    }
  const u32x4 o = {__float_as_uint(acc[0]) >> 16 | (__float_as_uint(acc[1]) & 0xFFFF0000u),
                   __float_as_uint(acc[2]) >> 16 | (__float_as_uint(acc[3]) & 0xFFFF0000u),
                   __float_as_uint(acc[4]) >> 16 | (__float_as_uint(acc[5]) & 0xFFFF0000u),
                   __float_as_uint(acc[6]) >> 16 | (__float_as_uint(acc[7]) & 0xFFFF0000u)};
  if (OUT == 0) keep(o, sink);
  else __builtin_nontemporal_store(o, out + (size_t)(OUT == 2 ? (t & 15) : t) * NV + part * 64 + lane);
}

int main(int argc, char **argv) {
  const int reps = argc > 1 ? atoi(argv[1]) : 10;
  u32x4 *x, *recv, *y, *out, *sink;
  int *seq, *zipf;
  CK(hipMalloc(&x, (size_t)T * NV * 16));
  CK(hipMalloc(&recv, (size_t)kVecs * 16));
  CK(hipMalloc(&y, (size_t)kVecs * 16));
  CK(hipMalloc(&out, (size_t)T * NV * 16));
  CK(hipMalloc(&sink, 256));
  CK(hipMalloc(&seq, kRows * 4));
  CK(hipMalloc(&zipf, kRows * 4));
  CK(hipMemset(x, 1, (size_t)T * NV * 16));
  CK(hipMemset(recv, 0, (size_t)kVecs * 16));
  CK(hipMemset(y, 1, (size_t)kVecs * 16));
  // destination rows: sequential, and a counting sort of a Zipf(s = 1) routing over 256 experts, 8 distinct per token
  std::vector<int> rm(kRows);
  std::iota(rm.begin(), rm.end(), 0);
  CK(hipMemcpy(seq, rm.data(), kRows * 4, hipMemcpyHostToDevice));
  {
    const int E = 256;
    std::mt19937 g(7);
    std::vector<double> p(E);
    for (int e = 0; e < E; ++e) p[e] = 1.0 / (e + 1);
    std::vector<int> idx(kRows), cnt(E, 0), off(E + 1, 0), fill(E, 0);
    for (int t = 0; t < T; ++t) {
      std::vector<double> q = p;
      for (int k = 0; k < K; ++k) {
        std::discrete_distribution<int> d(q.begin(), q.end());
        const int e = d(g);
        q[e] = 0.0;
        idx[t * K + k] = e;
        cnt[e]++;
      }
    }
    for (int e = 0; e < E; ++e) off[e + 1] = off[e] + cnt[e];
    for (long long i = 0; i < kRows; ++i) rm[i] = off[idx[i]] + fill[idx[i]]++;
  }
  CK(hipMemcpy(zipf, rm.data(), kRows * 4, hipMemcpyHostToDevice));
  // ... and of uniform routings (8 distinct experts per token) over 8, 32, 64 and 256 experts
  int *uni[4];
  const int uniE[4] = {8, 32, 64, 256};
  for (int u = 0; u < 4; ++u) {
    const int E = uniE[u];
    std::mt19937 g(11 + u);
    std::vector<int> idx(kRows), cnt(E, 0), off(E + 1, 0), fill(E, 0), perm(E);
    for (int t = 0; t < T; ++t) {
      std::iota(perm.begin(), perm.end(), 0);
      for (int k = 0; k < K; ++k) {  // partial Fisher-Yates
        std::swap(perm[k], perm[k + (int)(g() % (unsigned)(E - k))]);
        idx[t * K + k] = perm[k];
        cnt[perm[k]]++;
      }
    }
    for (int e = 0; e < E; ++e) off[e + 1] = off[e] + cnt[e];
    for (long long i = 0; i < kRows; ++i) rm[i] = off[idx[i]] + fill[idx[i]]++;
    CK(hipMalloc(&uni[u], kRows * 4));
    CK(hipMemcpy(uni[u], rm.data(), kRows * 4, hipMemcpyHostToDevice));
  }

  auto run = [&](auto launch) {
    for (int i = 0; i < 3 + reps; ++i) launch();
    CK(hipDeviceSynchronize());
    CK(hipGetLastError());
  };
  const dim3 blk(256);
  run([&] { hipLaunchKernelGGL(write_stream_in_launch_order<false>, dim3((unsigned)kBlocks), blk, 0, 0, recv); });
  run([&] { hipLaunchKernelGGL(write_stream_with_jittered_timing, dim3((unsigned)kBlocks), blk, 0, 0, recv); });
  run([&] { hipLaunchKernelGGL(write_interleaved_sequential_streams<8>, dim3((unsigned)kBlocks), blk, 0, 0, recv); });
  run([&] { hipLaunchKernelGGL(write_interleaved_sequential_streams<64>, dim3((unsigned)kBlocks), blk, 0, 0, recv); });
  run([&] { hipLaunchKernelGGL(write_interleaved_sequential_streams<256>, dim3((unsigned)kBlocks), blk, 0, 0, recv); });
  run([&] { hipLaunchKernelGGL(write_stream_in_scattered_chunks<4>, dim3((unsigned)kBlocks), blk, 0, 0, recv); });
  run([&] { hipLaunchKernelGGL(write_stream_in_scattered_chunks<16>, dim3((unsigned)kBlocks), blk, 0, 0, recv); });
  run([&] { hipLaunchKernelGGL(write_stream_in_scattered_chunks<64>, dim3((unsigned)kBlocks), blk, 0, 0, recv); });
  run([&] { hipLaunchKernelGGL(write_stream_in_scattered_chunks<256>, dim3((unsigned)kBlocks), blk, 0, 0, recv); });
  run([&] { hipLaunchKernelGGL(write_stream_in_scattered_chunks<1024>, dim3((unsigned)kBlocks), blk, 0, 0, recv); });
  run([&] { hipLaunchKernelGGL(write_stream_in_scattered_chunks<16384>, dim3((unsigned)kBlocks), blk, 0, 0, recv); });
  run([&] { hipLaunchKernelGGL(write_rows_in_order_one_row_per_workgroup, dim3((unsigned)kRows), dim3(896), 0, 0, recv, seq); });
  run([&] { hipLaunchKernelGGL((scatter_rows_dispatch_shape<0, false>), dim3(T), blk, 0, 0, x, recv, seq); });
  run([&] { hipLaunchKernelGGL((scatter_rows_dispatch_shape<0, true>), dim3(T), blk, 0, 0, x, recv, zipf); });
  run([&] { hipLaunchKernelGGL(scatter_rows_into_E_expert_regions<8>, dim3(T), blk, 0, 0, recv, uni[0]); });
  run([&] { hipLaunchKernelGGL(scatter_rows_into_E_expert_regions<32>, dim3(T), blk, 0, 0, recv, uni[1]); });
  run([&] { hipLaunchKernelGGL(scatter_rows_into_E_expert_regions<64>, dim3(T), blk, 0, 0, recv, uni[2]); });
  run([&] { hipLaunchKernelGGL(scatter_rows_into_E_expert_regions<256>, dim3(T), blk, 0, 0, recv, uni[3]); });
  run([&] { hipLaunchKernelGGL((scatter_rows_dispatch_shape<1, true>), dim3(T), blk, 0, 0, x, recv, zipf); });
  run([&] { hipLaunchKernelGGL((scatter_rows_dispatch_shape<2, true>), dim3(T), blk, 0, 0, x, recv, zipf); });
  run([&] { hipLaunchKernelGGL((read_stream<true, false>), dim3((unsigned)kBlocks), blk, 0, 0, y, sink); });
  run([&] { hipLaunchKernelGGL(gather_rows_combine_shape<0>, dim3(T * 14 / 4), blk, 0, 0, y, zipf, out, sink); });
  run([&] { hipLaunchKernelGGL(gather_rows_combine_shape<1>, dim3(T * 14 / 4), blk, 0, 0, y, zipf, out, sink); });
  run([&] { hipLaunchKernelGGL(gather_rows_combine_shape<2>, dim3(T * 14 / 4), blk, 0, 0, y, zipf, out, sink); });
  // a write stream into one buffer alternating with a read stream of ANOTHER buffer: streaming loads, then cached loads
  run([&] {
    hipLaunchKernelGGL(write_stream_in_launch_order<true>, dim3((unsigned)kBlocks), blk, 0, 0, recv);
    hipLaunchKernelGGL((read_stream<true, true>), dim3((unsigned)kBlocks), blk, 0, 0, y, sink);
  });
  run([&] {
    hipLaunchKernelGGL(write_stream_in_launch_order<true>, dim3((unsigned)kBlocks), blk, 0, 0, recv);
    hipLaunchKernelGGL((read_stream<false, true>), dim3((unsigned)kBlocks), blk, 0, 0, y, sink);
  });
  printf("mem_patterns: done (%d timed launches per kernel; read the averages from the profiler)\n", reps);
  return 0;
}
