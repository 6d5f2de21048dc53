// Layout (Section 2.1: sizes and destinations are recomputed from the router's output every step): counts,
// exclusive scans and slot indices as an integer counting sort built from LDS bit masks and popcounts.
#include "ep_device.h"

#include <mutex>

namespace ep {

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

// ------------------------------------------------- small routing tables: one launch
// A dozen flat tiles (768 tokens over all sources - a low-latency decode step) fit one workgroup:
// wave f owns tile f, the bit masks of all tiles stay in LDS, one thread per expert walks the tiles
// for the prefixes, and every wave finishes its own entries.  Nothing goes through memory between
// the steps, which for such sizes is most of what the two kernels above spend (their floor is the
// chain of round trips between them, about 12 us whatever the size).
constexpr int kSmallTiles = 16;

__global__ __launch_bounds__(1024) void layout_small_kernel(LayoutArgs a) {
  extern __shared__ unsigned long long q_lds[];
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int E = a.E, K = a.K, F = a.S * a.ntiles;
  unsigned long long *mask = q_lds;                                         // [F][E]
  unsigned short *pre = (unsigned short *)(q_lds + (size_t)kSmallTiles * E);  // [F][E] entries of e in earlier tiles
  int *s_off = (int *)(pre + (size_t)kSmallTiles * E);                      // [E + 1]
  int *s_tot = s_off + E + 1;                                               // [E]
  for (int i = tid; i < F * E; i += blockDim.x) mask[i] = 0ull;
  __syncthreads();

  const int f = wave, s = f < F ? f / a.ntiles : 0, tile = f < F ? f - s * a.ntiles : 0;
  const int t = tile * kLayoutTile + lane;
  const bool active = f < F && t < a.T;
  const size_t ebase = ((size_t)s * a.T + (active ? t : 0)) * K;
  const unsigned long long below = (1ull << lane) - 1ull;
  int ev[8], rk[8];
#pragma unroll
  for (int k = 0; k < 8; ++k) ev[k] = (active && k < K) ? a.idx[ebase + k] : -1;
  if (f < F) {  // (wave-uniform)
    unsigned long long *m = mask + (size_t)f * E;
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      const int e = ev[k];
      bool pend = e >= 0 && e < E;
      if (!pend && e != -1) dev_set_error(a.error, EP_EBOUNDS);
      // the two most common experts of the wave are written by one lane each (see the count kernel)
#pragma unroll
      for (int round = 0; round < 2; ++round) {
        const unsigned long long pm = __ballot(pend);
        if (pm == 0) break;
        const int leader = __builtin_ctzll(pm);
        const int e0 = __builtin_amdgcn_readlane(e, leader);
        const unsigned long long same = __ballot(pend && e == e0);
        if (lane == leader) atomicOr(&m[e0], same);
        pend = pend && e != e0;
      }
      if (pend) atomicOr(&m[e], 1ull << lane);
    }
  }
  __syncthreads();
  if (f < F) {
    const unsigned long long *m = mask + (size_t)f * E;
#pragma unroll
    for (int k = 0; k < 8; ++k) rk[k] = (ev[k] >= 0 && ev[k] < E) ? __popcll(m[ev[k]] & below) : 0;
  }
  // exclusive prefix over the flat tiles, one thread per expert; counts per source on the way
  for (int e = tid; e < E; e += blockDim.x) {
    int run = 0, src_first = 0;
    for (int g = 0; g < F; ++g) {
      if (g > 0 && g % a.ntiles == 0) {
        a.count[(size_t)(g / a.ntiles - 1) * E + e] = run - src_first;
        src_first = run;
      }
      pre[(size_t)g * E + e] = (unsigned short)run;
      run += __popcll(mask[(size_t)g * E + e]);
    }
    a.count[(size_t)(a.S - 1) * E + e] = run - src_first;
    s_tot[e] = run;
    a.expert_total[e] = run;
  }
  __syncthreads();
  if (wave == 0) {  // exclusive scan over experts: 64 lanes x contiguous runs
    const int per = (E + 63) / 64;
    const int lo = min(E, lane * per), hi = min(E, lo + per);
    int sum = 0;
    for (int i = lo; i < hi; ++i) sum += s_tot[i];
    const int incl = wave_inclusive_scan(sum, lane);
    int run = incl - sum;
    for (int i = lo; i < hi; ++i) {
      s_off[i] = run;
      a.expert_offset[i] = run;
      run += s_tot[i];
    }
    if (lane == 63) {
      s_off[E] = incl;
      a.expert_offset[E] = incl;
    }
  }
  __syncthreads();
  if (active) {
    const unsigned short *bp = pre + (size_t)f * E, *fp = pre + (size_t)s * a.ntiles * E;
#pragma unroll
    for (int k = 0; k < 8; ++k)
      if (k < K) {
        const int e = ev[k];
        if (e >= 0 && e < E) {
          const int before = bp[e];
          a.slot[ebase + k] = before - (int)fp[e] + rk[k];
          a.dst_row[ebase + k] = s_off[e] + before + rk[k];
        } else {
          a.slot[ebase + k] = -1;
          a.dst_row[ebase + k] = -1;
        }
      }
  }
  for (int i = tid; i < a.S * E; i += blockDim.x) {
    const int ss = i / E, e = i - ss * E;
    a.base[i] = s_off[e] + (int)pre[(size_t)ss * a.ntiles * E + e];
  }
  for (int r = tid; r <= a.R; r += blockDim.x) {
    const int o = s_off[r * a.E_loc];  // r == R reads the end sentinel s_off[E]
    a.rank_offset[r] = o;
    if (r < a.R) a.rank_total[r] = s_off[(r + 1) * a.E_loc] - o;
  }
}

// LDS bytes of the one-launch form, or 0 when the shape does not fit it.
static size_t small_layout_lds(const LayoutArgs &a) {
  const long long F = (long long)a.S * a.ntiles;
  // measured on MI355X (E = 256, top-8): 4.3 us against 11.7 for one tile, 8.5 / 15.7 for 4, 11.3 / 15.4 for 8,
  // 13.7 / 16.0 for 12; with all 16 waves busy the LDS atomics of the tiles slow each other down and
  // nothing is gained (16.5 / 15.8)
  if (a.T <= 0 || a.K > 8 || F <= 0 || F > 12) return 0;
  const size_t bytes = (size_t)kSmallTiles * a.E * (8 + 2) + (size_t)(2 * a.E + 1) * 4;
  return bytes <= 64 * 1024 ? bytes : 0;
}

// ------------------------------------------------- scratch that nobody allocates
// For callers that cannot allocate (ep_layout_static): the tile histograms, the tile prefixes, the ticket
// and an error sink live in a file-scope device array.  Every GPU holds its own copy at its own address
// until the process ends, so the address is looked up once per device, with that device current, and
// host code only ever uses the looked-up pointer (the array's name is a host-side stand-in, not a
// device address).
struct StaticLayoutScratch {
  unsigned ticket[64];  // one word used; a 256-byte line of its own
  int error_sink[64];   // where device-side errors go when the caller passes no status word
  int32_t hist[kStaticLayoutEntries];
  int32_t base[kStaticLayoutEntries];
};
static __device__ __align__(256) unsigned char scratch[sizeof(StaticLayoutScratch)];

constexpr int kMaxDevices = 64;
static std::mutex g_scratch_mu;
static void *g_scratch_ptr[kMaxDevices] = {};

int static_layout_scratch(LayoutArgs *a) {
  int dev = -1;
  hipError_t err = hipGetDevice(&dev);
  if (err != hipSuccess) return (int)err;
  if (dev < 0 || dev >= kMaxDevices) return (int)hipErrorInvalidDevice;
  void *p = nullptr;
  {
    std::lock_guard<std::mutex> g(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
      err = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
      if (err != hipSuccess) return (int)err;
      if (!p) return (int)hipErrorInvalidSymbol;
      g_scratch_ptr[dev] = p;
    }
    p = g_scratch_ptr[dev];
  }
  if (a) {
    StaticLayoutScratch *sc = (StaticLayoutScratch *)p;
    a->ticket = sc->ticket;
    a->tile_hist = sc->hist;
    a->tile_base = sc->base;
    if (!a->error) a->error = sc->error_sink;
  }
  return 0;
}

int launch_layout(const LayoutArgs &a, const Tunables &tune, void *stream, const LaunchTiming *timing) {
  hipStream_t st = (hipStream_t)stream;
  if (const size_t lds = tune.layout_small ? small_layout_lds(a) : 0) {
    launch_kernel(layout_small_kernel, dim3(1), dim3(1024), lds, st, timing ? timing->start : nullptr,
                  timing ? timing->stop : nullptr, a);
    return (int)hipGetLastError();
  }
  // Workgroups are 1024 threads so that the last one has many hands for the scan, but only a few
  // wavefronts of each own a tile: the LDS atomics of one tile then compete with few others.
  const int kBlock = 1024;
  int W = tune.layout_tpb;
  if (W != 1 && W != 2 && W != 4 && W != 8 && W != 16) W = 4;
  while (W > 1 && (size_t)W * a.E * sizeof(unsigned long long) > 65536 - 12288) W >>= 1;
  LayoutArgs b = a;
  b.tiles_per_block = W;
  b.scan_split = 1;  // threads per expert in the scan: a power of two, at most 16, all in one workgroup
  while (b.scan_split < 16 && b.scan_split * 2 * a.E <= kBlock) b.scan_split *= 2;
  const int nblk = (a.ntiles + W - 1) / W;
  const int grid1 = a.S * (nblk > 0 ? nblk : 1);
  const size_t lds = (size_t)W * a.E * sizeof(unsigned long long);
  const long long n = (long long)a.S * a.T * a.K;  // entries the second kernel finishes
  launch_kernel(layout_count_kernel, dim3(grid1), dim3(kBlock), lds, st, timing ? timing->start : nullptr,
                timing && n <= 0 ? timing->stop : nullptr, b);
  hipError_t err = hipGetLastError();
  if (err != hipSuccess) return (int)err;
  if (n > 0) {
    launch_kernel(layout_finish_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, nullptr,
                  timing ? timing->stop : nullptr, a);
    err = hipGetLastError();
  }
  return (int)err;
}

}  // namespace ep
