// Combine (weighted sum over the top-k expert outputs in token order) and the kernels of the deduplicating
// high-throughput mode: dedup, per-expert index list, partial reduce per group.
#include "ep_device.h"

namespace ep {

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

// The slices of one wave, one after the other: K loads in flight, the chain in ascending k, the packed
// result kept in registers; the stores of all slices leave together at the end, so that a wave's writes
// do not trickle into its reads.  STREAM: non-temporal loads (rows that no cache is expected to hold).
template <int VPL, int KT, bool STREAM>
EP_DEV void combine_slices(const u32x4 *y, u32x4 *out, const int (&rows)[KT], const float (&ws)[KT], int safe, int nvec,
                           int v0) {
  u32x4 res[VPL];
#pragma unroll
  for (int i = 0; i < VPL; ++i)
    if (v0 + i * 64 < nvec) {
      u32x4 ld[KT];
#pragma unroll
      for (int k = 0; k < KT; ++k) {
        const u32x4 *p = y + (size_t)(rows[k] >= 0 ? rows[k] : safe) * nvec + v0 + i * 64;
        ld[k] = STREAM ? __builtin_nontemporal_load(p) : *p;
      }
      float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int k = 0; k < KT; ++k)
        if (rows[k] >= 0) fma8(acc, ws[k], ld[k]);
      res[i] = u32x4{pack_bf16_rne(acc[0], acc[1]), pack_bf16_rne(acc[2], acc[3]), pack_bf16_rne(acc[4], acc[5]),
                     pack_bf16_rne(acc[6], acc[7])};
    }
#pragma unroll
  for (int i = 0; i < VPL; ++i)
    if (v0 + i * 64 < nvec) __builtin_nontemporal_store(res[i], out + v0 + i * 64);
}

template <int VPL, int KT>
__global__ __launch_bounds__(256) void combine_kernel(CombineArgs a) {
  const int wave = threadIdx.x >> 6, lane = lane_id();
  const long long item = (long long)blockIdx.x * 4 + wave;
  const int t_launch = (int)(item / a.parts), part = (int)(item % a.parts);
  if (t_launch >= a.T) return;
  // With fresh rows the grid starts at the end of the token range where they are (the last tokens,
  // or the first ones when the kernel that wrote them went backwards) and takes the newest first:
  // the rows written last are read before the rest of the traffic pushes them out of the
  // memory-side cache.
  const int n_fresh = a.T - a.fresh_from;
  const int t = (n_fresh > 0 && !a.fresh_head) ? a.T - 1 - t_launch : t_launch;
  const bool fresh = a.fresh_head ? t < n_fresh : t >= a.fresh_from;
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
    // (wave-uniform; two instances so that each keeps its own kind of load)
    if (fresh) {
      combine_slices<VPL, KT, false>(y, out, rows, ws, safe, nvec, v0);
      // (keeps the optimiser from folding the two instances into one, which drops the streaming hint of the other)
      asm volatile("" ::: "memory");
    } else {
      combine_slices<VPL, KT, true>(y, out, rows, ws, safe, nvec, v0);
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

// Column slices (64 lanes x 16 bytes) per wave.  One slice per wave - fewest registers, most waves in
// flight - is the general choice.  One WAVE PER TOKEN (all slices of the row, its stores together at the
// end) is faster by 3-5 us per 450 MB for rows of 9 to 15 slices (hidden 4608..7680) when the rows to read
// exceed the memory-side cache (256 MB) by half or more; it is slower for rows whose size is a power of two
// (hidden 4096, 8192: every wave is then at the same offset of a row that starts a multiple of that size
// away, i.e. on the same memory channels at the same time), and mixed below that amount of rows (few tokens:
// too few waves; a sparse table such as the second level of the hierarchical reduce: slower).  Measured for
// hidden 4096..8192, 1024..8192 tokens, Zipf, softmax and uniform routing.
static int tuned_combine_vpl(int forced, const CombineArgs &a) {
  static const int c[] = {1, 2, 4, 7, 9, 10, 11, 12, 13, 14, 15};
  for (int v : c)
    if (v == forced) return v;
  const int slices = (a.H / 8 + 63) / 64;
  const long long rows = (long long)a.T * a.K < a.y_rows ? (long long)a.T * a.K : a.y_rows;
  if (slices >= 9 && slices <= 15 && rows * a.H * 2 >= 384000000ll) return slices;
  return 1;
}

template <int VPL>
static void launch_combine_t(CombineArgs a, hipStream_t st, const LaunchTiming *tm) {
  const int nvec = a.H / 8;
  a.parts = (nvec + VPL * 64 - 1) / (VPL * 64);
  const long long items = (long long)a.T * a.parts;
  const unsigned grid = (unsigned)((items + 3) / 4);
  void *ev0 = tm ? tm->start : nullptr, *ev1 = tm ? tm->stop : nullptr;
  switch (a.K) {
    case 1: launch_kernel(combine_kernel<VPL, 1>, dim3(grid), dim3(256), 0, st, ev0, ev1, a); break;
    case 2: launch_kernel(combine_kernel<VPL, 2>, dim3(grid), dim3(256), 0, st, ev0, ev1, a); break;
    case 4: launch_kernel(combine_kernel<VPL, 4>, dim3(grid), dim3(256), 0, st, ev0, ev1, a); break;
    case 6: launch_kernel(combine_kernel<VPL, 6>, dim3(grid), dim3(256), 0, st, ev0, ev1, a); break;
    case 8: launch_kernel(combine_kernel<VPL, 8>, dim3(grid), dim3(256), 0, st, ev0, ev1, a); break;
    default: launch_kernel(combine_kernel<VPL, 0>, dim3(grid), dim3(256), 0, st, ev0, ev1, a); break;
  }
}

int launch_combine(const CombineArgs &a, const Tunables &tune, void *stream, const LaunchTiming *timing) {
  hipStream_t st = (hipStream_t)stream;
  if (a.T <= 0) return 0;
  if ((a.H / 8 + 63) / 64 > 65535) return (int)hipErrorInvalidValue;
  switch (tuned_combine_vpl(tune.combine_vpl, a)) {
    case 2: launch_combine_t<2>(a, st, timing); break;
    case 4: launch_combine_t<4>(a, st, timing); break;
    case 7: launch_combine_t<7>(a, st, timing); break;
    case 9: launch_combine_t<9>(a, st, timing); break;
    case 10: launch_combine_t<10>(a, st, timing); break;
    case 11: launch_combine_t<11>(a, st, timing); break;
    case 12: launch_combine_t<12>(a, st, timing); break;
    case 13: launch_combine_t<13>(a, st, timing); break;
    case 14: launch_combine_t<14>(a, st, timing); break;
    case 15: launch_combine_t<15>(a, st, timing); break;
    default: launch_combine_t<1>(a, st, timing); break;
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
    // every group's chain first, the packed sums kept in registers; then the stores, together
    u32x4 res[KT];
#pragma unroll
    for (int j = 0; j < KT; ++j) {
      if (!((leaders >> j) & 1)) continue;
      float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int k = 0; k < KT; ++k)
        if (rows[k] >= 0 && fks[k] == j) fma8(acc, ws[k], ld[k]);
      res[j] = u32x4{pack_bf16_rne(acc[0], acc[1]), pack_bf16_rne(acc[2], acc[3]), pack_bf16_rne(acc[4], acc[5]),
                     pack_bf16_rne(acc[6], acc[7])};
    }
#pragma unroll
    for (int j = 0; j < KT; ++j) {
      if (!((leaders >> j) & 1)) continue;
      const int pr = __builtin_amdgcn_readlane(prow, j);
      store_payload((u32x4 *)a.partial + (size_t)pr * nvec + vi, res[j]);
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
    case 1: hipLaunchKernelGGL(combine_partial_kernel<1>, dim3(grid), dim3(256), 0, st, a); break;
    case 2: hipLaunchKernelGGL(combine_partial_kernel<2>, dim3(grid), dim3(256), 0, st, a); break;
    case 4: hipLaunchKernelGGL(combine_partial_kernel<4>, dim3(grid), dim3(256), 0, st, a); break;
    case 6: hipLaunchKernelGGL(combine_partial_kernel<6>, dim3(grid), dim3(256), 0, st, a); break;
    case 8: hipLaunchKernelGGL(combine_partial_kernel<8>, dim3(grid), dim3(256), 0, st, a); break;
    default: hipLaunchKernelGGL(combine_partial_kernel<0>, dim3(grid), dim3(256), 0, st, a); break;
  }
  return (int)hipGetLastError();
}

}  // namespace ep
