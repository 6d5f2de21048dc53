// Internal declarations shared by the host side (handle, proxy threads) and the
// HIP kernels of libep.so.  Not part of the C ABI.
#pragma once

#include <stdint.h>

#include "../../include/ep.h"
#include "../../include/ep_diag.h"

namespace ep {

// One head index per channel sits alone in a 64-byte line of pinned host memory,
// so proxy threads that own different channels never share a line.
constexpr int kHeadStride = 8;  // in uint64 units
constexpr int kChunkRows = 32;  // rows per Write in EP_CMD_CHUNK32 (Section 3.3: "typically 32 tokens")
constexpr int kMaxChannels = 64;
constexpr int kMaxThreads = 16;
constexpr int kLayoutTile = 64;        // tokens per layout tile = one wavefront
constexpr int kMaxExperts = 1024;

// TransferCmd fields (layout documented in include/ep.h).
inline
#ifdef __HIPCC__
    __host__ __device__
#endif
    uint32_t
    cmd_w0(uint32_t op, uint32_t src, uint32_t dst_rank, uint32_t local_expert) {
  return (op << 28) | (src << 20) | (dst_rank << 12) | local_expert;
}

// Device-visible state of the FIFO channels (Section 3.1): slots and head live
// in pinned host memory, tail and the cached head in device memory.
struct RingDev {
  void *slots;                       // uint32x4 [channels * entries], pinned host
  const unsigned long long *head;    // [channels * kHeadStride], pinned host, written by the proxy
  unsigned long long *tail;          // [channels], device: next Idx to hand out
  unsigned long long *cached_head;   // [channels], device: last head value fetched over PCIe
  int *error;                        // pinned host sticky error word
  unsigned long long *stalls;        // device: times a push found the channel full
  unsigned *refresh_lock;            // [channels], device: held by the one lane re-reading a channel's head
  unsigned entries, log2_entries, channels;
  unsigned long long timeout_ticks;  // wall_clock64 ticks (100 MHz)
};

struct LayoutArgs {
  const int32_t *idx;  // [S,T,K]
  int32_t S, T, K, E, R, E_loc, ntiles;
  int32_t scan_split;  // threads per expert in the tile scan (set by the launcher)
  int32_t tiles_per_block;  // wavefronts of a layout workgroup that own a tile (set by the launcher)
  int32_t *tile_hist;  // scratch [S*ntiles][E]: histogram of every 64-token tile
  int32_t *tile_base;  // scratch [S*ntiles + 1][E]: exclusive scan over flat tiles, last row = totals
  unsigned *ticket;    // scratch: workgroups finished (self-resetting)
  int32_t *count, *expert_total, *rank_total, *base, *expert_offset, *rank_offset;
  int32_t *slot, *dst_row;
  int *error;
};

struct DispatchArgs {
  const void *x;           // bf16 [T,H]
  const int32_t *idx;      // [T,K]
  const int32_t *dst_row;  // [T,K]
  const int32_t *count;    // [E] of this source
  const int32_t *base;     // [E] of this source
  void *recv;              // bf16 [rows,H] or u8 [rows,H]
  float *recv_scale;       // [rows, H/128] (FP8)
  long long recv_rows;
  int32_t T, K, H, E, E_loc, src, filter;
  int32_t cmd_mode;        // ep_cmd_mode incl. flag bits
  uint32_t row_bytes;      // bytes of one token in a message
  int32_t parts;           // wavefronts per token
  int32_t tokens_per_block;
  int32_t block_cmds;      // the workgroup's first wave pushes the commands of all its tokens
  int32_t reverse;         // workgroups take the tokens from the last one down (see ep_dispatch)
  int32_t cache_hinted;    // the caller promised (EP_FLAG_CACHE_HINTS) that the rows are consumed out of the caches
  int32_t msg_rows;        // FP8 only: 0 = codes and scales go to the two receive arrays; 1 = every row is one message
                           // (codes, scales, padding: row_bytes) at its destination row of `recv`; 2 = one message
                           // per token at row t of `recv` (the proxy forwards it to every destination)
  int32_t chunks_per_expert;
  int32_t *chunk_cnt;      // scratch [E * chunks_per_expert], zero between calls
  int32_t *expert_done;    // scratch [E], zero between calls
  unsigned *waves_done;    // scratch of the Drain epilogue [1 + workgroups / 64], zero between calls
  unsigned *ht_seq;        // scratch [S*R]: next sequence number of each communication channel
  int32_t R;
  RingDev ring;
};

struct CombineArgs {
  const void *y;           // bf16 [rows,H]
  const float *w;          // [T,K]
  const int32_t *dst_row;  // [T,K]
  void *out;               // bf16 [T,H]
  long long y_rows;
  int32_t T, K, H, parts;
  int *error;
  // Tokens >= fresh_from had their rows written last, by the kernel that ran just before on this
  // stream (ep_combine knows this when it follows ep_dispatch into the same buffer): those rows
  // are read with cached loads and first, the rest with streaming loads.  fresh_from == T: none.
  // fresh_head: that kernel went through the tokens backwards, so the fresh ones are the FIRST
  // T - fresh_from tokens instead (and the grid keeps the ascending order).
  int32_t fresh_from;
  int32_t fresh_head;
};

struct DedupArgs {
  const int32_t *idx;  // [n_tokens, K]
  int32_t *group_idx, *first_k;
  long long n_tokens;
  int32_t K, E, E_loc, ranks_per_group;
  int *error;
};

struct GatherIndexArgs {
  const int32_t *dst_row, *dst_row_g, *first_k;  // [T,K]
  int32_t *index;                                // [rows]
  long long rows;
  int32_t T, K;
  int *error;
};

struct CombinePartialArgs {
  const void *y;       // bf16 [y_rows,H]
  const float *w;      // [T,K]
  const int32_t *dst_row, *first_k, *dst_row_g;  // [T,K]
  void *partial;       // bf16 [rows_g,H]
  long long y_rows, rows_g;
  int32_t T, K, H, parts;
  int *error;
};

// A batch of peer writes the proxy performs on behalf of the GPU (registered heaps).  Descriptors
// (offsets and lengths in 16-byte units) stay in pinned host memory; a workgroup fetches the 16 it
// serves with ONE coalesced read (a descriptor read per workgroup cost a PCIe round trip each and
// made the copy kernels 10x slower).
constexpr int kCopyBatchMax = 4096, kCopyGroup = 16;
struct CopyDesc {
  unsigned src16, dst16, len16;
};
struct CopyBatchArgs {
  const char *src_base;
  char *dst_base;
  const CopyDesc *descs;       // device address of the pinned array
  const CopyDesc *host_descs;  // the same array as the host sees it
  int n;
  unsigned max_len16;
};
// Large copies (chunks) are few per batch and want a workgroup per (copy, piece): their descriptors
// travel inside the kernel-argument block instead, up to this many per launch.
constexpr int kCopyArgMax = 256;
struct CopyArgBatch {
  const char *src_base;
  char *dst_base;
  CopyDesc d[kCopyArgMax];
};

// Ring-buffer channels of the high-throughput mode: one workgroup per slice, sending and receiving in turns.
struct HtRingArgs {
  const void *x;           // bf16 [T,H]
  const int32_t *idx;      // [T,K]
  const int32_t *dst_row;  // [T,K]
  void *ring_buf;          // [slices][R][W] slots of slot_bytes
  void *recv;              // bf16 [recv_rows,H], or E4M3 codes u8 [recv_rows,H]
  float *recv_scale;       // FP8: [recv_rows, H/128]
  long long recv_rows;
  int32_t T, K, H, E_loc, R, src, slices, slice_len, W, payload;
  unsigned slot_bytes;     // stride of a slot (header + 32 bf16 rows, whatever the payload)
  unsigned row_bytes;      // bytes of one row in a slot: 2H, or H codes + H/32 scale bytes padded to 16
  const int32_t *tail, *head;                       // pinned host [slices*R] of this source, written by the proxy
  unsigned *seq_fwd, *seq_rev, *cum_fwd, *cum_rev;  // device [slices*R] of this source
  unsigned *waves_done;
  RingDev fifo;
};

struct RecvWaitArgs {
  int *flags;        // pinned host [S*E]: 0 = not arrived, else posted count + 1 (written by the proxy)
  int32_t *out;      // device [E] or null
  int32_t E, E_loc, src, filter;
  int *error;
  unsigned long long timeout_ticks;
};

// Launch-shape overrides for sweeps and for tests that want every code path: read ONCE per handle, in
// ep_proxy_start, from EP_* environment variables (0 = the library's own choice).  No launch reads the
// environment.
struct Tunables {
  int dispatch_vpl = 0;      // EP_DISPATCH_VPL: 16-byte vectors per lane of a bf16 row
  int dispatch_fp8_vpl = 0;  // EP_DISPATCH_FP8_VPL: 16-channel groups per lane of an FP8 row
  int per_token_waves = 0;   // EP_PER_TOKEN_WAVES: data wavefronts per workgroup of a ring-on dispatch (0 = 12);
                             // in the plain form: wavefronts per workgroup of a per-token dispatch (0 = 16)
  int dispatch_pipeline = 0; // EP_DISPATCH_PIPELINE: 1 = ring-on dispatches run persistent workgroups with a command
                             // wave (measured: no faster in chunk mode, slower per token; see the kernel's comment)
  int combine_vpl = 0;       // EP_COMBINE_VPL: 16-byte column slices per lane
  int layout_small = 1;      // EP_LAYOUT_SMALL: 0 keeps small routing tables on the two-kernel form
  int layout_tpb = 4;        // EP_LAYOUT_TPB: tiles per workgroup of the count kernel
  int ht_threads = 1024;     // EP_HT_THREADS: threads per workgroup of the ring-buffer channels
  int combine_fresh_mb = 224;  // EP_COMBINE_FRESH_MB: see EP_FLAG_CACHE_HINTS
};

// Launchers implemented in the .hip files (layout, dispatch, combine, ht_ring, service).  All return a hipError_t as int.
// Optional kernel-exact timing of a launch (ep_profile): HIP events that receive the begin timestamp of the
// launch's first kernel and the end timestamp of its last one from the dispatch packets themselves, with no
// extra work on the stream.  Events are hipEvent_t, kept as plain pointers here.
struct LaunchTiming {
  void *start, *stop;
};
int launch_layout(const LayoutArgs &a, const Tunables &tune, void *stream, const LaunchTiming *timing = nullptr);
int launch_dispatch(const DispatchArgs &a, int payload, const Tunables &tune, void *stream,
                    const LaunchTiming *timing = nullptr);
int launch_combine(const CombineArgs &a, const Tunables &tune, void *stream, const LaunchTiming *timing = nullptr);
// ep_layout_static: points a's scratch (tile_hist, tile_base, ticket, and error when it is null) into the
// file-scope device array of layout.hip, looking its address up on the current device the first time.
// a == nullptr only does the look-up.  Holds (S * ntiles + 1) * E entries up to kStaticLayoutEntries.
constexpr long long kStaticLayoutEntries = 262144;
int static_layout_scratch(LayoutArgs *a);
int launch_recv_wait(const RecvWaitArgs &a, void *stream);
int launch_barrier(const RingDev &ring, void *stream);
int launch_fifo_stress(const RingDev &ring, int pushers, int per_pusher, unsigned long long *lat_sum,
                       unsigned long long *lat_max, void *stream);
int launch_ht_ring(const HtRingArgs &a, const Tunables &tune, void *stream);
int launch_copy_batch(const CopyBatchArgs &b, void *stream);
int launch_dedup(const DedupArgs &a, void *stream);
int launch_gather_index(const GatherIndexArgs &a, void *stream);
int launch_combine_partial(const CombinePartialArgs &a, void *stream);
int launch_fill_u32(uint32_t *p, uint32_t v, long long n, void *stream);
int launch_fp8_unpack(const void *msgs, long long rows, int H, unsigned row_bytes, void *q, float *scale, void *stream);
int launch_bw_probe(int kind, const void *src, void *dst, long long bytes, void *stream);
int launch_row_probe(int kind, const int32_t *rowmap, int k, long long items, int row_bytes, long long buf_rows,
                     void *buf, void *sink, void *stream);

}  // namespace ep
