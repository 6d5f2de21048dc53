/*
 * ep.h - C ABI of the MI355X expert-parallel dispatch/combine library (libep.so).
 *
 * One GPU runs its share of an expert-parallel (EP) group; the other EP ranks
 * are partitions of this GPU's HBM.  The calls follow the paper's statement of
 * the problem: tokens are dispatched to the ranks hosting their selected
 * experts and expert outputs are combined back in the original token order
 * (Section 2.1); transfers are initiated by the GPU as 16-byte commands pushed
 * into FIFO channels that a multithreaded CPU proxy drains (Section 3.1, 3.2);
 * the proxy enforces the receiver-side completion fence of the low-latency
 * mode with 32-bit immediate data and posts completion counters in pinned
 * host memory (Section 3.3, Section 4.1).
 *
 * Conventions
 *  - Every function returns 0 (EP_OK) or a negative ep_status; nothing is thrown.
 *  - Pointers named d_* are DEVICE pointers owned by the caller, 16-byte
 *    aligned, valid until the stream work that uses them has finished.
 *    All other pointers are HOST pointers.
 *  - `stream` is a hipStream_t passed as void* (NULL = the null stream).
 *    ep_layout / ep_dispatch / ep_combine only enqueue work on it and never
 *    synchronise the device.  Calls on one handle must be ordered on one
 *    stream (or otherwise serialised): they share the handle's scratch.
 *  - Argument errors found on the host return EP_EINVAL before anything is
 *    launched.  Errors found on the device (a destination row outside the
 *    receive buffer, an expert id outside [-1, E), a ring wait that timed out)
 *    skip the offending element, set a sticky error word and are reported by
 *    ep_wait / ep_stats as EP_EBOUNDS / EP_ETIMEOUT.
 *  - The library never falls back to the CPU: without a usable HIP device the
 *    compute entry points return EP_EHIP.
 *
 * Notation: R ranks, E experts (expert e lives on rank e / (E/R)), K = top-k,
 * T tokens of one source rank, H hidden size, S source ranks whose routing is
 * given.  bf16 data is raw 16-bit patterns.
 */
#ifndef EP_H_
#define EP_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct ep_handle ep_handle; /* opaque, owned by the library */

enum ep_status {
  EP_OK = 0,
  EP_EINVAL = -1,   /* bad argument or configuration                       */
  EP_ENOMEM = -2,   /* host or device allocation failed                    */
  EP_ESTATE = -3,   /* call not valid for this handle (e.g. host-only)     */
  EP_EHIP = -4,     /* a HIP runtime call failed / no device               */
  EP_ETIMEOUT = -5, /* a bounded wait (GPU ring push, ep_wait) expired     */
  EP_EBOUNDS = -6   /* an offset, row or expert id was out of range        */
};

/* Dispatch payload (Section 2.1: a token is ~7 KB in FP8 at hidden 7168). */
enum ep_payload {
  EP_BF16 = 0,     /* rows of H bf16                                               */
  EP_FP8_E4M3 = 1  /* rows of H OCP-E4M3 codes + one fp32 scale per 128 channels   */
};

/* How the dispatch kernel drives the control channel (Section 3.3: the
 * low-latency mode sends every token on its own; the high-throughput mode
 * moves chunks of typically 32 tokens). */
enum ep_cmd_mode {
  EP_CMD_PER_TOKEN = 0,       /* one Write command per (token, expert)                 */
  EP_CMD_CHUNK32 = 1,         /* one Write per run of <= 32 consecutive rows of an expert */
  EP_CMD_NONE = 2,            /* ring off: payload placement only                      */
  EP_CMD_CHUNK32_ORDERED = 3, /* high-throughput style (Section 3.3, "partial ordering"): per chunk an ordered
                                 Write and an ordered Atomic that advances the receiver's tail counter of the
                                 communication channel (source rank -> destination rank); both carry the
                                 channel's sequence number and go through the FIFO destination rank mod C; the
                                 receiver applies them strictly in sequence.  No per-expert count Atomics.
                                 Always ends with a Drain on every FIFO (EP_CMD_DRAIN is implied).          */
  EP_CMD_MODE_MASK = 0xFF,
  EP_CMD_ATOMICS_FIRST = 0x100, /* push every count Atomic before any Write (forces the fence path) */
  EP_CMD_DRAIN = 0x200,         /* last wave pushes Drain on every channel and blocks on Check-completion */
  EP_CMD_NO_PLACEMENT = 0x400   /* EP_CMD_PER_TOKEN with registered heaps (ep_register_heaps): the kernel places no
                                   row at its destination, it only pushes the commands; the proxy moves the rows.
                                   The low-latency mode as the paper runs it.  EP_BF16: nothing is stored at all,
                                   the source heap is d_x.  EP_FP8_E4M3: the kernel quantises every token once
                                   and stores it as ONE message (see ep_dispatch) at row t of the source heap. */
};

enum ep_flags {
  EP_FLAG_LOG_CMDS = 1,   /* proxy keeps every polled command (ep_cmd_log)          */
  EP_FLAG_LOG_EVENTS = 2, /* proxy keeps the receiver-side event trace (ep_event_log) */
  EP_FLAG_HOST_ONLY = 4,  /* no device: ring + proxy only, producer is ep_host_push  */
  EP_FLAG_SENDER_FENCE = 8, /* the alternative Section 3.3 weighs against the receiver-side fence: the SENDER half
                              holds a count Atomic back until the Writes it vouches for have completed, then
                              sends it; the receiver never has to buffer one.  Costs the sender a round trip. */
  EP_FLAG_CACHE_HINTS = 16 /* performance only, never the result; OFF unless asked for.  The caller promises that
                              every ep_combine of this handle reads the very buffer the preceding bf16 ep_dispatch
                              wrote (an identity expert, or experts that overwrite their rows in place right
                              before the combine), so that the rows of the tokens dispatched last are still in
                              the 256 MB memory-side cache: ep_combine then reads those rows first and with
                              cached loads (EP_COMBINE_FRESH_MB MiB worth at ep_proxy_start, default 224), and a
                              dispatch into the buffer of the previous dispatch hands the tokens to its
                              workgroups from the other end of the token range (and keeps the launch shape that
                              suits rows consumed out of that cache, whatever their volume).  Without the flag every
                              dispatch walks the tokens in ascending order and every combine reads all rows
                              with streaming loads, whatever ran before it. */
};

typedef struct ep_config {
  int32_t num_ranks;         /* R, 1..256                                              */
  int32_t num_experts;       /* E, multiple of R, <= 1024                              */
  int32_t top_k;             /* K, 1..64                                               */
  int32_t hidden;            /* H, multiple of 128, <= 65536                           */
  int32_t max_tokens;        /* capacity in tokens per source rank, < 2^19             */
  int32_t num_src;           /* S >= 1, <= 256                                         */
  int32_t self_rank;         /* this GPU's rank, informational                         */
  int32_t num_channels;      /* FIFO channels C, 1..64 (the paper runs 8)              */
  int32_t ring_entries;      /* slots per channel = the paper's kMaxInflight; power of two >= 2 */
  int32_t num_proxy_threads; /* 0..16 (the paper runs 4); channel c belongs to thread c mod N   */
  int32_t reorder_window;    /* test hook: receiver sees up to this many immediates out of order; 0 = in order, <= 16384 */
  int32_t spin_timeout_ms;   /* bound of every GPU-side and host-side wait; 0 = 5000   */
  uint64_t reorder_seed;
  int64_t heap_rows;         /* rows of the registered receive heap; 0 = S * max_tokens * K */
  int32_t flags;             /* ep_flags                                               */
  int32_t barrier_peers;     /* processes that take part in Barrier commands (0 or 1: only this one)   */
  char barrier_name[48];     /* name of the shared-memory barrier the peers of one node agree on; "" = private */
  int32_t max_outstanding;   /* pacing: messages a proxy thread may have in flight to one destination rank;
                                further ones wait at the sender (0 = unlimited)                              */
  int32_t pack_rows;         /* best-effort packing of per-token Writes: up to this many rows with consecutive
                                destination offsets, polled in one sweep, leave as one message (0, 1 = off; <= 16) */
  int32_t pack_hold_us;      /* ... and an open message may wait this long for more rows (0 = never beyond the
                                sweep that polled its first row; <= 1000)                                    */
  int32_t ht_slices;         /* ring-buffer channels: token slices per source (0 = ep_ht_dispatch unavailable), <= 4096 */
  int32_t ht_ring_slots;     /* ... chunk slots per channel ring (W); num_ranks * W <= 4096                           */
} ep_config;

typedef struct ep_stats_t {
  uint64_t cmds;             /* commands polled by all proxy threads                   */
  uint64_t writes, atomics, drains, barriers;
  uint64_t write_bytes;      /* sum of Write lengths                                   */
  uint64_t write_rows;       /* sum of rows carried by Writes                          */
  uint64_t atomics_applied;
  uint64_t atomics_deferred; /* atomics that had to wait in the control buffer         */
  uint64_t sender_held;      /* atomics the sender half held back (EP_FLAG_SENDER_FENCE) */
  uint64_t ordered_parked;   /* sequenced messages that arrived ahead of their turn    */
  uint64_t rejected;         /* commands that failed offset translation / bounds check */
  uint64_t write_msgs;       /* messages that carried the Writes (fewer than writes when rows were packed) */
  uint64_t paced;            /* messages that waited at the sender for the pacing limit  */
  uint64_t max_in_flight;    /* most messages any thread had in flight to one rank       */
  uint64_t copy_batches;     /* batched copy launches made by the proxy (registered heaps) */
  uint64_t copied_bytes;     /* bytes the proxy moved                                   */
  uint64_t gpu_ring_full;    /* times a GPU push saw "full" in its cached head and re-read the head over PCIe */
  uint64_t first_poll_ns;    /* CLOCK_MONOTONIC of the first command seen since ep_reset_stats */
  uint64_t last_apply_ns;    /* ... and of the last atomic applied                     */
  uint64_t per_thread_cmds[16];
  int32_t device_error;      /* sticky ep_status set by a kernel, 0 if none            */
  int32_t proxy_error;       /* sticky ep_status set by the proxy, 0 if none           */
} ep_stats_t;

/* ep_proxy_start - create a handle: validates *cfg, allocates the pinned-host
 * command rings, head indices and completion counters (Section 3.1: head on the
 * CPU, tail and a cached copy of the head on the GPU), device scratch, and
 * starts num_proxy_threads proxy threads that share no state (Section 3.2).
 * *out receives the handle.  EP_EINVAL / EP_ENOMEM / EP_EHIP on failure. */
int ep_proxy_start(const ep_config *cfg, ep_handle **out);

/* ep_proxy_stop - end of the proxy's life (Section 3.2: one proxy per GPU, created
 * with the communicator and torn down with it): waits for enqueued device work of
 * the handle, stops and joins the proxy threads, frees everything.  The handle is
 * dead afterwards. */
int ep_proxy_stop(ep_handle *h);

/* ep_layout - routing is only known at run time, so sizes and destinations of the
 * transfers are worked out anew for every step (Section 2.1, paragraph on irregular
 * communication): from the router's top-k expert ids compute
 *   count[s][e]      tokens of source s that chose expert e
 *   expert_total[e], rank_total[r]
 *   base[s][e]       first receive row of (s, e): rows are expert-major,
 *                    source-minor; expert_offset[E+1], rank_offset[R+1] are
 *                    the exclusive scans with end sentinels
 *   slot[s,t,k]      number of earlier tokens of s that chose the same expert
 *   dst_row[s,t,k]   base + slot
 * d_topk_idx is int32 [S,T,K], -1 = masked entry (slot = dst_row = -1); the
 * unmasked experts of one token must be distinct.  T <= max_tokens.  All
 * outputs are int32 device arrays of the shapes named above. */
int ep_layout(ep_handle *h, const int32_t *d_topk_idx, int32_t T,
              int32_t *d_count, int32_t *d_expert_total, int32_t *d_rank_total,
              int32_t *d_base, int32_t *d_expert_offset, int32_t *d_rank_offset,
              int32_t *d_slot, int32_t *d_dst_row, void *stream);

/* ep_layout_static - ep_layout for callers that cannot allocate device memory: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  It
 * needs no handle (ep_proxy_start allocates) and calls no hipMalloc, hipFree or any
 * other allocating routine: the scratch that ep_layout keeps in its handle (tile
 * histograms, tile prefixes, a ticket) lives in a device array that is part of the
 * library's code object, 2 MiB + 512 bytes per GPU, held until the process ends.
 * Same kernels, same outputs, bit for bit, as ep_layout with num_src = S, top_k = K,
 * num_experts = E, num_ranks = R (limits as in ep_config; 0 <= T < 2^19).
 *   Limit: (S * ceil(T/64) + 1) * E <= 262144 scratch entries (the 4096-token,
 *   256-expert table needs 16640); beyond that EP_EINVAL, with the figures in
 *   ep_last_error.
 *   d_status: device int32, may be NULL; receives EP_EBOUNDS when an expert id outside
 *   [-1, E) is met (that entry gets slot = dst_row = -1); never cleared by the call.
 * Every call on one GPU uses that GPU's one array: calls that overlap in time on the
 * same GPU (two streams, two threads) race; order them on one stream.  The first call
 * on a device looks the array's address up (not while the stream is being captured,
 * unless ep_proxy_start has run on that device before: it does the look-up too). */
int ep_layout_static(const int32_t *d_topk_idx, int32_t S, int32_t T, int32_t K, int32_t E, int32_t R,
                     int32_t *d_count, int32_t *d_expert_total, int32_t *d_rank_total,
                     int32_t *d_base, int32_t *d_expert_offset, int32_t *d_rank_offset,
                     int32_t *d_slot, int32_t *d_dst_row, int32_t *d_status, void *stream);

/* ep_dispatch - the dispatch phase (Section 2.1) for the T tokens of source
 * rank src_rank: every valid (t,k) whose expert lives on dst_rank_filter (or on
 * any rank if -1) gets x[t,:] written to receive row dst_row[t,k]:
 *   EP_BF16      d_recv is bf16 [recv_rows, H]; d_recv_scale must be NULL
 *   EP_FP8_E4M3  d_recv is uint8 [recv_rows, H], d_recv_scale fp32 [recv_rows, H/128]
 *                per 128-channel block: scale = amax/448 (1 if amax < 2^-100),
 *                code = e4m3_rne_sat(x * (448/amax)).
 * d_x bf16 [T,H]; d_topk_idx, d_dst_row int32 [T,K]; d_count, d_base int32 [E]
 * are row src_rank of ep_layout's outputs.  Rows not addressed keep their
 * contents.  Unless cmd_mode is EP_CMD_NONE the kernel also pushes the
 * transfer commands of Section 3.1 into the handle's FIFO channels (channel =
 * destination expert mod C): Writes at the granularity cmd_mode selects, after
 * the rows they describe are stored, and per destination expert one Atomic
 * carrying count[e] (also when 0).  A full channel blocks the pushing wave
 * until the proxy pops (bounded by spin_timeout_ms).
 * FP8 rows that the proxy moves (heaps registered, commands on; Section 2.1: the ~7 KB FP8 token is ONE
 * message): a row is then H codes followed by its H/128 fp32 scales, padded to a multiple of 16 bytes
 * (7392 bytes at H = 7168), d_recv_scale must be NULL, and d_recv is the source heap: [recv_rows] message
 * rows laid out like the receive heap for the chunk modes, [T] message rows (row t = token t) for
 * EP_CMD_PER_TOKEN | EP_CMD_NO_PLACEMENT.  The destination heap receives [recv_rows] message rows;
 * ep_fp8_unpack splits them into codes and scales. */
int ep_dispatch(ep_handle *h, const void *d_x, const int32_t *d_topk_idx,
                const int32_t *d_dst_row, const int32_t *d_count, const int32_t *d_base,
                int32_t T, int32_t src_rank, int32_t dst_rank_filter,
                int32_t payload, int32_t cmd_mode,
                void *d_recv, float *d_recv_scale, int64_t recv_rows, void *stream);

/* ep_combine - the combine phase (Section 2.1, 2.2: a weighted-sum reduce in
 * the original token order):
 *   out[t,:] = bf16( sum_k w[t,k] * y[dst_row[t,k], :] )
 * fp32 accumulator starting at +0, k ascending, fused multiply-add, one final
 * round-to-nearest-even; k with dst_row == -1 are skipped.  d_y bf16
 * [y_rows,H]; d_topk_w fp32 [T,K]; d_dst_row int32 [T,K]; d_out bf16 [T,H].
 * All rows are read with streaming loads in token order (see EP_FLAG_CACHE_HINTS
 * for the one exception a caller can ask for). */
int ep_combine(ep_handle *h, const void *d_y, const float *d_topk_w,
               const int32_t *d_dst_row, int32_t T, int64_t y_rows,
               void *d_out, void *stream);

/* ep_fp8_unpack - receiver side of FP8 rows that travelled as messages (Section 2.1: a token is one ~7 KB FP8
 * message; Section 3.2: the proxy moves it between registered heaps): splits `rows` message rows of d_msgs
 * (each H codes + H/128 fp32 scales, padded to 16 bytes) into d_recv (uint8 [rows, H]) and d_recv_scale
 * (fp32 [rows, H/128]).  Call it once the rows have arrived (after ep_wait, or after ep_recv_wait on `stream`). */
int ep_fp8_unpack(ep_handle *h, const void *d_msgs, int64_t rows, void *d_recv, float *d_recv_scale, void *stream);

/* ep_wait - the host-side view of completion (Section 3.3: an Atomic is applied
 * only when the Writes it vouches for have arrived; Section 4.1: completion is a
 * counter in host memory): host-blocks until the proxy has applied the count Atomic of every
 * destination expert of every dispatch enqueued so far (the data of those
 * dispatches is then in place and its counters are posted), or returns the
 * sticky device/proxy error, or EP_ETIMEOUT after spin_timeout_ms. */
int ep_wait(ep_handle *h);

/* ---- high-throughput mode (Section 2.2: message deduplication and hierarchical reduce) ----
 * A "group" is ranks_per_group consecutive ranks (1 = a GPU, 8 = a node of eight).
 *
 * ep_dedup - a token routed to several experts of one group travels once:
 *   group(e) = (e / (E/R)) / ranks_per_group; walking k ascending, the first
 *   entry of a token that names a group keeps it (group_idx[s,t,k] = group),
 *   later entries of that group are duplicates (group_idx = -1); first_k[s,t,k]
 *   is the k of that first entry (-1 for masked entries).  d_group_idx is a
 *   routing table over R/ranks_per_group "experts" that ep_layout / ep_dispatch
 *   of a second handle (num_ranks = num_experts = R/ranks_per_group, same K, H)
 *   consume unchanged: one receive row per (token, group).  All int32 [S,T,K]. */
int ep_dedup(ep_handle *h, const int32_t *d_topk_idx, int32_t T, int32_t ranks_per_group,
             int32_t *d_group_idx, int32_t *d_first_k, void *stream);

/* ep_gather_index - the per-expert index list: row i of the ordinary
 * (expert-major) layout reads its input from row d_index[i] of the deduplicated
 * receive buffer: d_index[dst_row[t,k]] = dst_row_g[t, first_k[t,k]] for every
 * valid (t,k) of one source.  d_dst_row, d_dst_row_g, d_first_k int32 [T,K];
 * d_index int32 [rows]; entries no (t,k) addresses keep their contents. */
int ep_gather_index(ep_handle *h, const int32_t *d_dst_row, const int32_t *d_dst_row_g, const int32_t *d_first_k,
                    int32_t T, int64_t rows, int32_t *d_index, void *stream);

/* ep_combine_partial - first level of the hierarchical reduce, done where the
 * experts live: one partial row per (token, group),
 *   partial[dst_row_g[t,j], :] = bf16( sum_{k : first_k[t,k] == j} w[t,k] * y[dst_row[t,k], :] )
 * (fp32 accumulator from +0, k ascending, fused multiply-add, one rounding to
 * bf16: the partial travels as bf16).  The second level is ep_combine over the
 * partial rows with dst_row_g and unit weights.  d_y bf16 [y_rows,H];
 * d_partial bf16 [rows_g,H]; the index arrays are int32 [T,K]. */
int ep_combine_partial(ep_handle *h, const void *d_y, const float *d_topk_w, const int32_t *d_dst_row,
                       const int32_t *d_first_k, const int32_t *d_dst_row_g, int32_t T, int64_t y_rows,
                       int64_t rows_g, void *d_partial, void *stream);

/* ep_register_heaps - symmetric-memory registration (Section 3.2): gives the
 * proxy the device base addresses and sizes of the source-side heap (what Write
 * commands' source offsets are relative to) and of the destination-side receive
 * heap.  While heaps are registered the proxy PERFORMS every Write command it
 * polls: after translating and bounds-checking the offsets it copies `length`
 * bytes from source heap + source offset to destination heap + destination
 * offset (batched copy kernels on a stream of the proxy's own, standing in
 * for the RDMA writes), and only when a batch has completed does it hand the
 * writes' immediates to the receiver half.  Count Atomics keep flowing at once,
 * so they regularly overtake their data and wait in the control buffer.
 *   chunk modes : ep_dispatch packs rows into the source heap (pass it as
 *                 d_recv); a chunk's source offset equals its destination offset.
 *   per-token   : with EP_CMD_NO_PLACEMENT the source heap is d_x itself (bf16), or
 *                 the [T] message rows the kernel quantises the tokens into (FP8;
 *                 pass them as d_recv).
 * FP8 rows travel as one message each: see ep_dispatch and ep_fp8_unpack.
 * Call it only while no dispatch is in flight; NULL bases unregister. */
int ep_register_heaps(ep_handle *h, const void *d_src_base, int64_t src_bytes, void *d_dst_base, int64_t dst_bytes);

/* ep_barrier - enqueues a one-wave kernel that pushes a Barrier command
 * (Section 3.1, "Types of TransferCmd") and blocks `stream` on
 * Check-completion of it.  The proxy pops the command only when all
 * barrier_peers processes that share barrier_name have pushed theirs (the
 * intra-node level of the paper's barrier: peers meet in shared memory), or
 * after spin_timeout_ms, in which case the proxy error becomes EP_ETIMEOUT.
 * The cross-node level (leaders exchanging immediates) needs a network and is
 * not part of this library. */
int ep_barrier(ep_handle *h, void *stream);

/* ep_recv_wait - the receiving side's wait, on the GPU (Section 4.1: the GPU
 * observes the host-allocated counters and uses them for control decisions).
 * Enqueues a kernel that blocks `stream` until the proxy has posted the
 * completion counter of every expert of dst_rank_filter (every expert if -1)
 * for source src_rank, i.e. until that dispatch's rows are in place and
 * announced.  The kernel then writes the posted counts to d_counts_out (int32
 * [E], device, may be NULL; experts outside the filter get -1) and clears the
 * arrival flags so the next dispatch of that source can be awaited.  One
 * ep_recv_wait per ep_dispatch of a (source, filter) pair, in stream order.
 * The wait is bounded by spin_timeout_ms: on expiry the kernel exits and the
 * sticky device error becomes EP_ETIMEOUT. */
int ep_recv_wait(ep_handle *h, int32_t src_rank, int32_t dst_rank_filter, int32_t *d_counts_out, void *stream);

/* ep_counters - *recv_count points at the pinned-host completion counters,
 * int32 [S, E] ([source][global expert]), written by the proxy when it applies
 * an Atomic (Section 4.1: host-allocated counters the GPU may also read).
 * *d_recv_count (may be NULL) receives the same memory's device address. */
int ep_counters(ep_handle *h, const int32_t **recv_count, const int32_t **d_recv_count);

/* ep_ht_dispatch - high-throughput-mode dispatch through ring-buffer
 * communication channels (Section 3.3, "partial ordering"; Section 3.3's
 * description of the HT kernel: rings of chunk slots, head and tail values).
 * The T tokens are cut into ht_slices slices of ceil(T/ht_slices) consecutive
 * tokens; a channel is (source, slice, destination rank) and owns a ring of
 * ht_ring_slots slots in d_ring.  One launch runs one workgroup per slice, which
 * plays both ends of the slice's channels in turns and never waits for the other
 * end (so a workgroup depends on nothing but the proxy, whatever the grid size):
 *   sender   - copies each valid (token, k) row into the next free row of its
 *              channel's current chunk (slot = chunk number mod W, a 128-byte
 *              header of int32 destination rows, then 32 rows); it may use a slot
 *              only when the head counter says chunk n - W was consumed; a full (or
 *              the last, partial) chunk is announced with a sequenced Write and a
 *              sequenced Atomic that adds its rows to the channel's tail;
 *   receiver - polls the tails, copies the rows of every announced chunk from the
 *              ring to their destination rows in d_recv (the packed receive buffer
 *              of ep_dispatch), then releases the slot with a sequenced Atomic that
 *              adds the rows to the channel's head (a channel in the other direction).
 * All three message kinds travel through the command rings and the proxy, which
 * applies each channel's messages strictly in sequence whatever order they were
 * delivered in; tail and head counters live in pinned host memory
 * (ep_ring_counters).  The launch ends with a Drain on every FIFO; ep_wait
 * returns when those are through.
 *   d_x [T,H] bf16, d_topk_idx / d_dst_row int32 [T,K] of source src_rank
 *   payload  EP_BF16: rows travel as they are.  EP_FP8_E4M3: the sender quantises (as ep_dispatch does) and a
 *            row in a slot is H codes followed by H/128 fp32 scales (padded to 16 bytes); the receiver splits it
 *            into d_recv (u8 [recv_rows, H]) and d_recv_scale (f32 [recv_rows, H/128]).  d_recv_scale is NULL
 *            exactly for EP_BF16.
 *   d_ring   device, ring_bytes >= ht_slices * R * W * (128 + 32 * 2H), 16-byte aligned (the slot stride is the
 *            same for both payloads)
 *   d_recv   device bf16 [recv_rows, H] (or the FP8 pair)
 * Needs ht_slices > 0 and proxy threads; one ep_ht_dispatch per source at a time
 * (wait with ep_wait before the next one of the same source).  Every wait in the
 * kernel is bounded by spin_timeout_ms (EP_ETIMEOUT in the sticky device error). */
int ep_ht_dispatch(ep_handle *h, const void *d_x, const int32_t *d_topk_idx, const int32_t *d_dst_row, int32_t T,
                   int32_t src_rank, int32_t payload, void *d_ring, int64_t ring_bytes, void *d_recv,
                   float *d_recv_scale, int64_t recv_rows, void *stream);

/* ep_ring_counters - pinned-host int32 [S, ht_slices, R] each: rows announced
 * (tail) and rows released (head) per ring-buffer channel, running totals. */
int ep_ring_counters(ep_handle *h, const int32_t **ring_tail, const int32_t **ring_head);

/* ep_tail_counters - *recv_tail points at pinned-host int32 [S, R]: rows
 * announced so far on the communication channel (source, destination rank) by
 * ordered Atomics (EP_CMD_CHUNK32_ORDERED), added up in sequence order. */
int ep_tail_counters(ep_handle *h, const int32_t **recv_tail);

/* ep_stats / ep_reset_stats - proxy and ring statistics: what Section 5.3 measures
 * of the channel (commands per second through the FIFOs, commands per proxy
 * thread) and what Section 3.3 describes of the receiver (Atomics that had to wait
 * in the control buffer).  Reset also zeroes the completion counters; call it only
 * when ep_wait has returned. */
int ep_stats(ep_handle *h, ep_stats_t *out);
int ep_reset_stats(ep_handle *h);

/* ep_cmd_log - the TransferCmds of Section 3.1 as the proxy's Poll saw them, for
 * replaying a dispatch from its commands alone: copies up to cap commands (16 bytes each, as polled, thread by
 * thread, in-channel order preserved) into buf; *n = number available.
 * Needs EP_FLAG_LOG_CMDS; call after ep_wait.
 * ep_event_log - same for the receiver-side trace (4 x uint32 per record:
 * kind | thread << 8, source rank, global expert, value; kind 1 = Write
 * delivered (value = rows), 2 = Atomic delivered, 3 = Atomic applied.  Ordered
 * mode: [2] is the destination rank and value the sequence number; kind 4 =
 * ordered Write delivered, 5 = ordered Atomic delivered, 6 = ordered Write
 * applied, 7 = ordered Atomic applied). */
int ep_cmd_log(ep_handle *h, void *buf, size_t cap, size_t *n);
int ep_event_log(ep_handle *h, void *buf, size_t cap, size_t *n);

/* Host-side producer for the same ring protocol, for handles made with
 * EP_FLAG_HOST_ONLY (tests and diagnostics of the proxy without a GPU; the
 * device-side Push lives in the kernels).  ep_host_push implements Push: it
 * blocks while channel is full (bounded by spin_timeout_ms), writes the four
 * words (lap-parity bits are set by the call) and returns the command's Idx.
 * ep_host_check_completion implements Check-completion(Idx): 1 if the proxy
 * has popped command idx of that channel, else 0. */
int ep_host_push(ep_handle *h, int32_t channel, uint32_t w0, uint32_t w1, uint32_t w2,
                 uint32_t w3, uint64_t *idx);
int ep_host_check_completion(ep_handle *h, int32_t channel, uint64_t idx);
/* ep_captured / ep_expect - ring-on launches inside a HIP graph.  ep_dispatch,
 * ep_ht_dispatch and ep_fifo_stress tell ep_wait at call time how many count
 * Atomics (or Drains) their kernel is going to push.  On a stream that is being
 * captured nothing runs at call time, so the call adds those numbers to a ledger
 * instead: ep_captured returns it (and clears it when reset != 0) once the capture
 * has ended, and the caller hands the numbers to ep_expect before (or right
 * after) every launch of the graph, so that ep_wait covers the replayed work.
 * Everything else these calls do is capturable as it is: their kernels clear
 * their own scratch, and no memset or copy is issued on the stream.
 * Host memory only; thread-compatible like the other calls. */
int ep_captured(ep_handle *h, int64_t *atomics, int64_t *drains, int32_t reset);
int ep_expect(ep_handle *h, int64_t atomics, int64_t drains);

/* Tells the proxy how many count Atomics ep_wait should expect in addition
 * (ep_dispatch does this itself for its own). */
int ep_host_expect_atomics(ep_handle *h, int32_t n);

/* ep_last_error - text describing the most recent failed HIP runtime call made
 * by the library on the calling thread ("" if none).  Static storage. */
const char *ep_last_error(void);

/* TransferCmd, 128 bits = four 32-bit words (Section 3.1 names the fields,
 * not their widths; this is the layout of this library):
 *   w0 [31] lap parity  [30:28] op  [27:20] source (connection) rank
 *      [19:12] destination rank  [11:0] expert index local to the destination
 *   w1 Write : [31:26] rows carried - 1, [25:0] length / 16
 *      Atomic: value      Drain: unused
 *   w2 Write : source offset / 16
 *   w3 [31] lap parity  [30:0] Write: destination offset / 16
 *                              Atomic: counter index = source * (E/R) + local expert
 * The lap parity of slot Idx is ((Idx / ring_entries) & 1) ^ 1; a slot is
 * ready when both parity bits match the lap the consumer is on.  The sequence
 * number of a command is its Idx (order inside one channel is kept). */
enum ep_cmd_op {
  EP_OP_WRITE = 1, EP_OP_ATOMIC = 2, EP_OP_DRAIN = 3, EP_OP_BARRIER = 4,
  /* Sequenced variants used by EP_CMD_CHUNK32_ORDERED: w2 carries the 32-bit sequence number of the
   * communication channel (source rank, destination rank); an ordered Write's source offset equals its
   * destination offset; an ordered Atomic ADDS w1 to the tail counter w3 = source * R + destination rank. */
  EP_OP_ORDERED_WRITE = 5, EP_OP_ORDERED_ATOMIC = 6,
  /* Messages of the ring-buffer channels (ep_ht_dispatch).  w0's local-expert field carries the slice, so
   * the channel is (source, slice, destination rank); w1[31:30] is the kind, w2 the channel's sequence number:
   *   kind 0 Write       w1[29:24] rows - 1, w1[23:0] length / 16 (header + rows), w3 = slot offset in the ring / 16
   *   kind 1 Atomic tail w1[29:0] rows to add to the channel's tail   (sender -> receiver, numbered with the Writes)
   *   kind 2 Atomic head w1[29:0] rows to add to the channel's head   (receiver -> sender, numbered on its own) */
  EP_OP_RING = 7
};
enum ep_ring_kind { EP_RING_WRITE = 0, EP_RING_TAIL = 1, EP_RING_HEAD = 2 };

#ifdef __cplusplus
}
#endif
#endif /* EP_H_ */
