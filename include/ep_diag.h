/*
 * ep_diag.h - measurement entry points of libep.so.  None of them is part of the
 * dispatch/combine path and no product call depends on them: they exist so that a
 * benchmark can time the path's kernels without an external profiler, load-test
 * the GPU->CPU channel the way Section 5.3 of the paper does, and measure this
 * device's plain streaming rates next to the path's kernels.  Conventions as in
 * ep.h.
 */
#ifndef EP_DIAG_H_
#define EP_DIAG_H_

#include "ep.h"

#ifdef __cplusplus
extern "C" {
#endif

/* ep_profile / ep_profile_read - kernel-exact durations of the three compute
 * calls, for callers that want them without an external profiler.  While
 * profiling is on, every ep_layout / ep_dispatch / ep_combine launch carries a
 * pair of HIP events that receive the begin timestamp of the call's first kernel
 * and the end timestamp of its last one from the launches themselves (nothing
 * extra is put on the stream, unlike a pair of recorded events, which delays
 * the kernel between them by a few microseconds).  ep_profile_read waits for the
 * timed launches of one call (0 layout, 1 dispatch, 2 combine), returns their
 * summed duration in milliseconds and their number, and forgets them when
 * reset != 0.  Launches on a capturing stream are not timed.  on = 0 switches
 * profiling off; on = n >= 1 switches it on and makes sure n pairs of events are
 * at hand, so that up to n timed launches create none (n <= 65536).  Events are
 * reused after a read with reset and freed when the handle stops; at most 65536
 * unread launches per call are kept, later ones run untimed. */
int ep_profile(ep_handle *h, int32_t on);
int ep_profile_read(ep_handle *h, int32_t call, double *total_ms, int32_t *launches, int32_t reset);

/* ep_fifo_stress - closed-loop load test of the GPU->CPU channel (the FIFO stress
 * test of Section 5.3): `pushers` wavefronts (lane 0 of each; channel = pusher
 * mod C) each push `cmds_per_pusher` commands, one after the other, waiting with
 * Check-completion until the proxy has popped each before pushing the next.  The
 * command is a count Atomic of value 0 for (source 0, expert 0): harmless, applied
 * at once (ep_wait accounts for them; do not run it while a dispatch of source 0
 * is being awaited).  d_lat_sum / d_lat_max (device, uint64 [pushers]) receive
 * each pusher's summed and largest push->popped time in ticks of 10 ns. */
int ep_fifo_stress(ep_handle *h, int32_t pushers, int32_t cmds_per_pusher, uint64_t *d_lat_sum, uint64_t *d_lat_max,
                   void *stream);

/* ep_bw_probe - plain streaming kernels for measuring this device's bandwidth
 * ceilings next to the path's kernels (no part of the method): kind 0 reads
 * `bytes` from d_src (16-byte non-temporal loads, one per lane), kind 1 writes
 * `bytes` to d_dst, kind 2 copies d_src to d_dst.  bytes must be a multiple of
 * 16; buffers are caller-owned device memory.  Needs no handle. */
int ep_bw_probe(int32_t kind, const void *d_src, void *d_dst, int64_t bytes, void *stream);

/* ep_row_probe - the memory access pattern of the path's two big kernels without the other half of their
 * traffic, to tell what the pattern itself can reach on this device (no part of the method): every item i
 * (a token) names k rows, d_rowmap[i*k .. i*k+k) (int32, device; entries < 0 or >= buf_rows are skipped), of
 * row_bytes bytes each in d_buf.  kind 0 stores a constant to every such row with the dispatch's kind of store
 * and wave shape (nothing is read); kind 1 reads every such row with the combine's kind of load and wave shape
 * (nothing is written; d_sink, 16 bytes of device memory, only keeps the loads alive).  row_bytes a multiple of
 * 16.  Needs no handle. */
int ep_row_probe(int32_t kind, const int32_t *d_rowmap, int32_t k, int64_t items, int32_t row_bytes, int64_t buf_rows,
                 void *d_buf, void *d_sink, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* EP_DIAG_H_ */
