#!/usr/bin/env python3
"""Benchmark of the expert-parallel hot path on one MI355X.

One step = one pass of the whole path over one batch of synthetic input:
ep_layout -> ep_dispatch (payload placement + transfer commands through the
FIFO channels to the CPU proxy) -> ep_combine over the experts' outputs, which
sit in a buffer of their own (as they do behind real experts) -> ep_wait (the
proxy has posted every completion counter of the step).

Workload: the 4096-token x hidden-7168 x 256-expert top-8 prefill share
(16 simulated ranks, Zipf-skewed routing), inputs resident in HBM before the
timed region.  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth


def algorithmic_bytes(T, H, K, rows, payload="bf16"):
    """Bytes the method itself must move (per launch).  dispatch bf16: read each token row once,
    write one row per valid (t,k), plus 8 bytes of (expert, row) metadata per (t,k).
    combine: read one row per valid (t,k), write each token row once, plus 8 bytes
    (row, weight) per (t,k)."""
    meta = 8 * T * K
    if payload == "bf16":
        disp = 2 * H * T + 2 * H * rows + meta
    else:
        disp = 2 * H * T + (H + H // 32) * rows + meta
    comb = 2 * H * rows + 2 * H * T + meta
    return disp, comb


def read_traffic(kernel_key: str):
    """HBM bytes per launch measured with rocprofv3 --pmc (FETCH_SIZE + WRITE_SIZE, scaled by a
    copy kernel of known size); taken from the committed summary under profiles/ if there is one."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic_cfg4.txt")
    if not os.path.exists(path):
        return None
    m = re.search(rf"^{kernel_key}\s+traffic_bytes_per_launch\s*=\s*([0-9.eE+]+)", open(path).read(), re.M)
    return float(m.group(1)) if m else None


def source_stamp() -> str:
    """Identifies the code that produced a table: the git revision when the tree has one (the GPU machine gets a
    copy without .git), and always a hash over the library's sources and this file, which anyone can recompute:
    cat include/*.h paper_2512_19849_amd/csrc/*.{h,hip,cpp} bench.py (sorted by path) | sha256sum."""
    import glob
    import hashlib
    import subprocess
    h = hashlib.sha256()
    files = sorted(glob.glob(os.path.join(ROOT, "include", "*.h")) +
                   [f for pat in ("*.h", "*.hip", "*.cpp")
                    for f in glob.glob(os.path.join(ROOT, "paper_2512_19849_amd", "csrc", pat))] +
                   [os.path.join(ROOT, "bench.py")])
    for f in files:
        h.update(open(f, "rb").read())
    rev = "n/a (no .git in this copy)"
    try:
        p = subprocess.run(["git", "-C", ROOT, "rev-parse", "--short", "HEAD"], capture_output=True, text=True, timeout=10)
        if p.returncode == 0 and p.stdout.strip():
            dirty = subprocess.run(["git", "-C", ROOT, "status", "--porcelain", "--untracked-files=no"],
                                   capture_output=True, text=True, timeout=10).stdout.strip()
            rev = p.stdout.strip() + (" + uncommitted changes" if dirty else "")
    except Exception:
        pass
    return f"git {rev}; sources sha256 {h.hexdigest()[:16]}"


SUITE_LEGEND = """Per-call timings of all five workloads, MI355X (HIP-event medians of 20 calls, microseconds).

command:  python3 bench.py --suite      (this file is written by that command, nothing is edited by hand)
code:     {stamp}
Every handle is made WITHOUT EP_FLAG_CACHE_HINTS: each call walks the tokens in ascending order and streams
its rows, whatever ran before it.
"warm": calls queued back to back.  Small workloads are launch-latency bound there (the host cannot
queue them faster than ~15 us apart); "cold": a 512 MiB fill runs before every call, which also keeps the
queue busy, so those figures are the kernel itself with cold caches.
Ring-on dispatches ("dispatch_*_per_token_us", "_chunk32_us", "_chunk32_ordered_us") are each followed by ep_wait
before the next call, so the GPU idles for some tens of microseconds between them: these figures read about
10 us higher than the same kernel inside a step (the headline's dispatch with chunk commands: 105 us, see
kernel_stats_cfg4_prefill_bf16_chunk32.txt).
"*_kernel_us": the kernels' own duration from their begin / end timestamps (ep_profile), mean of 16 warm launches.
"launch->last counter": host clock from the ep_dispatch call to ep_wait returning (all completion counters
posted by the proxy).  "proxy rate": commands / (last atomic applied - first command polled), proxy-side clocks.
GB/s = algorithmic bytes of that call / time.
"ll_step_*": one whole low-latency step (layout, per-token dispatch with commands through the proxy, GPU-side
wait for the posted counters, combine), host clock over 30 steps queued back to back: launched call by call
(four launches per step through Python) and replayed from a HIP graph (ep_captured / ep_expect).
"proxy_writes_*": heaps registered (ep_register_heaps), the proxy threads move the rows with batched copy
kernels on the proxy's stream and release arrival notices when a batch has completed; same host clock.
"*_rings_sized_for_the_dispatch": the same per-token dispatches on a handle whose rings hold all commands of one
dispatch (ring_entries as listed; every other section uses the default of 4096 slots per channel, which the two
large workloads overrun, so that producers wait for the proxy there).
"inbound_share_*" (the 32-source decode workload): the rows the other 31 source ranks send into this rank's
partition, 31 ep_dispatch calls with a rank filter queued back to back, event to event; "send_share" is this
rank's own dispatch to all 32 ranks.
"ht_step_*": the whole high-throughput step - dedup, group layout, group dispatch with chunk commands,
gather index, partial reduce per group, final reduce, wait - host clock over 20 steps queued back to back.
"""


def format_suite(out: dict) -> str:
    L = [SUITE_LEGEND.format(stamp=source_stamp())]
    for name, v in out.items():
        L.append(f"== {name}: T={v['T']} H={v['H']} E={v['E']} K={v['K']} R={v['R']} S={v['S']}  algorithmic bytes "
                 f"dispatch={v['dispatch_bytes']:,} combine={v['combine_bytes']:,}")
        for key in [k for k in v if k.startswith("threads")]:
            L.append(f"  [{key}]")
            for a, b in v[key].items():
                extra = ""
                if a.endswith("_us") and "dispatch_bf16" in a and "cold" not in a:
                    extra = f"   ({v['dispatch_bytes'] / b / 1e3:.0f} GB/s)"
                if a.endswith("_us") and "dispatch_fp8" in a and "cold" not in a:
                    extra = f"   ({v['dispatch_fp8_bytes'] / b / 1e3:.0f} GB/s)"
                if a in ("combine_us", "combine_kernel_us"):
                    extra = f"   ({v['combine_bytes'] / b / 1e3:.0f} GB/s)"
                L.append(f"    {a:50s} {b}{extra}")
        if "fifo_stress" in v:
            L.append("  [fifo_stress]  closed loop: each pusher (one wavefront) pushes a command, waits until the proxy "
                     "has popped it, pushes the next; 8 channels")
            for a, b in v["fifo_stress"].items():
                L.append(f"    {a:28s} {b['Mcmd_per_s']:8.2f} Mcmd/s   push->popped mean {b['mean_latency_us']:8.2f} us"
                         f"  max {b['max_latency_us']:8.1f} us")
        for key in [k for k in v if k.startswith("per_token_")]:
            L.append(f"  [{key}]  per-token dispatch with an option of the proxy (packing, pacing, where the fence sits)")
            for a, b in v[key].items():
                L.append(f"    {a:50s} {b}")
        for key in [k for k in v if k.startswith("ht_")]:
            what = ("ring-buffer channels: sending step -> ring slot -> receiving step -> packed buffer (one workgroup "
                    "per slice plays both ends in turns); Write / tail / head messages through the proxy; host clock "
                    "from the ep_ht_dispatch call to ep_wait (Drains popped)" if key.startswith("ht_ring")
                    else "high-throughput mode: one copy per (token, group of ranks), two-level reduce")
            L.append(f"  [{key}]  {what}")
            for a, b in v[key].items():
                L.append(f"    {a:50s} {b}")
    return "\n".join(L) + "\n"


def run_suite(args) -> int:
    """Per-call timings of all five workloads : layout, dispatch
    with the ring off / per-token / chunk32, FP8 where the workload names it, combine, the command
    rate the proxy sustains with 1 and 4 threads, warm and (small workloads) cold caches."""
    import numpy as np
    import torch

    import ep_inputs as g
    import paper_2512_19849_amd as ep
    from paper_2512_19849_amd.runner import EPRunner, bits_to_bf16

    ep.load_library(build_if_missing=False)
    scrub = torch.empty(512 << 20, dtype=torch.uint8, device="cuda")

    def timed(fn, n=20, warm=3, cold=False, after=None):
        """Median event-to-event time of one call.  Warm: calls are queued back to back (no host sync
        in between, so the time is the kernel plus its launch gap, not the idle-start latency).
        Cold: a 512 MiB fill runs before every call to push the call's data out of the caches."""
        for _ in range(warm):
            fn()
            if after:
                after()
        torch.cuda.synchronize()
        evs = []
        for _ in range(n):
            if cold:
                scrub.fill_(1)
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            fn()
            b.record()
            if after:
                after()
            evs.append((a, b))
        torch.cuda.synchronize()
        ts = sorted(a.elapsed_time(b) * 1e3 for a, b in evs)
        return round(ts[len(ts) // 2], 2)

    out = {}
    for cid in (1, 2, 3, 4, 5):
        cfg = g.config(cid)
        T, H, K, E, R, S = cfg.T, cfg.H, cfg.K, cfg.E, cfg.R, cfg.S
        idx, w = g.routing_all(cfg)
        rows = idx.size
        my_rows = T * K
        d_idx = torch.from_numpy(idx).cuda()
        d_w = torch.from_numpy(w[0]).cuda()
        d_x = bits_to_bf16(g.activations(cfg))
        recv = torch.zeros((rows, H), dtype=torch.bfloat16, device="cuda")
        rq = torch.zeros((rows, H), dtype=torch.uint8, device="cuda")
        rs = torch.zeros((rows, H // 128), dtype=torch.float32, device="cuda")
        o = torch.zeros((T, H), dtype=torch.bfloat16, device="cuda")
        db, cb = algorithmic_bytes(T, H, K, my_rows, "bf16")
        fb, _ = algorithmic_bytes(T, H, K, my_rows, "fp8")
        res = {"T": T, "H": H, "E": E, "K": K, "R": R, "S": S, "dispatch_bytes": db, "combine_bytes": cb,
               "dispatch_fp8_bytes": fb}
        small = rows * H * 2 < (128 << 20)
        for threads, chans in (((1, 8), (4, 8), (4, 64)) if cid in (4, 5) else ((4, 8),)):
            with EPRunner(R, E, K, H, T, S=S, num_proxy_threads=threads, num_channels=chans,
                          spin_timeout_ms=10000) as r:
                lay = r.layout(d_idx)
                key = f"threads{threads}_channels{chans}"
                rr = {}
                if threads == 4 and chans == 8:
                    rr["layout_us"] = timed(lambda: r.layout(d_idx))
                    rr["dispatch_bf16_ring_off_us"] = timed(
                        lambda: r.dispatch(d_x, d_idx[0], lay, recv, cmd_mode=ep.EP_CMD_NONE))
                    rr["combine_us"] = timed(lambda: r.combine(recv, d_w, lay.dst_row[0], o))
                    # the kernels' own durations (ep_profile), warm, beside the event-to-event figures above
                    for call, label, fn in ((0, "layout", lambda: r.layout(d_idx)),
                                            (1, "dispatch_bf16_ring_off",
                                             lambda: r.dispatch(d_x, d_idx[0], lay, recv, cmd_mode=ep.EP_CMD_NONE)),
                                            (2, "combine", lambda: r.combine(recv, d_w, lay.dst_row[0], o))):
                        ep.ep_profile(r.h, 16)
                        for _ in range(16):
                            fn()
                        ep.ep_profile(r.h, False)
                        ms, n = ep.ep_profile_read(r.h, call)
                        rr[f"{label}_kernel_us"] = round(ms / n * 1e3, 2)
                    if small:
                        rr["layout_cold_us"] = timed(lambda: r.layout(d_idx), cold=True)
                        rr["dispatch_bf16_ring_off_cold_us"] = timed(
                            lambda: r.dispatch(d_x, d_idx[0], lay, recv, cmd_mode=ep.EP_CMD_NONE), cold=True)
                        rr["combine_cold_us"] = timed(lambda: r.combine(recv, d_w, lay.dst_row[0], o), cold=True)
                    if cid in (3, 4, 5):
                        rr["dispatch_fp8_ring_off_us"] = timed(
                            lambda: r.dispatch(d_x, d_idx[0], lay, rq, rs, payload=ep.EP_FP8_E4M3,
                                               cmd_mode=ep.EP_CMD_NONE))
                for mode in ("per_token", "chunk32", "chunk32_ordered"):
                    cm = ep.CMD_MODES[mode]
                    rr[f"dispatch_bf16_{mode}_us"] = timed(
                        lambda: r.dispatch(d_x, d_idx[0], lay, recv, cmd_mode=cm), after=r.wait)
                    # one dispatch, host clock from launch to the last completion counter, and the proxy's own
                    # first-poll -> last-apply span
                    e2e, rate = [], []
                    for _ in range(10):
                        ep.ep_reset_stats(r.h)
                        torch.cuda.synchronize()
                        t0 = time.perf_counter()
                        r.dispatch(d_x, d_idx[0], lay, recv, cmd_mode=cm)
                        r.wait()
                        e2e.append((time.perf_counter() - t0) * 1e6)
                        st = r.stats()
                        span = (st["last_apply_ns"] - st["first_poll_ns"]) * 1e-9
                        rate.append(st["cmds"] / span / 1e6 if span > 0 else 0.0)
                    e2e.sort()
                    rate.sort()
                    rr[f"{mode}_cmds"] = st["cmds"]
                    rr[f"{mode}_launch_to_last_counter_us"] = round(e2e[len(e2e) // 2], 1)
                    rr[f"{mode}_proxy_Mcmd_per_s"] = round(rate[len(rate) // 2], 2)
                    if cid in (3, 4, 5):
                        rr[f"dispatch_fp8_{mode}_us"] = timed(
                            lambda: r.dispatch(d_x, d_idx[0], lay, rq, rs, payload=ep.EP_FP8_E4M3, cmd_mode=cm),
                            after=r.wait)
                if S > 1 and threads == 4 and chans == 8:
                    # the decode workload's inbound share: what the other S - 1 source ranks send into this rank's
                    # partition (rank filter = 0), one ep_dispatch per source, queued back to back
                    xs = [bits_to_bf16(g.activations(cfg, s_)) for s_ in range(1, S)]
                    inbound_rows = int((idx[1:] // cfg.E_loc == 0).sum())
                    for mode in ("none", "per_token"):
                        cm = ep.CMD_MODES[mode]

                        def inbound():
                            for s_ in range(1, S):
                                r.dispatch(xs[s_ - 1], d_idx[s_], lay, recv, src=s_, rank_filter=0, cmd_mode=cm)

                        rr[f"inbound_share_{S - 1}_sources_{mode}_us"] = timed(
                            inbound, n=10, after=(r.wait if cm != ep.EP_CMD_NONE else None))
                    rr["inbound_share_rows"] = inbound_rows
                    rr["send_share_per_token_us"] = rr["dispatch_bf16_per_token_us"]
                    del xs
                if threads == 4 and chans == 8 and T <= 512:
                    # one whole low-latency step - layout, per-token dispatch with commands through the proxy,
                    # GPU-side wait for the posted counters, combine - launched call by call and replayed
                    # from a HIP graph; host clock over 30 steps queued back to back, per step
                    counts = torch.zeros((E,), dtype=torch.int32, device="cuda")

                    def ll_step():
                        L = r.layout(d_idx)
                        r.dispatch(d_x, d_idx[0], L, recv, cmd_mode=ep.EP_CMD_PER_TOKEN)
                        r.recv_wait(counts)
                        r.combine(recv, d_w, L.dst_row[0], o)

                    def host_timed(fn, n=30):
                        for _ in range(3):
                            fn()
                        r.wait()
                        torch.cuda.synchronize()
                        t0 = time.perf_counter()
                        for _ in range(n):
                            fn()
                        r.wait()
                        torch.cuda.synchronize()
                        return round((time.perf_counter() - t0) / n * 1e6, 1)

                    rr["ll_step_call_by_call_us"] = host_timed(ll_step)
                    side, graph = torch.cuda.Stream(), torch.cuda.CUDAGraph()
                    with torch.cuda.stream(side):
                        with torch.cuda.graph(graph, stream=side):
                            ll_step()
                    cap = r.captured()

                    def ll_replay():
                        r.expect(*cap)
                        graph.replay()

                    rr["ll_step_hip_graph_us"] = host_timed(ll_replay)
                    del graph
                if threads == 4:
                    # the proxy performs the writes (registered heaps): per token straight out of x,
                    # chunks out of a packed send heap; host clock from launch to the last counter
                    send = torch.zeros((rows, H), dtype=torch.bfloat16, device="cuda")
                    for mode, src_heap, tgt, flag in (("per_token", d_x, recv, ep.EP_CMD_NO_PLACEMENT),
                                                      ("chunk32", send, send, 0),
                                                      ("chunk32_ordered", send, send, 0)):
                        r.register_heaps(src_heap, recv)
                        cm = ep.CMD_MODES[mode] | flag
                        e2e = []
                        for _ in range(13):
                            torch.cuda.synchronize()
                            t0 = time.perf_counter()
                            r.dispatch(d_x, d_idx[0], lay, tgt, cmd_mode=cm)
                            r.wait()
                            e2e.append((time.perf_counter() - t0) * 1e6)
                        e2e = sorted(e2e[3:])
                        rr[f"proxy_writes_{mode}_launch_to_last_counter_us"] = round(e2e[len(e2e) // 2], 1)
                    st = r.stats()
                    rr["proxy_writes_copy_batches_per_dispatch"] = round(st["copy_batches"] / 39, 1)
                    r.register_heaps(None, None)
                    del send
                res[key] = rr
        if cid in (4, 5):
            # per-token commands again, with rings that hold a whole dispatch's commands (twice a channel's fair
            # share of them), so that no producer has to wait for the proxy to make room
            big = 1 << max(12, int(np.ceil(np.log2(2.0 * rows / 8))))
            with EPRunner(R, E, K, H, T, S=S, num_channels=8, num_proxy_threads=4, ring_entries=big,
                          spin_timeout_ms=10000) as rb:
                layb = rb.layout(d_idx)
                rr = {"ring_entries_per_channel": big}
                for label, src_heap, flag in (("per_token", None, 0), ("proxy_writes_per_token", d_x, ep.EP_CMD_NO_PLACEMENT)):
                    if src_heap is not None:
                        rb.register_heaps(src_heap, recv)
                    e2e = []
                    for _ in range(13):
                        torch.cuda.synchronize()
                        t0 = time.perf_counter()
                        rb.dispatch(d_x, d_idx[0], layb, recv, cmd_mode=ep.EP_CMD_PER_TOKEN | flag)
                        rb.wait()
                        e2e.append((time.perf_counter() - t0) * 1e6)
                    e2e = sorted(e2e[3:])
                    rr[f"{label}_launch_to_last_counter_us"] = round(e2e[len(e2e) // 2], 1)
                rr["gpu_ring_full"] = rb.stats()["gpu_ring_full"]
                rb.register_heaps(None, None)
                res["threads4_channels8_rings_sized_for_the_dispatch"] = rr
            # high-throughput mode: one copy per (token, group), partial reduce per group, final reduce
            for G in ((1, 8) if cid == 4 else (1,)):
                NG = R // G
                with EPRunner(R, E, K, H, T, num_proxy_threads=0) as r1, \
                        EPRunner(NG, NG, K, H, T, num_proxy_threads=4, spin_timeout_ms=10000) as rg:
                    gi, fk = torch.empty_like(d_idx), torch.empty_like(d_idx)
                    ep.ep_dedup(r1.h, d_idx, T, G, gi, fk)
                    L = r1.layout(d_idx)
                    Lg = rg.layout(gi)
                    torch.cuda.synchronize()
                    rows_g = int((gi >= 0).sum().item())
                    recv_g = torch.zeros((rows_g, H), dtype=torch.bfloat16, device="cuda")
                    partial = torch.zeros((rows_g, H), dtype=torch.bfloat16, device="cuda")
                    index = torch.zeros((rows,), dtype=torch.int32, device="cuda")
                    ones = torch.ones_like(d_w)
                    hh = {"groups": NG, "rows_per_token_expert": rows, "rows_per_token_group": rows_g,
                          "wire_bytes_ratio": round(rows_g / rows, 4)}
                    hh["dedup_us"] = timed(lambda: ep.ep_dedup(r1.h, d_idx, T, G, gi, fk))
                    hh["layout_groups_us"] = timed(lambda: rg.layout(gi))
                    hh["dispatch_groups_chunk32_us"] = timed(
                        lambda: rg.dispatch(d_x, gi[0], Lg, recv_g, cmd_mode=ep.EP_CMD_CHUNK32), after=rg.wait)
                    hh["gather_index_us"] = timed(
                        lambda: ep.ep_gather_index(r1.h, L.dst_row[0], Lg.dst_row[0], fk[0], T, rows, index))
                    hh["combine_partial_us"] = timed(
                        lambda: ep.ep_combine_partial(r1.h, recv, d_w, L.dst_row[0], fk[0], Lg.dst_row[0], T, rows,
                                                      rows_g, partial))
                    hh["combine_final_us"] = timed(lambda: rg.combine(partial, ones, Lg.dst_row[0], o))

                    # the whole high-throughput step, host clock over 20 steps queued back to back; the experts'
                    # outputs y sit in a buffer of their own (here: the flat receive buffer of the plain path)
                    def ht_step():
                        ep.ep_dedup(r1.h, d_idx, T, G, gi, fk)
                        L2 = r1.layout(d_idx)
                        Lg2 = rg.layout(gi)
                        rg.dispatch(d_x, gi[0], Lg2, recv_g, cmd_mode=ep.EP_CMD_CHUNK32)
                        ep.ep_gather_index(r1.h, L2.dst_row[0], Lg2.dst_row[0], fk[0], T, rows, index)
                        ep.ep_combine_partial(r1.h, recv, d_w, L2.dst_row[0], fk[0], Lg2.dst_row[0], T, rows, rows_g,
                                              partial)
                        rg.combine(partial, ones, Lg2.dst_row[0], o)
                        rg.wait()

                    for _ in range(3):
                        ht_step()
                    torch.cuda.synchronize()
                    c0 = time.perf_counter()
                    for _ in range(20):
                        ht_step()
                    torch.cuda.synchronize()
                    hh["ht_step_us"] = round((time.perf_counter() - c0) / 20 * 1e6, 1)
                    res[f"ht_ranks_per_group{G}"] = hh
                    del recv_g, partial
            # sender-side policies of the proxy on the per-token stream: best-effort packing, pacing
            for label, kw in (("pack8", dict(pack_rows=8)), ("pack8_hold50us", dict(pack_rows=8, pack_hold_us=50)),
                              ("pace32_window256", dict(max_outstanding=32, reorder_window=256)),
                              ("receiver_fence_window64", dict(reorder_window=64)),
                              ("sender_fence_window64", dict(reorder_window=64, flags=ep.EP_FLAG_SENDER_FENCE))):
                with EPRunner(R, E, K, H, T, num_proxy_threads=4, spin_timeout_ms=10000, **kw) as rp:
                    Lp = rp.layout(d_idx)
                    e2e = []
                    for _ in range(13):
                        torch.cuda.synchronize()
                        t0 = time.perf_counter()
                        rp.dispatch(d_x, d_idx[0], Lp, recv, cmd_mode=ep.EP_CMD_PER_TOKEN)
                        rp.wait()
                        e2e.append((time.perf_counter() - t0) * 1e6)
                    e2e = sorted(e2e[3:])
                    st = rp.stats()
                    res[f"per_token_{label}"] = {
                        "launch_to_last_counter_us": round(e2e[len(e2e) // 2], 1), "writes_per_dispatch": st["writes"] // 13,
                        "messages_per_dispatch": st["write_msgs"] // 13, "paced_per_dispatch": st["paced"] // 13,
                        "max_in_flight": st["max_in_flight"], "atomics_deferred_per_dispatch": st["atomics_deferred"] // 13,
                        "sender_held_per_dispatch": st["sender_held"] // 13}
            # ring-buffer channels: sender -> ring slot -> receiver -> packed buffer, head/tail through the proxy
            for slices, W in ((128, 2), (128, 4), (256, 2)):
                with EPRunner(R, E, K, H, T, num_proxy_threads=4, spin_timeout_ms=10000, ht_slices=slices,
                              ht_ring_slots=W) as rr_:
                    Lr = rr_.layout(d_idx)
                    ring = torch.zeros(rr_.ht_ring_bytes(), dtype=torch.uint8, device="cuda")
                    e2e = []
                    for _ in range(13):
                        torch.cuda.synchronize()
                        t0 = time.perf_counter()
                        rr_.ht_dispatch(d_x, d_idx[0], Lr, ring, recv)
                        rr_.wait()
                        e2e.append((time.perf_counter() - t0) * 1e6)
                    e2e = sorted(e2e[3:])
                    st = rr_.stats()
                    res[f"ht_ring_slices{slices}_slots{W}"] = {
                        "launch_to_drained_us": round(e2e[len(e2e) // 2], 1), "cmds_per_dispatch": st["cmds"] // 13,
                        "ring_MiB": rr_.ht_ring_bytes() >> 20,
                        "GBs_rows_delivered": round(my_rows * H * 2 / e2e[len(e2e) // 2] / 1e3, 1)}
                    if cid == 5 and (slices, W) == (128, 2):
                        e2e = []
                        for _ in range(13):
                            torch.cuda.synchronize()
                            t0 = time.perf_counter()
                            rr_.ht_dispatch(d_x, d_idx[0], Lr, ring, rq, recv_scale=rs)
                            rr_.wait()
                            e2e.append((time.perf_counter() - t0) * 1e6)
                        e2e = sorted(e2e[3:])
                        res["ht_ring_fp8_slices128_slots2"] = {"launch_to_drained_us": round(e2e[len(e2e) // 2], 1)}
                    del ring
        if cid == 4:
            # closed-loop FIFO stress: commands per second and push -> popped latency against the number of pushers
            fs = {}
            for threads in (1, 4):
                for pushers in (1, 16, 256, 4096):
                    per = 400 if pushers <= 256 else 50
                    with EPRunner(R, E, K, H, T, num_proxy_threads=threads, spin_timeout_ms=10000) as rf:
                        ls = torch.zeros(pushers, dtype=torch.int64, device="cuda")
                        lm = torch.zeros(pushers, dtype=torch.int64, device="cuda")
                        ep.ep_fifo_stress(rf.h, pushers, 20, ls, lm)
                        rf.wait()
                        torch.cuda.synchronize()
                        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                        a.record()
                        ep.ep_fifo_stress(rf.h, pushers, per, ls, lm)
                        b.record()
                        rf.wait()
                        torch.cuda.synchronize()
                        us = a.elapsed_time(b) * 1e3
                        fs[f"threads{threads}_pushers{pushers}"] = {
                            "Mcmd_per_s": round(pushers * per / us, 2),
                            "mean_latency_us": round(float(ls.sum().item()) / (pushers * per) / 100.0, 2),
                            "max_latency_us": round(float(lm.max().item()) / 100.0, 1)}
            res["fifo_stress"] = fs
        out[cfg.name] = res
        del recv, rq, rs, d_x, o
        torch.cuda.empty_cache()
    table = format_suite(out)
    os.makedirs(os.path.dirname(os.path.abspath(args.suite_out)), exist_ok=True)
    with open(args.suite_out, "w") as f:
        f.write(table)
    print(json.dumps({"suite": out, "table": args.suite_out}))
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=4, help="workload id (4 = the headline prefill share)")
    ap.add_argument("--payload", default=None, choices=["bf16", "fp8"])
    ap.add_argument("--cmd-mode", default=None, choices=["per_token", "chunk32", "none"])
    ap.add_argument("--proxy-threads", type=int, default=4)
    ap.add_argument("--channels", type=int, default=8)
    ap.add_argument("--ring-entries", type=int, default=4096)
    ap.add_argument("--timed-launches", type=int, default=8,
                    help="how many launches of each of ep_layout, ep_dispatch and ep_combine inside the timed "
                         "region carry HIP events that receive the kernel's own begin/end timestamps (ep_profile), "
                         "spread evenly over the steps; a timed launch costs the stream ~3 us, so timing every "
                         "call would slow the path being measured by 5 %%")
    ap.add_argument("--no-in-place", action="store_true",
                    help="skip the second, labelled measurement (identity expert in place, EP_FLAG_CACHE_HINTS)")
    ap.add_argument("--gpu-wait", action="store_true",
                    help="put ep_recv_wait between dispatch and combine: the combine kernel starts only after the "
                         "proxy's completion counters reached the GPU (the GPU->CPU->GPU loop of the paper)")
    ap.add_argument("--no-verify", action="store_true")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibrate-copy", type=int, default=0,
                    help="also launch N plain device copies of 1 GiB (counter calibration for rocprofv3 --pmc)")
    ap.add_argument("--suite", action="store_true", help="per-call timings of all five workloads instead")
    ap.add_argument("--suite-out", default=os.path.join(ROOT, "profiles", "per_call_timings_all_workloads.txt"),
                    help="where --suite writes its formatted table")
    args = ap.parse_args()
    if args.suite and args.gpus == 1:
        return run_suite(args)
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (the other EP ranks are partitions of its HBM); "
              "--gpus must be 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    import ep_inputs as g
    import paper_2512_19849_amd as ep
    from paper_2512_19849_amd.runner import EPRunner, bf16_to_bits, bits_to_bf16

    if not torch.cuda.is_available():
        print("bench.py: no HIP device; there is no CPU path", file=sys.stderr)
        return 3
    ep.load_library(build_if_missing=False)

    cfg = g.config(args.config, S=1)
    payload = args.payload or cfg.payload
    cmd_mode_name = args.cmd_mode or cfg.cmd_mode
    cmd_mode = ep.CMD_MODES[cmd_mode_name]
    T, H, K, E, R = cfg.T, cfg.H, cfg.K, cfg.E, cfg.R
    idx, w = g.routing_all(cfg)
    x = g.activations(cfg)
    rows = int((idx >= 0).sum())
    disp_bytes, comb_bytes = algorithmic_bytes(T, H, K, rows, payload)

    threads = args.proxy_threads if cmd_mode != ep.EP_CMD_NONE else 0
    r = EPRunner(R, E, K, H, T, S=1, num_channels=args.channels, ring_entries=args.ring_entries,
                 num_proxy_threads=max(threads, 0), spin_timeout_ms=10000)
    d_idx = torch.from_numpy(idx).cuda()
    d_w = torch.from_numpy(w[0]).cuda()
    d_x = bits_to_bf16(x)
    if payload == "bf16":
        recv = torch.zeros((rows, H), dtype=torch.bfloat16, device="cuda")
        scale = None
        # the experts' outputs live in a buffer of their own (filled below, before anything is timed, with what
        # identity experts would write: a copy of the received rows), so the combine reads rows that no kernel
        # of the step has touched - nothing it reads can still be in a cache
        y = torch.empty_like(recv)
    else:
        recv = torch.zeros((rows, H), dtype=torch.uint8, device="cuda")
        scale = torch.zeros((rows, H // 128), dtype=torch.float32, device="cuda")
        y = bits_to_bf16(g.activations(cfg, 0, tid=g.TID_Y, T=rows))   # expert outputs are bf16
    out = torch.zeros((T, H), dtype=torch.bfloat16, device="cuda")
    pl = ep.PAYLOADS[payload]

    def step(run=None, y_buf=None, timed=()):
        # `timed` names the calls of this step (0 layout, 1 dispatch, 2 combine) that are launched with
        # events that receive their kernels' own begin and end timestamps (ep_profile); nothing else goes
        # onto the stream
        run = run or r
        prof = lambda call, on: ep.ep_profile(run.h, on) if call in timed else None
        prof(0, True)
        lay = run.layout(d_idx)
        prof(0, False)
        prof(1, True)
        run.dispatch(d_x, d_idx[0], lay, recv, scale, payload=pl, cmd_mode=cmd_mode)
        prof(1, False)
        if args.gpu_wait and cmd_mode != ep.EP_CMD_NONE:
            run.recv_wait(None)
        prof(2, True)
        run.combine(y if y_buf is None else y_buf, d_w, lay.dst_row[0], out)
        prof(2, False)
        if cmd_mode != ep.EP_CMD_NONE:
            run.wait()
        return lay

    # measured ceilings of this device with plain streaming kernels over a buffer of the receive
    # buffer's size (best of 10 launches each), reported beside the published peak
    ceilings = {}
    probe_a = torch.zeros(rows * H * 2, dtype=torch.uint8, device="cuda")
    probe_b = torch.zeros(rows * H * 2, dtype=torch.uint8, device="cuda")
    for kind, name in ((0, "read"), (1, "write"), (2, "copy")):
        best = 1e9
        for i in range(13):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            ep.ep_bw_probe(kind, probe_a, probe_b, probe_a.numel())
            e1.record()
            torch.cuda.synchronize()
            if i >= 3:
                best = min(best, e0.elapsed_time(e1))
        ceilings[name + "_GBs"] = round(probe_a.numel() * (2 if kind == 2 else 1) / best / 1e6, 1)
    del probe_a, probe_b
    torch.cuda.empty_cache()
    # ... and of the two access patterns themselves, on this workload's own destination rows: the dispatch's
    # stores without its loads, the combine's loads without its stores (plain write and read streams are the
    # only traffic that reaches the figures above; rows scattered over expert regions do not)
    if payload == "bf16":
        lay0 = r.layout(d_idx)
        sink = torch.zeros(64, dtype=torch.uint8, device="cuda")
        for kind, name, buf in ((0, "row_scatter_write", recv), (1, "row_gather_read", y)):
            best = 1e9
            for i in range(13):
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                ep.ep_row_probe(kind, lay0.dst_row[0], K, T, 2 * H, buf, sink)
                e1.record()
                torch.cuda.synchronize()
                if i >= 3:
                    best = min(best, e0.elapsed_time(e1))
            ceilings[name + "_GBs"] = round(rows * 2 * H / best / 1e6, 1)
    if args.calibrate_copy:
        a = torch.zeros(1 << 28, dtype=torch.float32, device="cuda")
        b = torch.empty_like(a)
        for _ in range(args.calibrate_copy):
            b.copy_(a)
        torch.cuda.synchronize()
        del a, b
    if payload == "bf16":
        step(y_buf=recv)                           # fills recv ...
        torch.cuda.synchronize()
        y.copy_(recv)                              # ... and the identity experts' outputs, once, untimed
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    if cmd_mode != ep.EP_CMD_NONE:
        ep.ep_reset_stats(r.h)
    # Which calls of which steps are timed: --timed-launches launches of every kernel, spread evenly over the
    # steps; layout and combine of one step (they are not neighbours on the stream), dispatch of the next.
    n_t = min(args.timed_launches, max(1, args.steps // 2))
    plan = {}
    for i in sorted({int(j * args.steps / n_t) for j in range(n_t)}):
        plan[i] = plan.get(i, ()) + (0, 2)
        plan[(i + 1) % args.steps] = plan.get((i + 1) % args.steps, ()) + (1,)
    ep.ep_profile(r.h, 3 * n_t)  # the timed launches' events, made ahead
    ep.ep_profile(r.h, False)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        lay = step(timed=plan.get(i, ()))
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    st = r.stats()

    (lay_sum, n_lay), (disp_sum, n_disp), (comb_sum, n_comb) = (ep.ep_profile_read(r.h, c) for c in (0, 1, 2))
    nan = float("nan")
    lay_ms = lay_sum / n_lay if n_lay else nan
    disp_ms = disp_sum / n_disp if n_disp else nan
    comb_ms = comb_sum / n_comb if n_comb else nan
    total_bytes = disp_bytes + comb_bytes
    value = total_bytes / (ms_per_step * 1e-3) / 1e9

    dom = "dispatch" if (n_disp and not n_comb) or disp_ms >= comb_ms else "combine"
    dom_ms, dom_bytes = (disp_ms, disp_bytes) if dom == "dispatch" else (comb_ms, comb_bytes)
    n_timed = n_disp if dom == "dispatch" else n_comb
    achieved = dom_bytes / (dom_ms * 1e-3) / 1e9
    roofline = {"kernel": f"{dom}_{payload if dom == 'dispatch' else 'bf16'}", "bound": "hbm",
                "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": read_traffic(dom),
                "avg_launch_ms": round(dom_ms, 4), "algorithmic_bytes": dom_bytes,
                "launches_timed": n_timed}

    verified = None
    cpu_baseline = None
    if not (args.no_verify and args.no_cpu_baseline):
        from oracle import ep_oracle as oracle
        ncores = min(oracle.max_threads(), len(os.sched_getaffinity(0)), 16)
        best = {}
        parts = {}
        res = {}
        for nthr in ([1, ncores] if not args.no_cpu_baseline else [ncores]):
            oracle.set_threads(nthr)
            for rep in range(2 if not args.no_cpu_baseline else 1):
                c0 = time.perf_counter()
                olay = oracle.layout(idx, E, R)
                c1 = time.perf_counter()
                if payload == "bf16":
                    orecv, _ = oracle.dispatch_bf16(x, idx[0], olay["dst_row"][0], cfg.E_loc, rows)
                    oy = orecv
                else:
                    oq, os_, _ = oracle.dispatch_fp8(x, idx[0], olay["dst_row"][0], cfg.E_loc, rows)
                    oy = bf16_to_bits(y)
                c2 = time.perf_counter()
                oout = oracle.combine(oy, w[0], olay["dst_row"][0])
                dt = time.perf_counter() - c0
                if dt < best.get(nthr, 1e9):
                    best[nthr] = dt
                    parts[nthr] = {"layout": round((c1 - c0) * 1e3, 2), "dispatch": round((c2 - c1) * 1e3, 2),
                                   "combine": round((c0 + dt - c2) * 1e3, 2)}
            res = dict(olay=olay, oout=oout)
        if not args.no_cpu_baseline:
            cpu_baseline = {"value": round(total_bytes / best[ncores] / 1e9, 3), "unit": "GB/s", "cores": ncores,
                            "kind": "oracle",
                            "sample": f"the full {cfg.name} workload ({T} tokens), one pass of layout+dispatch+combine, "
                                      f"best of 2",
                            "value_1_thread": round(total_bytes / best[1] / 1e9, 3),
                            "ms": parts[ncores], "ms_1_thread": parts[1],
                            "tokens_per_s": round(T / best[ncores], 1)}
        if not args.no_verify:
            got = lay.numpy()
            ok = all(np.array_equal(got[k], v) for k, v in res["olay"].items())
            if payload == "bf16":
                ok = ok and np.array_equal(bf16_to_bits(recv), oy) and np.array_equal(bf16_to_bits(y), oy)
            else:
                ok = ok and np.array_equal(recv.cpu().numpy(), oq) and np.array_equal(scale.cpu().numpy(), os_)
            ok = ok and int(oracle.bf16_ulp_distance(bf16_to_bits(out), res["oout"]).max()) <= 1
            verified = bool(ok)

    # Second, labelled measurement: the identity expert IN PLACE - the combine reads the receive buffer the
    # dispatch has just written, on a handle that was told so (EP_FLAG_CACHE_HINTS): part of what it reads is
    # then served by the 256 MB memory-side cache.  Not the headline: real experts sit between the two calls.
    in_place = None
    if payload == "bf16" and not args.no_in_place:
        r2 = EPRunner(R, E, K, H, T, S=1, num_channels=args.channels, ring_entries=args.ring_entries,
                      num_proxy_threads=max(threads, 0), spin_timeout_ms=10000, flags=ep.EP_FLAG_CACHE_HINTS)
        for _ in range(args.warmup):
            step(run=r2, y_buf=recv)
        torch.cuda.synchronize()
        c0 = time.perf_counter()
        for _ in range(args.steps):
            step(run=r2, y_buf=recv)
        torch.cuda.synchronize()
        ms2 = (time.perf_counter() - c0) * 1e3 / args.steps
        r2.close()
        in_place = {"what": "same step, but the combine reads the receive buffer itself (identity expert in place) "
                            "on a handle made with EP_FLAG_CACHE_HINTS",
                    "ms_per_step": round(ms2, 4), "value": round(total_bytes / (ms2 * 1e-3) / 1e9, 1),
                    "frac_hbm_peak": round(total_bytes / (ms2 * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}
    r.close()
    line = {
        "metric": "dispatch+combine GB/s and tokens/s on 1 GPU; % of HBM peak",
        "metric_detail": "value = algorithmic bytes of dispatch + combine / time of one step; a step is one pass of "
                         "layout + dispatch (with transfer commands through the CPU proxy) + combine + wait for the "
                         "proxy's completion counters",
        "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if payload == "bf16" else "fp8_e4m3+bf16", "data": "synthetic",
        "config": {"workload": f"{cfg.name}: {T} tokens x hidden {H}, {E} experts top-{K}, {R} simulated ranks, "
                               f"{cfg.routing} routing, payload {payload}, commands {cmd_mode_name}",
                   "rows": rows, "proxy_threads": threads, "channels": args.channels, "gpu_wait": args.gpu_wait,
                   "ring_entries": args.ring_entries,
                   "expert_outputs": "own buffer (copy of the received rows, written before the timed region)"
                                     if payload == "bf16" else "own buffer (seeded bf16 rows)"},
        "tokens_per_s": round(T / (ms_per_step * 1e-3), 1),
        "frac_hbm_peak": round(value / HBM_PEAK_GBS, 4),
        "kernels_ms": {"layout": round(lay_ms, 4), "dispatch": round(disp_ms, 4), "combine": round(comb_ms, 4)},
        "kernels_gbs": {"dispatch": round(disp_bytes / disp_ms / 1e6, 1), "combine": round(comb_bytes / comb_ms / 1e6, 1)},
        "ring": {"cmds_per_step": st["cmds"] / max(1, args.steps), "gpu_ring_full": st["gpu_ring_full"],
                 "atomics_deferred": st["atomics_deferred"]},
        "measured_ceilings": ceilings,
        "ring_rate": {"Mcmd_per_s_step_average": round(st["cmds"] / max(1, args.steps) / (ms_per_step * 1e3), 2),
                      "note": "commands through the rings per step / step time; proxy-side peak rates are in "
                              "profiles/per_call_timings_all_workloads.txt"},
        "paper_context": {
            "note": "the paper's own figures, other hardware, context only - not a target",
            "absolute_kernel_path_numbers": "none in the text (plots only)",
            "fifo_rate": "about 8 M commands/s through 8 FIFOs, unbatched 7 KB messages (H200 + AWS EFA testbed and "
                         "MI300X + Broadcom Thor-2 testbed, Section 5.3)",
            "required_rate": "up to 7 M commands/s per GPU for a 400 Gb/s network with 7 KB tokens (Section 1)",
            "dispatch_latency": "EP32 dispatch 2.3x lower than PPLX, combine 1.1-1.5x lower, on 4 x (8 x H200, "
                                "16 x EFA 200G) (Section 5.2)",
            "ht_vs_deepep": "within 5 % of DeepEP on 4 x (8 x H100, 8 x ConnectX-7 400G) (Section 5.2)",
            "proxy_threads": "one proxy thread is the bottleneck, four are used everywhere (Section 5.3)"},
        "identity_expert_in_place": in_place,
        "kernels_timed_launches": {"layout": n_lay, "dispatch": n_disp, "combine": n_comb},
        "roofline": roofline, "cpu_baseline": cpu_baseline, "verified_vs_oracle": verified,
    }
    print(json.dumps(line))
    return 0


if __name__ == "__main__":
    sys.exit(main())
