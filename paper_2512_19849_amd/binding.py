"""Thin ctypes binding of libep.so: same names as the C ABI, argument
marshalling only.  Every step of the path runs in the library's HIP kernels and
proxy threads; torch tensors are used for device memory and streams.

There is no CPU fallback: if the library is missing or no HIP device is usable
the calls raise.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

import numpy as np

from . import build as _build

EP_OK, EP_EINVAL, EP_ENOMEM, EP_ESTATE, EP_EHIP, EP_ETIMEOUT, EP_EBOUNDS = 0, -1, -2, -3, -4, -5, -6
EP_BF16, EP_FP8_E4M3 = 0, 1
EP_CMD_PER_TOKEN, EP_CMD_CHUNK32, EP_CMD_NONE, EP_CMD_CHUNK32_ORDERED = 0, 1, 2, 3
EP_CMD_ATOMICS_FIRST, EP_CMD_DRAIN, EP_CMD_NO_PLACEMENT = 0x100, 0x200, 0x400
EP_FLAG_LOG_CMDS, EP_FLAG_LOG_EVENTS, EP_FLAG_HOST_ONLY, EP_FLAG_SENDER_FENCE, EP_FLAG_CACHE_HINTS = 1, 2, 4, 8, 16
EP_OP_WRITE, EP_OP_ATOMIC, EP_OP_DRAIN, EP_OP_BARRIER, EP_OP_ORDERED_WRITE, EP_OP_ORDERED_ATOMIC = 1, 2, 3, 4, 5, 6
EP_OP_RING = 7
EP_RING_WRITE, EP_RING_TAIL, EP_RING_HEAD = 0, 1, 2

_STATUS = {0: "EP_OK", -1: "EP_EINVAL", -2: "EP_ENOMEM", -3: "EP_ESTATE", -4: "EP_EHIP", -5: "EP_ETIMEOUT",
           -6: "EP_EBOUNDS"}
PAYLOADS = {"bf16": EP_BF16, "fp8": EP_FP8_E4M3}
CMD_MODES = {"per_token": EP_CMD_PER_TOKEN, "chunk32": EP_CMD_CHUNK32, "none": EP_CMD_NONE,
             "chunk32_ordered": EP_CMD_CHUNK32_ORDERED}


class EPError(RuntimeError):
    def __init__(self, fn: str, rc: int):
        detail = ""
        if _lib is not None and rc == EP_EHIP or rc == EP_ENOMEM:
            detail = (_lib.ep_last_error() or b"").decode(errors="replace") if _lib is not None else ""
        super().__init__(f"{fn} failed: {_STATUS.get(rc, rc)}" + (f" [{detail}]" if detail else ""))
        self.rc = rc


class ep_config(C.Structure):
    _fields_ = [("num_ranks", C.c_int32), ("num_experts", C.c_int32), ("top_k", C.c_int32), ("hidden", C.c_int32),
                ("max_tokens", C.c_int32), ("num_src", C.c_int32), ("self_rank", C.c_int32),
                ("num_channels", C.c_int32), ("ring_entries", C.c_int32), ("num_proxy_threads", C.c_int32),
                ("reorder_window", C.c_int32), ("spin_timeout_ms", C.c_int32), ("reorder_seed", C.c_uint64),
                ("heap_rows", C.c_int64), ("flags", C.c_int32), ("barrier_peers", C.c_int32),
                ("barrier_name", C.c_char * 48), ("max_outstanding", C.c_int32), ("pack_rows", C.c_int32), ("pack_hold_us", C.c_int32),
                ("ht_slices", C.c_int32), ("ht_ring_slots", C.c_int32)]


class ep_stats_t(C.Structure):
    _fields_ = [(n, C.c_uint64) for n in ("cmds", "writes", "atomics", "drains", "barriers", "write_bytes", "write_rows",
                                          "atomics_applied", "atomics_deferred", "sender_held", "ordered_parked", "rejected",
                                          "write_msgs", "paced", "max_in_flight",
                                          "copy_batches", "copied_bytes", "gpu_ring_full",
                                          "first_poll_ns", "last_apply_ns")] + \
               [("per_thread_cmds", C.c_uint64 * 16), ("device_error", C.c_int32), ("proxy_error", C.c_int32)]

    def as_dict(self):
        d = {n: int(getattr(self, n)) for n, _ in self._fields_ if n != "per_thread_cmds"}
        d["per_thread_cmds"] = [int(v) for v in self.per_thread_cmds]
        return d


EXPORTS = ["ep_proxy_start", "ep_proxy_stop", "ep_layout", "ep_layout_static", "ep_dispatch", "ep_combine", "ep_fp8_unpack", "ep_recv_wait", "ep_wait",
           "ep_counters", "ep_tail_counters", "ep_barrier", "ep_dedup", "ep_gather_index", "ep_combine_partial",
           "ep_stats", "ep_reset_stats", "ep_cmd_log", "ep_event_log", "ep_host_push",
           "ep_host_check_completion", "ep_host_expect_atomics", "ep_last_error", "ep_bw_probe",
           "ep_register_heaps", "ep_ht_dispatch", "ep_ring_counters", "ep_fifo_stress", "ep_captured", "ep_expect", "ep_profile", "ep_profile_read",
           "ep_row_probe"]

_lib = None


def lib_path() -> str:
    return _build.LIB


def load_library(build_if_missing: bool = True) -> C.CDLL:
    """Load libep.so (building it only when no built library exists)."""
    global _lib
    if _lib is not None:
        return _lib
    try:
        # torch ships its own HIP runtime; it must be the one this process uses, so it has to be
        # loaded before libep.so resolves libamdhip64 (two runtimes in one process do not mix)
        import torch  # noqa: F401
    except ImportError:
        pass
    if not os.path.exists(_build.LIB):
        if not build_if_missing:
            raise FileNotFoundError(_build.LIB)
        _build.build_lib()
    L = C.CDLL(_build.LIB)
    vp, i32, i64, u32, u64 = C.c_void_p, C.c_int32, C.c_int64, C.c_uint32, C.c_uint64
    L.ep_proxy_start.argtypes = [C.POINTER(ep_config), C.POINTER(vp)]
    L.ep_proxy_stop.argtypes = [vp]
    L.ep_layout.argtypes = [vp, vp, i32] + [vp] * 8 + [vp]
    L.ep_layout_static.argtypes = [vp, i32, i32, i32, i32, i32] + [vp] * 8 + [vp, vp]
    L.ep_dispatch.argtypes = [vp, vp, vp, vp, vp, vp, i32, i32, i32, i32, i32, vp, vp, i64, vp]
    L.ep_combine.argtypes = [vp, vp, vp, vp, i32, i64, vp, vp]
    L.ep_fp8_unpack.argtypes = [vp, vp, i64, vp, vp, vp]
    L.ep_wait.argtypes = [vp]
    L.ep_barrier.argtypes = [vp, vp]
    L.ep_dedup.argtypes = [vp, vp, i32, i32, vp, vp, vp]
    L.ep_gather_index.argtypes = [vp, vp, vp, vp, i32, i64, vp, vp]
    L.ep_combine_partial.argtypes = [vp, vp, vp, vp, vp, vp, i32, i64, i64, vp, vp]
    L.ep_recv_wait.argtypes = [vp, i32, i32, vp, vp]
    L.ep_counters.argtypes = [vp, C.POINTER(vp), C.POINTER(vp)]
    L.ep_stats.argtypes = [vp, C.POINTER(ep_stats_t)]
    L.ep_tail_counters.argtypes = [vp, C.POINTER(vp)]
    L.ep_reset_stats.argtypes = [vp]
    L.ep_cmd_log.argtypes = [vp, vp, C.c_size_t, C.POINTER(C.c_size_t)]
    L.ep_event_log.argtypes = [vp, vp, C.c_size_t, C.POINTER(C.c_size_t)]
    L.ep_host_push.argtypes = [vp, i32, u32, u32, u32, u32, C.POINTER(u64)]
    L.ep_host_check_completion.argtypes = [vp, i32, u64]
    L.ep_host_expect_atomics.argtypes = [vp, i32]
    L.ep_bw_probe.argtypes = [i32, vp, vp, i64, vp]
    L.ep_row_probe.argtypes = [i32, vp, i32, i64, i32, i64, vp, vp, vp]
    L.ep_register_heaps.argtypes = [vp, vp, i64, vp, i64]
    L.ep_ht_dispatch.argtypes = [vp, vp, vp, vp, i32, i32, i32, vp, i64, vp, vp, i64, vp]
    L.ep_ring_counters.argtypes = [vp, C.POINTER(vp), C.POINTER(vp)]
    L.ep_fifo_stress.argtypes = [vp, i32, i32, vp, vp, vp]
    L.ep_captured.argtypes = [vp, C.POINTER(i64), C.POINTER(i64), i32]
    L.ep_expect.argtypes = [vp, i64, i64]
    L.ep_profile.argtypes = [vp, i32]
    L.ep_profile_read.argtypes = [vp, i32, C.POINTER(C.c_double), C.POINTER(i32), i32]
    for name in EXPORTS:
        getattr(L, name).restype = C.c_int
    L.ep_last_error.argtypes = []
    L.ep_last_error.restype = C.c_char_p
    _lib = L
    return L


def _check(fn: str, rc: int) -> None:
    if rc != EP_OK:
        raise EPError(fn, rc)


def _ptr(t) -> Optional[int]:
    """Device (or host) address of a torch tensor / numpy array / None."""
    if t is None:
        return None
    if hasattr(t, "data_ptr"):
        if not t.is_contiguous():
            raise ValueError("tensor must be contiguous")
        return t.data_ptr()
    return t.ctypes.data


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    return getattr(stream, "cuda_stream", stream)


def ep_proxy_start(num_ranks: int, num_experts: int, top_k: int, hidden: int, max_tokens: int, num_src: int = 1,
                   self_rank: int = 0, num_channels: int = 8, ring_entries: int = 4096, num_proxy_threads: int = 4,
                   reorder_window: int = 0, reorder_seed: int = 0, spin_timeout_ms: int = 0, heap_rows: int = 0,
                   flags: int = 0, barrier_peers: int = 0, barrier_name: str = "", ht_slices: int = 0,
                   ht_ring_slots: int = 0, max_outstanding: int = 0, pack_rows: int = 0,
                   pack_hold_us: int = 0) -> int:
    """Returns the opaque handle (an integer address)."""
    cfg = ep_config(num_ranks, num_experts, top_k, hidden, max_tokens, num_src, self_rank, num_channels,
                    ring_entries, num_proxy_threads, reorder_window, spin_timeout_ms, reorder_seed, heap_rows,
                    flags, barrier_peers, barrier_name.encode(), max_outstanding, pack_rows, pack_hold_us, ht_slices,
                    ht_ring_slots)
    h = C.c_void_p()
    _check("ep_proxy_start", load_library().ep_proxy_start(C.byref(cfg), C.byref(h)))
    return h.value


def ep_proxy_stop(h: int) -> None:
    _check("ep_proxy_stop", load_library().ep_proxy_stop(h))


def ep_layout(h: int, topk_idx, T: int, count, expert_total, rank_total, base, expert_offset, rank_offset, slot,
              dst_row, stream=None) -> None:
    _check("ep_layout", load_library().ep_layout(h, _ptr(topk_idx), T, _ptr(count), _ptr(expert_total),
                                                 _ptr(rank_total), _ptr(base), _ptr(expert_offset),
                                                 _ptr(rank_offset), _ptr(slot), _ptr(dst_row), _stream(stream)))


def ep_layout_static(topk_idx, S: int, T: int, K: int, E: int, R: int, count, expert_total, rank_total, base,
                     expert_offset, rank_offset, slot, dst_row, status=None, stream=None) -> None:
    """ep_layout without a handle and without any allocation (scratch in a static device array)."""
    _check("ep_layout_static", load_library().ep_layout_static(
        _ptr(topk_idx), S, T, K, E, R, _ptr(count), _ptr(expert_total), _ptr(rank_total), _ptr(base),
        _ptr(expert_offset), _ptr(rank_offset), _ptr(slot), _ptr(dst_row), _ptr(status), _stream(stream)))


def ep_dispatch(h: int, x, topk_idx, dst_row, count, base, T: int, src_rank: int, dst_rank_filter: int,
                payload: int, cmd_mode: int, recv, recv_scale, recv_rows: int, stream=None) -> None:
    _check("ep_dispatch", load_library().ep_dispatch(h, _ptr(x), _ptr(topk_idx), _ptr(dst_row), _ptr(count),
                                                     _ptr(base), T, src_rank, dst_rank_filter, payload, cmd_mode,
                                                     _ptr(recv), _ptr(recv_scale), recv_rows, _stream(stream)))


def ep_combine(h: int, y, topk_w, dst_row, T: int, y_rows: int, out, stream=None) -> None:
    _check("ep_combine", load_library().ep_combine(h, _ptr(y), _ptr(topk_w), _ptr(dst_row), T, y_rows, _ptr(out),
                                                   _stream(stream)))


def ep_fp8_unpack(h: int, msgs, rows: int, recv, recv_scale, stream=None) -> None:
    _check("ep_fp8_unpack", load_library().ep_fp8_unpack(h, _ptr(msgs), rows, _ptr(recv), _ptr(recv_scale),
                                                         _stream(stream)))


def ep_dedup(h: int, topk_idx, T: int, ranks_per_group: int, group_idx, first_k, stream=None) -> None:
    _check("ep_dedup", load_library().ep_dedup(h, _ptr(topk_idx), T, ranks_per_group, _ptr(group_idx),
                                               _ptr(first_k), _stream(stream)))


def ep_gather_index(h: int, dst_row, dst_row_g, first_k, T: int, rows: int, index, stream=None) -> None:
    _check("ep_gather_index", load_library().ep_gather_index(h, _ptr(dst_row), _ptr(dst_row_g), _ptr(first_k), T,
                                                             rows, _ptr(index), _stream(stream)))


def ep_combine_partial(h: int, y, topk_w, dst_row, first_k, dst_row_g, T: int, y_rows: int, rows_g: int, partial,
                       stream=None) -> None:
    _check("ep_combine_partial", load_library().ep_combine_partial(h, _ptr(y), _ptr(topk_w), _ptr(dst_row),
                                                                   _ptr(first_k), _ptr(dst_row_g), T, y_rows,
                                                                   rows_g, _ptr(partial), _stream(stream)))


def ep_register_heaps(h: int, src, dst) -> None:
    """src/dst: device tensors spanning the source-side and destination-side heaps, or None/None to unregister."""
    nbytes = lambda t: 0 if t is None else t.numel() * t.element_size()
    _check("ep_register_heaps", load_library().ep_register_heaps(h, _ptr(src), nbytes(src), _ptr(dst), nbytes(dst)))


def ep_barrier(h: int, stream=None) -> None:
    _check("ep_barrier", load_library().ep_barrier(h, _stream(stream)))


def ep_recv_wait(h: int, src_rank: int, dst_rank_filter: int, counts_out, stream=None) -> None:
    _check("ep_recv_wait", load_library().ep_recv_wait(h, src_rank, dst_rank_filter, _ptr(counts_out),
                                                       _stream(stream)))


def ep_wait(h: int) -> None:
    _check("ep_wait", load_library().ep_wait(h))


def ep_counters(h: int, S: int, E: int) -> np.ndarray:
    """numpy view (no copy) of the pinned-host completion counters [S, E]."""
    host, dev = C.c_void_p(), C.c_void_p()
    _check("ep_counters", load_library().ep_counters(h, C.byref(host), C.byref(dev)))
    buf = (C.c_int32 * (S * E)).from_address(host.value)
    return np.frombuffer(buf, dtype=np.int32).reshape(S, E)


def ep_ht_dispatch(h: int, x, topk_idx, dst_row, T: int, src_rank: int, ring, recv, recv_rows: int,
                   stream=None, payload: int = EP_BF16, recv_scale=None) -> None:
    _check("ep_ht_dispatch", load_library().ep_ht_dispatch(h, _ptr(x), _ptr(topk_idx), _ptr(dst_row), T, src_rank,
                                                           payload, _ptr(ring), ring.numel() * ring.element_size(),
                                                           _ptr(recv), _ptr(recv_scale), recv_rows,
                                                           _stream(stream)))


def ep_fifo_stress(h: int, pushers: int, cmds_per_pusher: int, lat_sum, lat_max, stream=None) -> None:
    _check("ep_fifo_stress", load_library().ep_fifo_stress(h, pushers, cmds_per_pusher, _ptr(lat_sum), _ptr(lat_max),
                                                           _stream(stream)))


def ep_ring_counters(h: int, S: int, slices: int, R: int):
    """numpy views (no copy) of the pinned-host tail and head counters [S, slices, R] of the ring-buffer channels."""
    tail, head = C.c_void_p(), C.c_void_p()
    _check("ep_ring_counters", load_library().ep_ring_counters(h, C.byref(tail), C.byref(head)))
    n = S * slices * R
    return tuple(np.frombuffer((C.c_int32 * n).from_address(p.value), dtype=np.int32).reshape(S, slices, R)
                 for p in (tail, head))


def ep_tail_counters(h: int, S: int, R: int) -> np.ndarray:
    """numpy view (no copy) of the pinned-host tail counters [S, R] of the ordered mode."""
    host = C.c_void_p()
    _check("ep_tail_counters", load_library().ep_tail_counters(h, C.byref(host)))
    buf = (C.c_int32 * (S * R)).from_address(host.value)
    return np.frombuffer(buf, dtype=np.int32).reshape(S, R)


def ep_stats(h: int) -> dict:
    st = ep_stats_t()
    _check("ep_stats", load_library().ep_stats(h, C.byref(st)))
    return st.as_dict()


def ep_reset_stats(h: int) -> None:
    _check("ep_reset_stats", load_library().ep_reset_stats(h))


def _log(fn_name: str, h: int) -> np.ndarray:
    fn = getattr(load_library(), fn_name)
    n = C.c_size_t(0)
    _check(fn_name, fn(h, None, 0, C.byref(n)))
    out = np.zeros((n.value, 4), np.uint32)
    if n.value:
        _check(fn_name, fn(h, out.ctypes.data, n.value, C.byref(n)))
    return out


def ep_cmd_log(h: int) -> np.ndarray:
    """uint32 [n, 4]: the commands the proxy polled."""
    return _log("ep_cmd_log", h)


def ep_event_log(h: int) -> np.ndarray:
    """uint32 [n, 4]: receiver-side trace (kind | thread << 8, source, expert, value)."""
    return _log("ep_event_log", h)


def ep_host_push(h: int, channel: int, w0: int, w1: int, w2: int, w3: int) -> int:
    idx = C.c_uint64(0)
    _check("ep_host_push", load_library().ep_host_push(h, channel, w0, w1, w2, w3, C.byref(idx)))
    return idx.value


def ep_host_check_completion(h: int, channel: int, idx: int) -> bool:
    rc = load_library().ep_host_check_completion(h, channel, idx)
    if rc < 0:
        raise EPError("ep_host_check_completion", rc)
    return bool(rc)


def ep_bw_probe(kind: int, src, dst, nbytes: int, stream=None) -> None:
    """kind 0 read src, 1 write dst, 2 copy src -> dst (plain streaming kernels, for ceilings)."""
    _check("ep_bw_probe", load_library().ep_bw_probe(kind, _ptr(src), _ptr(dst), nbytes, _stream(stream)))


def ep_row_probe(kind: int, rowmap, k: int, items: int, row_bytes: int, buf, sink, stream=None) -> None:
    """kind 0: the dispatch's stores without its loads; 1: the combine's loads without its stores (see ep_diag.h)."""
    _check("ep_row_probe", load_library().ep_row_probe(kind, _ptr(rowmap), k, items, row_bytes, buf.shape[0], _ptr(buf),
                                                       _ptr(sink), _stream(stream)))


def ep_last_error() -> str:
    return (load_library().ep_last_error() or b"").decode(errors="replace")


def ep_profile(h: int, on) -> None:
    """on: False/0 off; True/1 on; n > 1 on, with n event pairs made ahead of the launches."""
    _check("ep_profile", load_library().ep_profile(h, int(on)))


def ep_profile_read(h: int, call: int, reset: bool = True):
    """(summed kernel time in ms, launches) of the timed ep_layout (0) / ep_dispatch (1) / ep_combine (2) calls."""
    ms, n = C.c_double(0.0), C.c_int32(0)
    _check("ep_profile_read", load_library().ep_profile_read(h, call, C.byref(ms), C.byref(n), 1 if reset else 0))
    return float(ms.value), int(n.value)


def ep_captured(h: int, reset: bool = True):
    """(atomics, drains) that calls on capturing streams have put into the handle's ledger."""
    a, d = C.c_int64(0), C.c_int64(0)
    _check("ep_captured", load_library().ep_captured(h, C.byref(a), C.byref(d), 1 if reset else 0))
    return int(a.value), int(d.value)


def ep_expect(h: int, atomics: int, drains: int) -> None:
    _check("ep_expect", load_library().ep_expect(h, atomics, drains))


def ep_host_expect_atomics(h: int, n: int) -> None:
    _check("ep_host_expect_atomics", load_library().ep_host_expect_atomics(h, n))
