"""Device-buffer plumbing around the binding: allocates the torch tensors one
workload needs and sequences ep_layout -> ep_dispatch -> ep_combine on the
current stream.  No arithmetic of the method happens here."""
from __future__ import annotations

from dataclasses import dataclass
from typing import Optional

import numpy as np
import torch

from . import binding as ep


def bits_to_bf16(a: np.ndarray, device="cuda") -> torch.Tensor:
    """uint16 bit patterns -> torch.bfloat16 tensor on the device (a reinterpretation)."""
    return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).to(device).view(torch.bfloat16)


def bf16_to_bits(t: torch.Tensor) -> np.ndarray:
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


@dataclass
class LayoutOut:
    count: torch.Tensor
    expert_total: torch.Tensor
    rank_total: torch.Tensor
    base: torch.Tensor
    expert_offset: torch.Tensor
    rank_offset: torch.Tensor
    slot: torch.Tensor
    dst_row: torch.Tensor

    def numpy(self) -> dict:
        return {k: getattr(self, k).cpu().numpy() for k in self.__dataclass_fields__}


class EPRunner:
    """One handle plus the buffers of one workload shape."""

    def __init__(self, R: int, E: int, K: int, H: int, max_tokens: int, S: int = 1, self_rank: int = 0,
                 num_channels: int = 8, ring_entries: int = 4096, num_proxy_threads: int = 4,
                 reorder_window: int = 0, reorder_seed: int = 0, spin_timeout_ms: int = 0, heap_rows: int = 0,
                 flags: int = 0, device: str = "cuda", barrier_peers: int = 0, barrier_name: str = "",
                 ht_slices: int = 0, ht_ring_slots: int = 0, max_outstanding: int = 0, pack_rows: int = 0,
                 pack_hold_us: int = 0):
        if not torch.cuda.is_available():
            raise RuntimeError("EPRunner needs a HIP device; there is no CPU path")
        self.R, self.E, self.K, self.H, self.S, self.T_cap = R, E, K, H, S, max_tokens
        self.E_loc = E // R
        self.dev = torch.device(device)
        self.heap_rows = heap_rows or S * max_tokens * K
        self.h = ep.ep_proxy_start(R, E, K, H, max_tokens, S, self_rank, num_channels, ring_entries,
                                   num_proxy_threads, reorder_window, reorder_seed, spin_timeout_ms, heap_rows,
                                   flags, barrier_peers, barrier_name, ht_slices, ht_ring_slots, max_outstanding,
                                   pack_rows, pack_hold_us)
        self.ht_slices, self.ht_ring_slots = ht_slices, ht_ring_slots
        i32 = dict(dtype=torch.int32, device=self.dev)
        self.lay = LayoutOut(
            count=torch.zeros((S, E), **i32), expert_total=torch.zeros(E, **i32), rank_total=torch.zeros(R, **i32),
            base=torch.zeros((S, E), **i32), expert_offset=torch.zeros(E + 1, **i32),
            rank_offset=torch.zeros(R + 1, **i32), slot=torch.zeros((S, max_tokens, K), **i32),
            dst_row=torch.zeros((S, max_tokens, K), **i32))

    def close(self) -> None:
        if self.h:
            ep.ep_proxy_stop(self.h)
            self.h = 0

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()

    # ---- the three calls -------------------------------------------------
    def layout(self, topk_idx: torch.Tensor) -> LayoutOut:
        """topk_idx int32 [S,T,K] on the device."""
        S, T, K = topk_idx.shape
        assert S == self.S and K == self.K and T <= self.T_cap and topk_idx.dtype == torch.int32
        L = self.lay
        slot, dst = L.slot, L.dst_row
        if T != self.T_cap:
            slot = torch.zeros((S, T, K), dtype=torch.int32, device=self.dev)
            dst = torch.zeros((S, T, K), dtype=torch.int32, device=self.dev)
        ep.ep_layout(self.h, topk_idx, T, L.count, L.expert_total, L.rank_total, L.base, L.expert_offset,
                     L.rank_offset, slot, dst)
        return LayoutOut(L.count, L.expert_total, L.rank_total, L.base, L.expert_offset, L.rank_offset, slot, dst)

    def dispatch(self, x: torch.Tensor, topk_idx_s: torch.Tensor, lay: LayoutOut, recv: torch.Tensor,
                 recv_scale: Optional[torch.Tensor] = None, src: int = 0, rank_filter: int = -1,
                 payload: int = ep.EP_BF16, cmd_mode: int = ep.EP_CMD_NONE, recv_rows: Optional[int] = None) -> None:
        """recv_rows: rows of the destination; defaults to recv's own row count (it differs when recv is the [T]
        message rows of a per-token FP8 dispatch that the proxy forwards)."""
        T = x.shape[0]
        ep.ep_dispatch(self.h, x, topk_idx_s, lay.dst_row[src], lay.count[src], lay.base[src], T, src, rank_filter,
                       payload, cmd_mode, recv, recv_scale, recv.shape[0] if recv_rows is None else recv_rows)

    def fp8_unpack(self, msgs: torch.Tensor, recv: torch.Tensor, recv_scale: torch.Tensor) -> None:
        ep.ep_fp8_unpack(self.h, msgs, recv.shape[0], recv, recv_scale)

    def combine(self, y: torch.Tensor, topk_w_s: torch.Tensor, dst_row_s: torch.Tensor, out: torch.Tensor) -> None:
        ep.ep_combine(self.h, y, topk_w_s, dst_row_s, out.shape[0], y.shape[0], out)

    def register_heaps(self, src: Optional[torch.Tensor], dst: Optional[torch.Tensor]) -> None:
        ep.ep_register_heaps(self.h, src, dst)

    def ht_ring_bytes(self) -> int:
        return self.ht_slices * self.R * self.ht_ring_slots * (128 + 32 * 2 * self.H)

    def ht_dispatch(self, x: torch.Tensor, topk_idx_s: torch.Tensor, lay: LayoutOut, ring: torch.Tensor,
                    recv: torch.Tensor, src: int = 0, recv_scale: Optional[torch.Tensor] = None) -> None:
        payload = ep.EP_BF16 if recv_scale is None else ep.EP_FP8_E4M3
        ep.ep_ht_dispatch(self.h, x, topk_idx_s, lay.dst_row[src], x.shape[0], src, ring, recv, recv.shape[0],
                          payload=payload, recv_scale=recv_scale)

    def recv_wait(self, counts_out: Optional[torch.Tensor] = None, src: int = 0, rank_filter: int = -1) -> None:
        ep.ep_recv_wait(self.h, src, rank_filter, counts_out)

    def wait(self) -> None:
        ep.ep_wait(self.h)

    def captured(self, reset: bool = True):
        """What the ring-on launches captured into a HIP graph will push per replay: (atomics, drains)."""
        return ep.ep_captured(self.h, reset)

    def expect(self, atomics: int, drains: int) -> None:
        """Before (or right after) launching such a graph: lets wait() cover the replayed work."""
        ep.ep_expect(self.h, atomics, drains)

    def stats(self) -> dict:
        return ep.ep_stats(self.h)

    def counters(self) -> np.ndarray:
        return ep.ep_counters(self.h, self.S, self.E)
