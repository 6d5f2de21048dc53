"""numpy front end of the CPU oracle (test infrastructure, not product).

Loads ``libep_oracle.so`` (built from ``ep_oracle.c`` by ``build_oracle``) and
adds the command-stream side of the oracle, which is small enough for plain
Python: the multiset of transfer commands a dispatch must emit (Section 3.1,
"Types of TransferCmd"), a replay of a drained command log onto the oracle's
own receive buffer, and a checker for the receiver-side completion fence of
the low-latency mode (Section 3.3, "partial completion fence"), and the checkers
of the other receiver- and sender-side rules: per-channel sequence order,
ring-buffer channels with head/tail flow control (Section 3.3, "partial
ordering"), and pacing (Section 6).

Only tests, the smoke check and the benchmark's cpu_baseline leg may import
this module.  It imports nothing from the HIP package.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from collections import Counter
from typing import Dict, Iterable, List, Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ep_oracle.c")
_LIB = os.path.join(_HERE, "libep_oracle.so")
_lib = None


def build_oracle(force: bool = False) -> str:
    """Compile the C oracle with gcc.  -ffp-contract=off: no multiply-add is
    fused unless the source says fmaf."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=gnu11", "-ffp-contract=off", "-fno-fast-math", "-fopenmp",
               "-fPIC", "-shared", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build_oracle()
        L = C.CDLL(_LIB)
        i32p, u16p, u8p, f32p, f64p = (C.POINTER(C.c_int32), C.POINTER(C.c_uint16), C.POINTER(C.c_uint8),
                                       C.POINTER(C.c_float), C.POINTER(C.c_double))
        L.oracle_layout.argtypes = [i32p] + [C.c_int] * 5 + [i32p] * 8
        L.oracle_layout.restype = C.c_int
        L.oracle_dispatch_bf16.argtypes = [u16p, i32p, i32p, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int,
                                           u16p, C.c_long, u8p]
        L.oracle_dispatch_bf16.restype = C.c_int
        L.oracle_dispatch_fp8.argtypes = [u16p, i32p, i32p, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int,
                                          u8p, f32p, C.c_long, u8p]
        L.oracle_dispatch_fp8.restype = C.c_int
        L.oracle_e4m3_decode.argtypes = [C.c_uint8]
        L.oracle_e4m3_decode.restype = C.c_float
        L.oracle_e4m3_encode.argtypes = [C.c_float]
        L.oracle_e4m3_encode.restype = C.c_uint8
        L.oracle_quant_block.argtypes = [u16p, C.c_int, u8p, f32p]
        L.oracle_quant_block.restype = None
        L.oracle_quant_rows.argtypes = [u16p, C.c_int, C.c_int, u8p, f32p]
        L.oracle_quant_rows.restype = None
        L.oracle_dequant_rows.argtypes = [u8p, f32p, C.c_long, C.c_int, u16p]
        L.oracle_dequant_rows.restype = None
        L.oracle_combine.argtypes = [u16p, f32p, i32p, C.c_int, C.c_int, C.c_int, C.c_long, u16p]
        L.oracle_combine.restype = C.c_int
        L.oracle_combine_f64.argtypes = [u16p, f32p, i32p, C.c_int, C.c_int, C.c_int, C.c_long, f64p, f64p]
        L.oracle_combine_f64.restype = C.c_int
        L.oracle_f32_to_bf16.argtypes = [C.c_float]
        L.oracle_f32_to_bf16.restype = C.c_uint16
        L.oracle_bf16_to_f32.argtypes = [C.c_uint16]
        L.oracle_bf16_to_f32.restype = C.c_float
        L.oracle_dedup.argtypes = [i32p, C.c_long, C.c_int, C.c_int, C.c_int, i32p, i32p]
        L.oracle_dedup.restype = C.c_int
        L.oracle_gather_index.argtypes = [i32p, i32p, i32p, C.c_long, C.c_int, C.c_long, i32p]
        L.oracle_gather_index.restype = C.c_int
        L.oracle_combine_partial.argtypes = [u16p, f32p, i32p, i32p, i32p, C.c_int, C.c_int, C.c_int, C.c_long,
                                             C.c_long, u16p]
        L.oracle_combine_partial.restype = C.c_int
        L.oracle_set_threads.argtypes = [C.c_int]
        L.oracle_max_threads.restype = C.c_int
        L.oracle_get_threads.restype = C.c_int
        _lib = L
    return _lib


def _p(a: np.ndarray, ct):
    return a.ctypes.data_as(C.POINTER(ct))


def _c(a, dt) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=dt)


def set_threads(n: int) -> None:
    _load().oracle_set_threads(int(n))


def max_threads() -> int:
    return int(_load().oracle_max_threads())


def get_threads() -> int:
    return int(_load().oracle_get_threads())


# ------------------------------------------------------------------ layout
def layout(idx: np.ndarray, E: int, R: int) -> Dict[str, np.ndarray]:
    """idx int32 [S,T,K] (or [T,K]) -> counts, scans, slots (see ep_oracle.c)."""
    idx = _c(idx, np.int32)
    if idx.ndim == 2:
        idx = idx[None]
    S, T, K = idx.shape
    o = dict(count=np.zeros((S, E), np.int32), expert_total=np.zeros(E, np.int32),
             rank_total=np.zeros(R, np.int32), base=np.zeros((S, E), np.int32),
             expert_offset=np.zeros(E + 1, np.int32), rank_offset=np.zeros(R + 1, np.int32),
             slot=np.zeros((S, T, K), np.int32), dst_row=np.zeros((S, T, K), np.int32))
    rc = _load().oracle_layout(_p(idx, C.c_int32), S, T, K, E, R,
                               *[_p(o[n], C.c_int32) for n in ("count", "expert_total", "rank_total", "base",
                                                               "expert_offset", "rank_offset", "slot", "dst_row")])
    if rc != 0:
        raise ValueError(f"oracle_layout rejected its input (rc={rc})")
    return o


# ---------------------------------------------------------------- dispatch
def dispatch_bf16(x, idx, dst_row, E_loc: int, recv_rows: int, rank_filter: int = -1,
                  recv: Optional[np.ndarray] = None, fill: int = 0xA5A5):
    """x uint16 [T,H]; idx/dst_row int32 [T,K] -> (recv uint16 [recv_rows,H], write_count uint8)."""
    x = _c(x, np.uint16); idx = _c(idx, np.int32); dst_row = _c(dst_row, np.int32)
    T, H = x.shape
    K = idx.shape[1]
    if recv is None:
        recv = np.full((recv_rows, H), fill, np.uint16)
    wc = np.zeros(recv_rows, np.uint8)
    rc = _load().oracle_dispatch_bf16(_p(x, C.c_uint16), _p(idx, C.c_int32), _p(dst_row, C.c_int32),
                                      T, K, H, E_loc, rank_filter, _p(recv, C.c_uint16), recv_rows,
                                      _p(wc, C.c_uint8))
    if rc != 0:
        raise ValueError(f"oracle_dispatch_bf16: destination row out of range (rc={rc})")
    return recv, wc


def dispatch_fp8(x, idx, dst_row, E_loc: int, recv_rows: int, rank_filter: int = -1,
                 recv_q: Optional[np.ndarray] = None, recv_scale: Optional[np.ndarray] = None,
                 fill: int = 0xA5):
    x = _c(x, np.uint16); idx = _c(idx, np.int32); dst_row = _c(dst_row, np.int32)
    T, H = x.shape
    K = idx.shape[1]
    if recv_q is None:
        recv_q = np.full((recv_rows, H), fill, np.uint8)
    if recv_scale is None:
        recv_scale = np.full((recv_rows, H // 128), -1.0, np.float32)
    wc = np.zeros(recv_rows, np.uint8)
    rc = _load().oracle_dispatch_fp8(_p(x, C.c_uint16), _p(idx, C.c_int32), _p(dst_row, C.c_int32),
                                     T, K, H, E_loc, rank_filter, _p(recv_q, C.c_uint8),
                                     _p(recv_scale, C.c_float), recv_rows, _p(wc, C.c_uint8))
    if rc != 0:
        raise ValueError(f"oracle_dispatch_fp8: destination row out of range (rc={rc})")
    return recv_q, recv_scale, wc


def e4m3_decode(code: int) -> float:
    return float(_load().oracle_e4m3_decode(int(code)))


def e4m3_encode(y: float) -> int:
    return int(_load().oracle_e4m3_encode(C.c_float(y)))


def e4m3_encode_array(y: np.ndarray) -> np.ndarray:
    """Encode via quant-free path: element-wise oracle_e4m3_encode."""
    y = _c(y, np.float32).ravel()
    L = _load()
    return np.fromiter((L.oracle_e4m3_encode(C.c_float(v)) for v in y), dtype=np.uint8, count=y.size)


def quant_block(v_bits: np.ndarray) -> Tuple[np.ndarray, float]:
    v = _c(v_bits, np.uint16).ravel()
    q = np.zeros(v.size, np.uint8)
    s = C.c_float(0)
    _load().oracle_quant_block(_p(v, C.c_uint16), v.size, _p(q, C.c_uint8), C.byref(s))
    return q, float(s.value)


def quant_rows(x: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    x = _c(x, np.uint16)
    T, H = x.shape
    q = np.zeros((T, H), np.uint8)
    s = np.zeros((T, H // 128), np.float32)
    _load().oracle_quant_rows(_p(x, C.c_uint16), T, H, _p(q, C.c_uint8), _p(s, C.c_float))
    return q, s


def dequant_rows(q: np.ndarray, scale: np.ndarray) -> np.ndarray:
    q = _c(q, np.uint8); scale = _c(scale, np.float32)
    rows, H = q.shape
    y = np.zeros((rows, H), np.uint16)
    _load().oracle_dequant_rows(_p(q, C.c_uint8), _p(scale, C.c_float), rows, H, _p(y, C.c_uint16))
    return y


# ----------------------------------------------------------------- combine
def combine(y, w, dst_row) -> np.ndarray:
    """y uint16 [rows,H]; w float32 [T,K]; dst_row int32 [T,K] -> out uint16 [T,H]."""
    y = _c(y, np.uint16); w = _c(w, np.float32); dst_row = _c(dst_row, np.int32)
    rows, H = y.shape
    T, K = dst_row.shape
    out = np.zeros((T, H), np.uint16)
    rc = _load().oracle_combine(_p(y, C.c_uint16), _p(w, C.c_float), _p(dst_row, C.c_int32), T, K, H, rows,
                                _p(out, C.c_uint16))
    if rc != 0:
        raise ValueError("oracle_combine: row out of range")
    return out


def combine_f64(y, w, dst_row) -> Tuple[np.ndarray, np.ndarray]:
    """Plain fp64 weighted sum and the sum of |terms| (for the error bound)."""
    y = _c(y, np.uint16); w = _c(w, np.float32); dst_row = _c(dst_row, np.int32)
    rows, H = y.shape
    T, K = dst_row.shape
    out = np.zeros((T, H), np.float64)
    mag = np.zeros((T, H), np.float64)
    rc = _load().oracle_combine_f64(_p(y, C.c_uint16), _p(w, C.c_float), _p(dst_row, C.c_int32), T, K, H, rows,
                                    _p(out, C.c_double), _p(mag, C.c_double))
    if rc != 0:
        raise ValueError("oracle_combine_f64: row out of range")
    return out, mag


# ------------------------------------------------ high-throughput mode
def dedup(idx: np.ndarray, E_loc: int, ranks_per_group: int) -> Tuple[np.ndarray, np.ndarray]:
    """idx int32 [..., K] -> (group_idx, first_k), same shape (see ep_oracle.c)."""
    idx = _c(idx, np.int32)
    K = idx.shape[-1]
    g = np.zeros_like(idx)
    f = np.zeros_like(idx)
    _load().oracle_dedup(_p(idx, C.c_int32), idx.size // K, K, E_loc, ranks_per_group, _p(g, C.c_int32),
                         _p(f, C.c_int32))
    return g, f


def gather_index(dst_row, dst_row_g, first_k, rows: int) -> np.ndarray:
    dst_row = _c(dst_row, np.int32); dst_row_g = _c(dst_row_g, np.int32); first_k = _c(first_k, np.int32)
    T, K = dst_row.shape
    out = np.zeros(rows, np.int32)
    rc = _load().oracle_gather_index(_p(dst_row, C.c_int32), _p(dst_row_g, C.c_int32), _p(first_k, C.c_int32), T, K,
                                     rows, _p(out, C.c_int32))
    if rc != 0:
        raise ValueError("oracle_gather_index: row out of range")
    return out


def combine_partial(y, w, dst_row, first_k, dst_row_g, rows_g: int, fill: int = 0) -> np.ndarray:
    y = _c(y, np.uint16); w = _c(w, np.float32)
    dst_row = _c(dst_row, np.int32); first_k = _c(first_k, np.int32); dst_row_g = _c(dst_row_g, np.int32)
    rows, H = y.shape
    T, K = dst_row.shape
    partial = np.full((rows_g, H), fill, np.uint16)
    rc = _load().oracle_combine_partial(_p(y, C.c_uint16), _p(w, C.c_float), _p(dst_row, C.c_int32),
                                        _p(first_k, C.c_int32), _p(dst_row_g, C.c_int32), T, K, H, rows, rows_g,
                                        _p(partial, C.c_uint16))
    if rc != 0:
        raise ValueError("oracle_combine_partial: row out of range")
    return partial


def f32_to_bf16(a: np.ndarray) -> np.ndarray:
    a = _c(a, np.float32)
    L = _load()
    return np.fromiter((L.oracle_f32_to_bf16(C.c_float(v)) for v in a.ravel()), dtype=np.uint16,
                       count=a.size).reshape(a.shape)


def bf16_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.asarray(b, np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def bf16_ulp_distance(a_bits: np.ndarray, b_bits: np.ndarray) -> np.ndarray:
    """Distance in units of representable bf16 values between two bit patterns
    (sign-magnitude order mapped to a line; +0 and -0 coincide)."""
    def line(b):
        b = np.asarray(b, np.uint16).astype(np.int32)
        mag = b & 0x7FFF
        return np.where(b & 0x8000, -mag, mag)
    return np.abs(line(a_bits) - line(b_bits))


# ------------------------------------------------------- command stream
# TransferCmd = four 32-bit words (16 bytes, Section 3.1 "FIFO channels").
# The paper names the fields (destination peer, offsets, length, sequence)
# but not their widths; this is the reading the build uses:
#   w0: [31] lap parity  [30:28] op  [27:20] source (connection) rank
#       [19:12] destination rank  [11:0] expert index local to the destination
#   w1: Write: [31:26] rows carried - 1, [25:0] bytes to move / 16;  Atomic: value
#   w2: Write: source offset / 16
#   w3: [31] lap parity  [30:0] Write: destination offset / 16;
#                               Atomic: counter index src * E_loc + local expert
OP_WRITE, OP_ATOMIC, OP_DRAIN, OP_BARRIER, OP_ORDERED_WRITE, OP_ORDERED_ATOMIC = 1, 2, 3, 4, 5, 6
CHUNK_ROWS = 32


def row_bytes(H: int, payload: str) -> int:
    """Bytes one token occupies in a message: bf16 row, or FP8 codes plus one
    fp32 scale per 128 channels, padded to the 16-byte offset granule."""
    if payload == "bf16":
        return 2 * H
    return (H + H // 32 + 15) // 16 * 16


def fp8_message_rows(q: np.ndarray, scale: np.ndarray) -> np.ndarray:
    """FP8 rows as they travel when the proxy moves them (Section 2.1: a token is ONE ~7 KB FP8 message):
    per row the H codes, then the H/128 fp32 scales as stored (little-endian), then zero bytes up to the
    16-byte offset granule.  uint8 [rows, row_bytes(H, "fp8")]."""
    rows, H = q.shape
    assert scale.shape == (rows, H // 128) and q.dtype == np.uint8 and scale.dtype == np.float32
    out = np.zeros((rows, row_bytes(H, "fp8")), np.uint8)
    out[:, :H] = q
    out[:, H:H + H // 32] = np.ascontiguousarray(scale).view(np.uint8).reshape(rows, H // 32)
    return out


def fp8_split_messages(msgs: np.ndarray, H: int):
    """Inverse of fp8_message_rows: (codes uint8 [rows, H], scales fp32 [rows, H/128])."""
    rows = msgs.shape[0]
    assert msgs.shape[1] == row_bytes(H, "fp8")
    q = np.ascontiguousarray(msgs[:, :H])
    scale = np.ascontiguousarray(msgs[:, H:H + H // 32]).view(np.float32).reshape(rows, H // 128)
    return q, scale


def decode_cmd(words: Iterable[int]) -> Dict[str, int]:
    w0, w1, w2, w3 = (int(v) & 0xFFFFFFFF for v in words)
    return dict(gen=w0 >> 31, gen_hi=w3 >> 31, op=(w0 >> 28) & 7, src=(w0 >> 20) & 0xFF,
                dst_rank=(w0 >> 12) & 0xFF, local_expert=w0 & 0xFFF, w1=w1,
                nbytes=(w1 & 0x3FFFFFF) << 4, rows=(w1 >> 26) + 1, src_off=w2 << 4,
                dst_off=(w3 & 0x7FFFFFFF) << 4, counter=w3 & 0x7FFFFFFF)


def expected_cmds(idx_s: np.ndarray, lay: Dict[str, np.ndarray], s: int, E_loc: int, H: int,
                  payload: str, mode: str, rank_filter: int = -1) -> Counter:
    """Multiset of commands one dispatch of source rank s must push.

    per_token: one Write per valid (t,k).  chunk32: per expert one Write per
    run of <= 32 consecutive slots.  Both: one Atomic per destination expert
    carrying count[s][e] (also when it is 0), the doorbell the receiver holds
    back until that many writes arrived.  Keys are tuples
    (op, src, dst_rank, local_expert, bytes_or_value, src_off, dst_off_or_counter).
    """
    rb = row_bytes(H, payload)
    E = lay["count"].shape[1]
    out: Counter = Counter()
    T, K = idx_s.shape
    passes = lambda e: rank_filter < 0 or e // E_loc == rank_filter
    if mode == "per_token":
        for t in range(T):
            for k in range(K):
                e = int(idx_s[t, k])
                if e < 0 or not passes(e):
                    continue
                row = int(lay["dst_row"][s, t, k])
                out[(OP_WRITE, s, e // E_loc, e % E_loc, rb, t * rb, row * rb)] += 1
    elif mode == "chunk32":
        for e in range(E):
            if not passes(e):
                continue
            c = int(lay["count"][s, e]); b = int(lay["base"][s, e])
            for j in range(0, c, CHUNK_ROWS):
                n = min(CHUNK_ROWS, c - j)
                out[(OP_WRITE, s, e // E_loc, e % E_loc, n * rb, (b + j) * rb, (b + j) * rb)] += 1
    elif mode != "none":
        raise ValueError(mode)
    if mode != "none":
        for e in range(E):
            if passes(e):
                out[(OP_ATOMIC, s, e // E_loc, e % E_loc, int(lay["count"][s, e]), 0,
                     s * E_loc + e % E_loc)] += 1
    return out


def cmd_multiset(log_words: np.ndarray, ops=(OP_WRITE, OP_ATOMIC)) -> Counter:
    """Multiset (same key shape as expected_cmds) of a drained command log uint32 [n,4]."""
    out: Counter = Counter()
    for w in np.asarray(log_words, np.uint32).reshape(-1, 4):
        d = decode_cmd(w)
        if d["op"] not in ops:
            continue
        if d["op"] == OP_WRITE:
            out[(OP_WRITE, d["src"], d["dst_rank"], d["local_expert"], d["nbytes"], d["src_off"], d["dst_off"])] += 1
        else:
            out[(OP_ATOMIC, d["src"], d["dst_rank"], d["local_expert"], d["w1"], 0, d["counter"])] += 1
    return out


def replay_writes_per_token(log_words: np.ndarray, x_rows: np.ndarray, recv_rows: int,
                            fill_byte: int = 0xA5) -> Tuple[np.ndarray, np.ndarray]:
    """Apply the Write commands of a per-token log to a fresh receive buffer:
    each command moves `len` bytes from offset src_off of the packed send rows
    (x_rows: uint8 [T, row_bytes]) to offset dst_off of the receive heap.
    Shows the commands alone determine the receive buffer."""
    rb = x_rows.shape[1]
    heap = np.full(recv_rows * rb, fill_byte, np.uint8)
    hits = np.zeros(recv_rows, np.int32)
    src = np.ascontiguousarray(x_rows).reshape(-1)
    for w in np.asarray(log_words, np.uint32).reshape(-1, 4):
        d = decode_cmd(w)
        if d["op"] != OP_WRITE:
            continue
        n, so, do = d["nbytes"], d["src_off"], d["dst_off"]
        if so + n > src.size or do + n > heap.size or n % rb or do % rb or d["rows"] != n // rb:
            raise ValueError(f"command outside the registered regions: {d}")
        heap[do:do + n] = src[so:so + n]
        hits[do // rb:(do + n) // rb] += 1
    return heap.reshape(recv_rows, rb), hits


def check_chunk_cover(log_words: np.ndarray, lay: Dict[str, np.ndarray], s: int, E_loc: int, rb: int) -> None:
    """chunk32 logs: the Writes of source s must tile exactly the rows
    [base[s][e], base[s][e]+count[s][e]) of every destination expert, each chunk
    inside one expert, none longer than 32 rows."""
    E = lay["count"].shape[1]
    covered = np.zeros(int(lay["expert_offset"][E]), np.int32)
    for w in np.asarray(log_words, np.uint32).reshape(-1, 4):
        d = decode_cmd(w)
        if d["op"] != OP_WRITE or d["src"] != s:
            continue
        e = d["dst_rank"] * E_loc + d["local_expert"]
        r0, n = d["dst_off"] // rb, d["nbytes"] // rb
        assert d["dst_off"] % rb == 0 and d["nbytes"] % rb == 0 and 1 <= n <= CHUNK_ROWS and d["rows"] == n, d
        b, c = int(lay["base"][s, e]), int(lay["count"][s, e])
        assert b <= r0 and r0 + n <= b + c and (r0 - b) % CHUNK_ROWS == 0, (d, b, c)
        covered[r0:r0 + n] += 1
    want = np.zeros_like(covered)
    for e in range(E):
        b, c = int(lay["base"][s, e]), int(lay["count"][s, e])
        want[b:b + c] = 1
    assert np.array_equal(covered, want), "chunk writes do not tile the destination rows exactly once"


def check_ordered_cmds(log_words: np.ndarray, lay: Dict[str, np.ndarray], s: int, E_loc: int, rb: int,
                       first_seq: Optional[Dict[int, int]] = None) -> Dict[int, int]:
    """High-throughput-style command stream of source s (Section 3.3, "partial ordering"): per
    communication channel (s -> destination rank) the sequence numbers form one contiguous run
    (starting at first_seq[rank], default 0); every ordered Write with number n is paired with the
    ordered Atomic n + 1 whose value is the Write's row count; the Writes tile every expert's rows
    exactly once in chunks of <= 32 that start at multiples of 32 from the expert's first row; the
    Atomics of a rank add up to the rows that rank receives from s.  Returns the next sequence
    number per rank."""
    E = lay["count"].shape[1]
    R = E // E_loc
    per_rank: Dict[int, Dict[int, dict]] = {r: {} for r in range(R)}
    covered = np.zeros(int(lay["expert_offset"][E]), np.int32)
    for w in np.asarray(log_words, np.uint32).reshape(-1, 4):
        d = decode_cmd(w)
        if d["op"] not in (OP_ORDERED_WRITE, OP_ORDERED_ATOMIC) or d["src"] != s:
            continue
        seq = int(w[2])
        assert seq not in per_rank[d["dst_rank"]], f"sequence number {seq} used twice on rank {d['dst_rank']}"
        per_rank[d["dst_rank"]][seq] = d
        if d["op"] == OP_ORDERED_WRITE:
            e = d["dst_rank"] * E_loc + d["local_expert"]
            r0, n = d["dst_off"] // rb, d["nbytes"] // rb
            assert d["dst_off"] % rb == 0 and d["nbytes"] % rb == 0 and 1 <= n <= CHUNK_ROWS and d["rows"] == n, d
            b, c = int(lay["base"][s, e]), int(lay["count"][s, e])
            assert b <= r0 and r0 + n <= b + c and (r0 - b) % CHUNK_ROWS == 0, (d, b, c)
            covered[r0:r0 + n] += 1
        else:
            assert d["counter"] == s * R + d["dst_rank"], d
    want = np.zeros_like(covered)
    for e in range(E):
        b, c = int(lay["base"][s, e]), int(lay["count"][s, e])
        want[b:b + c] = 1
    assert np.array_equal(covered, want), "ordered writes do not tile the destination rows exactly once"
    nxt = {}
    for r in range(R):
        seqs = sorted(per_rank[r])
        lo = (first_seq or {}).get(r, 0)
        assert seqs == list(range(lo, lo + len(seqs))), f"rank {r}: sequence numbers are not one contiguous run"
        assert len(seqs) % 2 == 0
        total = 0
        for q in seqs[::2]:
            wr, at = per_rank[r][q], per_rank[r][q + 1]
            assert wr["op"] == OP_ORDERED_WRITE and at["op"] == OP_ORDERED_ATOMIC and at["w1"] == wr["rows"], (wr, at)
            total += wr["rows"]
        assert total == int(lay["count"][s, r * E_loc:(r + 1) * E_loc].sum())
        nxt[r] = lo + len(seqs)
    return nxt


EV_ORD_WRITE_IN, EV_ORD_ATOMIC_IN, EV_ORD_WRITE_APPLIED, EV_ORD_ATOMIC_APPLIED = 4, 5, 6, 7


def check_order_trace(events: np.ndarray, first_seq: Optional[Dict[Tuple[int, int], int]] = None) -> Dict[str, int]:
    """Receiver-side partial ordering (Section 3.3): on every communication channel (source,
    destination rank) messages are applied strictly in sequence-number order starting at
    first_seq[(source, rank)] (default 0), each exactly once and only after it was delivered; a
    message delivered ahead of its turn waits; every delivered message is eventually applied.
    Returns how many messages were applied and how many had to wait."""
    ev = np.asarray(events, np.uint32).reshape(-1, 4)
    delivered: Dict[Tuple[int, int], set] = {}
    nxt: Dict[Tuple[int, int], int] = {}
    owner: Dict[Tuple[int, int], int] = {}
    kinds: Dict[Tuple[int, int, int], int] = {}
    waited = applied = 0
    for kind_thr, src, dr, seq in ev.tolist():
        kind, thr = kind_thr & 0xFF, kind_thr >> 8
        if kind not in (EV_ORD_WRITE_IN, EV_ORD_ATOMIC_IN, EV_ORD_WRITE_APPLIED, EV_ORD_ATOMIC_APPLIED):
            continue
        key = (src, dr)
        assert owner.setdefault(key, thr) == thr, f"channel {key} handled by two threads"
        nxt.setdefault(key, (first_seq or {}).get(key, 0))
        if kind in (EV_ORD_WRITE_IN, EV_ORD_ATOMIC_IN):
            assert seq not in delivered.setdefault(key, set()), f"{key}: sequence {seq} delivered twice"
            delivered[key].add(seq)
            kinds[(src, dr, seq)] = kind
            if seq != nxt[key]:
                waited += 1
        else:
            assert seq in delivered.get(key, set()), f"{key}: sequence {seq} applied before it was delivered"
            assert kinds[(src, dr, seq)] == kind - 2, f"{key}: sequence {seq} applied as the wrong kind"
            assert seq == nxt[key], f"{key}: applied {seq}, expected {nxt[key]} (out of order)"
            nxt[key] = seq + 1
            applied += 1
    for key, got in delivered.items():
        assert all(q < nxt[key] for q in got), f"{key}: delivered but never applied: {sorted(q for q in got if q >= nxt[key])}"
    return dict(applied=applied, waited=waited)


# Receiver-side event log (one record = 4 x uint32):
#   [0] kind | thread << 8   kind 1: Write delivered (value = rows it carried)
#                            kind 2: Atomic delivered (value = X)
#                            kind 3: Atomic applied   (value = X)
#   [1] source rank   [2] global expert   [3] value
EV_WRITE, EV_ATOMIC_IN, EV_ATOMIC_APPLIED = 1, 2, 3
# Sender half: kind 14 = a message handed to the transport; [1] source, [2] destination rank,
# [3] messages this thread then had in flight to that rank.
EV_SENT = 14
# kind 15 = a count Atomic held back by the sender half (sender-side fence); [2] global expert, [3] X
EV_SENDER_HELD = 15


def check_fence_trace(events: np.ndarray, count: np.ndarray) -> Dict[str, int]:
    """Completion-fence check (Section 3.3): within the receiving thread's own
    order, an Atomic(src, e, X) may only be applied once at least X rows for
    (src, e) were delivered; rows for other experts do not count; every
    delivered atomic is applied exactly once; the final counters equal count.
    Returns how many atomics had to wait."""
    ev = np.asarray(events, np.uint32).reshape(-1, 4)
    seen: Dict[Tuple[int, int], int] = {}
    pending: Dict[Tuple[int, int], List[int]] = {}
    owner: Dict[Tuple[int, int], int] = {}
    applied: Dict[Tuple[int, int], int] = {}
    waited = 0
    for kind_thr, src, e, val in ev.tolist():
        kind, thr = kind_thr & 0xFF, kind_thr >> 8
        if EV_ORD_WRITE_IN <= kind <= EV_SENDER_HELD:
            continue                                   # records of the other protocols and of the sender half
        key = (src, e)
        assert owner.setdefault(key, thr) == thr, f"(src,expert) {key} handled by two threads"
        if kind == EV_WRITE:
            seen[key] = seen.get(key, 0) + val
        elif kind == EV_ATOMIC_IN:
            pending.setdefault(key, []).append(val)
            if seen.get(key, 0) < val:
                waited += 1
        elif kind == EV_ATOMIC_APPLIED:
            assert key in pending and val in pending[key], f"atomic applied but never delivered: {key} {val}"
            pending[key].remove(val)
            assert seen.get(key, 0) >= val, (
                f"fence violated: atomic X={val} for {key} applied after only {seen.get(key, 0)} rows")
            applied[key] = val
        else:
            raise AssertionError(f"unknown event kind {kind}")
    left = {k: v for k, v in pending.items() if v}
    assert not left, f"atomics delivered but never applied: {left}"
    S, E = count.shape
    for (src, e), val in applied.items():
        assert int(count[src, e]) == val, f"counter ({src},{e}) = {val}, layout says {int(count[src, e])}"
    return dict(waited=waited, applied=len(applied))


# ---------------------------------------------------------------------------
# High-throughput mode through ring-buffer channels (Section 3.3, "partial
# ordering": ring buffers as communication channels, head and tail values,
# chunks of typically 32 tokens).  The paper fixes neither the split into
# channels nor the message fields; the reading used:
#   * the T tokens of a source are cut into C slices of slice_len = ceil(T/C)
#     consecutive tokens; a communication channel is (source, slice, destination
#     rank) and owns a ring of W slots at the receiver;
#   * a slot holds one chunk: a 128-byte header (the destination row of each of
#     its <= 32 rows in the packed receive buffer, int32) followed by the rows;
#     slot (c, r, w) starts at ((c*R + r)*W + w) * (128 + 32*row_bytes);
#   * the n-th chunk of a channel (n from 0 within one dispatch) goes to slot
#     n mod W and carries min(32, rows - 32n) rows; the sender may write it only
#     when chunk n - W has been consumed (head), the receiver may read it only
#     when the tail covers it;
#   * messages (op 7; w0 as for every command with the slice in the local-expert
#     field; w1[31:30] kind; w2 = sequence number):
#       kind 0 Write       w1 = (rows-1) << 24 | bytes/16, w3 = slot offset/16,
#                          sequence base + 2n            (sender -> receiver)
#       kind 1 Atomic tail w1 = rows, sequence base + 2n + 1
#       kind 2 Atomic head w1 = rows, sequence rbase + n (receiver -> sender,
#                          a channel of its own in the other direction)
OP_RING = 7
RING_WRITE, RING_TAIL, RING_HEAD = 0, 1, 2
RING_HEADER_BYTES = 128


def ring_slot_bytes(H: int) -> int:
    return RING_HEADER_BYTES + CHUNK_ROWS * row_bytes(H, "bf16")


def ring_bytes(H: int, R: int, slices: int, W: int) -> int:
    return slices * R * W * ring_slot_bytes(H)


def ring_channel_rows(idx_s: np.ndarray, E_loc: int, R: int, slices: int) -> np.ndarray:
    """rows[c][r]: valid (token, k) entries of slice c whose expert lives on rank r."""
    idx_s = np.asarray(idx_s)
    T = idx_s.shape[0]
    out = np.zeros((slices, R), np.int64)
    if T == 0:
        return out
    slice_len = -(-T // slices)
    for t in range(T):
        for e in idx_s[t]:
            if e >= 0:
                out[t // slice_len, int(e) // E_loc] += 1
    return out


def decode_ring_cmd(words: Iterable[int]) -> Dict[str, int]:
    w0, w1, w2, w3 = (int(v) & 0xFFFFFFFF for v in words)
    kind = w1 >> 30
    d = dict(op=(w0 >> 28) & 7, src=(w0 >> 20) & 0xFF, dst_rank=(w0 >> 12) & 0xFF, slice=w0 & 0xFFF,
             kind=kind, seq=w2, gen=w0 >> 31, gen_hi=w3 >> 31)
    if kind == RING_WRITE:
        d.update(rows=((w1 >> 24) & 0x3F) + 1, nbytes=(w1 & 0xFFFFFF) << 4, dst_off=(w3 & 0x7FFFFFFF) << 4)
    else:
        d.update(rows=w1 & 0x3FFFFFFF, nbytes=0, dst_off=0)
    return d


def expected_ring_cmds(idx_s: np.ndarray, s: int, E_loc: int, R: int, H: int, slices: int, W: int,
                       seq_base: Optional[np.ndarray] = None, rseq_base: Optional[np.ndarray] = None,
                       payload: str = "bf16") -> Counter:
    """Multiset of the ring-mode messages of one dispatch of source s; seq_base / rseq_base [slices, R]
    are the channels' sequence numbers before the dispatch (they keep running across dispatches)."""
    rows = ring_channel_rows(idx_s, E_loc, R, slices)
    rb, sb = row_bytes(H, payload), ring_slot_bytes(H)      # the slot stride does not depend on the payload
    out: Counter = Counter()
    for c in range(slices):
        for r in range(R):
            b = int(seq_base[c, r]) if seq_base is not None else 0
            rbase = int(rseq_base[c, r]) if rseq_base is not None else 0
            n, left = 0, int(rows[c, r])
            while left > 0:
                m = min(CHUNK_ROWS, left)
                off = ((c * R + r) * W + n % W) * sb
                out[(RING_WRITE, s, r, c, b + 2 * n, m, RING_HEADER_BYTES + m * rb, off)] += 1
                out[(RING_TAIL, s, r, c, b + 2 * n + 1, m, 0, 0)] += 1
                out[(RING_HEAD, s, r, c, rbase + n, m, 0, 0)] += 1
                left -= m
                n += 1
    return out


def ring_cmd_multiset(log_words: np.ndarray) -> Counter:
    out: Counter = Counter()
    for w in np.asarray(log_words, np.uint32).reshape(-1, 4):
        d = decode_ring_cmd(w)
        if d["op"] != OP_RING:
            continue
        assert d["gen"] == d["gen_hi"]
        out[(d["kind"], d["src"], d["dst_rank"], d["slice"], d["seq"], d["rows"], d["nbytes"], d["dst_off"])] += 1
    return out


# Receiver-side events of the ring mode: [0] kind | thread << 8, [1] source,
# [2] slice << 8 | destination rank, [3] sequence number.
EV_RING_WRITE_IN, EV_RING_TAIL_IN, EV_RING_HEAD_IN = 8, 9, 10
EV_RING_WRITE_APPLIED, EV_RING_TAIL_APPLIED, EV_RING_HEAD_APPLIED = 11, 12, 13


def check_ring_trace(events: np.ndarray, W: int, first_seq: Optional[Dict[Tuple[int, int, int], int]] = None,
                     first_rseq: Optional[Dict[Tuple[int, int, int], int]] = None) -> Dict[str, int]:
    """What the ring-buffer protocol needs from the proxy, checked on the receiving thread's own log:
      * both directions of a channel are handled by one thread;
      * forward messages (Write 2n, tail Atomic 2n+1) are applied in sequence order, each once and only
        after it was delivered; likewise the head Atomics of the reverse direction;
      * no overwrite: when the Write of chunk n is delivered, the head Atomic of chunk n - W has been
        applied (the sender could not have known the slot was free otherwise);
      * no stale read: the head Atomic of chunk n is delivered only after the tail Atomic of chunk n was
        applied (the receiver consumed a chunk it had been told about);
      * nothing delivered stays unapplied.
    Sequence numbers are taken relative to first_seq / first_rseq of the channel (default 0)."""
    ev = np.asarray(events, np.uint32).reshape(-1, 4)
    fwd_in: Dict[Tuple[int, int, int], set] = {}
    rev_in: Dict[Tuple[int, int, int], set] = {}
    fwd_next: Dict[Tuple[int, int, int], int] = {}
    rev_next: Dict[Tuple[int, int, int], int] = {}
    owner: Dict[Tuple[int, int, int], int] = {}
    waited = applied = 0
    for kind_thr, src, cr, seq in ev.tolist():
        kind, thr = kind_thr & 0xFF, kind_thr >> 8
        if kind < EV_RING_WRITE_IN or kind > EV_RING_HEAD_APPLIED:
            continue
        key = (src, cr >> 8, cr & 0xFF)
        assert owner.setdefault(key, thr) == thr, f"channel {key} handled by two threads"
        f0 = (first_seq or {}).get(key, 0)
        r0 = (first_rseq or {}).get(key, 0)
        fwd_next.setdefault(key, 0)
        rev_next.setdefault(key, 0)
        if kind in (EV_RING_WRITE_IN, EV_RING_TAIL_IN):
            n = seq - f0
            assert n >= 0 and n not in fwd_in.setdefault(key, set()), f"{key}: forward {seq} delivered twice"
            assert (n % 2 == 0) == (kind == EV_RING_WRITE_IN), f"{key}: forward {seq} has the wrong kind"
            fwd_in[key].add(n)
            if n != fwd_next[key]:
                waited += 1
            if kind == EV_RING_WRITE_IN:
                chunk = n // 2
                assert rev_next[key] >= chunk - W + 1, (
                    f"{key}: chunk {chunk} written while chunk {chunk - W} was not yet released (overwrite)")
        elif kind == EV_RING_HEAD_IN:
            n = seq - r0
            assert n >= 0 and n not in rev_in.setdefault(key, set()), f"{key}: head {seq} delivered twice"
            rev_in[key].add(n)
            if n != rev_next[key]:
                waited += 1
            assert fwd_next[key] >= 2 * n + 2, f"{key}: chunk {n} released before its tail update was applied"
        elif kind in (EV_RING_WRITE_APPLIED, EV_RING_TAIL_APPLIED):
            n = seq - f0
            assert n in fwd_in.get(key, set()), f"{key}: forward {seq} applied before it was delivered"
            assert (n % 2 == 0) == (kind == EV_RING_WRITE_APPLIED), f"{key}: forward {seq} applied as the wrong kind"
            assert n == fwd_next[key], f"{key}: forward {seq} applied out of order (next {fwd_next[key] + f0})"
            fwd_next[key] = n + 1
            applied += 1
        else:
            n = seq - r0
            assert n in rev_in.get(key, set()), f"{key}: head {seq} applied before it was delivered"
            assert n == rev_next[key], f"{key}: head {seq} applied out of order (next {rev_next[key] + r0})"
            rev_next[key] = n + 1
            applied += 1
    for key, got in fwd_in.items():
        assert fwd_next[key] == len(got), f"{key}: forward messages delivered but never applied"
    for key, got in rev_in.items():
        assert rev_next[key] == len(got), f"{key}: head updates delivered but never applied"
    return dict(applied=applied, waited=waited,
                chunks={k: v // 2 for k, v in fwd_next.items()}, released=dict(rev_next))


def check_pacing_trace(events: np.ndarray, limit: int, E_loc: int) -> Dict[str, int]:
    """Pacing at the sender (Section 6, congestion control by the proxy): per proxy thread and
    destination rank, the messages handed to the transport and not yet arrived never exceed
    `limit`; every message sent arrives.  Recomputed from the send and arrival records alone (the
    in-flight figure the proxy logs with each send must agree).  Returns the peak seen."""
    ev = np.asarray(events, np.uint32).reshape(-1, 4)
    flying: Dict[Tuple[int, int], int] = {}
    peak = sent = 0
    for kind_thr, src, where, val in ev.tolist():
        kind, thr = kind_thr & 0xFF, kind_thr >> 8
        if kind == EV_SENT:
            key = (thr, where)
            flying[key] = flying.get(key, 0) + 1
            assert flying[key] == val, f"thread {thr} rank {where}: proxy counted {val} in flight, the log shows {flying[key]}"
            assert limit <= 0 or flying[key] <= limit, f"thread {thr} has {flying[key]} messages in flight to rank {where}"
            peak = max(peak, flying[key])
            sent += 1
        elif kind in (EV_WRITE, EV_ATOMIC_IN):
            key = (thr, where // E_loc)                # [2] is the global expert
        elif kind in (EV_ORD_WRITE_IN, EV_ORD_ATOMIC_IN):
            key = (thr, where)                         # [2] is the destination rank
        elif kind in (EV_RING_WRITE_IN, EV_RING_TAIL_IN, EV_RING_HEAD_IN):
            key = (thr, where & 0xFF)                  # [2] is slice << 8 | destination rank
        else:
            continue
        if kind != EV_SENT:
            assert flying.get(key, 0) > 0, f"arrival at rank {key[1]} (thread {thr}) of a message never sent"
            flying[key] -= 1
    left = {k: v for k, v in flying.items() if v}
    assert not left, f"messages sent but never arrived: {left}"
    return dict(peak=peak, sent=sent)
