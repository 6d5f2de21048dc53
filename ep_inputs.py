"""Seeded synthetic inputs for the expert-parallel dispatch/combine path.

This module only *draws inputs*: activations, gating logits, the top-k expert
choice a router would hand over, and its weights.  It contains none of the
method's arithmetic (no layout, no packing, no quantisation, no weighted sum);
both the CPU oracle's tests and the HIP path's tests/bench consume the arrays
it returns, and neither of those two imports the other.

Everything is counter based: element ``i`` of tensor ``tid`` under ``seed`` is a
pure function of ``(seed, tid, i)`` (splitmix64 -> Box-Muller), so a sub-range
can be regenerated without the rest.

Workload shapes follow the paper's description of expert-parallel traffic
(Section 1 and Section 2.1: hidden size 7168, 8 experts per token, batches of
4096 tokens, data-dependent and imbalanced routing).  bf16 values are carried
as ``uint16`` bit patterns in numpy.
"""
from __future__ import annotations

from dataclasses import dataclass, field, replace
from typing import Dict, Optional

import numpy as np

_U64 = np.uint64
_GOLDEN = _U64(0x9E3779B97F4A7C15)
_M1 = _U64(0xBF58476D1CE4E5B9)
_M2 = _U64(0x94D049BB133111EB)

# tensor ids (streams) of the counter-based generator
TID_X = 1
TID_LOGITS = 2
TID_PERM = 3
TID_ROUTE = 4
TID_WLOGITS = 5
TID_Y = 6

BASE_SEED = 20251219


def splitmix64(x: np.ndarray) -> np.ndarray:
    """One splitmix64 output step on an array of uint64 counters."""
    with np.errstate(over="ignore"):
        z = (x + _GOLDEN).astype(_U64)
        z = ((z ^ (z >> _U64(30))) * _M1).astype(_U64)
        z = ((z ^ (z >> _U64(27))) * _M2).astype(_U64)
        return (z ^ (z >> _U64(31))).astype(_U64)


def _stream_key(seed: int, tid: int) -> np.uint64:
    k = splitmix64(np.array([seed & 0xFFFFFFFFFFFFFFFF], dtype=_U64))
    with np.errstate(over="ignore"):
        k = splitmix64(k ^ (_U64(tid) * _M1))
    return k[0]


def uniform_u64(seed: int, tid: int, start: int, n: int) -> np.ndarray:
    """n raw 64-bit draws: counters start .. start+n-1 of stream (seed, tid)."""
    key = _stream_key(seed, tid)
    idx = np.arange(start, start + n, dtype=_U64)
    with np.errstate(over="ignore"):
        return splitmix64(key + idx * _GOLDEN)


def uniform01(seed: int, tid: int, start: int, n: int) -> np.ndarray:
    """float64 uniforms in (0, 1]."""
    u = uniform_u64(seed, tid, start, n)
    return ((u >> _U64(11)).astype(np.float64) + 1.0) * (1.0 / 9007199254740992.0)


def normal_f32(seed: int, tid: int, n: int, chunk: int = 1 << 22) -> np.ndarray:
    """n standard normals (float32) by Box-Muller on counter pairs (2j, 2j+1)."""
    out = np.empty(n, dtype=np.float32)
    npairs = (n + 1) // 2
    for p0 in range(0, npairs, chunk):
        p1 = min(npairs, p0 + chunk)
        u = uniform01(seed, tid, 2 * p0, 2 * (p1 - p0))
        r = np.sqrt(-2.0 * np.log(u[0::2]))
        th = (2.0 * np.pi) * u[1::2]
        z = np.empty(2 * (p1 - p0), dtype=np.float64)
        z[0::2] = r * np.cos(th)
        z[1::2] = r * np.sin(th)
        hi = min(n, 2 * p1)
        out[2 * p0:hi] = z[: hi - 2 * p0].astype(np.float32)
    return out


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (nearest, ties to even); returns uint16 bit
    patterns.  Inputs are finite.  Used only to *produce inputs*."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = u + np.uint32(0x7FFF) + lsb
    return (r >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Exact widening of bf16 bit patterns to float32."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


@dataclass(frozen=True)
class EPConfig:
    """One workload.  R ranks (simulated partitions), E experts, K = top-k,
    T tokens per source rank, H hidden, S source ranks whose routing is given."""
    name: str
    T: int
    H: int
    E: int
    K: int
    R: int
    S: int = 1
    self_rank: int = 0
    routing: str = "softmax"      # "softmax" | "zipf" | "uniform"
    zipf_identity_perm: bool = False
    payload: str = "bf16"         # "bf16" | "fp8"
    cmd_mode: str = "per_token"   # "per_token" | "chunk32" | "none"
    seed: int = BASE_SEED

    @property
    def E_loc(self) -> int:
        return self.E // self.R


# The five workloads the build is measured/tested on (index = config id).
CONFIGS: Dict[int, EPConfig] = {
    1: EPConfig("cfg1_tiny", T=64, H=1024, E=16, K=2, R=4, seed=BASE_SEED + 1),
    2: EPConfig("cfg2_ll_decode", T=128, H=7168, E=256, K=8, R=32, S=32, self_rank=0,
                seed=BASE_SEED + 2),
    3: EPConfig("cfg3_tiny_fp8", T=64, H=1024, E=16, K=2, R=4, payload="fp8", seed=BASE_SEED + 3),
    4: EPConfig("cfg4_prefill", T=4096, H=7168, E=256, K=8, R=16, routing="zipf",
                cmd_mode="chunk32", seed=BASE_SEED + 4),
    5: EPConfig("cfg5_stress", T=8192, H=4096, E=128, K=8, R=8, routing="uniform",
                cmd_mode="chunk32", seed=BASE_SEED + 5),
}


def config(cid: int, **over) -> EPConfig:
    return replace(CONFIGS[cid], **over) if over else CONFIGS[cid]


def rank_seed(cfg: EPConfig, s: int) -> int:
    return cfg.seed * 1000 + s


def activations(cfg: EPConfig, s: int = 0, tid: int = TID_X, T: Optional[int] = None) -> np.ndarray:
    """bf16(N(0,1)) activations of source rank s: uint16 [T, H]."""
    T = cfg.T if T is None else T
    z = normal_f32(rank_seed(cfg, s), tid, T * cfg.H)
    return f32_to_bf16_bits(z).reshape(T, cfg.H)


def expert_popularity_logit(cfg: EPConfig) -> np.ndarray:
    """log p_e with p_e proportional to 1/(pi(e)+1): Zipf(s=1) popularity over a
    seeded permutation pi of the experts (identity if zipf_identity_perm)."""
    if cfg.zipf_identity_perm:
        pi = np.arange(cfg.E)
    else:
        keys = uniform_u64(cfg.seed, TID_PERM, 0, cfg.E)
        pi = np.empty(cfg.E, dtype=np.int64)
        pi[np.argsort(keys, kind="stable")] = np.arange(cfg.E)
    p = 1.0 / (pi.astype(np.float64) + 1.0)
    p /= p.sum()
    return np.log(p).astype(np.float32)


def routing(cfg: EPConfig, s: int = 0, T: Optional[int] = None):
    """Router output of source rank s.

    Returns (topk_idx int32 [T,K], topk_w float32 [T,K]).  Experts of one token
    are distinct.  "softmax"/"zipf": fp32 softmax over all E logits, top-k by
    score with ties to the lower expert id, listed in descending score, weights
    renormalised over the k chosen.  "uniform": K distinct experts uniformly at
    random (partial Fisher-Yates), weights = softmax of K N(0,1) draws.
    """
    T = cfg.T if T is None else T
    E, K = cfg.E, cfg.K
    seed = rank_seed(cfg, s)
    if cfg.routing in ("softmax", "zipf"):
        logits = normal_f32(seed, TID_LOGITS, T * E).reshape(T, E)
        if cfg.routing == "zipf":
            logits = (logits + expert_popularity_logit(cfg)[None, :]).astype(np.float32)
        m = logits.max(axis=1, keepdims=True)
        ex = np.exp((logits - m).astype(np.float32)).astype(np.float32)
        sm = (ex / ex.sum(axis=1, keepdims=True, dtype=np.float32)).astype(np.float32)
        order = np.argsort(-sm, axis=1, kind="stable")[:, :K]
        w = np.take_along_axis(sm, order, axis=1).astype(np.float32)
        w = (w / w.sum(axis=1, keepdims=True, dtype=np.float32)).astype(np.float32)
        return order.astype(np.int32), w
    if cfg.routing == "uniform":
        u = uniform_u64(seed, TID_ROUTE, 0, T * K).reshape(T, K)
        perm = np.tile(np.arange(E, dtype=np.int64), (T, 1))
        rows = np.arange(T)
        for k in range(K):  # partial Fisher-Yates, vectorised over tokens
            j = k + (u[:, k] % _U64(E - k)).astype(np.int64)
            a = perm[rows, k].copy()
            perm[rows, k] = perm[rows, j]
            perm[rows, j] = a
        idx = perm[:, :K].astype(np.int32)
        wl = normal_f32(seed, TID_WLOGITS, T * K).reshape(T, K)
        ex = np.exp((wl - wl.max(axis=1, keepdims=True)).astype(np.float32)).astype(np.float32)
        w = (ex / ex.sum(axis=1, keepdims=True, dtype=np.float32)).astype(np.float32)
        return idx, w
    raise ValueError(f"unknown routing {cfg.routing!r}")


def routing_all(cfg: EPConfig, T: Optional[int] = None):
    """Routing of all S source ranks: (int32 [S,T,K], float32 [S,T,K])."""
    idx, w = zip(*(routing(cfg, s, T) for s in range(cfg.S)))
    return np.stack(idx), np.stack(w)


def mask_random(idx: np.ndarray, frac: float, seed: int) -> np.ndarray:
    """Copy of idx with about ``frac`` of the entries masked (-1): dropped
    (token, k) pairs, as a router with capacity limits would produce."""
    u = uniform01(seed, 77, 0, idx.size).reshape(idx.shape)
    out = idx.copy()
    out[u < frac] = -1
    return out


def validate_routing(idx: np.ndarray, E: int) -> None:
    """Debug validator for the contract the kernels assume: every entry is -1 or
    in [0,E), and the unmasked experts of one token are distinct."""
    a = np.asarray(idx)
    if a.dtype != np.int32:
        raise ValueError("topk_idx must be int32")
    if ((a < -1) | (a >= E)).any():
        raise ValueError("topk_idx entry outside [-1, E)")
    flat = a.reshape(-1, a.shape[-1])
    srt = np.sort(flat, axis=1)
    dup = (srt[:, 1:] == srt[:, :-1]) & (srt[:, 1:] >= 0)
    if dup.any():
        raise ValueError("a token lists the same expert twice")
