"""Pins for the oracle's layout and bf16 dispatch (CPU only).

The paper prints no worked values for these steps, so the oracle is pinned by a
hand-worked example, by library routines that compute the same thing another
way (bincount, stable argsort = counting sort), by brute force on small inputs,
by invariants, and by special cases.
"""
import os

import numpy as np
import pytest

import ep_inputs as g

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _read_hand_example():
    vals, cur = {}, None
    for line in open(os.path.join(GOLD, "layout_hand_example.txt")):
        line = line.split("#")[0].strip()
        if not line:
            continue
        tok = line.split()
        if tok[0].isalpha() or "_" in tok[0]:
            cur = tok[0]
            vals[cur] = [int(v) for v in tok[1:]]
        else:
            vals[cur] += [int(v) for v in tok]
    return vals


def test_layout_hand_example(oracle):
    v = _read_hand_example()
    S, T, K, E, R = (v[n][0] for n in "STKER")
    idx = np.array(v["idx"], np.int32).reshape(S, T, K)
    lay = oracle.layout(idx, E, R)
    assert lay["count"].ravel().tolist() == v["count"]
    assert lay["expert_total"].tolist() == v["expert_total"]
    assert lay["rank_total"].tolist() == v["rank_total"]
    assert lay["expert_offset"].tolist() == v["expert_offset"]
    assert lay["rank_offset"].tolist() == v["rank_offset"]
    assert lay["base"].ravel().tolist() == v["base"]
    assert lay["slot"].ravel().tolist() == v["slot"]
    assert lay["dst_row"].ravel().tolist() == v["dst_row"]


def _library_layout(idx, E, R):
    """Same quantities from numpy library routines: bincount, cumsum and the
    inverse of a stable argsort keyed by (expert, source, token)."""
    S, T, K = idx.shape
    valid = idx >= 0
    count = np.stack([np.bincount(idx[s][valid[s]], minlength=E) for s in range(S)])
    expert_total = count.sum(0)
    expert_offset = np.concatenate([[0], np.cumsum(expert_total)])
    flat_e = idx.reshape(-1)
    pos = np.flatnonzero(flat_e >= 0)          # already ordered by (s, t, k)
    order = pos[np.argsort(flat_e[pos], kind="stable")]
    dst = np.full(flat_e.shape, -1, np.int64)
    dst[order] = np.arange(order.size)
    return count, expert_total, expert_offset, dst.reshape(S, T, K)


@pytest.mark.parametrize("cid,T", [(1, None), (2, 64), (4, 512), (5, 700)])
def test_layout_matches_library_counting_sort(oracle, cid, T):
    cfg = g.config(cid)
    idx, _ = g.routing_all(cfg, T)
    lay = oracle.layout(idx, cfg.E, cfg.R)
    count, etot, eoff, dst = _library_layout(idx, cfg.E, cfg.R)
    assert np.array_equal(lay["count"], count)
    assert np.array_equal(lay["expert_total"], etot)
    assert np.array_equal(lay["expert_offset"], eoff)
    assert np.array_equal(lay["dst_row"], dst)
    E_loc = cfg.E_loc
    assert np.array_equal(lay["rank_total"], etot.reshape(cfg.R, E_loc).sum(1))
    assert np.array_equal(lay["rank_offset"][:-1], eoff[:-1:E_loc])
    assert lay["rank_offset"][-1] == eoff[-1]


def test_layout_brute_force_and_invariants(oracle):
    cfg = g.config(1)
    idx, _ = g.routing_all(g.config(1, S=3))
    idx = g.mask_random(idx, 0.15, seed=5)
    S, T, K = idx.shape
    lay = oracle.layout(idx, cfg.E, cfg.R)
    # brute force: slot = number of earlier (t', any k') of the same source with the same expert
    for s in range(S):
        for t in range(T):
            for k in range(K):
                e = idx[s, t, k]
                if e < 0:
                    assert lay["slot"][s, t, k] == -1 and lay["dst_row"][s, t, k] == -1
                    continue
                want = sum(1 for t2 in range(t) for k2 in range(K) if idx[s, t2, k2] == e)
                assert lay["slot"][s, t, k] == want
                # brute-force base: all rows of smaller experts, then smaller sources of this expert
                b = int((idx[idx >= 0] < e).sum()) + int((idx[:s] == e).sum())
                assert lay["base"][s, e] == b
                assert lay["dst_row"][s, t, k] == b + want
    nvalid = int((idx >= 0).sum())
    assert lay["count"].sum() == nvalid
    rows = lay["dst_row"][idx >= 0]
    assert sorted(rows.tolist()) == list(range(nvalid))           # bijection onto [0, rows)
    # rows of expert e occupy [expert_offset[e], expert_offset[e+1]) ascending in (s, t)
    for e in range(cfg.E):
        r = lay["dst_row"][idx == e]
        assert np.array_equal(r, np.arange(lay["expert_offset"][e], lay["expert_offset"][e + 1]))


def test_layout_counts_sum_to_tokens_times_k(oracle):
    for cid in (1, 2, 4, 5):
        cfg = g.config(cid)
        idx, _ = g.routing_all(cfg, min(cfg.T, 256))
        lay = oracle.layout(idx, cfg.E, cfg.R)
        assert int(lay["count"].sum()) == idx.shape[0] * idx.shape[1] * cfg.K
        assert lay["rank_offset"][-1] == lay["expert_offset"][-1] == idx.size


def test_layout_special_cases(oracle):
    T = 37
    # one expert, k = 1: identity placement
    lay = oracle.layout(np.zeros((1, T, 1), np.int32), 1, 1)
    assert np.array_equal(lay["dst_row"].ravel(), np.arange(T))
    # all tokens to one expert of many; the others are empty
    idx = np.full((1, T, 1), 5, np.int32)
    lay = oracle.layout(idx, 8, 4)
    assert lay["count"][0].tolist() == [0, 0, 0, 0, 0, T, 0, 0]
    assert lay["rank_total"].tolist() == [0, 0, T, 0]
    assert np.array_equal(lay["dst_row"].ravel(), np.arange(T))
    assert lay["expert_offset"].tolist() == [0] * 6 + [T] * 3
    # single rank
    cfg = g.config(1)
    idx, _ = g.routing_all(cfg)
    lay = oracle.layout(idx, cfg.E, 1)
    assert lay["rank_total"].tolist() == [cfg.T * cfg.K] and lay["rank_offset"].tolist() == [0, cfg.T * cfg.K]
    # everything masked
    lay = oracle.layout(np.full((2, 5, 3), -1, np.int32), 4, 2)
    assert lay["count"].sum() == 0 and (lay["dst_row"] == -1).all() and lay["rank_offset"].tolist() == [0, 0, 0]
    # T = 0
    lay = oracle.layout(np.zeros((1, 0, 2), np.int32), 4, 2)
    assert lay["expert_offset"].tolist() == [0] * 5


def test_layout_rejects_bad_input(oracle):
    with pytest.raises(ValueError):
        oracle.layout(np.array([[[0, 9]]], np.int32), 4, 2)
    with pytest.raises(ValueError):
        oracle.layout(np.array([[[0, 1]]], np.int32), 5, 2)       # E % R != 0


def test_layout_is_stable_by_source_then_token(oracle):
    """Slot order inside an expert is (source rank, token): swapping two
    tokens' routing swaps their rows."""
    idx = np.array([[[1], [1], [0]], [[1], [0], [1]]], np.int32)
    lay = oracle.layout(idx, 2, 1)
    assert lay["dst_row"][:, :, 0].tolist() == [[2, 3, 0], [4, 1, 5]]


# ------------------------------------------------------------------ dispatch
@pytest.mark.parametrize("cid,T", [(1, None), (4, 96), (5, 100)])
def test_dispatch_equals_library_permutation(oracle, cid, T):
    cfg = g.config(cid)
    idx, _ = g.routing(cfg, 0, T)
    x = g.activations(cfg, 0, T=T)
    lay = oracle.layout(idx, cfg.E, cfg.R)
    rows = idx.size
    recv, wc = oracle.dispatch_bf16(x, idx, lay["dst_row"][0], cfg.E_loc, rows)
    # library pin: repeat every token K times, reorder by a stable sort of the expert ids
    want = np.repeat(x, cfg.K, axis=0)[np.argsort(idx.reshape(-1), kind="stable")]
    assert np.array_equal(recv, want)
    assert (wc == 1).all()
    # element definition
    for t in range(0, idx.shape[0], 7):
        for k in range(cfg.K):
            assert np.array_equal(recv[lay["dst_row"][0, t, k]], x[t])


def test_dispatch_masked_filter_and_sentinel(oracle):
    cfg = g.config(1)
    idx, _ = g.routing(cfg)
    idx = g.mask_random(idx, 0.3, seed=9)
    x = g.activations(cfg)
    lay = oracle.layout(idx, cfg.E, cfg.R)
    nvalid = int((idx >= 0).sum())
    cap = nvalid + 5                              # spare rows stay untouched
    recv, wc = oracle.dispatch_bf16(x, idx, lay["dst_row"][0], cfg.E_loc, cap)
    assert (wc[:nvalid] == 1).all() and (wc[nvalid:] == 0).all()
    assert (recv[nvalid:] == 0xA5A5).all()
    # only rank 2's partition is written under the filter
    recv2, wc2 = oracle.dispatch_bf16(x, idx, lay["dst_row"][0], cfg.E_loc, cap, rank_filter=2)
    lo, hi = lay["rank_offset"][2], lay["rank_offset"][3]
    assert (wc2[lo:hi] == 1).all() and wc2.sum() == hi - lo
    assert np.array_equal(recv2[lo:hi], recv[lo:hi])
    assert (recv2[:lo] == 0xA5A5).all() and (recv2[hi:] == 0xA5A5).all()


def test_dispatch_rejects_row_outside_buffer(oracle):
    cfg = g.config(1)
    idx, _ = g.routing(cfg)
    x = g.activations(cfg)
    lay = oracle.layout(idx, cfg.E, cfg.R)
    with pytest.raises(ValueError):
        oracle.dispatch_bf16(x, idx, lay["dst_row"][0], cfg.E_loc, idx.size - 1)


def test_each_token_lands_once_per_chosen_expert(oracle):
    cfg = g.config(2)
    idx, _ = g.routing_all(cfg, 32)
    lay = oracle.layout(idx, cfg.E, cfg.R)
    S, T, K = idx.shape
    owner = np.full(idx.size, -1, np.int64)
    ids = np.arange(idx.size).reshape(idx.shape)
    owner[lay["dst_row"].ravel()] = ids.ravel()
    assert (owner >= 0).all()
    # row r belongs to expert e iff expert_offset[e] <= r < expert_offset[e+1]
    e_of_row = np.searchsorted(lay["expert_offset"], np.arange(idx.size), side="right") - 1
    assert np.array_equal(e_of_row[lay["dst_row"].ravel()], idx.ravel())
