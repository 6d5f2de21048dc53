"""Ring-buffer communication channels of the high-throughput mode (Section 3.3,
"partial ordering") without a GPU: the oracle's channel arithmetic is pinned
against independent counts, and the real proxy (driven through ep_host_push by
an emulated sender and receiver that obey the head/tail rules) is checked with
the oracle's trace checker - which is itself shown to catch planted violations."""
import time

import numpy as np
import pytest

import ep_inputs as g


@pytest.fixture(scope="module")
def ep():
    import paper_2512_19849_amd as ep
    ep.load_library()
    return ep


def _w0(op, src, dr, le):
    return (op << 28) | (src << 20) | (dr << 12) | le


# ------------------------------------------------------------- oracle pins
@pytest.mark.parametrize("cid,T,slices,W,mask", [(1, None, 4, 2, 0.0), (1, 50, 7, 1, 0.3), (4, 700, 16, 3, 0.0),
                                                 (5, 300, 1, 4, 0.1), (2, 128, 128, 2, 0.0), (1, 3, 8, 2, 0.0)])
def test_ring_channel_arithmetic(oracle, cid, T, slices, W, mask):
    cfg = g.config(cid, S=1)
    idx, _ = g.routing_all(cfg, T)
    if mask:
        idx = g.mask_random(idx, mask, seed=3)
    idx_s = idx[0]
    T = idx_s.shape[0]
    rows = oracle.ring_channel_rows(idx_s, cfg.E_loc, cfg.R, slices)
    # independent counts: a 2-D histogram over (slice of the token, rank of the expert)
    slice_len = -(-T // slices)
    tt, kk = np.nonzero(idx_s >= 0)
    want = np.zeros((slices, cfg.R), np.int64)
    np.add.at(want, (tt // slice_len, idx_s[tt, kk] // cfg.E_loc), 1)
    assert np.array_equal(rows, want)
    # summed over slices they are the layout's rank totals
    lay = oracle.layout(idx, cfg.E, cfg.R)
    assert np.array_equal(rows.sum(axis=0), lay["rank_total"])

    cm = oracle.expected_ring_cmds(idx_s, 0, cfg.E_loc, cfg.R, cfg.H, slices, W)
    sb, rb = oracle.ring_slot_bytes(cfg.H), 2 * cfg.H
    assert sb == 128 + 32 * rb
    per = {}
    for (kind, s, r, c, seq, m, nbytes, off), mult in cm.items():
        assert mult == 1 and s == 0 and 1 <= m <= 32
        per.setdefault((c, r), {}).setdefault(kind, []).append((seq, m, nbytes, off))
    for (c, r), d in per.items():
        w, t, h = (sorted(d[k]) for k in (oracle.RING_WRITE, oracle.RING_TAIL, oracle.RING_HEAD))
        n = len(w)
        assert n == len(t) == len(h) == -(-int(rows[c, r]) // 32)
        assert [x[0] for x in w] == list(range(0, 2 * n, 2)) and [x[0] for x in t] == list(range(1, 2 * n, 2))
        assert [x[0] for x in h] == list(range(n))
        assert sum(x[1] for x in w) == sum(x[1] for x in t) == sum(x[1] for x in h) == rows[c, r]
        assert all(x[1] == 32 for x in w[:-1])                        # only the last chunk may be partial
        first = (c * cfg.R + r) * W * sb
        for i, (_, m, nbytes, off) in enumerate(w):
            assert nbytes == 128 + m * rb and off == first + (i % W) * sb
            assert off + nbytes <= oracle.ring_bytes(cfg.H, cfg.R, slices, W)
    assert set(per) == {(c, r) for c in range(slices) for r in range(cfg.R) if rows[c, r] > 0}


# ------------------------------------------------- the proxy, driven by hand
def _start(ep, **kw):
    base = dict(num_ranks=4, num_experts=16, top_k=2, hidden=1024, max_tokens=4096, num_src=1, num_channels=4,
                ring_entries=64, num_proxy_threads=2, spin_timeout_ms=2000, ht_slices=3, ht_ring_slots=2,
                flags=ep.EP_FLAG_HOST_ONLY | ep.EP_FLAG_LOG_CMDS | ep.EP_FLAG_LOG_EVENTS)
    base.update(kw)
    return ep.ep_proxy_start(**base), base


def _ring_push(ep, h, cfg, kind, c, r, seq, rows, n=0, src=0, off=None, nbytes=None):
    sb = 128 + 32 * 2 * cfg["hidden"]
    fifo = (c * cfg["num_ranks"] + r) % cfg["num_channels"]
    if kind == ep.EP_RING_WRITE:
        if off is None:
            off = ((c * cfg["num_ranks"] + r) * cfg["ht_ring_slots"] + n % cfg["ht_ring_slots"]) * sb
        if nbytes is None:
            nbytes = 128 + rows * 2 * cfg["hidden"]
        w1, w3 = (kind << 30) | ((rows - 1) << 24) | (nbytes >> 4), off >> 4
    else:
        w1, w3 = (kind << 30) | rows, 0
    return ep.ep_host_push(h, fifo, _w0(ep.EP_OP_RING, src, r, c), w1, seq, w3)


def _drain_all(ep, h, C):
    ids = [ep.ep_host_push(h, c, _w0(3, 0, 0, 0), 0, 0, 0) for c in range(C)]
    deadline = time.time() + 5
    for c, i in enumerate(ids):
        while not ep.ep_host_check_completion(h, c, i):
            assert time.time() < deadline
            time.sleep(0.0005)


def _emulate(ep, h, cfg, totals, rng, seq0=None, rseq0=None, cum0=None):
    """An emulated sender and receiver per channel: the sender announces chunk n only once the head
    counter shows chunk n - W released, the receiver releases chunk n only once the tail counter
    covers it.  Which channel moves next, and in which role, is drawn at random."""
    S, C, R, W = 1, cfg["ht_slices"], cfg["num_ranks"], cfg["ht_ring_slots"]
    tail, head = ep.ep_ring_counters(h, S, C, R)
    sent = np.zeros((C, R), int)
    taken = np.zeros((C, R), int)
    nch = -(-totals // 32)
    seq0 = np.zeros((C, R), int) if seq0 is None else seq0
    rseq0 = np.zeros((C, R), int) if rseq0 is None else rseq0
    cum0 = np.zeros((C, R), int) if cum0 is None else cum0
    deadline = time.time() + 20
    while (taken < nch).any():
        assert time.time() < deadline, "protocol stalled"
        c, r = int(rng.integers(C)), int(rng.integers(R))
        if rng.random() < 0.5:
            n = sent[c, r]
            if n < nch[c, r] and (n < W or int(head[0, c, r]) - cum0[c, r] >= 32 * (n - W + 1)):
                m = min(32, totals[c, r] - 32 * n)
                # the two messages of a chunk may enter the FIFO in either order
                a = (ep.EP_RING_WRITE, int(seq0[c, r] + 2 * n))
                b = (ep.EP_RING_TAIL, int(seq0[c, r] + 2 * n + 1))
                for kind, seq in ((a, b) if rng.random() < 0.5 else (b, a)):
                    _ring_push(ep, h, cfg, kind, c, r, seq, m, n)
                sent[c, r] += 1
        else:
            n = taken[c, r]
            if n < nch[c, r] and int(tail[0, c, r]) - cum0[c, r] >= min(32 * (n + 1), totals[c, r]):
                _ring_push(ep, h, cfg, ep.EP_RING_HEAD, c, r, int(rseq0[c, r] + n), min(32, totals[c, r] - 32 * n))
                taken[c, r] += 1
    _drain_all(ep, h, cfg["num_channels"])
    return tail, head


@pytest.mark.parametrize("window,W,threads", [(0, 2, 2), (6, 1, 1), (40, 3, 4)])
def test_ring_protocol_through_the_proxy(ep, oracle, window, W, threads):
    h, cfg = _start(ep, reorder_window=window, reorder_seed=11, ht_ring_slots=W, num_proxy_threads=threads)
    try:
        rng = np.random.default_rng(window + W)
        C, R = cfg["ht_slices"], cfg["num_ranks"]
        totals = rng.integers(0, 230, size=(C, R))
        totals[0, 0] = 0                                             # an idle channel
        totals[1, 1] = 64                                            # ends on a chunk boundary
        tail, head = _emulate(ep, h, cfg, totals, rng)
        assert np.array_equal(tail[0], totals) and np.array_equal(head[0], totals)
        st = ep.ep_stats(h)
        nch = int((-(-totals // 32)).sum())
        assert st["rejected"] == 0 and st["proxy_error"] == 0
        assert st["writes"] == nch and st["atomics"] == 2 * nch and st["write_rows"] == totals.sum()
        res = oracle.check_ring_trace(ep.ep_event_log(h), W)
        assert res["applied"] == 3 * nch
        assert res["chunks"] == {(0, c, r): -(-int(totals[c, r]) // 32) for c in range(C) for r in range(R)
                                 if totals[c, r] > 0}
        # second dispatch on the same channels: numbering and counters keep running
        totals2 = rng.integers(0, 100, size=(C, R))
        seq0, rseq0 = 2 * (-(-totals // 32)), -(-totals // 32)
        ep.ep_reset_stats(h)                                         # clears logs; ring counters are left alone
        tail, head = _emulate(ep, h, cfg, totals2, rng, seq0, rseq0, totals.copy())
        assert np.array_equal(tail[0], totals + totals2) and np.array_equal(head[0], totals + totals2)
        first = {(0, c, r): int(seq0[c, r]) for c in range(C) for r in range(R)}
        rfirst = {(0, c, r): int(rseq0[c, r]) for c in range(C) for r in range(R)}
        oracle.check_ring_trace(ep.ep_event_log(h), W, first, rfirst)
        assert ep.ep_stats(h)["proxy_error"] == 0
    finally:
        ep.ep_proxy_stop(h)


def test_ring_trace_checker_catches_planted_violations(ep, oracle):
    h, cfg = _start(ep, num_proxy_threads=1, ht_ring_slots=2)
    try:
        rng = np.random.default_rng(5)
        totals = np.full((cfg["ht_slices"], cfg["num_ranks"]), 0)
        totals[1, 2] = 150                                           # 5 chunks through 2 slots
        _emulate(ep, h, cfg, totals, rng)
        ev = ep.ep_event_log(h).reshape(-1, 4).copy()
    finally:
        ep.ep_proxy_stop(h)
    oracle.check_ring_trace(ev, 2)
    kinds = ev[:, 0] & 0xFF

    def pos(kind, seq):
        (i,) = np.nonzero((kinds == kind) & (ev[:, 3] == seq))[0][:1]
        return int(i)

    def moved(src, dst):                                             # event src re-inserted at position dst
        order = [i for i in range(len(ev)) if i != src]
        order.insert(dst, src)
        return ev[order]
    # the Write of chunk 2 shows up before chunk 0 was released: a slot overwritten while unread
    with pytest.raises(AssertionError, match="overwrite"):
        oracle.check_ring_trace(moved(pos(oracle.EV_RING_WRITE_IN, 4), pos(oracle.EV_RING_HEAD_APPLIED, 0)), 2)
    # with one slot per ring already chunk 1 must wait for the release of chunk 0
    with pytest.raises(AssertionError, match="overwrite"):
        oracle.check_ring_trace(moved(pos(oracle.EV_RING_WRITE_IN, 2), pos(oracle.EV_RING_HEAD_APPLIED, 0)), 1)
    # a chunk released before its tail update was applied: the receiver read what it had not been told about
    with pytest.raises(AssertionError, match="released before"):
        oracle.check_ring_trace(moved(pos(oracle.EV_RING_HEAD_IN, 1), pos(oracle.EV_RING_TAIL_APPLIED, 3)), 2)
    # applied out of sequence
    i, j = pos(oracle.EV_RING_WRITE_APPLIED, 2), pos(oracle.EV_RING_TAIL_APPLIED, 3)
    swapped = ev.copy()
    swapped[[i, j]] = swapped[[j, i]]
    with pytest.raises(AssertionError, match="out of order|before it was delivered"):
        oracle.check_ring_trace(swapped, 2)
    # delivered, never applied
    with pytest.raises(AssertionError, match="never applied"):
        oracle.check_ring_trace(np.delete(ev, pos(oracle.EV_RING_HEAD_APPLIED, 4), axis=0), 2)
    # delivered twice
    with pytest.raises(AssertionError, match="twice"):
        oracle.check_ring_trace(np.concatenate([ev, ev[pos(oracle.EV_RING_TAIL_IN, 1)][None]]), 2)


def test_ring_commands_are_bounds_checked(ep):
    """A Write must name a slot of its own channel's ring and carry exactly header + rows bytes
    (Section 3.2: offsets are translated and checked by the proxy before it acts)."""
    h, cfg = _start(ep, num_proxy_threads=1)
    try:
        sb = 128 + 32 * 2048
        ok0 = _ring_push(ep, h, cfg, ep.EP_RING_WRITE, 1, 2, 0, 32, 0)
        bad = [
            dict(kind=ep.EP_RING_WRITE, c=1, r=2, seq=2, rows=32, off=((1 * 4 + 3) * 2) * sb),      # slot of channel (1,3)
            dict(kind=ep.EP_RING_WRITE, c=1, r=2, seq=2, rows=32, off=((1 * 4 + 2) * 2) * sb + 16),  # not a slot start
            dict(kind=ep.EP_RING_WRITE, c=1, r=2, seq=2, rows=31, nbytes=128 + 32 * 2048),           # length != header + rows
            dict(kind=ep.EP_RING_WRITE, c=3, r=0, seq=0, rows=1),                                    # slice 3 of 3
            dict(kind=ep.EP_RING_TAIL, c=0, r=4, seq=0, rows=1),                                     # rank 4 of 4
            dict(kind=ep.EP_RING_HEAD, c=0, r=0, seq=0, rows=1, src=1),                              # source 1 of 1
            dict(kind=3, c=0, r=0, seq=0, rows=1),                                                   # no such kind
            dict(kind=ep.EP_RING_TAIL, c=0, r=0, seq=0, rows=1 << 15),                               # value beyond the immediate
        ]
        for b in bad:
            _ring_push(ep, h, cfg, **b)
        _ring_push(ep, h, cfg, ep.EP_RING_TAIL, 1, 2, 1, 32)
        _drain_all(ep, h, cfg["num_channels"])
        st = ep.ep_stats(h)
        assert st["rejected"] == len(bad) and st["writes"] == 1 and st["atomics"] == 1
        assert st["proxy_error"] == ep.EP_EBOUNDS and ok0 == 0
        tail, head = ep.ep_ring_counters(h, 1, 3, 4)
        assert tail[0, 1, 2] == 32 and tail.sum() == 32 and head.sum() == 0
    finally:
        ep.ep_proxy_stop(h)


def test_ring_sequence_gap_is_reported_by_drain(ep, oracle):
    h, cfg = _start(ep, num_proxy_threads=2, spin_timeout_ms=300)
    try:
        _ring_push(ep, h, cfg, ep.EP_RING_WRITE, 0, 1, 0, 32, 0)
        _ring_push(ep, h, cfg, ep.EP_RING_TAIL, 0, 1, 1, 32)
        _ring_push(ep, h, cfg, ep.EP_RING_TAIL, 0, 1, 3, 20)           # its Write (2) never comes
        _ring_push(ep, h, cfg, ep.EP_RING_HEAD, 0, 1, 0, 32)
        _drain_all(ep, h, cfg["num_channels"])
        tail, head = ep.ep_ring_counters(h, 1, 3, 4)
        assert tail[0, 0, 1] == 32 and head[0, 0, 1] == 32
        assert ep.ep_stats(h)["proxy_error"] == ep.EP_ESTATE
        with pytest.raises(AssertionError, match="never applied"):
            oracle.check_ring_trace(ep.ep_event_log(h), 2)
    finally:
        ep.ep_proxy_stop(h)


def test_ring_configuration_is_validated(ep):
    for kw in (dict(ht_slices=3, ht_ring_slots=0), dict(ht_slices=0, ht_ring_slots=2), dict(ht_slices=4097),
               dict(ht_ring_slots=65), dict(num_ranks=128, num_experts=128, ht_ring_slots=33),
               dict(num_proxy_threads=0)):
        with pytest.raises(ep.EPError) as ei:
            h, _ = _start(ep, **kw)
            ep.ep_proxy_stop(h)
        assert ei.value.rc == ep.EP_EINVAL
    # a handle without ring channels has no ring counters and rejects ring messages
    h, cfg = _start(ep, ht_slices=0, ht_ring_slots=0)
    try:
        with pytest.raises(ep.EPError) as ei:
            ep.ep_ring_counters(h, 1, 1, 4)
        assert ei.value.rc == ep.EP_ESTATE
        ep.ep_host_push(h, 0, _w0(ep.EP_OP_RING, 0, 0, 0), 1, 0, 0)
        _drain_all(ep, h, cfg["num_channels"])
        assert ep.ep_stats(h)["rejected"] == 1
    finally:
        ep.ep_proxy_stop(h)
