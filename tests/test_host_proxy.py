"""Host logic of libep.so without a GPU: the library loads and exports what the
header declares, and the ring + proxy (Poll/Pop, bounds check, immediates,
completion fence, Drain, back-pressure) behave as Section 3 of the paper
describes.  The producer is ep_host_push, which speaks the same slot protocol
as the kernels' device-side Push."""
import os
import re
import threading
import time

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def ep():
    import paper_2512_19849_amd as ep
    ep.load_library()
    return ep


def test_library_exports_every_declared_symbol(ep):
    hdr = "".join(open(os.path.join(ROOT, "include", f)).read() for f in ("ep.h", "ep_diag.h"))
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    names = set(re.findall(r"\b(ep_[a-z0-9_]+)\s*\(", hdr))
    assert {"ep_proxy_start", "ep_proxy_stop", "ep_layout", "ep_dispatch", "ep_combine"} <= names
    lib = ep.load_library()
    for n in sorted(names):
        assert getattr(lib, n) is not None, n
    assert names == set(ep.EXPORTS)


def _w0(op, src, dr, le):
    return (op << 28) | (src << 20) | (dr << 12) | le


def _write(ep, h, ch, src, dr, le, rows, rb, row0):
    off = row0 * rb
    return ep.ep_host_push(h, ch, _w0(1, src, dr, le), ((rows - 1) << 26) | ((rows * rb) >> 4), off >> 4, off >> 4)


def _atomic(ep, h, ch, src, dr, le, value, E_loc):
    return ep.ep_host_push(h, ch, _w0(2, src, dr, le), value, 0, src * E_loc + le)


def _start(ep, **kw):
    base = dict(num_ranks=4, num_experts=16, top_k=2, hidden=1024, max_tokens=4096, num_src=2, num_channels=4,
                ring_entries=64, num_proxy_threads=2, spin_timeout_ms=2000,
                flags=ep.EP_FLAG_HOST_ONLY | ep.EP_FLAG_LOG_CMDS | ep.EP_FLAG_LOG_EVENTS)
    base.update(kw)
    return ep.ep_proxy_start(**base)


def test_compute_calls_refuse_a_host_only_handle(ep):
    h = _start(ep)
    try:
        lib = ep.load_library()
        assert lib.ep_layout(h, None, 0, *([None] * 8), None) == ep.EP_ESTATE
        assert lib.ep_combine(h, None, None, None, 0, 0, None, None) == ep.EP_ESTATE
        assert lib.ep_dispatch(h, None, None, None, None, None, 0, 0, -1, 0, 2, None, None, 0, None) == ep.EP_ESTATE
    finally:
        ep.ep_proxy_stop(h)


@pytest.mark.parametrize("window", [0, 4, 64])
@pytest.mark.parametrize("atomics_first", [False, True])
def test_completion_fence_under_reordering(ep, oracle, window, atomics_first):
    E, R, E_loc, C, rb = 16, 4, 4, 4, 2048
    rng = np.random.default_rng(window * 2 + atomics_first)
    count = rng.integers(0, 40, size=(2, E)).astype(np.int32)
    count[0, 3] = 0
    h = _start(ep, reorder_window=window, reorder_seed=11)
    try:
        ep.ep_host_expect_atomics(h, 2 * E)
        row = 0
        jobs = []
        for s in range(2):
            for e in range(E):
                dr, le = e // E_loc, e % E_loc
                ws = []
                left = int(count[s, e])
                while left:
                    n = min(32, left, int(rng.integers(1, 33)))
                    ws.append(("w", s, dr, le, n, row))
                    row += n
                    left -= n
                a = [("a", s, dr, le, int(count[s, e]))]
                jobs.append((a + ws) if atomics_first else (ws + a))
        order = rng.permutation(len(jobs))
        for j in order:                                         # per (src, expert) order kept, experts interleaved
            for item in jobs[j]:
                ch = item[2] % C
                if item[0] == "w":
                    _write(ep, h, ch, item[1], item[2], item[3], item[4], rb, item[5])
                else:
                    _atomic(ep, h, ch, item[1], item[2], item[3], item[4], E_loc)
        ep.ep_wait(h)
        st = ep.ep_stats(h)
        assert st["rejected"] == 0 and st["proxy_error"] == 0
        assert st["atomics_applied"] == 2 * E and st["write_rows"] == int(count.sum())
        assert np.array_equal(ep.ep_counters(h, 2, E), count)
        res = oracle.check_fence_trace(ep.ep_event_log(h), count)
        assert res["applied"] == 2 * E and res["waited"] == st["atomics_deferred"]
        if atomics_first and window == 0:
            assert res["waited"] == int((count > 0).sum())      # every non-empty expert's atomic had to wait
        if not atomics_first and window == 0:
            assert res["waited"] == 0                           # in-order delivery: never early
    finally:
        ep.ep_proxy_stop(h)


def test_fifo_order_wraparound_and_backpressure(ep, oracle):
    """10 000 commands through 8-slot rings: nothing lost or overwritten, order
    inside a channel is the push order, Idx is the sequence number, and the
    producer has to wait for the consumer (stall count > 0)."""
    C, n = 2, 5000
    h = _start(ep, num_channels=C, ring_entries=8, num_proxy_threads=2, num_src=1)
    try:
        for i in range(n):
            for ch in range(C):
                idx = ep.ep_host_push(h, ch, _w0(1, 0, ch, 0), (0 << 26) | (2048 >> 4), i, (i % 1000) * 128)
                assert idx == i
        for ch in range(C):
            deadline = time.time() + 5
            while not ep.ep_host_check_completion(h, ch, n - 1):
                assert time.time() < deadline
                time.sleep(0.001)
            assert ep.ep_host_check_completion(h, ch, 0) and not ep.ep_host_check_completion(h, ch, n)
        log = ep.ep_cmd_log(h)
        assert len(log) == C * n
        for ch in range(C):
            mine = log[((log[:, 0] >> 12) & 0xFF) == ch]
            assert np.array_equal(mine[:, 2], np.arange(n, dtype=np.uint32))      # w2 carried the push index
            gens = (mine[:, 0] >> 31).astype(np.int64)
            assert np.array_equal(gens, ((np.arange(n) // 8) & 1) ^ 1)              # lap parity alternates per lap
            assert np.array_equal(mine[:, 0] >> 31, mine[:, 3] >> 31)
        st = ep.ep_stats(h)
        assert st["cmds"] == C * n and st["gpu_ring_full"] > 0 and st["rejected"] == 0
    finally:
        ep.ep_proxy_stop(h)


def test_concurrent_producers_share_a_channel(ep):
    h = _start(ep, num_channels=1, ring_entries=16, num_proxy_threads=1, num_src=1)
    try:
        n, nthr = 2000, 4
        seen = [[] for _ in range(nthr)]

        def work(k):
            for i in range(n):
                seen[k].append(ep.ep_host_push(h, 0, _w0(1, 0, 0, k), 2048 >> 4, i, 0))
        ts = [threading.Thread(target=work, args=(k,)) for k in range(nthr)]
        [t.start() for t in ts]
        [t.join() for t in ts]
        allidx = sorted(i for s in seen for i in s)
        assert allidx == list(range(n * nthr))                   # every Idx handed out exactly once
        deadline = time.time() + 5
        while not ep.ep_host_check_completion(h, 0, n * nthr - 1):
            assert time.time() < deadline
            time.sleep(0.001)
        log = ep.ep_cmd_log(h)
        assert len(log) == n * nthr
        for k in range(nthr):                                    # each producer's own commands stay in order
            mine = log[(log[:, 0] & 0xFFF) == k]
            assert np.array_equal(mine[:, 2], np.arange(n, dtype=np.uint32))
    finally:
        ep.ep_proxy_stop(h)


def test_bounds_check_rejects_bad_commands(ep):
    """Offsets are translated against the registered heap and checked
    (Section 3.2, "Symmetric memory"); bad field values are rejected too."""
    heap_rows, H = 100, 1024
    heap = heap_rows * 2 * H
    h = _start(ep, heap_rows=heap_rows, num_src=1)
    try:
        good = ep.ep_host_push(h, 0, _w0(1, 0, 0, 0), 2048 >> 4, 0, (heap - 2048) >> 4)
        bad = [
            (_w0(1, 0, 0, 0), 2048 >> 4, 0, (heap - 2048 + 16) >> 4),     # destination runs past the heap
            (_w0(1, 0, 0, 0), 2048 >> 4, (4096 * 2 * H - 1024) >> 4, 0),  # source runs past a source's max_tokens rows
            (_w0(1, 0, 0, 0), 0, 0, 0),                                   # zero length
            (_w0(1, 1, 0, 0), 2048 >> 4, 0, 0),                           # source rank 1 of 1
            (_w0(1, 0, 4, 0), 2048 >> 4, 0, 0),                           # destination rank 4 of 4
            (_w0(1, 0, 0, 4), 2048 >> 4, 0, 0),                           # local expert 4 of 4
            (_w0(2, 0, 1, 2), 5, 0, 3),                                   # atomic whose counter index is not src*E_loc+le
            (_w0(2, 0, 1, 2), 1 << 19, 0, 2),                             # atomic value too large for the immediate
            (_w0(7, 0, 0, 0), 0, 0, 0),                                   # no such command type
        ]
        for w in bad:
            ep.ep_host_push(h, 0, *w)
        last = ep.ep_host_push(h, 0, _w0(1, 0, 0, 0), 2048 >> 4, 0, 0)
        deadline = time.time() + 5
        while not ep.ep_host_check_completion(h, 0, last):
            assert time.time() < deadline
            time.sleep(0.001)
        st = ep.ep_stats(h)
        assert st["rejected"] == len(bad) and st["writes"] == 2 and st["proxy_error"] == ep.EP_EBOUNDS
        assert good == 0
        ep.ep_host_expect_atomics(h, 1)
        with pytest.raises(ep.EPError) as ei:
            ep.ep_wait(h)
        assert ei.value.rc == ep.EP_EBOUNDS
    finally:
        ep.ep_proxy_stop(h)


def test_drain_completes_everything_in_flight(ep, oracle):
    """With a large reordering window nothing is delivered until the window
    overflows; a Drain forces every outstanding notice to land before it pops."""
    E_loc = 4
    h = _start(ep, reorder_window=1000, num_channels=1, num_proxy_threads=1, num_src=1)
    try:
        ep.ep_host_expect_atomics(h, 1)
        _atomic(ep, h, 0, 0, 2, 1, 5, E_loc)
        for i in range(5):
            _write(ep, h, 0, 0, 2, 1, 1, 2048, i)
        d = ep.ep_host_push(h, 0, _w0(3, 0, 0, 0), 0, 0, 0)
        deadline = time.time() + 5
        while not ep.ep_host_check_completion(h, 0, d):
            assert time.time() < deadline
            time.sleep(0.0005)
        st = ep.ep_stats(h)
        assert st["drains"] == 1 and st["atomics_applied"] == 1
        ev = ep.ep_event_log(h)
        ev = ev[(ev[:, 0] & 0xFF) != oracle.EV_SENT]                   # receiver-half records only
        assert len(ev) == 5 + 1 + 1
        count = np.zeros((1, 16), np.int32)
        count[0, 2 * E_loc + 1] = 5
        oracle.check_fence_trace(ev, count)
    finally:
        ep.ep_proxy_stop(h)


def test_full_ring_with_no_consumer_times_out_instead_of_hanging(ep):
    h = _start(ep, num_proxy_threads=0, num_channels=1, ring_entries=2, spin_timeout_ms=50, num_src=1)
    try:
        ep.ep_host_push(h, 0, _w0(1, 0, 0, 0), 2048 >> 4, 0, 0)
        ep.ep_host_push(h, 0, _w0(1, 0, 0, 0), 2048 >> 4, 0, 0)
        t0 = time.time()
        with pytest.raises(ep.EPError) as ei:
            ep.ep_host_push(h, 0, _w0(1, 0, 0, 0), 2048 >> 4, 0, 0)
        assert ei.value.rc == ep.EP_ETIMEOUT and time.time() - t0 < 2
        assert ep.ep_stats(h)["device_error"] == ep.EP_ETIMEOUT
        with pytest.raises(ep.EPError):
            ep.ep_wait(h)                                        # sticky
    finally:
        ep.ep_proxy_stop(h)


def test_wait_times_out_when_an_atomic_never_gets_its_writes(ep):
    h = _start(ep, spin_timeout_ms=100, num_src=1)
    try:
        ep.ep_host_expect_atomics(h, 1)
        _atomic(ep, h, 1, 0, 1, 0, 3, 4)
        _write(ep, h, 1, 0, 1, 0, 2, 2048, 0)                    # only 2 of the 3 rows ever arrive
        _write(ep, h, 1, 0, 1, 1, 32, 2048, 2)                   # rows for another expert must not count
        with pytest.raises(ep.EPError) as ei:
            ep.ep_wait(h)
        assert ei.value.rc == ep.EP_ETIMEOUT
        assert ep.ep_stats(h)["atomics_applied"] == 0 and ep.ep_counters(h, 1, 16).sum() == 0
        _write(ep, h, 1, 0, 1, 0, 1, 2048, 40)                   # the missing row
        ep.ep_wait(h)
        assert ep.ep_counters(h, 1, 16)[0, 4] == 3
    finally:
        ep.ep_proxy_stop(h)


def test_config_validation(ep):
    ok = dict(num_ranks=4, num_experts=16, top_k=2, hidden=1024, max_tokens=64, flags=ep.EP_FLAG_HOST_ONLY)
    for bad in (dict(num_ranks=0), dict(num_experts=18), dict(num_experts=2048, num_ranks=1), dict(top_k=0),
                dict(hidden=100), dict(max_tokens=0), dict(max_tokens=1 << 19), dict(ring_entries=48),
                dict(ring_entries=1), dict(num_channels=0), dict(num_channels=65), dict(num_proxy_threads=17),
                dict(self_rank=4), dict(num_src=0), dict(heap_rows=1 << 40)):
        with pytest.raises(ep.EPError) as ei:
            ep.ep_proxy_start(**{**ok, **bad})
        assert ei.value.rc == ep.EP_EINVAL, bad
    h = ep.ep_proxy_start(**ok)
    ep.ep_proxy_stop(h)


def test_reset_stats_and_repeat(ep):
    h = _start(ep, num_src=1)
    try:
        for rep in range(3):
            ep.ep_host_expect_atomics(h, 1)
            _write(ep, h, 0, 0, 0, 1, 7, 2048, 0)
            _atomic(ep, h, 0, 0, 0, 1, 7, 4)
            ep.ep_wait(h)
            st = ep.ep_stats(h)
            assert st["cmds"] == 2 and st["write_rows"] == 7 and st["first_poll_ns"] <= st["last_apply_ns"]
            assert ep.ep_counters(h, 1, 16)[0, 1] == 7
            ep.ep_reset_stats(h)
            assert ep.ep_stats(h)["cmds"] == 0 and ep.ep_counters(h, 1, 16).sum() == 0
    finally:
        ep.ep_proxy_stop(h)


# ------------------------------------------ high-throughput style: per-channel sequence order
def _owrite(ep, h, ch, src, dr, seq, rows, rb, row0):
    return ep.ep_host_push(h, ch, _w0(5, src, dr, 0), ((rows - 1) << 26) | ((rows * rb) >> 4), seq, (row0 * rb) >> 4)


def _oatomic(ep, h, ch, src, dr, seq, value, R):
    return ep.ep_host_push(h, ch, _w0(6, src, dr, 0), value, seq, src * R + dr)


def _drain_all(ep, h, C):
    ids = [ep.ep_host_push(h, c, _w0(3, 0, 0, 0), 0, 0, 0) for c in range(C)]
    deadline = time.time() + 5
    for c, i in enumerate(ids):
        while not ep.ep_host_check_completion(h, c, i):
            assert time.time() < deadline
            time.sleep(0.0005)


@pytest.mark.parametrize("window", [0, 5, 200])
def test_partial_ordering_per_communication_channel(ep, oracle, window):
    """Messages of one communication channel (source -> destination rank) are pushed in a
    scrambled order and additionally reordered in flight; the receiver applies them strictly by
    sequence number, channel by channel, and the tail counters end at the rows announced."""
    R, C, rb = 4, 4, 2048
    rng = np.random.default_rng(window)
    h = _start(ep, reorder_window=window, reorder_seed=7, num_src=2)
    try:
        want_tail = np.zeros((2, R), np.int64)
        msgs = []
        for s in range(2):
            for dr in range(R):
                n = int(rng.integers(1, 40))
                row = 0
                for i in range(n):
                    rows = int(rng.integers(1, 33))
                    msgs.append(("w", s, dr, 2 * i, rows, row))
                    msgs.append(("a", s, dr, 2 * i + 1, rows))
                    row += rows
                    want_tail[s, dr] += rows
        # scramble within a sliding window so the FIFO order differs from the sequence order
        order = np.arange(len(msgs))
        for i in range(0, len(order) - 6, 3):
            rng.shuffle(order[i:i + 6])
        for j in order:
            m = msgs[j]
            if m[0] == "w":
                _owrite(ep, h, m[2] % C, m[1], m[2], m[3], m[4], rb, m[5])
            else:
                _oatomic(ep, h, m[2] % C, m[1], m[2], m[3], m[4], R)
        _drain_all(ep, h, C)
        st = ep.ep_stats(h)
        assert st["rejected"] == 0 and st["proxy_error"] == 0 and st["drains"] == C
        assert np.array_equal(ep.ep_tail_counters(h, 2, R), want_tail)
        res = oracle.check_order_trace(ep.ep_event_log(h))
        assert res["applied"] == len(msgs) and res["waited"] == st["ordered_parked"] and res["waited"] > 0
    finally:
        ep.ep_proxy_stop(h)


def test_partial_ordering_sequence_gap_is_reported(ep, oracle):
    """If a sequence number never arrives, everything behind it on that channel stays in the
    control buffer; the Drain reports the gap, other channels are unaffected."""
    R, C = 4, 4
    h = _start(ep, num_src=1, spin_timeout_ms=300)
    try:
        _owrite(ep, h, 1, 0, 1, 0, 4, 2048, 0)
        _oatomic(ep, h, 1, 0, 1, 1, 4, R)
        _oatomic(ep, h, 1, 0, 1, 3, 9, R)                        # 2 is missing
        _owrite(ep, h, 2, 0, 2, 0, 7, 2048, 0)
        _oatomic(ep, h, 2, 0, 2, 1, 7, R)
        _drain_all(ep, h, C)
        tails = ep.ep_tail_counters(h, 1, R)
        assert tails[0].tolist() == [0, 4, 7, 0]                 # the 9 rows behind the gap were never announced
        assert ep.ep_stats(h)["proxy_error"] == ep.EP_ESTATE
        with pytest.raises(ep.EPError):
            ep.ep_wait(h)
        with pytest.raises(AssertionError, match="never applied"):
            oracle.check_order_trace(ep.ep_event_log(h))
    finally:
        ep.ep_proxy_stop(h)


def test_partial_ordering_long_run_ahead_of_a_late_message(ep, oracle):
    """The first message of a channel arrives last, behind 1400 later ones (more than the receiver's
    reorder window holds, so both the window and its overflow are in play), twice in a row on the same
    channel; nothing is applied before it, everything in sequence after it."""
    R = 4
    h = _start(ep, num_src=1, ring_entries=4096)
    try:
        base = 0
        for rnd, n in enumerate((1400, 700)):
            for q in range(2, n, 2):
                _owrite(ep, h, 2, 0, 2, base + q, 1, 2048, 0)
                _oatomic(ep, h, 2, 0, 2, base + q + 1, 3, R)
            _oatomic(ep, h, 2, 0, 2, base + 1, 3, R)
            time.sleep(0.05)
            assert ep.ep_tail_counters(h, 1, R)[0, 2] == rnd * 2100   # nothing new announced yet
            _owrite(ep, h, 2, 0, 2, base, 1, 2048, 0)                     # the late one
            _drain_all(ep, h, 4)
            base += n
            assert ep.ep_tail_counters(h, 1, R)[0, 2] == 3 * base // 2
        st = ep.ep_stats(h)
        assert st["proxy_error"] == 0 and st["rejected"] == 0 and st["ordered_parked"] == 1399 + 699
        res = oracle.check_order_trace(ep.ep_event_log(h))
        assert res["applied"] == 2100 and res["waited"] == 1399 + 699
    finally:
        ep.ep_proxy_stop(h)


def test_partial_ordering_sequence_numbers_wrap_16_bits(ep, oracle):
    """The immediate carries 16 bits of the number; the receiver rebuilds the full value."""
    R = 4
    h = _start(ep, num_src=1, reorder_window=16, reorder_seed=3, flags=ep.EP_FLAG_HOST_ONLY)
    try:
        n = 70000
        for q in range(0, n, 2):
            _owrite(ep, h, 3, 0, 3, q, 1, 2048, 0)
            _oatomic(ep, h, 3, 0, 3, q + 1, 1, R)
        _drain_all(ep, h, 4)
        assert ep.ep_tail_counters(h, 1, R)[0, 3] == n // 2
        assert ep.ep_stats(h)["proxy_error"] == 0
    finally:
        ep.ep_proxy_stop(h)


# ------------------------------------------------------------------- Barrier across processes
def _barrier_peer(name, delay, rounds, q):
    """Child process: its own handle and proxy; pushes `rounds` Barrier commands."""
    import time as _t
    import paper_2512_19849_amd as ep_
    h = ep_.ep_proxy_start(4, 16, 2, 1024, 64, num_channels=1, ring_entries=8, num_proxy_threads=1,
                           spin_timeout_ms=5000, flags=ep_.EP_FLAG_HOST_ONLY, barrier_peers=2, barrier_name=name)
    out = []
    try:
        for r in range(rounds):
            _t.sleep(delay)
            t_push = _t.time()
            i = ep_.ep_host_push(h, 0, 4 << 28, 0, 0, 0)
            while not ep_.ep_host_check_completion(h, 0, i):
                _t.sleep(0.0005)
            out.append((t_push, _t.time()))
        st = ep_.ep_stats(h)
        q.put((out, st["barriers"], st["proxy_error"]))
    finally:
        ep_.ep_proxy_stop(h)


def test_barrier_releases_only_when_every_peer_process_has_entered(ep):
    """Two processes share a named barrier: a Barrier command is popped only after
    both proxies have received one; three generations in a row."""
    import multiprocessing as mp
    ctx = mp.get_context("spawn")
    name = f"t{os.getpid()}"
    q = ctx.Queue()
    rounds, delay = 3, 0.25
    child = ctx.Process(target=_barrier_peer, args=(name, delay, rounds, q))
    child.start()
    h = _start(ep, num_channels=1, num_proxy_threads=1, num_src=1, barrier_peers=2, barrier_name=name,
               spin_timeout_ms=20000)
    try:
        mine = []
        for r in range(rounds):
            t_push = time.time()
            i = ep.ep_host_push(h, 0, _w0(4, 0, 0, 0), 0, 0, 0)
            time.sleep(0.05)
            deadline = time.time() + 20
            while not ep.ep_host_check_completion(h, 0, i):
                assert time.time() < deadline
                time.sleep(0.0005)
            mine.append((t_push, time.time()))
        theirs, nbar, perr = q.get(timeout=30)
        child.join(timeout=30)
        assert child.exitcode == 0 and nbar == rounds and perr == 0
        st = ep.ep_stats(h)
        assert st["barriers"] == rounds and st["proxy_error"] == 0
        for (p0, d0), (p1, d1) in zip(mine, theirs):
            # nobody leaves before the later of the two pushes
            assert min(d0, d1) >= max(p0, p1) - 1e-3
        # the parent always pushes first and must have been held for about the child's delay
        assert all(d - p > 0.1 for p, d in mine[1:])
    finally:
        ep.ep_proxy_stop(h)
        if child.is_alive():
            child.terminate()


def test_barrier_alone_and_timeout(ep):
    h = _start(ep, num_channels=1, num_proxy_threads=1, num_src=1)          # no peers: trivially satisfied
    try:
        i = ep.ep_host_push(h, 0, _w0(4, 0, 0, 0), 0, 0, 0)
        deadline = time.time() + 5
        while not ep.ep_host_check_completion(h, 0, i):
            assert time.time() < deadline
        assert ep.ep_stats(h)["barriers"] == 1
    finally:
        ep.ep_proxy_stop(h)
    h = _start(ep, num_channels=1, num_proxy_threads=1, num_src=1, barrier_peers=2,
               barrier_name=f"lonely{os.getpid()}", spin_timeout_ms=100)
    try:
        t0 = time.time()
        i = ep.ep_host_push(h, 0, _w0(4, 0, 0, 0), 0, 0, 0)
        while not ep.ep_host_check_completion(h, 0, i):
            assert time.time() - t0 < 5
        assert time.time() - t0 >= 0.09                                    # held for the bound, then given up
        assert ep.ep_stats(h)["proxy_error"] == ep.EP_ETIMEOUT
    finally:
        ep.ep_proxy_stop(h)
    with pytest.raises(ep.EPError):
        _start(ep, barrier_peers=2, barrier_name="")                       # peers need a name
    with pytest.raises(ep.EPError):
        _start(ep, barrier_peers=2, barrier_name="a/b")


# ------------------------------------------------ pacing and packing (Section 6)
class _Burst:
    """Lets a test queue a whole burst before the proxy sees any of it: the proxy thread is parked in
    a two-party Barrier (first command of the FIFO) that a second handle completes on release()."""

    def __init__(self, ep, name, **kw):
        self.ep = ep
        kw.update(num_proxy_threads=1, num_channels=1, num_src=1, ring_entries=2048, barrier_peers=2,
                  barrier_name=name, spin_timeout_ms=10000)
        self.h = _start(ep, **kw)
        self.peer = _start(ep, num_proxy_threads=1, num_channels=1, num_src=1, barrier_peers=2, barrier_name=name,
                           spin_timeout_ms=10000)
        ep.ep_host_push(self.h, 0, _w0(4, 0, 0, 0), 0, 0, 0)

    def release(self):
        self.ep.ep_host_push(self.peer, 0, _w0(4, 0, 0, 0), 0, 0, 0)

    def close(self):
        self.ep.ep_proxy_stop(self.h)
        self.ep.ep_proxy_stop(self.peer)


@pytest.mark.parametrize("limit,window", [(1, 0), (4, 64), (16, 1000), (3, 7)])
def test_pacing_bounds_the_messages_in_flight_per_destination(ep, oracle, limit, window):
    """With max_outstanding set, a proxy thread never has more than that many messages on their way to
    one destination rank; the rest wait at the sender, in order, and everything still arrives and
    passes the completion fence."""
    E_loc, rb = 4, 2048
    b = _Burst(ep, f"pace{limit}_{window}_{os.getpid()}", reorder_window=window, reorder_seed=3, max_outstanding=limit)
    h = b.h
    try:
        rng = np.random.default_rng(limit)
        count = np.zeros((1, 16), np.int64)
        ep.ep_host_expect_atomics(h, 16)
        for row in range(600):                                  # a burst, most of it to rank 2 (an incast)
            e = int(rng.choice([8, 9, 10, 11])) if rng.random() < 0.7 else int(rng.integers(16))
            _write(ep, h, 0, 0, e // E_loc, e % E_loc, 1, rb, row)
            count[0, e] += 1
        for e in range(16):
            _atomic(ep, h, 0, 0, e // E_loc, e % E_loc, int(count[0, e]), E_loc)
        b.release()
        ep.ep_wait(h)
        _drain_all(ep, h, 1)
        st = ep.ep_stats(h)
        assert st["rejected"] == 0 and st["proxy_error"] == 0 and st["atomics_applied"] == 16
        assert st["max_in_flight"] == limit if window else st["max_in_flight"] == 1
        assert (st["paced"] > 0) == (window > 0)
        ev = ep.ep_event_log(h)
        res = oracle.check_pacing_trace(ev, limit, E_loc)
        assert res["sent"] == 600 + 16 and res["peak"] == st["max_in_flight"]
        oracle.check_fence_trace(ev, count)
        assert np.array_equal(ep.ep_counters(h, 1, 16), count)
    finally:
        b.close()


def test_without_pacing_the_transport_fills_with_one_destination(ep, oracle):
    """The same kind of burst without a limit: as many messages in flight to the hot rank as the
    transport holds (what the limit is there to prevent); the checker rejects that trace for any
    smaller limit, and notices a send record that is missing."""
    b = _Burst(ep, f"nopace_{os.getpid()}", reorder_window=64)
    h = b.h
    try:
        ep.ep_host_expect_atomics(h, 1)
        for i in range(300):
            _write(ep, h, 0, 0, 2, 1, 1, 2048, i)
        _atomic(ep, h, 0, 0, 2, 1, 300, 4)
        b.release()
        ep.ep_wait(h)
        _drain_all(ep, h, 1)
        st = ep.ep_stats(h)
        assert st["max_in_flight"] == 65 and st["paced"] == 0
        ev = ep.ep_event_log(h)
        assert oracle.check_pacing_trace(ev, 0, 4)["peak"] == 65
        with pytest.raises(AssertionError, match="in flight to rank 2"):
            oracle.check_pacing_trace(ev, 64, 4)
        sent = np.nonzero((ev[:, 0] & 0xFF) == oracle.EV_SENT)[0]
        with pytest.raises(AssertionError, match="never sent|proxy counted"):
            oracle.check_pacing_trace(np.delete(ev, sent[0], axis=0), 0, 4)
    finally:
        b.close()


@pytest.mark.parametrize("pack,window", [(4, 0), (16, 9), (2, 0)])
def test_best_effort_packing_of_one_row_writes(ep, oracle, pack, window):
    """One-row Writes to consecutive destination offsets of one expert, polled in the same sweep, leave
    as one message of up to pack_rows rows; a gap or the expert's count Atomic closes a message, another
    expert's rows in between do not.  Rows, bytes and the fence are unaffected; the message count drops."""
    E_loc, rb = 4, 2048
    b = _Burst(ep, f"pack{pack}_{window}_{os.getpid()}", reorder_window=window, pack_rows=pack)
    h = b.h
    try:
        ep.ep_host_expect_atomics(h, 3)
        # expert 5: rows 0..19 contiguous; expert 6: rows 100,101 then a gap, 103; expert 7: a single row
        for i in range(20):
            _write(ep, h, 0, 0, 1, 1, 1, rb, i)
            if i == 3:
                _write(ep, h, 0, 0, 1, 2, 1, rb, 100)
        _write(ep, h, 0, 0, 1, 2, 1, rb, 101)
        _write(ep, h, 0, 0, 1, 2, 1, rb, 103)
        _write(ep, h, 0, 0, 1, 3, 1, rb, 200)
        _atomic(ep, h, 0, 0, 1, 1, 20, E_loc)
        _atomic(ep, h, 0, 0, 1, 2, 3, E_loc)
        _atomic(ep, h, 0, 0, 1, 3, 1, E_loc)
        b.release()
        ep.ep_wait(h)
        _drain_all(ep, h, 1)
        st = ep.ep_stats(h)
        assert st["writes"] == 24 and st["write_rows"] == 24 and st["write_bytes"] == 24 * rb
        assert st["atomics_applied"] == 3 and st["rejected"] == 0 and st["proxy_error"] == 0
        assert st["write_msgs"] == -(-20 // pack) + 2 + 1       # the whole burst is polled in one sweep
        ev = ep.ep_event_log(h)
        count = np.zeros((1, 16), np.int64)
        count[0, 5], count[0, 6], count[0, 7] = 20, 3, 1
        oracle.check_fence_trace(ev, count)
        wr = ev[(ev[:, 0] & 0xFF) == oracle.EV_WRITE]
        assert sorted(wr[wr[:, 2] == 5][:, 3].tolist(), reverse=True) == [pack] * (20 // pack) + ([20 % pack] if 20 % pack else [])
        assert sorted(wr[wr[:, 2] == 6][:, 3].tolist()) == [1, 2] and wr[wr[:, 2] == 7][:, 3].tolist() == [1]
        oracle.check_pacing_trace(ev, 0, E_loc)
    finally:
        b.close()


def test_packing_hold_time_spans_poll_sweeps_and_expires(ep, oracle):
    """With pack_hold_us an open message may wait for rows that arrive in later sweeps; once its time is
    up it leaves although nothing else arrives."""
    h = _start(ep, num_proxy_threads=1, num_channels=1, num_src=1, pack_rows=8, pack_hold_us=1000)
    try:
        for burst in range(2):
            for i in range(8):                                   # pushed one by one: the proxy sweeps in between
                _write(ep, h, 0, 0, 1, 1, 1, 2048, 8 * burst + i)
            time.sleep(0.005)
        _write(ep, h, 0, 0, 1, 1, 1, 2048, 16)                   # a lone row, nothing follows it
        deadline = time.time() + 5
        while ep.ep_stats(h)["write_rows"] < 17 or ep.ep_stats(h)["write_msgs"] < 3:
            assert time.time() < deadline, "the open message never left"
            time.sleep(0.001)
        time.sleep(0.01)
        ev = ep.ep_event_log(h)
        wr = ev[(ev[:, 0] & 0xFF) == oracle.EV_WRITE][:, 3].tolist()
        # normally [8, 8, 1]; a producer that stalls for more than the hold time splits a run, no more
        assert sum(wr) == 17 and max(wr) <= 8 and wr[-1] == 1 and len(wr) <= 9, wr
        ep.ep_host_expect_atomics(h, 1)
        _atomic(ep, h, 0, 0, 1, 1, 17, 4)
        ep.ep_wait(h)
        assert ep.ep_counters(h, 1, 16)[0, 5] == 17
    finally:
        ep.ep_proxy_stop(h)


def test_pacing_and_packing_configuration_is_validated(ep):
    for kw in (dict(max_outstanding=-1), dict(pack_rows=17), dict(pack_rows=-1), dict(pack_hold_us=1001)):
        with pytest.raises(ep.EPError) as ei:
            ep.ep_proxy_stop(_start(ep, **kw))
        assert ei.value.rc == ep.EP_EINVAL


# ------------------------------------- sender-side fence (Section 3.3, the alternative)
@pytest.mark.parametrize("window", [0, 8, 300])
def test_sender_side_fence_holds_atomics_at_the_sender(ep, oracle, window):
    """With EP_FLAG_SENDER_FENCE the sender half keeps a count Atomic until the rows it vouches for have
    arrived, so the receiver never buffers one - whatever the push order and the reordering in flight -
    and the counters come out the same.  Two rounds on the same experts: the second round's Atomic waits
    for the first to be applied."""
    E_loc, rb, C = 4, 2048, 4
    h = _start(ep, reorder_window=window, reorder_seed=21, num_src=1,
               flags=ep.EP_FLAG_HOST_ONLY | ep.EP_FLAG_LOG_CMDS | ep.EP_FLAG_LOG_EVENTS | ep.EP_FLAG_SENDER_FENCE)
    try:
        rng = np.random.default_rng(window)
        row = 0
        for rnd in range(2):
            count = rng.integers(0, 30, size=(1, 16))
            count[0, 3] = 0
            ep.ep_host_expect_atomics(h, 16)
            order = rng.permutation(16)
            for e in order[:8]:                                   # these Atomics come before their rows
                _atomic(ep, h, int(e) % C, 0, int(e) // E_loc, int(e) % E_loc, int(count[0, e]), E_loc)
            for e in rng.permutation(np.repeat(np.arange(16), count[0])):
                _write(ep, h, int(e) % C, 0, int(e) // E_loc, int(e) % E_loc, 1, rb, row)
                row += 1
            for e in order[8:]:
                _atomic(ep, h, int(e) % C, 0, int(e) // E_loc, int(e) % E_loc, int(count[0, e]), E_loc)
            ep.ep_wait(h)
            assert np.array_equal(ep.ep_counters(h, 1, 16), count)
        _drain_all(ep, h, C)
        st = ep.ep_stats(h)
        assert st["atomics_deferred"] == 0 and st["atomics_applied"] == 32 and st["proxy_error"] == 0
        assert st["sender_held"] >= 1
        ev = ep.ep_event_log(h)
        held = ev[(ev[:, 0] & 0xFF) == oracle.EV_SENDER_HELD]
        assert len(held) == st["sender_held"]
        # at the receiver every Atomic found its rows there already
        seen, waited = {}, 0
        for kind_thr, src, e, val in ev.tolist():
            kind = kind_thr & 0xFF
            if kind == oracle.EV_WRITE:
                seen[e] = seen.get(e, 0) + val
            elif kind == oracle.EV_ATOMIC_IN:
                waited += seen.get(e, 0) < val
            elif kind == oracle.EV_ATOMIC_APPLIED:
                seen[e] = seen.get(e, 0) - val
        assert waited == 0
        oracle.check_pacing_trace(ev, 0, E_loc)
    finally:
        ep.ep_proxy_stop(h)


def test_capture_ledger_and_expectations_on_a_host_handle(ep):
    """ep_captured / ep_expect are host bookkeeping: the ledger starts empty, ep_expect makes ep_wait wait for
    that many more count Atomics, negative numbers are refused."""
    h = _start(ep, num_channels=2, ring_entries=16, num_proxy_threads=1)
    try:
        assert ep.ep_captured(h) == (0, 0)
        ep.ep_expect(h, 1, 0)
        with pytest.raises(ep.EPError):
            ep.ep_expect(h, -1, 0)
        _atomic(ep, h, 0, 0, 0, 0, 0, 4)              # a count of zero rows for (source 0, rank 0, expert 0)
        ep.ep_wait(h)
        assert ep.ep_stats(h)["atomics_applied"] == 1
    finally:
        ep.ep_proxy_stop(h)


def test_profile_calls_refuse_a_host_only_handle(ep):
    h = _start(ep)
    try:
        with pytest.raises(ep.EPError):
            ep.ep_profile(h, True)
        with pytest.raises(ep.EPError):
            ep.ep_profile_read(h, 0)
    finally:
        ep.ep_proxy_stop(h)
