"""Pins for the command-stream side of the oracle (CPU only): the multiset of
transfer commands a dispatch must emit, the replay of a command log, and the
completion-fence checker.  Mistakes are planted on the CPU, in hand-built logs."""
import numpy as np
import pytest

import ep_inputs as g


def _encode(op, src, dst_rank, local, w1, src_off, dst_or_counter, gen=1, rb=None):
    """Build the four words by hand from the documented bit layout.  For a
    Write, w1 arrives as a byte count and rb is the bytes of one row."""
    w0 = (gen << 31) | (op << 28) | (src << 20) | (dst_rank << 12) | local
    if op == 1:
        w1 = ((w1 // rb - 1) << 26) | (w1 >> 4)
    w3 = (gen << 31) | (dst_or_counter >> 4 if op == 1 else dst_or_counter)
    return [w0, w1, src_off >> 4, w3]


def _log_from(ms, rb):
    rows = []
    for key, n in ms.items():
        rows += [_encode(*key, rb=rb)] * n
    return np.array(rows, np.uint32).reshape(-1, 4)


@pytest.mark.parametrize("payload", ["bf16", "fp8"])
def test_expected_per_token_commands_replay_to_the_dispatch_result(oracle, payload):
    cfg = g.config(1)
    idx, _ = g.routing(cfg)
    idx = g.mask_random(idx, 0.2, seed=2)
    x = g.activations(cfg)
    lay = oracle.layout(idx, cfg.E, cfg.R)
    rows = int((idx >= 0).sum())
    ms = oracle.expected_cmds(idx, lay, 0, cfg.E_loc, cfg.H, payload, "per_token")
    nW = sum(n for k, n in ms.items() if k[0] == oracle.OP_WRITE)
    nA = sum(n for k, n in ms.items() if k[0] == oracle.OP_ATOMIC)
    assert nW == rows and nA == cfg.E
    rb = oracle.row_bytes(cfg.H, payload)
    assert sum(k[4] * n for k, n in ms.items() if k[0] == oracle.OP_WRITE) == rows * rb
    assert sum(k[4] * n for k, n in ms.items() if k[0] == oracle.OP_ATOMIC) == rows
    log = _log_from(ms, rb)
    assert oracle.cmd_multiset(log) == ms                       # decode is the inverse of the layout
    if payload == "bf16":
        send = x.view(np.uint8).reshape(cfg.T, rb)
        want, _ = oracle.dispatch_bf16(x, idx, lay["dst_row"][0], cfg.E_loc, rows, fill=0xA5A5)
        want = want.view(np.uint8).reshape(rows, rb)
    else:
        q, s = oracle.quant_rows(x)
        send = np.zeros((cfg.T, rb), np.uint8)
        send[:, :cfg.H] = q
        send[:, cfg.H:cfg.H + cfg.H // 32] = s.view(np.uint8).reshape(cfg.T, -1)
        rq, rs, _ = oracle.dispatch_fp8(x, idx, lay["dst_row"][0], cfg.E_loc, rows)
        want = np.zeros((rows, rb), np.uint8)
        want[:, :cfg.H] = rq
        want[:, cfg.H:cfg.H + cfg.H // 32] = rs.view(np.uint8).reshape(rows, -1)
    heap, hits = oracle.replay_writes_per_token(log, send, rows)
    assert (hits == 1).all()
    assert np.array_equal(heap[:, :want.shape[1]], want)


def test_fp8_message_rows_are_codes_then_scales_then_padding(oracle):
    """The message a token travels as when the proxy moves FP8 rows: built here by hand from the quantiser's
    outputs, byte for byte, for a row length with padding (H = 128 -> 132 -> 144) and one without."""
    rng = np.random.default_rng(5)
    for H in (128, 1024):
        rows = 7
        q = rng.integers(0, 255, (rows, H), dtype=np.uint8)
        s = rng.standard_normal((rows, H // 128)).astype(np.float32)
        m = oracle.fp8_message_rows(q, s)
        rb = oracle.row_bytes(H, "fp8")
        assert m.shape == (rows, rb) and m.dtype == np.uint8
        for r in range(rows):
            want = bytes(q[r]) + b"".join(np.float32(v).tobytes() for v in s[r])
            assert bytes(m[r, :len(want)]) == want and not m[r, len(want):].any()
        q2, s2 = oracle.fp8_split_messages(m, H)
        assert np.array_equal(q2, q) and np.array_equal(s2.view(np.uint32), s.view(np.uint32))


def test_row_bytes(oracle):
    assert oracle.row_bytes(7168, "bf16") == 14336
    assert oracle.row_bytes(7168, "fp8") == 7168 + 224          # the paper's "7 KB" token
    assert oracle.row_bytes(128, "fp8") == 144                  # 132 padded to the 16-byte granule


def test_expected_chunk_commands_tile_every_expert(oracle):
    cfg = g.config(4)
    idx, _ = g.routing(cfg, 0, 300)
    lay = oracle.layout(idx, cfg.E, cfg.R)
    ms = oracle.expected_cmds(idx, lay, 0, cfg.E_loc, cfg.H, "bf16", "chunk32")
    nW = sum(n for k, n in ms.items() if k[0] == oracle.OP_WRITE)
    assert nW == int(np.ceil(lay["count"][0] / 32).sum())
    log = _log_from(ms, 14336)
    oracle.check_chunk_cover(log, lay, 0, cfg.E_loc, oracle.row_bytes(cfg.H, "bf16"))
    # planted mistakes: a dropped chunk, a chunk that crosses into the next expert
    writes = [i for i, w in enumerate(log) if oracle.decode_cmd(w)["op"] == oracle.OP_WRITE]
    with pytest.raises(AssertionError):
        oracle.check_chunk_cover(np.delete(log, writes[3], axis=0), lay, 0, cfg.E_loc, 14336)
    bad = log.copy()
    bad[writes[0], 1] += (1 << 26) + (14336 >> 4)
    with pytest.raises(AssertionError):
        oracle.check_chunk_cover(bad, lay, 0, cfg.E_loc, 14336)
    # filter keeps only one rank's experts
    ms2 = oracle.expected_cmds(idx, lay, 0, cfg.E_loc, cfg.H, "bf16", "chunk32", rank_filter=3)
    assert all(k[2] == 3 for k in ms2)
    assert sum(n for k, n in ms2.items() if k[0] == oracle.OP_ATOMIC) == cfg.E_loc


def test_replay_rejects_out_of_region_commands(oracle):
    send = np.zeros((4, 64), np.uint8)
    ok = np.array([_encode(1, 0, 0, 0, 64, 64, 128, rb=64)], np.uint32)
    oracle.replay_writes_per_token(ok, send, 3)
    for bad in (_encode(1, 0, 0, 0, 64, 64 * 4, 0, rb=64), _encode(1, 0, 0, 0, 64, 0, 64 * 3, rb=64),
                _encode(1, 0, 0, 0, 48, 0, 0, rb=48), _encode(1, 0, 0, 0, 128, 0, 0, rb=128)):
        with pytest.raises(ValueError):
            oracle.replay_writes_per_token(np.array([bad], np.uint32), send, 3)


def _ev(kind, src, e, val, thr=0):
    return [kind | (thr << 8), src, e, val]


def test_fence_checker_accepts_valid_and_catches_planted_violations(oracle):
    count = np.array([[2, 1, 0]], np.int32)
    W, A, AP = oracle.EV_WRITE, oracle.EV_ATOMIC_IN, oracle.EV_ATOMIC_APPLIED
    good = [_ev(A, 0, 0, 2), _ev(W, 0, 0, 1), _ev(W, 0, 1, 1), _ev(A, 0, 1, 1), _ev(AP, 0, 1, 1),
            _ev(W, 0, 0, 1), _ev(AP, 0, 0, 2), _ev(A, 0, 2, 0), _ev(AP, 0, 2, 0)]
    r = oracle.check_fence_trace(np.array(good, np.uint32), count)
    assert r == dict(waited=1, applied=3)
    # applied before its writes arrived (writes to another expert must not count)
    early = [_ev(A, 0, 0, 2), _ev(W, 0, 0, 1), _ev(W, 0, 1, 1), _ev(AP, 0, 0, 2), _ev(W, 0, 0, 1)]
    with pytest.raises(AssertionError, match="fence violated"):
        oracle.check_fence_trace(np.array(early, np.uint32), count)
    # never applied
    with pytest.raises(AssertionError, match="never applied"):
        oracle.check_fence_trace(np.array(good[:6], np.uint32), count)
    # applied without having been delivered
    with pytest.raises(AssertionError, match="never delivered"):
        oracle.check_fence_trace(np.array([_ev(W, 0, 1, 1), _ev(AP, 0, 1, 1)], np.uint32), count)
    # wrong final value
    wrong = [_ev(W, 0, 1, 1), _ev(A, 0, 1, 1), _ev(AP, 0, 1, 1)]
    with pytest.raises(AssertionError, match="layout says"):
        oracle.check_fence_trace(np.array(wrong, np.uint32), np.array([[0, 2, 0]], np.int32))
    # one (src, expert) handled by two threads breaks the share-nothing rule
    two = [_ev(W, 0, 1, 1, thr=0), _ev(A, 0, 1, 1, thr=1)]
    with pytest.raises(AssertionError, match="two threads"):
        oracle.check_fence_trace(np.array(two, np.uint32), count)


def test_order_trace_checker_accepts_valid_and_catches_planted_violations(oracle):
    WI, AI, WA, AA = (oracle.EV_ORD_WRITE_IN, oracle.EV_ORD_ATOMIC_IN, oracle.EV_ORD_WRITE_APPLIED,
                      oracle.EV_ORD_ATOMIC_APPLIED)
    # channel (0,1): atomic 1 arrives before write 0; channel (0,2) in order and independent
    good = [_ev(AI, 0, 1, 1), _ev(WI, 0, 2, 0), _ev(WA, 0, 2, 0), _ev(WI, 0, 1, 0), _ev(WA, 0, 1, 0),
            _ev(AA, 0, 1, 1), _ev(AI, 0, 2, 1), _ev(AA, 0, 2, 1)]
    assert oracle.check_order_trace(np.array(good, np.uint32)) == dict(applied=4, waited=1)
    # an atomic applied while an earlier message of its channel is still missing
    early = [_ev(AI, 0, 1, 1), _ev(AA, 0, 1, 1), _ev(WI, 0, 1, 0), _ev(WA, 0, 1, 0)]
    with pytest.raises(AssertionError, match="out of order"):
        oracle.check_order_trace(np.array(early, np.uint32))
    with pytest.raises(AssertionError, match="before it was delivered"):
        oracle.check_order_trace(np.array([_ev(WA, 0, 1, 0)], np.uint32))
    with pytest.raises(AssertionError, match="never applied"):
        oracle.check_order_trace(np.array(good[:5], np.uint32))
    with pytest.raises(AssertionError, match="delivered twice"):
        oracle.check_order_trace(np.array([_ev(WI, 0, 1, 0), _ev(WI, 0, 1, 0)], np.uint32))
    with pytest.raises(AssertionError, match="wrong kind"):
        oracle.check_order_trace(np.array([_ev(WI, 0, 1, 0), _ev(AA, 0, 1, 0)], np.uint32))
    # a run that starts later (second dispatch on the same handle)
    later = [_ev(WI, 0, 1, 6), _ev(WA, 0, 1, 6)]
    assert oracle.check_order_trace(np.array(later, np.uint32), {(0, 1): 6})["applied"] == 1
    with pytest.raises(AssertionError):
        oracle.check_order_trace(np.array(later, np.uint32))


def test_ordered_command_checker(oracle):
    cfg = g.config(1)
    idx, _ = g.routing(cfg)
    lay = oracle.layout(idx, cfg.E, cfg.R)
    rb = oracle.row_bytes(cfg.H, "bf16")
    log, seq = [], {r: 0 for r in range(cfg.R)}
    for e in range(cfg.E):
        c, b = int(lay["count"][0, e]), int(lay["base"][0, e])
        dr, le = e // cfg.E_loc, e % cfg.E_loc
        for j in range(0, c, 32):
            n = min(32, c - j)
            q = seq[dr]
            seq[dr] += 2
            log.append([(1 << 31) | (5 << 28) | (dr << 12) | le, ((n - 1) << 26) | ((n * rb) >> 4), q,
                        (1 << 31) | (((b + j) * rb) >> 4)])
            log.append([(1 << 31) | (6 << 28) | (dr << 12), n, q + 1, (1 << 31) | dr])
    log = np.array(log, np.uint32)
    assert oracle.check_ordered_cmds(log, lay, 0, cfg.E_loc, rb) == seq
    bad = log.copy()
    bad[1, 1] += 1                                               # atomic value != rows of its write
    with pytest.raises(AssertionError):
        oracle.check_ordered_cmds(bad, lay, 0, cfg.E_loc, rb)
    with pytest.raises(AssertionError):
        oracle.check_ordered_cmds(np.delete(log, [2, 3], axis=0), lay, 0, cfg.E_loc, rb)   # a chunk is missing
    bad = log.copy()
    bad[0, 2], bad[2, 2] = bad[2, 2], bad[0, 2]                  # still a permutation of the numbers: allowed
    if (bad[0, 0] >> 12) & 0xFF == (bad[2, 0] >> 12) & 0xFF:
        with pytest.raises(AssertionError):                      # ...but then write n is no longer followed by atomic n+1
            oracle.check_ordered_cmds(bad, lay, 0, cfg.E_loc, rb)
