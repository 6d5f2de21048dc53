"""Pins for the oracle's FP8 quantiser and its combine (CPU only)."""
import os

import numpy as np
import pytest

import ep_inputs as g

GOLD = os.path.join(os.path.dirname(__file__), "golden")


# ----------------------------------------------------------- independent E4M3
def _e4m3_table():
    """All non-negative finite E4M3 values from the format definition
    (S.EEEE.MMM, bias 7, subnormals M*2^-9, top code 0x7F is NaN)."""
    vals = []
    for c in range(0x7F):
        ex, m = c >> 3, c & 7
        vals.append(m * 2.0 ** -9 if ex == 0 else (1 + m / 8) * 2.0 ** (ex - 7))
    return np.array(vals, np.float64)


def _table_search_encode(y: np.ndarray) -> np.ndarray:
    """Nearest table entry, ties to the even code, beyond the top -> 0x7E.
    Brute force by definition; independent of the oracle's arithmetic."""
    tab = _e4m3_table()
    y = np.asarray(y, np.float32)
    a = np.abs(y.astype(np.float64))
    hi = np.searchsorted(tab, a, side="left").clip(1, len(tab) - 1)
    lo = hi - 1
    dlo, dhi = a - tab[lo], tab[hi] - a
    code = np.where(dlo < dhi, lo, np.where(dhi < dlo, hi, np.where(lo % 2 == 0, lo, hi)))
    code = np.where(a >= tab[-1], 0x7E, code).astype(np.uint8)
    return code | (np.signbit(y).astype(np.uint8) << 7)


def test_e4m3_format_values_from_spec(oracle):
    for line in open(os.path.join(GOLD, "e4m3_format_values.txt")):
        line = line.split("#")[0].strip()
        if not line:
            continue
        val, code = line.split()
        assert oracle.e4m3_encode(float(val)) == int(code, 16), line
        assert oracle.e4m3_decode(int(code, 16)) == float(val), line


def test_e4m3_codes_round_trip_and_match_table(oracle):
    tab = _e4m3_table()
    for c in range(0x7F):
        assert oracle.e4m3_decode(c) == tab[c]
        assert oracle.e4m3_decode(c | 0x80) == -tab[c]
        assert oracle.e4m3_encode(tab[c]) == c
        assert oracle.e4m3_encode(-tab[c]) == (c | 0x80)
    assert np.isnan(oracle.e4m3_decode(0x7F)) and np.isnan(oracle.e4m3_decode(0xFF))


def test_e4m3_midpoints_go_to_even_and_saturate(oracle):
    tab = _e4m3_table()
    for c in range(0x7E):
        mid = np.float32((tab[c] + tab[c + 1]) / 2)          # exactly representable in fp32
        assert float(mid) == (tab[c] + tab[c + 1]) / 2
        want = c if c % 2 == 0 else c + 1
        assert oracle.e4m3_encode(float(mid)) == want
        assert oracle.e4m3_encode(float(np.nextafter(mid, np.float32(0)))) == c
        assert oracle.e4m3_encode(float(np.nextafter(mid, np.float32(1e9)))) == c + 1
    for v in (448.0, 463.99, 464.0, 480.0, 512.0, 1e30, 3.0e38):
        assert oracle.e4m3_encode(v) == 0x7E and oracle.e4m3_encode(-v) == 0xFE
    assert oracle.e4m3_encode(2.0 ** -10) == 0x00            # tie between 0 and 2^-9 -> even (0)
    assert oracle.e4m3_encode(-(2.0 ** -10)) == 0x80
    assert oracle.e4m3_encode(1e-30) == 0x00 and oracle.e4m3_encode(-1e-30) == 0x80


def test_e4m3_encode_exhaustive_bf16_times_inv_vs_table_search(oracle):
    """Every finite bf16 input times a set of fp32 reciprocal scales, against
    the brute-force table search."""
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    v = g.bf16_bits_to_f32(bits)
    v = v[np.isfinite(v)]
    invs = np.array([1.0, 448.0 / 3.0078125, 448.0 / 0.0123, 448.0 / 417.0, 0.37, 2.0 ** -20, 1.9e4], np.float32)
    for inv in invs:
        with np.errstate(over="ignore"):
            y = (v * inv).astype(np.float32)
        y = y[np.isfinite(y)]
        y = y[:: 3] if inv != 1.0 else y
        got = oracle.e4m3_encode_array(y)
        assert np.array_equal(got, _table_search_encode(y)), f"inv={inv}"


def test_e4m3_encode_agrees_with_torch_float8_cast(oracle):
    """Second opinion from a library: torch's float32 -> float8_e4m3fn cast
    (values clamped to +-448 first, since the library cast does not saturate)."""
    torch = pytest.importorskip("torch")
    if not hasattr(torch, "float8_e4m3fn"):
        pytest.skip("torch build has no float8_e4m3fn")
    rng = np.random.default_rng(3)
    y = np.concatenate([rng.normal(0, 100, 20000), rng.normal(0, 1, 20000), rng.normal(0, 0.01, 20000),
                        rng.uniform(-500, 500, 20000)]).astype(np.float32)
    t = torch.from_numpy(np.clip(y, -448, 448)).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    assert np.array_equal(oracle.e4m3_encode_array(y), t)


def test_quant_block_scale_amax_code_and_error_bound(oracle):
    cfg = g.config(3)
    x = g.activations(cfg)
    q, s = oracle.quant_rows(x)
    v = g.bf16_bits_to_f32(x).astype(np.float64).reshape(cfg.T, -1, 128)
    amax = np.abs(v).max(axis=2)
    # scale = amax/448 rounded once to fp32 (closed form, recomputed in fp64)
    assert np.array_equal(s, (amax / 448.0).astype(np.float32))
    qb = q.reshape(cfg.T, -1, 128)
    # the element with |v| = amax encodes to +-448
    am = np.abs(v).argmax(axis=2)
    top = np.take_along_axis(qb, am[..., None], axis=2)[..., 0]
    assert ((top & 0x7F) == 0x7E).all()
    # half-ulp bound of the round trip, per binade of y = v * 448/amax
    tab = np.concatenate([_e4m3_table(), [np.nan]])
    dec = np.where(qb & 0x80, -1.0, 1.0) * tab[(qb & 0x7F).astype(np.int64)]
    deq = dec * s.astype(np.float64)[..., None]
    yabs = np.abs(v) * (448.0 / amax)[..., None]
    half_ulp = np.where(yabs >= 2.0 ** -6, 2.0 ** (np.floor(np.log2(np.maximum(yabs, 1e-300))) - 4), 2.0 ** -10)
    bound = (amax / 448.0)[..., None] * half_ulp * (1 + 2.0 ** -20) + 1e-30
    assert (np.abs(deq - v) <= bound).all()
    assert (np.abs(deq - v) <= amax[..., None] / 28 * (1 + 2.0 ** -20) + 1e-30).all()
    # per-element definition through the independent table search
    inv = (np.float32(448.0) / amax.astype(np.float32)).astype(np.float32)
    y = (g.bf16_bits_to_f32(x).reshape(cfg.T, -1, 128) * inv[..., None]).astype(np.float32)
    assert np.array_equal(qb, _table_search_encode(y))


def test_quant_block_zero_and_tiny_blocks(oracle):
    zero = np.zeros(128, np.uint16)
    zero[5] = 0x8000                                            # -0.0
    q, s = oracle.quant_block(zero)
    assert s == 1.0 and q[5] == 0x80 and (np.delete(q, 5) == 0).all()
    tiny = np.full(128, 0x0080, np.uint16)                      # smallest bf16 normal, 2^-126
    tiny[1] = 0x8080
    q, s = oracle.quant_block(tiny)
    assert s == 1.0 and q[0] == 0x00 and q[1] == 0x80
    # amax just at/above the threshold 2^-100 takes the common path: the peak encodes to 448
    blk = np.zeros(128, np.uint16)
    blk[0] = g.f32_to_bf16_bits(np.array([2.0 ** -100], np.float32))[0]
    blk[1] = g.f32_to_bf16_bits(np.array([-(2.0 ** -101)], np.float32))[0]
    q, s = oracle.quant_block(blk)
    assert s == np.float32(2.0 ** -100) / np.float32(448) and q[0] == 0x7E and q[1] == (0x80 | 0x76)
    below = np.zeros(128, np.uint16)
    below[0] = g.f32_to_bf16_bits(np.array([2.0 ** -101], np.float32))[0]
    q, s = oracle.quant_block(below)
    assert s == 1.0 and (q == 0).all()


def test_dispatch_fp8_rows_equal_quantised_source(oracle):
    cfg = g.config(3)
    idx, _ = g.routing(cfg)
    idx = g.mask_random(idx, 0.2, seed=4)
    x = g.activations(cfg)
    lay = oracle.layout(idx, cfg.E, cfg.R)
    rows = int((idx >= 0).sum())
    rq, rs, wc = oracle.dispatch_fp8(x, idx, lay["dst_row"][0], cfg.E_loc, rows + 3)
    q, s = oracle.quant_rows(x)
    assert (wc[:rows] == 1).all() and (wc[rows:] == 0).all()
    assert (rq[rows:] == 0xA5).all() and (rs[rows:] == -1.0).all()
    for t in range(cfg.T):
        for k in range(cfg.K):
            r = lay["dst_row"][0, t, k]
            if r >= 0:
                assert np.array_equal(rq[r], q[t]) and np.array_equal(rs[r], s[t])


def test_dequant_is_decode_times_scale_rounded_to_bf16(oracle):
    cfg = g.config(3)
    x = g.activations(cfg)[:8]
    q, s = oracle.quant_rows(x)
    y = oracle.dequant_rows(q, s)
    tab = np.concatenate([_e4m3_table(), [np.nan]])
    dec = (np.where(q & 0x80, -1.0, 1.0) * tab[(q & 0x7F).astype(np.int64)]).astype(np.float32)
    prod = (dec * np.repeat(s, 128, axis=1)).astype(np.float32)
    assert np.array_equal(y, g.f32_to_bf16_bits(prod))


# ------------------------------------------------------------------ combine
def _setup(oracle, cid, T=None, mask=0.0):
    cfg = g.config(cid)
    idx, w = g.routing(cfg, 0, T)
    if mask:
        idx = g.mask_random(idx, mask, seed=11)
    x = g.activations(cfg, 0, T=T)
    lay = oracle.layout(idx, cfg.E, cfg.R)
    rows = int((idx >= 0).sum())
    recv, _ = oracle.dispatch_bf16(x, idx, lay["dst_row"][0], cfg.E_loc, rows)
    return cfg, idx, w, x, lay, recv


@pytest.mark.parametrize("cid,T,mask", [(1, None, 0.0), (1, None, 0.3), (4, 40, 0.0), (5, 33, 0.1)])
def test_combine_within_bound_of_fp64_definition(oracle, cid, T, mask):
    cfg, idx, w, x, lay, recv = _setup(oracle, cid, T, mask)
    y = g.activations(cfg, 0, tid=g.TID_Y, T=recv.shape[0])     # arbitrary expert outputs
    out = oracle.combine(y, w, lay["dst_row"][0])
    ref, mag = oracle.combine_f64(y, w, lay["dst_row"][0])
    # independent fp64 gather + einsum for the definition itself
    yf = g.bf16_bits_to_f32(y).astype(np.float64)
    dr = lay["dst_row"][0]
    gathered = np.where((dr >= 0)[..., None], yf[np.maximum(dr, 0)], 0.0)
    ref2 = np.einsum("tk,tkh->th", w.astype(np.float64), gathered)
    assert np.allclose(ref, ref2, rtol=1e-13, atol=1e-300)
    got = g.bf16_bits_to_f32(out).astype(np.float64)
    K = cfg.K
    bound = 2.0 ** -8 * np.abs(ref) + K * 2.0 ** -24 * mag * (1 + 2.0 ** -7) + 2.0 ** -133
    assert (np.abs(got - ref) <= bound).all()
    # a correctly rounded fp64 sum is at most one bf16 step away
    near = g.f32_to_bf16_bits(ref.astype(np.float32))
    assert oracle.bf16_ulp_distance(out, near).max() <= 1


def test_combine_identity_expert_k1_is_bit_exact_permutation_inverse(oracle):
    cfg = g.config(1, K=1)
    idx, _ = g.routing(cfg)
    x = g.activations(cfg)
    lay = oracle.layout(idx, cfg.E, cfg.R)
    recv, _ = oracle.dispatch_bf16(x, idx, lay["dst_row"][0], cfg.E_loc, idx.size)
    out = oracle.combine(recv, np.ones((cfg.T, 1), np.float32), lay["dst_row"][0])
    assert np.array_equal(out, x)


def test_combine_round_trip_scales_input_by_weight_sum(oracle):
    cfg, idx, w, x, lay, recv = _setup(oracle, 1)
    out = oracle.combine(recv, w, lay["dst_row"][0])
    xf = g.bf16_bits_to_f32(x).astype(np.float64)
    want = xf * w.astype(np.float64).sum(1, keepdims=True)
    got = g.bf16_bits_to_f32(out).astype(np.float64)
    assert (np.abs(got - want) <= 2.0 ** -8 * np.abs(want) * (1 + 2.0 ** -10) + 2.0 ** -133).all()
    assert oracle.bf16_ulp_distance(out, x).max() <= 1          # weights renormalised: sum = 1 +- 2^-23


def test_combine_fixed_k_order_and_fused_multiply_add(oracle):
    """The accumulation is the k-ascending fmaf chain in fp32: reproduce it
    with exact rational arithmetic rounded step by step."""
    from fractions import Fraction
    rng = np.random.default_rng(0)
    K, H = 4, 64
    y = g.f32_to_bf16_bits(rng.normal(0, 1, (K, H)).astype(np.float32))
    w = rng.normal(0, 1, (1, K)).astype(np.float32)
    dr = np.arange(K, dtype=np.int32)[None]
    out = oracle.combine(y, w, dr)
    yf = g.bf16_bits_to_f32(y)
    want = np.zeros(H, np.float32)
    for h in range(H):
        acc = Fraction(0)
        for k in range(K):
            exact = Fraction(float(w[0, k])) * Fraction(float(yf[k, h])) + acc
            acc = Fraction(float(np.float32(float(exact))))     # one rounding per fused step
        want[h] = np.float32(float(acc))
    assert np.array_equal(out[0], g.f32_to_bf16_bits(want))
    # order pin: (1 - 1) + 2^-30 = 2^-30 in ascending k, but (1 + 2^-30) - 1 = 0
    one, tiny = 0x3F80, int(g.f32_to_bf16_bits(np.array([2.0 ** -30], np.float32))[0])
    yo = np.array([[one], [one], [tiny]], np.uint16)
    dr3 = np.arange(3, dtype=np.int32)[None]
    asc = oracle.combine(yo, np.array([[1.0, -1.0, 1.0]], np.float32), dr3)
    assert asc[0, 0] == tiny
    swapped = oracle.combine(yo[[0, 2, 1]], np.array([[1.0, 1.0, -1.0]], np.float32), dr3)
    assert swapped[0, 0] == 0
    # fusion pin: (1+2^-23)*(1+2^-7) - (1+2^-7) keeps the 2^-30 term only when the product is not rounded
    yb = int(g.f32_to_bf16_bits(np.array([1 + 2.0 ** -7], np.float32))[0])
    yf2 = np.array([[yb], [yb]], np.uint16)
    wf = np.array([[-1.0, np.float32(1 + 2.0 ** -23)]], np.float32)
    fused = oracle.combine(yf2, wf, np.arange(2, dtype=np.int32)[None])
    assert fused[0, 0] == int(g.f32_to_bf16_bits(np.array([2.0 ** -23 * (1 + 2.0 ** -7)], np.float32))[0])
    assert fused[0, 0] != int(g.f32_to_bf16_bits(np.array([2.0 ** -23], np.float32))[0])


def test_combine_linearity_permutation_masking(oracle):
    cfg, idx, w, x, lay, recv = _setup(oracle, 1, mask=0.25)
    dr = lay["dst_row"][0]
    out = oracle.combine(recv, w, dr)
    # doubling all weights doubles the result exactly (power of two)
    out2 = oracle.combine(recv, (2 * w).astype(np.float32), dr)
    assert np.array_equal(g.bf16_bits_to_f32(out2), 2 * g.bf16_bits_to_f32(out))
    # permuting tokens permutes the output
    perm = np.random.default_rng(1).permutation(cfg.T)
    outp = oracle.combine(recv, w[perm], dr[perm])
    assert np.array_equal(outp, out[perm])
    # a token with every k masked yields +0
    dr0 = dr.copy()
    dr0[3] = -1
    assert (oracle.combine(recv, w, dr0)[3] == 0).all()
    # masked k contribute nothing: zeroing their weight changes nothing
    wz = w.copy()
    wz[dr < 0] = 123.0
    assert np.array_equal(oracle.combine(recv, wz, dr), out)


def test_f32_to_bf16_rounding_pins(oracle):
    cases = {1.0: 0x3F80, 1.00390625: 0x3F80, 1.01171875: 0x3F82, 1.0078125: 0x3F81,
             -2.5: 0xC020, 0.0: 0x0000, 3.3895313892515355e38: 0x7F7F}
    # 1 + 2^-8 ties to even (down); 1 + 3*2^-8 ties to even (up)
    for v, b in cases.items():
        assert int(oracle.f32_to_bf16(np.array([v], np.float32))[0]) == b, v
    rng = np.random.default_rng(5)
    a = rng.normal(0, 10, 5000).astype(np.float32)
    assert np.array_equal(oracle.f32_to_bf16(a), g.f32_to_bf16_bits(a))
    torch = pytest.importorskip("torch")
    tb = torch.from_numpy(a).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(oracle.f32_to_bf16(a), tb)
